// LTI complex-diagonal scan for gfx950:  x_k = lambda (.) x_{k-1} + v_k  (Eq. 2 of the
// paper with a constant diagonal A; the recurrence of the S5 / LRU layers, Sec. 2.2.1).
//
// v and x are [B,L,P] with P contiguous, so the lanes run along P (coalesced 8-byte
// complex elements) and the time axis is cut into chunks that different workgroups take.
// Because lambda is constant the affine aggregate of a chunk is (lambda^len, end state
// from zero): only the end state is stored.  Two launches: the end state of every chunk, then
// the rescan of every chunk from its true carry-in, which each workgroup first rebuilds for
// itself from the end states of the chunks before it (Horner in lambda^len over an L2-resident
// array; the second read of v is served by the L2 / Infinity Cache at these sizes).
#include "kernels.hpp"

namespace lrnnx {

__device__ __forceinline__ float2 cmul(float2 a, float2 b) {
    return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x);
}
__device__ __forceinline__ float2 cpow(float2 a, int64_t e) {            // a^e by repeated squaring
    float2 r = make_float2(1.0f, 0.0f);
    while (e > 0) {
        if (e & 1) r = cmul(r, a);
        a = cmul(a, a);
        e >>= 1;
    }
    return r;
}
__device__ __forceinline__ float2 cfma(float2 a, float2 b, float2 c) {   // a*b + c
    return make_float2(__builtin_fmaf(a.x, b.x, __builtin_fmaf(-a.y, b.y, c.x)),
                       __builtin_fmaf(a.x, b.y, __builtin_fmaf(a.y, b.x, c.y)));
}

constexpr int kLtiThreads = 256;

// APPLY = false: end state of each chunk started from zero -> ws_S[b,c,p].
// APPLY = true : carry-in = x0 pushed through the chunks before this one (from their end states), then
//                rescan and store x.
template <bool APPLY>
__global__ __launch_bounds__(kLtiThreads) void k_lti_chunk(const LtiParams p) {
    const int pp = blockIdx.x * kLtiThreads + threadIdx.x;
    if (pp >= p.P) return;
    const int c = blockIdx.y, b = blockIdx.z;
    const int64_t k0 = (int64_t)c * p.chunk;
    const int64_t k1 = (k0 + p.chunk < p.L) ? k0 + p.chunk : p.L;
    const float2 lam = p.lambda[pp];
    float2 x = make_float2(0.0f, 0.0f);
    if (APPLY) {
        if (p.x0) x = p.x0[(int64_t)b * p.P + pp];
        if (c > 0) {                                  // in_{j+1} = lambda^chunk in_j + S_j  (every chunk before c is full)
            const float2 lp = cpow(lam, p.chunk);
            const float2 *S = p.ws_S + (int64_t)b * p.nchunks * p.P + pp;
            int j = 0;
            for (; j + 4 <= c; j += 4) {
                const float2 s0 = S[(int64_t)j * p.P], s1 = S[(int64_t)(j + 1) * p.P];
                const float2 s2 = S[(int64_t)(j + 2) * p.P], s3 = S[(int64_t)(j + 3) * p.P];
                x = cfma(lp, x, s0); x = cfma(lp, x, s1); x = cfma(lp, x, s2); x = cfma(lp, x, s3);
            }
            for (; j < c; ++j) x = cfma(lp, x, S[(int64_t)j * p.P]);
        }
    }
    const float2 *v = p.v + ((int64_t)b * p.L + k0) * p.P + pp;
    float2 *xo = p.x + ((int64_t)b * p.L + k0) * p.P + pp;
    int64_t k = k0;
    for (; k + 4 <= k1; k += 4) {          // four loads in flight per lane
        float2 v0 = v[0], v1 = v[p.P], v2 = v[2 * (int64_t)p.P], v3 = v[3 * (int64_t)p.P];
        v += 4 * (int64_t)p.P;
        x = cfma(lam, x, v0); if (APPLY) xo[0] = x;
        x = cfma(lam, x, v1); if (APPLY) xo[p.P] = x;
        x = cfma(lam, x, v2); if (APPLY) xo[2 * (int64_t)p.P] = x;
        x = cfma(lam, x, v3); if (APPLY) xo[3 * (int64_t)p.P] = x;
        if (APPLY) xo += 4 * (int64_t)p.P;
    }
    for (; k < k1; ++k) {
        x = cfma(lam, x, v[0]); v += p.P;
        if (APPLY) { xo[0] = x; xo += p.P; }
    }
    if (!APPLY) p.ws_S[((int64_t)b * p.nchunks + c) * p.P + pp] = x;
    else if (p.x_last && k1 == p.L) p.x_last[(int64_t)b * p.P + pp] = x;
}

hipError_t launch_lti(const LtiParams &p, hipStream_t s) {
    dim3 grid((p.P + kLtiThreads - 1) / kLtiThreads, p.nchunks, p.B);
    if (p.nchunks > 1) {
        hipLaunchKernelGGL(k_lti_chunk<false>, grid, dim3(kLtiThreads), 0, s, p);
    }
    hipLaunchKernelGGL(k_lti_chunk<true>, grid, dim3(kLtiThreads), 0, s, p);
    return hipGetLastError();
}

}  // namespace lrnnx
