// LTI complex-diagonal scan for gfx950:  x_k = lambda (.) x_{k-1} + v_k  (Eq. 2 of the
// paper with a constant diagonal A; the recurrence of the S5 / LRU layers, Sec. 2.2.1).
//
// v and x are [B,L,P] with P contiguous, so the lanes run along P (coalesced 8-byte
// complex elements) and the time axis is cut into chunks that different workgroups take.
// Because lambda is constant the affine aggregate of a chunk is (lambda^len, end state
// from zero): only end states are stored.  Two launches.  The first scans every chunk from zero
// and, inside each workgroup (4 consecutive chunks), chains the end states through LDS.  The
// second rebuilds each chunk's true carry-in from the end states of the groups before it and its in-group
// prefix, rescans the chunk and writes x (the second read of v is served by the L2 / Infinity
// Cache at these sizes, so v comes from HBM once and x is written once).
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

constexpr int kLtiWaves = 4;                  // wavefronts per workgroup = consecutive chunks of one group
constexpr int kLtiThreads = kLtiWaves * 64;

// Lanes run along p (64 complex values = 512 contiguous bytes per time step); wavefront w of a workgroup takes
// chunk 4*group + w of the same (b, p-slab).
// APPLY = false: scan each chunk from zero; through LDS, the state entering each chunk if its group had started
//                from zero -> ws_S[b,c,p], and the group's end state -> ws_G[b,group,p].
// APPLY = true : carry-in = (x0 pushed through the groups before, Horner over the group end states) pushed
//                through the w chunks before this one in its group, plus ws_S; then rescan and store x.
template <bool APPLY>
__global__ __launch_bounds__(kLtiThreads) void k_lti_chunk(const LtiParams p) {
    __shared__ float2 sS[kLtiWaves][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int pp = blockIdx.x * 64 + lane;
    const bool okp = pp < p.P;
    const int grp = blockIdx.y, b = blockIdx.z;
    const int c = grp * kLtiWaves + w;
    const bool okc = c < p.nchunks;
    const int64_t k0 = (int64_t)c * p.chunk;
    const int64_t k1 = (k0 + p.chunk < p.L) ? k0 + p.chunk : p.L;
    const float2 lam = okp ? p.lambda[pp] : make_float2(0.0f, 0.0f);
    const float2 lp = cpow(lam, p.chunk);                        // every chunk but the very last is full
    float2 x = make_float2(0.0f, 0.0f);
    if (APPLY && okp && okc) {
        if (p.x0) x = p.x0[(int64_t)b * p.P + pp];
        if (p.nchunks > 1) {
            const float2 lg = cpow(lp, kLtiWaves);
            const float2 *G = p.ws_G + (int64_t)b * p.ngroups * p.P + pp;
            for (int g = 0; g < grp; ++g) x = cfma(lg, x, G[(int64_t)g * p.P]);
            x = cfma(cpow(lp, w), x, p.ws_S[((int64_t)b * p.nchunks + c) * p.P + pp]);
        }
    }
    if (okp && okc) {
        const float2 *v = p.v + ((int64_t)b * p.L + k0) * p.P + pp;
        float2 *xo = p.x + ((int64_t)b * p.L + k0) * p.P + pp;
        const int64_t P = p.P;
        int64_t k = k0;
        for (; k + 8 <= k1; k += 8) {          // eight loads in flight per lane
            float2 vv[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) vv[i] = v[i * P];
            v += 8 * P;
#pragma unroll
            for (int i = 0; i < 8; ++i) { x = cfma(lam, x, vv[i]); if (APPLY) xo[i * P] = x; }
            if (APPLY) xo += 8 * P;
        }
        for (; k < k1; ++k) {
            x = cfma(lam, x, v[0]); v += P;
            if (APPLY) { xo[0] = x; xo += P; }
        }
        if (APPLY && p.x_last && k1 == p.L) p.x_last[(int64_t)b * p.P + pp] = x;
    }
    if (!APPLY) {
        sS[w][lane] = (okp && okc) ? x : make_float2(0.0f, 0.0f);
        __syncthreads();
        float2 e = make_float2(0.0f, 0.0f);
        for (int ww = 0; ww < w; ++ww) e = cfma(lp, e, sS[ww][lane]);
        if (okp && okc) p.ws_S[((int64_t)b * p.nchunks + c) * p.P + pp] = e;
        if (okp && w == kLtiWaves - 1) p.ws_G[((int64_t)b * p.ngroups + grp) * p.P + pp] = cfma(lp, e, sS[w][lane]);
    }
}

hipError_t launch_lti(const LtiParams &p, hipStream_t s) {
    dim3 grid((p.P + 63) / 64, p.ngroups, p.B);
    if (p.nchunks > 1) hipLaunchKernelGGL(k_lti_chunk<false>, grid, dim3(kLtiThreads), 0, s, p);
    hipLaunchKernelGGL(k_lti_chunk<true>, grid, dim3(kLtiThreads), 0, s, p);
    return hipGetLastError();
}

}  // namespace lrnnx
