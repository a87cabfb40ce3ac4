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

// ---------------------------------------------------------------- single pass
// One launch, v read once and x written once.  A wavefront keeps its 32 steps of v in registers, scans them from
// zero, the 8 wavefronts of a workgroup (one group = 256 consecutive steps of 64 values of p) chain their end
// states through LDS, and the groups of one (b, p-slab) are chained through global memory: every group publishes
// its end-state-from-zero T_g (flag 1) as soon as it has it, then rebuilds its carry-in from the T_j of the groups
// before it, back to the last "anchor" group, whose true end state X (flag 2) it takes.  Every T_g is available
// after one load phase, so only anchors wait on a chain (one hop per 16 groups).  Workgroups are ordered so that a
// group is dispatched after the groups it looks back on (blockIdx.y = group), and every wait is bounded: after
// kSpinLimit polls a wavefront gives up, raises *err and finishes with a NaN carry rather than hang.
constexpr int kOneCS = 32;
constexpr int kOneBwdCS = 16;               // the adjoint also holds the saved states of its steps in registers
constexpr int kOneGW = 8;
constexpr int kSpinLimit = 1 << 22;
constexpr int kAnchor = 16;                  // every 16th group publishes its true end state

// BWD = false: the scan itself.  BWD = true: its adjoint (Sec. 2.2.1's recurrence differentiated): the same chain
// run over reversed time with the conjugate pole, g_k = gx_k + conj(lambda) g_{k+1}, reading gx through p.v and
// writing dv = g through p.x; each wavefront also loads the saved forward state before each of its steps and
// accumulates dlambda += conj(x_{k-1}) g_k, reduced over the workgroup in LDS and added to p.dlambda with one
// atomic pair per lane.  The scan position j maps to time k = j (forward) or k = L-1-j (adjoint).
template <int CS, bool BWD>
__global__ __launch_bounds__(kOneGW * 64) void k_lti_onepass(const LtiParams p) {
    __shared__ float2 sS[kOneGW][64];
    __shared__ float2 sCarry[64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int npslab = (p.P + 63) / 64;
    const int pslab = blockIdx.x % npslab, b = blockIdx.x / npslab;
    const int g = blockIdx.y;
    const int pp = pslab * 64 + lane;
    const bool okp = pp < p.P;
    const int64_t P = p.P;
    const int64_t k0 = ((int64_t)g * kOneGW + w) * CS;
    float2 lam = okp ? p.lambda[pp] : make_float2(0.0f, 0.0f);
    if (BWD) lam.y = -lam.y;
    const float2 lp = cpow(lam, CS), lg = cpow(lp, kOneGW);
    const int64_t tstep = BWD ? -P : P;                        // element stride between consecutive scan positions
    const int64_t first = ((int64_t)b * p.L + (BWD ? p.L - 1 - k0 : k0)) * P + pp;

    // ---- this wavefront's steps, all loads in flight at once
    float2 v[CS];
    const float2 *vp = p.v + first;
#pragma unroll
    for (int i = 0; i < CS; ++i)
        v[i] = (okp && k0 + i < p.L) ? vp[i * tstep] : make_float2(0.0f, 0.0f);
    float2 xprev[BWD ? CS : 1];
    if constexpr (BWD) {
        // state before time step k = L-1-(k0+i): the saved x at k-1, or x0 (zero if absent) for k = 0
        const float2 *xp = p.xs + first - P;
#pragma unroll
        for (int i = 0; i < CS; ++i) {
            const int64_t k = p.L - 1 - (k0 + i);
            xprev[i] = make_float2(0.0f, 0.0f);
            if (okp && k > 0) xprev[i] = xp[i * tstep];
            else if (okp && k == 0 && p.x0) xprev[i] = p.x0[(int64_t)b * P + pp];
        }
    }
    float2 x = make_float2(0.0f, 0.0f);
#pragma unroll
    for (int i = 0; i < CS; ++i) x = cfma(lam, x, v[i]);
    sS[w][lane] = x;
    __syncthreads();
    float2 e = make_float2(0.0f, 0.0f);                       // state entering this chunk if the group started from zero
    for (int ww = 0; ww < w; ++ww) e = cfma(lp, e, sS[ww][lane]);

    if (w == 0) {
        float2 T = make_float2(0.0f, 0.0f);                   // end state of the group started from zero
#pragma unroll
        for (int ww = 0; ww < kOneGW; ++ww) T = cfma(lp, T, sS[ww][lane]);
        int *flags = p.flags + ((int64_t)b * npslab + pslab) * p.ngroups;
        const int64_t gi = ((int64_t)b * p.ngroups) * P + pp;
        if (okp) p.ws_T[gi + (int64_t)g * P] = T;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
        if (lane == 0) __hip_atomic_store(flags + g, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

        // Carry-in of this group, always by the same arithmetic (so x is bitwise reproducible): start from the true
        // end state X_m of the last "anchor" group before g (every 16th group publishes one; x0 before the first)
        // and push it through the end-states-from-zero of the groups in between, oldest first.
        const int m = (g / kAnchor) * kAnchor - 1;
        const int need = g - 1 - m;                            // groups m+1 .. g-1 contribute their T (at most 15)
        // one poll covers every flag this group depends on: lane i < need watches group m+1+i (needs >= 1),
        // lane `need` watches the anchor m (needs 2)
        bool failed = false;
        {
            const bool watch = lane < need || (lane == need && m >= 0);
            const int idx = lane < need ? m + 1 + lane : m;
            const int want = lane < need ? 1 : 2;
            int spins = 0;
            bool ok;
            do {
                const int f = watch ? __hip_atomic_load(flags + idx, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : want;
                ok = __builtin_amdgcn_ballot_w64(f < want) == 0;
            } while (!ok && ++spins < kSpinLimit);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
            failed = !ok;
        }
        float2 acc = make_float2(0.0f, 0.0f);
        if (m >= 0) { if (okp) acc = p.ws_X[gi + (int64_t)m * P]; }
        else if (!BWD && p.x0 && okp) acc = p.x0[(int64_t)b * P + pp];   // the adjoint starts from g_{L+1} = 0
        float2 Tj[kAnchor - 1];
#pragma unroll
        for (int i = 0; i < kAnchor - 1; ++i)                  // all loads in flight before the Horner chain
            Tj[i] = (i < need && okp) ? p.ws_T[gi + (int64_t)(m + 1 + i) * P] : make_float2(0.0f, 0.0f);
#pragma unroll
        for (int i = 0; i < kAnchor - 1; ++i)
            if (i < need) acc = cfma(lg, acc, Tj[i]);
        if (failed) {                                          // never hand back a plausible but wrong state
            if (lane == 0) *p.err = 1;
            acc = make_float2(__builtin_nanf(""), __builtin_nanf(""));
        }
        if (g % kAnchor == kAnchor - 1) {
            if (okp) p.ws_X[gi + (int64_t)g * P] = cfma(lg, acc, T);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            if (lane == 0) __hip_atomic_store(flags + g, 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        sCarry[lane] = acc;
    }
    __syncthreads();

    // ---- replay from the true carry-in, out of registers
    x = cfma(cpow(lp, w), sCarry[lane], e);
    float2 *xo = p.x + first;
    float2 dl = make_float2(0.0f, 0.0f);
#pragma unroll
    for (int i = 0; i < CS; ++i) {
        x = cfma(lam, x, v[i]);
        if (okp && k0 + i < p.L) {
            xo[i * tstep] = x;
            if constexpr (BWD) {                               // conj(xprev) * g
                dl.x = __builtin_fmaf(xprev[i].x, x.x, __builtin_fmaf(xprev[i].y, x.y, dl.x));
                dl.y = __builtin_fmaf(xprev[i].x, x.y, __builtin_fmaf(-xprev[i].y, x.x, dl.y));
            }
            if (p.x_last && k0 + i == p.L - 1) p.x_last[(int64_t)b * P + pp] = BWD ? cmul(lam, x) : x;
        }
    }
    if constexpr (BWD) {
        __syncthreads();                                       // sS is free again: every wavefront has read its prefix
        sS[w][lane] = dl;
        __syncthreads();
        if (w == 0 && okp) {
#pragma unroll
            for (int ww = 1; ww < kOneGW; ++ww) { dl.x += sS[ww][lane].x; dl.y += sS[ww][lane].y; }
            atomicAdd(p.dlambda + 2 * pp, dl.x);
            atomicAdd(p.dlambda + 2 * pp + 1, dl.y);
        }
    }
}

hipError_t launch_lti_onepass(const LtiParams &p, hipStream_t s) {
    const int npslab = (p.P + 63) / 64;
    dim3 grid((unsigned)(npslab * p.B), p.ngroups);
    hipLaunchKernelGGL((k_lti_onepass<kOneCS, false>), grid, dim3(kOneGW * 64), 0, s, p);
    return hipGetLastError();
}
int lti_onepass_group_steps() { return kOneCS * kOneGW; }

hipError_t launch_lti_onepass_bwd(const LtiParams &p, hipStream_t s) {
    const int npslab = (p.P + 63) / 64;
    dim3 grid((unsigned)(npslab * p.B), p.ngroups);
    hipLaunchKernelGGL((k_lti_onepass<kOneBwdCS, true>), grid, dim3(kOneGW * 64), 0, s, p);
    return hipGetLastError();
}
int lti_onepass_bwd_group_steps() { return kOneBwdCS * kOneGW; }

hipError_t launch_lti(const LtiParams &p, hipStream_t s) {
    dim3 grid((p.P + 63) / 64, p.ngroups, p.B);
    if (p.nchunks > 1) hipLaunchKernelGGL(k_lti_chunk<false>, grid, dim3(kLtiThreads), 0, s, p);
    hipLaunchKernelGGL(k_lti_chunk<true>, grid, dim3(kLtiThreads), 0, s, p);
    return hipGetLastError();
}

}  // namespace lrnnx
