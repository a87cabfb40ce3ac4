// LTI complex-diagonal scan for gfx950:  x_k = lambda (.) x_{k-1} + v_k  (Eq. 2 of the
// paper with a constant diagonal A; the recurrence of the S5 / LRU layers, Sec. 2.2.1).
//
// v and x are [B,L,P] with P contiguous, so the lanes run along P (coalesced 8-byte
// complex elements) and the time axis is cut into chunks that different workgroups take.
// Because lambda is constant the affine aggregate of a chunk is (lambda^len, end state
// from zero): only end states are stored.  Two forms.  The default is the single-launch chained scan
// further down (k_lti_onepass, also used for the adjoint).  The other takes two launches and no
// inter-workgroup waiting: the first scans every chunk from zero and, inside each workgroup (4 consecutive
// chunks), chains the end states through LDS; the second rebuilds each chunk's true carry-in from the end
// states of the groups before it and its in-group prefix, rescans the chunk and writes x (the second read
// of v is served by the L2 / Infinity Cache at these sizes).
#include "kernels.hpp"
#include "chain.hpp"

namespace lrnnx {

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
            const float2 lg = cpow(lam, p.chunk * kLtiWaves);
            const float2 *G = p.ws_G + (int64_t)b * p.ngroups * p.P + pp;
            for (int g = 0; g < grp; ++g) x = cfma(lg, x, G[(int64_t)g * p.P]);
            x = cfma(cpow(lam, p.chunk * w), x, p.ws_S[((int64_t)b * p.nchunks + c) * p.P + pp]);
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
// zero, the 4 or 8 wavefronts of a workgroup (one group = 128 or 256 consecutive steps of 64 values of p) chain their end
// states through LDS, and the groups of one (b, p-slab) are chained through global memory: every group publishes
// its end-state-from-zero T_g as soon as it has it, then rebuilds its carry-in from the T_j of the groups
// before it, back to the last "anchor" group, whose true end state X it takes.  Every T_g is available
// after one load phase, so only anchors wait on a chain (one hop per 16 groups).  A published value is its own
// ready flag (see publish() in chain.hpp), so a hop costs one store and one load round trip and needs no fence.
// Workgroups are ordered so that a group is dispatched after the groups it looks back on (blockIdx.y = group),
// and every wait is bounded: after kSpinLimit polls a wavefront gives up, raises *err and finishes with a NaN
// carry rather than hang.
constexpr int kOneCS = 32;                   // steps a wavefront keeps in registers
constexpr int kOneGWSmall = 4, kOneGWLarge = 8;   // wavefronts per group: see lti_onepass_group_steps()
constexpr int kOneBwdCS = 32, kOneBwdGW = 4;      // the adjoint also holds the saved states of its steps

// BWD = false: the scan itself.  BWD = true: its adjoint (Sec. 2.2.1's recurrence differentiated): the same chain
// run over reversed time with the conjugate pole, g_k = gx_k + conj(lambda) g_{k+1}, reading gx through p.v and
// writing dv = g through p.x; each wavefront also loads the saved forward state before each of its steps and
// accumulates dlambda += conj(x_{k-1}) g_k, reduced over the workgroup in LDS and added to p.dlambda with one
// atomic pair per lane.  The scan position j maps to time k = j (forward) or k = L-1-j (adjoint).
template <int CS, int kOneGW, bool BWD>
__global__ __launch_bounds__(kOneGW * 64) void k_lti_onepass(const LtiParams p) {
    __shared__ float2 sS[kOneGW][64];
    __shared__ float2 sCarry[64];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int npslab = (p.P + 63) / 64;
    const int pslab = blockIdx.x % npslab, b = blockIdx.x / npslab;
    const int g = blockIdx.y;
    const int pp = pslab * 64 + lane;
    const unsigned boff = (unsigned)pp * 8u;                   // the lane's byte offset within a row of P values
    const bool okp = pp < p.P;
    const int64_t P = p.P;
    const int64_t k0 = ((int64_t)g * kOneGW + w) * CS;
    float2 lam = okp ? p.lambda[pp] : make_float2(0.0f, 0.0f);
    if (BWD) lam.y = -lam.y;
    const float2 lp = cpow(lam, CS), lg = cpow(lam, CS * kOneGW);
    // Row pointers are wave-uniform (scalar registers) and the lane adds only its p, so a whole chunk needs one
    // vector offset register; scan position k0+i is time k0+i (forward) or L-1-(k0+i) (adjoint).
    const int64_t tstep = BWD ? -P : P;                        // element stride between consecutive scan positions
    const int64_t row0 = ((int64_t)b * p.L + (BWD ? p.L - 1 - k0 : k0)) * P;
    const bool full = k0 + CS <= p.L;                          // no step of this chunk is beyond the sequence

    // ---- this wavefront's steps, all loads in flight at once
    float2 v[CS];
#pragma unroll
    for (int i = 0; i < CS; ++i) v[i] = make_float2(0.0f, 0.0f);
    const float2 *vrow = p.v + row0;
    if (full) {
        if (okp) {
#pragma unroll
            for (int i = 0; i < CS; ++i) v[i] = at(vrow + i * tstep, boff);
        }
    } else if (okp) {
#pragma unroll
        for (int i = 0; i < CS; ++i)
            if (k0 + i < p.L) v[i] = at(vrow + i * tstep, boff);
    }
    float2 xprev[BWD ? CS : 1];
    if constexpr (BWD) {
        // state before time step k = L-1-(k0+i): the saved x at k-1, or x0 (zero if absent) for k = 0
#pragma unroll
        for (int i = 0; i < CS; ++i) xprev[i] = make_float2(0.0f, 0.0f);
        const float2 *xrow = p.xs + row0 - P;
        if (k0 + CS < p.L) {                                   // every k of this chunk is at least 1
            if (okp) {
#pragma unroll
                for (int i = 0; i < CS; ++i) xprev[i] = at(xrow + i * tstep, boff);
            }
        } else if (okp) {
#pragma unroll
            for (int i = 0; i < CS; ++i) {
                const int64_t k = p.L - 1 - (k0 + i);
                if (k > 0) xprev[i] = at(xrow + i * tstep, boff);
                else if (k == 0 && p.x0) xprev[i] = p.x0[(int64_t)b * P + pp];
            }
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
        const int nanch = p.ngroups / kAnchor + 1;
        float2 *wsT = p.ws_T + ((int64_t)b * p.ngroups) * P + pp;
        float2 *wsX = p.ws_X + ((int64_t)b * nanch) * P + pp;
        if (okp) publish(wsT + (int64_t)g * P, T);

        // Carry-in of this group, always by the same arithmetic (so x is bitwise reproducible): start from the true
        // end state X_m of the last "anchor" group before g (every 16th group publishes one; x0 before the first)
        // and push it through the end-states-from-zero of the groups in between, oldest first.
        const int m = (g / kAnchor) * kAnchor - 1;
        const int need = g - 1 - m;                            // groups m+1 .. g-1 contribute their T (at most 15)
        // Every lane polls the slots of its own p: all loads of one round are in flight together, and a slot is
        // its own ready flag (it holds kNotReady until its 8-byte value is stored), so no fence is involved.
        unsigned long long tb[kAnchor - 1] = {}, xb = 0;
        int spins = 0;
        bool ok;
        do {
            bool mine = true;
#pragma unroll
            for (int i = 0; i < kAnchor - 1; ++i)
                if (i < need && okp) { tb[i] = peek(wsT + (int64_t)(m + 1 + i) * P); mine &= tb[i] != kNotReady; }
            if (m >= 0 && okp) { xb = peek(wsX + (int64_t)(m / kAnchor) * P); mine &= xb != kNotReady; }
            ok = __builtin_amdgcn_ballot_w64(!mine) == 0;
        } while (!ok && ++spins < kSpinLimit);
        float2 acc = make_float2(0.0f, 0.0f);
        if (m >= 0) acc = from_bits(xb);
        else if (!BWD && p.x0 && okp) acc = p.x0[(int64_t)b * P + pp];   // the adjoint starts from g_{L+1} = 0
#pragma unroll
        for (int i = 0; i < kAnchor - 1; ++i)
            if (i < need) acc = cfma(lg, acc, from_bits(tb[i]));
        if (!ok) {                                             // never hand back a plausible but wrong state
            if (lane == 0) { *p.err = 1; if (p.status) *p.status = 1; }
            acc = make_float2(__builtin_nanf(""), __builtin_nanf(""));
        }
        if (g % kAnchor == kAnchor - 1 && okp) publish(wsX + (int64_t)(g / kAnchor) * P, cfma(lg, acc, T));
        sCarry[lane] = acc;
    }
    __syncthreads();

    // ---- replay from the true carry-in, out of registers
    x = cfma(cpow(lam, CS * w), sCarry[lane], e);
    float2 *xrow_out = p.x + row0;
    float2 dl = make_float2(0.0f, 0.0f);
    float2 xl = x;                                             // state at the last scan position of the sequence
    auto dlam_term = [&](int i) {                              // dl += conj(xprev) * g
        dl.x = __builtin_fmaf(xprev[BWD ? i : 0].x, x.x, __builtin_fmaf(xprev[BWD ? i : 0].y, x.y, dl.x));
        dl.y = __builtin_fmaf(xprev[BWD ? i : 0].x, x.y, __builtin_fmaf(-xprev[BWD ? i : 0].y, x.x, dl.y));
    };
    if (full) {
        if (okp) {
#pragma unroll
            for (int i = 0; i < CS; ++i) {
                x = cfma(lam, x, v[i]);
                at(xrow_out + i * tstep, boff) = x;
                if constexpr (BWD) dlam_term(i);
            }
        }
        xl = x;
    } else if (okp) {
#pragma unroll
        for (int i = 0; i < CS; ++i) {
            x = cfma(lam, x, v[i]);
            if (k0 + i < p.L) {
                at(xrow_out + i * tstep, boff) = x;
                if constexpr (BWD) dlam_term(i);
                xl = x;
            }
        }
    }
    if (p.x_last && okp && k0 < p.L && p.L <= k0 + CS) p.x_last[(int64_t)b * P + pp] = BWD ? cmul(lam, xl) : xl;
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

// Wavefronts per group of the forward scan.  With many independent chains (one per batch entry and 64 values of
// p) the chip is filled by chains alone and small workgroups overlap their load, wait and store phases best
// (two per compute unit); with few chains the time is the length of a chain, and longer groups halve it.
static int onepass_gw(int64_t B, int64_t P) { return B * ((P + 63) / 64) >= 64 ? kOneGWSmall : kOneGWLarge; }
int lti_onepass_group_steps(int64_t B, int64_t P) { return kOneCS * onepass_gw(B, P); }
int lti_onepass_min_group_steps() { return kOneCS * kOneGWSmall; }
int lti_onepass_bwd_group_steps() { return kOneBwdCS * kOneBwdGW; }
int lti_onepass_anchor() { return kAnchor; }
int lti_chunk_group() { return kLtiWaves; }

hipError_t launch_lti_onepass(const LtiParams &p, hipStream_t s) {
    const int npslab = (p.P + 63) / 64;
    dim3 grid((unsigned)(npslab * p.B), p.ngroups);
    if (onepass_gw(p.B, p.P) == kOneGWSmall)
        hipLaunchKernelGGL((k_lti_onepass<kOneCS, kOneGWSmall, false>), grid, dim3(kOneGWSmall * 64), 0, s, p);
    else
        hipLaunchKernelGGL((k_lti_onepass<kOneCS, kOneGWLarge, false>), grid, dim3(kOneGWLarge * 64), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_lti_onepass_bwd(const LtiParams &p, hipStream_t s) {
    const int npslab = (p.P + 63) / 64;
    dim3 grid((unsigned)(npslab * p.B), p.ngroups);
    hipLaunchKernelGGL((k_lti_onepass<kOneBwdCS, kOneBwdGW, true>), grid, dim3(kOneBwdGW * 64), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_lti(const LtiParams &p, hipStream_t s) {
    dim3 grid((p.P + 63) / 64, p.ngroups, p.B);
    if (p.nchunks > 1) hipLaunchKernelGGL(k_lti_chunk<false>, grid, dim3(kLtiThreads), 0, s, p);
    hipLaunchKernelGGL(k_lti_chunk<true>, grid, dim3(kLtiThreads), 0, s, p);
    return hipGetLastError();
}

}  // namespace lrnnx
