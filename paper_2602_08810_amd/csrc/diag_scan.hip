// Diagonal scan with caller-supplied coefficients for gfx950:  x_k = a_k (.) x_{k-1} + b_k   (Eq. 2 of the paper
// with A(k) = diag(a_k) and b_k = B(k) u_k formed by the caller: the recurrence of the time-varying S5-style
// layers of Sec. 2.2.2, of gated real recurrences, and of event-driven discretisation, Sec. 3).
//
// a, b and x are [B,L,P] with P contiguous, real (float) or complex (float2).  Same structure as the single-launch
// LTI scan: lanes along p, a wavefront keeps CS steps of (a, b) in registers, the wavefronts of a workgroup chain
// their aggregates through LDS, and the groups of one (b, 64 values of p) are chained through global memory.
// Because a_k varies, the aggregate of a span is the pair (product of its a, end state from zero) and composing
// two spans is (A2, S2) o (A1, S1) = (A2 A1, A2 S1 + S2).  A real pair is published as one 8-byte slot, a complex
// pair as two.  HBM-bound: 3 elements per step (a and b read once, x written once).
#include "kernels.hpp"
#include "chain.hpp"

namespace lrnnx {

template <bool CPLX> struct Elem;
template <> struct Elem<false> {
    using T = float;
    static __device__ __forceinline__ T zero() { return 0.0f; }
    static __device__ __forceinline__ T one() { return 1.0f; }
    static __device__ __forceinline__ T mul(T a, T b) { return a * b; }
    static __device__ __forceinline__ T fma(T a, T x, T b) { return __builtin_fmaf(a, x, b); }
    static __device__ __forceinline__ T nan() { return __builtin_nanf(""); }
    static __device__ __forceinline__ T conj(T a) { return a; }
};
template <> struct Elem<true> {
    using T = float2;
    static __device__ __forceinline__ T zero() { return make_float2(0.0f, 0.0f); }
    static __device__ __forceinline__ T one() { return make_float2(1.0f, 0.0f); }
    static __device__ __forceinline__ T mul(T a, T b) { return cmul(a, b); }
    static __device__ __forceinline__ T fma(T a, T x, T b) { return cfma(a, x, b); }
    static __device__ __forceinline__ T nan() { return make_float2(__builtin_nanf(""), __builtin_nanf("")); }
    static __device__ __forceinline__ T conj(T a) { return make_float2(a.x, -a.y); }
};

template <typename E>
__device__ __forceinline__ const E &el(const E *row, unsigned byte_off) {
    return *reinterpret_cast<const E *>(reinterpret_cast<const char *>(row) + byte_off);
}
template <typename E>
__device__ __forceinline__ E &el(E *row, unsigned byte_off) {
    return *reinterpret_cast<E *>(reinterpret_cast<char *>(row) + byte_off);
}

// ANCH: every ANCH-th group publishes its true end state; a group looks back over at most ANCH-1 aggregates.
// BWD = false: the scan.  BWD = true: its adjoint, the same chain over reversed time (scan position j is time
// k = L-1-j): g_k = gx_k + conj(a_{k+1}) g_{k+1}, read through p.b = gx and written through p.x = db; the coefficient
// of a position is therefore the NEXT time step's a, conjugated.  Each step also loads the saved state before it
// and writes da_k = conj(x_{k-1}) g_k; the last position writes dx0 = conj(a_0) g_0 through p.x_last.
template <bool CPLX, int CS, int GW, int ANCH, bool BWD>
__global__ __launch_bounds__(GW * 64) void k_diag_scan(const DiagParams p) {
    using EL = Elem<CPLX>;
    using E = typename EL::T;
    constexpr int NS = CPLX ? 2 : 1;                           // 8-byte slots per published aggregate
    __shared__ E sA[GW][64], sS[GW][64], sCarry[64];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int npslab = (p.P + 63) / 64;
    const int pslab = blockIdx.x % npslab, b = blockIdx.x / npslab;
    const int g = blockIdx.y;
    const int pp = pslab * 64 + lane;
    const unsigned boff = (unsigned)pp * (unsigned)sizeof(E);
    const bool okp = pp < p.P;
    const int64_t P = p.P;
    const int64_t k0 = ((int64_t)g * GW + w) * CS;
    const int64_t tstep = BWD ? -P : P;                        // element stride between consecutive scan positions
    const int64_t row0 = ((int64_t)b * p.L + (BWD ? p.L - 1 - k0 : k0)) * P;
    const bool full = k0 + CS <= p.L;

    // ---- this wavefront's steps of (a, b), all loads in flight at once; steps beyond the sequence are identities
    E a[CS], bv[CS];
#pragma unroll
    for (int i = 0; i < CS; ++i) { a[i] = EL::one(); bv[i] = EL::zero(); }
    // forward: a of the step itself; adjoint: a of the next time step (one row further), none for the last time step
    const E *arow = reinterpret_cast<const E *>(p.a) + row0 + (BWD ? P : 0);
    const E *brow = reinterpret_cast<const E *>(p.b) + row0;
    if (full && (!BWD || k0 > 0)) {
        if (okp) {
#pragma unroll
            for (int i = 0; i < CS; ++i) { a[i] = el(arow + i * tstep, boff); bv[i] = el(brow + i * tstep, boff); }
        }
    } else if (okp) {
#pragma unroll
        for (int i = 0; i < CS; ++i)
            if (k0 + i < p.L) {
                if (!BWD || k0 + i > 0) a[i] = el(arow + i * tstep, boff);
                bv[i] = el(brow + i * tstep, boff);
            }
    }
    E xprev[BWD ? CS : 1];
    if constexpr (BWD) {
#pragma unroll
        for (int i = 0; i < CS; ++i) { a[i] = EL::conj(a[i]); xprev[i] = EL::zero(); }
        // state before time step k = L-1-(k0+i): the saved x at k-1, or x0 (zero if absent) for k = 0
        const E *xrow = reinterpret_cast<const E *>(p.xs) + row0 - P;
        if (k0 + CS < p.L) {
            if (okp) {
#pragma unroll
                for (int i = 0; i < CS; ++i) xprev[i] = el(xrow + i * tstep, boff);
            }
        } else if (okp) {
#pragma unroll
            for (int i = 0; i < CS; ++i) {
                const int64_t k = p.L - 1 - (k0 + i);
                if (k > 0) xprev[i] = el(xrow + i * tstep, boff);
                else if (k == 0 && p.x0) xprev[i] = reinterpret_cast<const E *>(p.x0)[(int64_t)b * P + pp];
            }
        }
    }
    E A = EL::one(), x = EL::zero();
#pragma unroll
    for (int i = 0; i < CS; ++i) { x = EL::fma(a[i], x, bv[i]); A = EL::mul(a[i], A); }
    sA[w][lane] = A;
    sS[w][lane] = x;
    __syncthreads();
    E Ae = EL::one(), e = EL::zero();                          // aggregate of the chunks before this one in its group
    for (int ww = 0; ww < w; ++ww) { e = EL::fma(sA[ww][lane], e, sS[ww][lane]); Ae = EL::mul(sA[ww][lane], Ae); }

    if (w == 0) {
        E AG = EL::one(), SG = EL::zero();                     // aggregate of the whole group
#pragma unroll
        for (int ww = 0; ww < GW; ++ww) { SG = EL::fma(sA[ww][lane], SG, sS[ww][lane]); AG = EL::mul(sA[ww][lane], AG); }
        const int nanch = p.ngroups / ANCH + 1;
        float2 *wsT = p.ws_T + ((int64_t)b * p.ngroups) * NS * P + pp;     // [B, ngroups, NS, P]
        float2 *wsX = p.ws_X + ((int64_t)b * nanch) * P + pp;              // [B, nanch, P]
        if (okp) {
            if constexpr (CPLX) {
                publish(wsT + ((int64_t)g * NS + 0) * P, AG);
                publish(wsT + ((int64_t)g * NS + 1) * P, SG);
            } else {
                publish(wsT + (int64_t)g * P, make_float2(AG, SG));
            }
        }
        // carry-in: the true end state of the last anchor group before g (x0 before the first), pushed through the
        // aggregates of the groups in between, oldest first; always the same arithmetic, so x is reproducible
        const int m = (g / ANCH) * ANCH - 1;
        const int need = g - 1 - m;
        unsigned long long tb[(ANCH - 1) * NS] = {}, xb = 0;
        int spins = 0;
        bool ok;
        do {
            bool mine = true;
#pragma unroll
            for (int i = 0; i < ANCH - 1; ++i)
                if (i < need && okp) {
#pragma unroll
                    for (int s = 0; s < NS; ++s) {
                        tb[i * NS + s] = peek(wsT + ((int64_t)(m + 1 + i) * NS + s) * P);
                        mine &= tb[i * NS + s] != kNotReady;
                    }
                }
            if (m >= 0 && okp) { xb = peek(wsX + (int64_t)(m / ANCH) * P); mine &= xb != kNotReady; }
            ok = __builtin_amdgcn_ballot_w64(!mine) == 0;
        } while (!ok && ++spins < kSpinLimit);
        E acc = EL::zero();
        if (m >= 0) {
            const float2 f = from_bits(xb);
            if constexpr (CPLX) acc = f; else acc = f.x;
        } else if (!BWD && p.x0 && okp) {                      // the adjoint starts from zero
            acc = reinterpret_cast<const E *>(p.x0)[(int64_t)b * P + pp];
        }
#pragma unroll
        for (int i = 0; i < ANCH - 1; ++i)
            if (i < need) {
                if constexpr (CPLX) acc = cfma(from_bits(tb[2 * i]), acc, from_bits(tb[2 * i + 1]));
                else { const float2 f = from_bits(tb[i]); acc = __builtin_fmaf(f.x, acc, f.y); }
            }
        if (!ok) {                                             // never hand back a plausible but wrong state
            if (lane == 0) { *p.err = 1; if (p.status) *p.status = 1; }
            acc = EL::nan();
        }
        if (g % ANCH == ANCH - 1 && okp) {
            const E X = EL::fma(AG, acc, SG);
            if constexpr (CPLX) publish(wsX + (int64_t)(g / ANCH) * P, X);
            else publish(wsX + (int64_t)(g / ANCH) * P, make_float2(X, 0.0f));
        }
        sCarry[lane] = acc;
    }
    __syncthreads();

    // ---- replay from the true carry-in, out of registers
    x = EL::fma(Ae, sCarry[lane], e);
    E *xrow_out = reinterpret_cast<E *>(p.x) + row0;
    E *darow = BWD ? reinterpret_cast<E *>(p.da) + row0 : nullptr;
    E xl = x;
    if (full) {
        if (okp) {
#pragma unroll
            for (int i = 0; i < CS; ++i) {
                x = EL::fma(a[i], x, bv[i]);
                el(xrow_out + i * tstep, boff) = x;
                if constexpr (BWD) el(darow + i * tstep, boff) = EL::mul(EL::conj(xprev[i]), x);
            }
        }
        xl = x;
    } else if (okp) {
#pragma unroll
        for (int i = 0; i < CS; ++i) {
            x = EL::fma(a[i], x, bv[i]);
            if (k0 + i < p.L) {
                el(xrow_out + i * tstep, boff) = x;
                if constexpr (BWD) el(darow + i * tstep, boff) = EL::mul(EL::conj(xprev[i]), x);
                xl = x;
            }
        }
    }
    if (p.x_last && okp && k0 < p.L && p.L <= k0 + CS) {
        if constexpr (BWD) {                                   // dx0 = conj(a at time 0) g_0
            const E a0 = reinterpret_cast<const E *>(p.a)[((int64_t)b * p.L) * P + pp];
            xl = EL::mul(EL::conj(a0), xl);
        }
        reinterpret_cast<E *>(p.x_last)[(int64_t)b * P + pp] = xl;
    }
}

// ---------------------------------------------------------------- launchers
constexpr int kDsCS = 32;                        // steps of (a, b) a wavefront keeps in registers
constexpr int kDsGWSmall = 4, kDsGWLarge = 8;    // real: wavefronts per group, by the number of independent chains
constexpr int kDsCplxGW = 4, kDsCplxAnchor = 8;  // complex: twice the registers per step and two slots per aggregate
// adjoint: three arrays per step (coefficient, gx, saved state); real keeps 32 steps, complex 16
constexpr int kDsBwdGW = 4, kDsBwdCplxCS = 16;

static int ds_gw(int64_t B, int64_t P, int is_complex) {
    if (is_complex) return kDsCplxGW;
    return B * ((P + 63) / 64) >= 64 ? kDsGWSmall : kDsGWLarge;
}
int diag_scan_group_steps(int64_t B, int64_t P, int is_complex) { return kDsCS * ds_gw(B, P, is_complex); }
int diag_scan_min_group_steps(int is_complex) { return kDsCS * (is_complex ? kDsCplxGW : kDsGWSmall); }
int diag_scan_anchor(int is_complex) { return is_complex ? kDsCplxAnchor : kAnchor; }
int diag_scan_bwd_group_steps(int is_complex) { return (is_complex ? kDsBwdCplxCS : kDsCS) * kDsBwdGW; }

hipError_t launch_diag_scan(const DiagParams &p, hipStream_t s) {
    const int npslab = (p.P + 63) / 64;
    dim3 grid((unsigned)(npslab * p.B), p.ngroups);
    if (p.is_complex)
        hipLaunchKernelGGL((k_diag_scan<true, kDsCS, kDsCplxGW, kDsCplxAnchor, false>), grid, dim3(kDsCplxGW * 64), 0, s, p);
    else if (ds_gw(p.B, p.P, 0) == kDsGWSmall)
        hipLaunchKernelGGL((k_diag_scan<false, kDsCS, kDsGWSmall, kAnchor, false>), grid, dim3(kDsGWSmall * 64), 0, s, p);
    else
        hipLaunchKernelGGL((k_diag_scan<false, kDsCS, kDsGWLarge, kAnchor, false>), grid, dim3(kDsGWLarge * 64), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_diag_scan_bwd(const DiagParams &p, hipStream_t s) {
    const int npslab = (p.P + 63) / 64;
    dim3 grid((unsigned)(npslab * p.B), p.ngroups);
    if (p.is_complex)
        hipLaunchKernelGGL((k_diag_scan<true, kDsBwdCplxCS, kDsBwdGW, kDsCplxAnchor, true>), grid, dim3(kDsBwdGW * 64), 0, s, p);
    else
        hipLaunchKernelGGL((k_diag_scan<false, kDsCS, kDsBwdGW, kAnchor, true>), grid, dim3(kDsBwdGW * 64), 0, s, p);
    return hipGetLastError();
}

}  // namespace lrnnx
