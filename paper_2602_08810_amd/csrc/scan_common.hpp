// Device-side building blocks shared by the gfx950 scan kernels: I/O element access,
// transcendental helpers, the fused discretisations (schemes named in Sec. 3 of the
// paper) and the wavefront scans over affine pairs.
//
// The recurrence x_k = a_k x_{k-1} + b_k (Eq. 2, line 1, diagonal A) is the
// composition of affine maps (a, b): x -> a x + b.  Two maps compose as
//     (a2, b2) o (a1, b1) = (a2 a1, a2 b1 + b2),
// which is associative, so a wavefront can take an inclusive prefix over its 64
// lanes in six cross-lane steps.  Out-of-range lanes hold the identity (1, 0).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lrnnx {

constexpr int kWave = 64;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

struct bf16_t { unsigned short v; };

// ---------------------------------------------------------------- bit casts and cross-lane moves
__device__ __forceinline__ int f2i(float x) { return __builtin_bit_cast(int, x); }
__device__ __forceinline__ float i2f(int x) { return __builtin_bit_cast(float, x); }

// DPP move: lanes whose source lane does not exist (or whose row is masked off) keep `old`.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp(float old, float src) {
    return i2f(__builtin_amdgcn_update_dpp(f2i(old), f2i(src), CTRL, ROW_MASK, 0xF, false));
}
constexpr int DPP_ROW_SHL1 = 0x101, DPP_ROW_SHR1 = 0x111;
constexpr int DPP_WAVE_SHL1 = 0x130, DPP_WAVE_SHR1 = 0x138;
constexpr int DPP_ROW_BCAST15 = 0x142, DPP_ROW_BCAST31 = 0x143;

__device__ __forceinline__ float readlane(float x, int lane) { return i2f(__builtin_amdgcn_readlane(f2i(x), lane)); }
// copy of `old` with lane `lane` replaced by the wave-uniform value v: one v_writelane_b32.  This compiler has no
// builtin for it, so the LLVM intrinsic is declared by its name (the compiler still sees an ordinary instruction
// and handles its hazards).
extern "C" __device__ int lrnnx_llvm_writelane_i32(int value, int lane, int old) __asm("llvm.amdgcn.writelane.i32");
__device__ __forceinline__ float writelane(float old, float v, int lane) {
    return i2f(lrnnx_llvm_writelane_i32(f2i(v), lane, f2i(old)));
}
__device__ __forceinline__ float bpermute(int src_lane, float x) { return i2f(__builtin_amdgcn_ds_bpermute(src_lane << 2, f2i(x))); }
// v[lane] + v[lane ^ 16]: the row-pair swap of gfx950 exchanges the odd rows of one copy with the even rows of the
// other, all in the vector ALU (a swizzle through the LDS crossbar would cost a round trip of a hundred cycles)
__device__ __forceinline__ float sum_xor16(float v) {
    const auto r = __builtin_amdgcn_permlane16_swap((unsigned)f2i(v), (unsigned)f2i(v), false, false);
    return i2f((int)r[0]) + i2f((int)r[1]);
}
// LDS accumulate without a returned value: the wavefront does not wait for it
__device__ __forceinline__ void lds_add(float *p, float v) {
    (void)__hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// ---------------------------------------------------------------- transcendentals (fp32, ~1 ulp hardware ops)
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32
__device__ __forceinline__ float log2_fast(float x) { return __builtin_amdgcn_logf(x); }    // v_log_f32
__device__ __forceinline__ float rcp_fast(float x) { return __builtin_amdgcn_rcpf(x); }     // v_rcp_f32

// softplus(s) = log(1 + e^s) and its derivative sigmoid(s) = e^s / (1 + e^s).
// For s > 20 both saturate (softplus = s to 2e-9).  The logarithm of 1 + w rounds its argument, which leaves an
// ABSOLUTE error of 2^-24 in the step size: for float32 I/O (PRECISE) small w take the series of log(1 + w) instead,
// which keeps full relative accuracy; with bfloat16 I/O, whose inputs and outputs carry relative errors of 2^-9, the
// absolute 6e-8 is far below anything the step size is multiplied into, and the series is left out.
template <bool PRECISE = true>
__device__ __forceinline__ void softplus_sigmoid(float s, float &sp, float &sg) {
    float w = exp2_fast(fminf(s, 20.0f) * kLog2e);
    float r = rcp_fast(1.0f + w);
    float v = log2_fast(1.0f + w) * kLn2;
    if constexpr (PRECISE) {
        const float series = w * (1.0f - w * (0.5f - w * (0.33333334f - w * 0.25f)));
        v = w < 0.015625f ? series : v;
    }
    sp = s > 20.0f ? s : v;
    sg = s > 20.0f ? 1.0f : w * r;
}
__device__ __forceinline__ float sigmoid_fast(float zz) { return rcp_fast(1.0f + exp2_fast(-zz * kLog2e)); }

// Input gain of the exact zero-order hold, g = (e^{dt A} - 1) / A, given a = e^{dt A} and rA = 1/A (0 for A = 0).
// For |dt A| >= 1/64 the difference a - 1 loses at most 6 bits (relative error <= 64 eps = 4e-6); below, and for
// A = 0, g = dt (1 + x/2 + x^2/6) with x = dt A, whose first omitted term x^3/24 is below 2e-7.
__device__ __forceinline__ float zoh_gain(float dt, float A, float rA, float a) {
    const float x = dt * A;
    const float small = dt * __builtin_fmaf(x, __builtin_fmaf(x, 0.16666667f, 0.5f), 1.0f);
    return fabsf(x) < 0.015625f ? small : (a - 1.0f) * rA;
}

// ---------------------------------------------------------------- fused discretisation (Sec. 3 schemes)
enum : int { DISC_ZOH_S6 = 0, DISC_ZOH = 1, DISC_BILINEAR = 2, DISC_DIRAC = 3 };

// Per-(d,n) constants derived once from A[d,n].
struct ACoef {
    float A;      // A[d,n]
    float A2;     // A * log2(e), so that exp(dt*A) = exp2(dt*A2)
    float rA;     // 1/A (exact ZOH only; 0 for A == 0, where the series branch of the gain applies)
    float hA;     // A/2 (bilinear only)
};
template <int DISC>
__device__ __forceinline__ ACoef make_acoef(float A) {
    ACoef c; c.A = A; c.A2 = A * kLog2e;
    if constexpr (DISC == 1) c.rA = (A != 0.0f) ? rcp_fast(A) : 0.0f; else c.rA = 0.0f;
    c.hA = 0.5f * A;
    return c;
}

// State multiplier a and input gain g of one step.
template <int DISC>
__device__ __forceinline__ void disc_ag(float dt, const ACoef &c, float &a, float &g) {
    if constexpr (DISC == DISC_BILINEAR) {
        // q = 1 / (1 - dt A / 2); a = (1 + dt A / 2) q = 2 q - 1.  v_rcp_f32 is accurate to 1 ulp, like the
        // exponential of the other schemes
        const float q = rcp_fast(__builtin_fmaf(-dt, c.hA, 1.0f));
        a = __builtin_fmaf(2.0f, q, -1.0f);
        g = dt * q;
    } else {
        a = exp2_fast(dt * c.A2);
        if constexpr (DISC == DISC_ZOH_S6) g = dt;
        else if constexpr (DISC == DISC_DIRAC) g = 1.0f;
        else g = zoh_gain(dt, c.A, c.rA, a);
    }
}

// Partials (da/ddt, da/dA, dg/ddt, dg/dA) given a, g of the same step.
template <int DISC>
__device__ __forceinline__ void disc_partials(float dt, const ACoef &c, float a, float g,
                                              float &a_t, float &a_A, float &g_t, float &g_A) {
    if constexpr (DISC == DISC_BILINEAR) {
        const float q = __builtin_fmaf(a, 0.5f, 0.5f);               // 1 / (1 - dt A / 2) = (a + 1) / 2
        const float q2 = q * q;
        a_t = c.A * q2; a_A = dt * q2; g_t = q2; g_A = 0.5f * dt * dt * q2;
    } else {
        a_t = c.A * a; a_A = dt * a;
        if constexpr (DISC == DISC_ZOH_S6) { g_t = 1.0f; g_A = 0.0f; }
        else if constexpr (DISC == DISC_DIRAC) { g_t = 0.0f; g_A = 0.0f; }
        else {
            g_t = a;
            // (dt A a - (a - 1)) / A^2 = (dt a - g) / A = dt^2 (1/2 + x/3 + x^2/8 + x^3/30 + ...), x = dt A.  A
            // rounding error e in a reaches the difference dt a - g as e / A, i.e. 2 eps / x^2 relative to it: the
            // closed form is used from |x| = 1/8 on (1e-5), the series below (first omitted term x^4/144 < 4e-6)
            const float x = dt * c.A;
            const float small = dt * dt * __builtin_fmaf(x, __builtin_fmaf(x, __builtin_fmaf(x, 0.033333335f, 0.125f), 0.33333334f), 0.5f);
            g_A = (fabsf(x) < 0.125f) ? small : __builtin_fmaf(dt, a, -g) * c.rA;
        }
    }
}

// ---------------------------------------------------------------- per-step inputs of the backward pass
// From the raw step input s = delta + bias, the upstream gradient dy and the gate input z of one time step:
// Delta and d Delta / d s, the gradient reaching ypre (y = ypre z sigmoid(z)) and the factor that turns ypre into dz
// (dz = dy ypre sigmoid(z) (1 + z (1 - sigmoid(z)))).
template <bool PRECISE = true>
__device__ __forceinline__ void bwd_step_inputs(float s, float dy, float z, bool softplus, bool has_z,
                                                float &sp, float &sg, float &dyp, float &zf) {
    if (softplus) softplus_sigmoid<PRECISE>(s, sp, sg); else { sp = s; sg = 1.0f; }
    if (has_z) {
        const float sz = sigmoid_fast(z);
        const float dsz = dy * sz;
        dyp = dsz * z;
        zf = dsz * __builtin_fmaf(z, 1.0f - sz, 1.0f);
    } else { zf = 0.0f; dyp = dy; }
}

// ---------------------------------------------------------------- wavefront scans over affine pairs
// One Hillis-Steele step on the pair held in (P,S): the pair of the lane named by the DPP
// control is composed in from the earlier side.  Both updates are single VALU instructions
// with a DPP source operand; a lane whose source lane does not exist, or whose row is
// masked off, is left unchanged (= composed with the identity).  The leading s_nop covers
// the two wait states a DPP read needs after a VALU write of the same register.
#define LRNNX_PAIR_STEP(P, S, CTRL)                                                   \
    asm("s_nop 1\n\t"                                                                 \
        "v_fmac_f32_dpp %0, %0, %1 " CTRL "\n\t"                                      \
        "v_mul_f32_dpp %1, %1, %1 " CTRL                                              \
        : "+v"(S), "+v"(P))

// The same step on two independent pairs at once.  Each pair's instructions give the other pair the wait states its
// next DPP read needs, so only the first step of a sequence carries the s_nop; the two dependent chains also fill
// each other's issue gaps.
#define LRNNX_PAIR_STEP2(NOP, P, S, CTRL, Q, R, CTRL2)                                \
    asm(NOP "v_fmac_f32_dpp %0, %0, %1 " CTRL "\n\t"                                  \
            "v_mul_f32_dpp %1, %1, %1 " CTRL "\n\t"                                   \
            "v_fmac_f32_dpp %2, %2, %3 " CTRL2 "\n\t"                                 \
            "v_mul_f32_dpp %3, %3, %3 " CTRL2                                         \
        : "+v"(S), "+v"(P), "+v"(R), "+v"(Q))

// Inclusive prefix over the 64 lanes, lane 0 first:  (P,S)_i <- (P,S)_i o ... o (P,S)_0.
__device__ __forceinline__ void wave_scan_fwd(float &P, float &S) {
    LRNNX_PAIR_STEP(P, S, "row_shr:1 row_mask:0xf bank_mask:0xf");
    LRNNX_PAIR_STEP(P, S, "row_shr:2 row_mask:0xf bank_mask:0xf");
    LRNNX_PAIR_STEP(P, S, "row_shr:4 row_mask:0xf bank_mask:0xf");
    LRNNX_PAIR_STEP(P, S, "row_shr:8 row_mask:0xf bank_mask:0xf");
    LRNNX_PAIR_STEP(P, S, "row_bcast:15 row_mask:0xa bank_mask:0xf");   // lane 15 of rows 0,2 -> rows 1,3
    LRNNX_PAIR_STEP(P, S, "row_bcast:31 row_mask:0xc bank_mask:0xf");   // lane 31 -> rows 2,3
}

// Inclusive prefixes of two independent pairs at once (two states of one channel): see LRNNX_PAIR_STEP2.
__device__ __forceinline__ void wave_scan_fwd2(float &P, float &S, float &Q, float &R) {
    LRNNX_PAIR_STEP2("s_nop 1\n\t", P, S, "row_shr:1 row_mask:0xf bank_mask:0xf", Q, R, "row_shr:1 row_mask:0xf bank_mask:0xf");
    LRNNX_PAIR_STEP2("", P, S, "row_shr:2 row_mask:0xf bank_mask:0xf", Q, R, "row_shr:2 row_mask:0xf bank_mask:0xf");
    LRNNX_PAIR_STEP2("", P, S, "row_shr:4 row_mask:0xf bank_mask:0xf", Q, R, "row_shr:4 row_mask:0xf bank_mask:0xf");
    LRNNX_PAIR_STEP2("", P, S, "row_shr:8 row_mask:0xf bank_mask:0xf", Q, R, "row_shr:8 row_mask:0xf bank_mask:0xf");
    LRNNX_PAIR_STEP2("", P, S, "row_bcast:15 row_mask:0xa bank_mask:0xf", Q, R, "row_bcast:15 row_mask:0xa bank_mask:0xf");
    LRNNX_PAIR_STEP2("", P, S, "row_bcast:31 row_mask:0xc bank_mask:0xf", Q, R, "row_bcast:31 row_mask:0xc bank_mask:0xf");
}

// ---------------------------------------------------------------- both scans of the backward pass, NK states at once
// The state prefix (P,S) and the adjoint suffix (Pr,Sr) of each of NK states advance together, one Hillis-Steele
// step of all 2 NK pairs per block of instructions.  The chains of different states are independent, so each fills
// the others' wait states (no s_nop between DPP steps) and, above all, the one LDS round trip of the suffix scan
// (the hand-over between rows: no DPP control moves data towards lower rows) is paid once per call instead of once
// per state: all 2 NK lane permutes are in flight while the prefix scans take their two broadcast steps.
// Hazards inside the blocks are kept by construction (a DPP read of a register comes at least three instructions
// after its last write); every block starts with s_nop 1 in case the compiler placed a copy right before it.
#define LRNNX_FR_STATE(s, p, r, q, CF, CR)                                             \
    "v_fmac_f32_dpp %" #s ", %" #s ", %" #p " " CF "\n\t"                               \
    "v_mul_f32_dpp %" #p ", %" #p ", %" #p " " CF "\n\t"                                \
    "v_fmac_f32_dpp %" #r ", %" #r ", %" #q " " CR "\n\t"                               \
    "v_mul_f32_dpp %" #q ", %" #q ", %" #q " " CR "\n\t"
#define LRNNX_F_STATE(s, p, CF)                                                        \
    "v_fmac_f32_dpp %" #s ", %" #s ", %" #p " " CF "\n\t"                               \
    "v_mul_f32_dpp %" #p ", %" #p ", %" #p " " CF "\n\t"
#define LRNNX_ALLROWS " row_mask:0xf bank_mask:0xf"

// One state only (NK = 1): the four in-row steps of its prefix and of its suffix in one block (four instructions per
// step, so a DPP read comes at least two instructions after the last write of its register) ...
__device__ __forceinline__ void scan_fr_rows_one(float &P, float &S, float &Pr, float &Sr) {
    asm("s_nop 1\n\t"
        LRNNX_FR_STATE(0, 1, 2, 3, "row_shr:1" LRNNX_ALLROWS, "row_shl:1" LRNNX_ALLROWS)
        LRNNX_FR_STATE(0, 1, 2, 3, "row_shr:2" LRNNX_ALLROWS, "row_shl:2" LRNNX_ALLROWS)
        LRNNX_FR_STATE(0, 1, 2, 3, "row_shr:4" LRNNX_ALLROWS, "row_shl:4" LRNNX_ALLROWS)
        LRNNX_FR_STATE(0, 1, 2, 3, "row_shr:8" LRNNX_ALLROWS, "row_shl:8" LRNNX_ALLROWS)
        : "+v"(S), "+v"(P), "+v"(Sr), "+v"(Pr));
}
// ... and the two steps of its prefix that cross rows (lane 15 of rows 0,2 -> rows 1,3; lane 31 -> rows 2,3; the
// last one leaves the product alone, nobody needs it afterwards)
__device__ __forceinline__ void scan_f_cross_one(float &P, float &S) {
    asm("s_nop 1\n\t" LRNNX_F_STATE(0, 1, "row_bcast:15 row_mask:0xa bank_mask:0xf")
        "s_nop 0\n\t"
        "v_fmac_f32_dpp %0, %0, %1 row_bcast:31 row_mask:0xc bank_mask:0xf"
        : "+v"(S), "+v"(P));
}

// All steps of the NK suffix scans inside their rows, and all steps of the NK prefix scans, as one block of
// instructions each (NK = 2 or 4).  Every leading s_nop and every boundary between blocks costs the wavefront an issue
// slot of its own, and a wavefront of the backward kernel is bound by the length of its own instruction stream.
// A step touches every state once, so a DPP read of a register comes at least two instructions after its last write.
#define LRNNX_STEP2(CTRL) LRNNX_F_STATE(0, 1, CTRL) LRNNX_F_STATE(2, 3, CTRL)
#define LRNNX_STEP4(CTRL) LRNNX_STEP2(CTRL) LRNNX_F_STATE(4, 5, CTRL) LRNNX_F_STATE(6, 7, CTRL)
#define LRNNX_S_ONLY(s, p, CTRL) "v_fmac_f32_dpp %" #s ", %" #s ", %" #p " " CTRL "\n\t"
template <int NK>
__device__ __forceinline__ void scan_r_rows(float *Pr, float *Sr) {
    static_assert(NK == 2 || NK == 4, "states per block");
    if constexpr (NK == 2) {
        asm("s_nop 1\n\t" LRNNX_STEP2("row_shl:1" LRNNX_ALLROWS) LRNNX_STEP2("row_shl:2" LRNNX_ALLROWS)
            LRNNX_STEP2("row_shl:4" LRNNX_ALLROWS) LRNNX_STEP2("row_shl:8" LRNNX_ALLROWS)
            : "+v"(Sr[0]), "+v"(Pr[0]), "+v"(Sr[1]), "+v"(Pr[1]));
    } else {
        asm("s_nop 1\n\t" LRNNX_STEP4("row_shl:1" LRNNX_ALLROWS) LRNNX_STEP4("row_shl:2" LRNNX_ALLROWS)
            LRNNX_STEP4("row_shl:4" LRNNX_ALLROWS) LRNNX_STEP4("row_shl:8" LRNNX_ALLROWS)
            : "+v"(Sr[0]), "+v"(Pr[0]), "+v"(Sr[1]), "+v"(Pr[1]), "+v"(Sr[2]), "+v"(Pr[2]), "+v"(Sr[3]), "+v"(Pr[3]));
    }
}
// inclusive prefixes of NK states, complete (lane 15 of rows 0,2 -> rows 1,3, then lane 31 -> rows 2,3; the last
// step leaves the products alone, nobody needs them afterwards)
template <int NK>
__device__ __forceinline__ void scan_f_all(float *P, float *S) {
    static_assert(NK == 2 || NK == 4, "states per block");
    if constexpr (NK == 2) {
        asm("s_nop 1\n\t" LRNNX_STEP2("row_shr:1" LRNNX_ALLROWS) LRNNX_STEP2("row_shr:2" LRNNX_ALLROWS)
            LRNNX_STEP2("row_shr:4" LRNNX_ALLROWS) LRNNX_STEP2("row_shr:8" LRNNX_ALLROWS)
            LRNNX_STEP2("row_bcast:15 row_mask:0xa bank_mask:0xf")
            LRNNX_S_ONLY(0, 1, "row_bcast:31 row_mask:0xc bank_mask:0xf") LRNNX_S_ONLY(2, 3, "row_bcast:31 row_mask:0xc bank_mask:0xf")
            : "+v"(S[0]), "+v"(P[0]), "+v"(S[1]), "+v"(P[1]));
    } else {
        asm("s_nop 1\n\t" LRNNX_STEP4("row_shr:1" LRNNX_ALLROWS) LRNNX_STEP4("row_shr:2" LRNNX_ALLROWS)
            LRNNX_STEP4("row_shr:4" LRNNX_ALLROWS) LRNNX_STEP4("row_shr:8" LRNNX_ALLROWS)
            LRNNX_STEP4("row_bcast:15 row_mask:0xa bank_mask:0xf")
            LRNNX_S_ONLY(0, 1, "row_bcast:31 row_mask:0xc bank_mask:0xf") LRNNX_S_ONLY(2, 3, "row_bcast:31 row_mask:0xc bank_mask:0xf")
            LRNNX_S_ONLY(4, 5, "row_bcast:31 row_mask:0xc bank_mask:0xf") LRNNX_S_ONLY(6, 7, "row_bcast:31 row_mask:0xc bank_mask:0xf")
            : "+v"(S[0]), "+v"(P[0]), "+v"(S[1]), "+v"(P[1]), "+v"(S[2]), "+v"(P[2]), "+v"(S[3]), "+v"(P[3]));
    }
}

// On return S holds the inclusive prefix (lane 0 first) and Sr the inclusive suffix (lane 63 first) of every state;
// P and Pr are left in an unspecified state.
template <int NK>
__device__ __forceinline__ void wave_scan_fwd_rev_multi(float *P, float *S, float *Pr, float *Sr, int lane) {
    // suffixes: rows 0 and 2 take the pair held by the first lane of the next row
    const int src = ((lane & 0x30) + 16) & 63;
    float Pp[NK], Sp[NK];
    if constexpr (NK == 1) {
        scan_fr_rows_one(P[0], S[0], Pr[0], Sr[0]);
        Pp[0] = bpermute(src, Pr[0]); Sp[0] = bpermute(src, Sr[0]);
        scan_f_cross_one(P[0], S[0]);
    } else {
        // the suffixes go first, so that the lane permutes of their hand-over between rows (one round trip through
        // the LDS crossbar) are in flight during all of the prefix scans
        scan_r_rows<NK>(Pr, Sr);
#pragma unroll
        for (int k = 0; k < NK; ++k) { Pp[k] = bpermute(src, Pr[k]); Sp[k] = bpermute(src, Sr[k]); }
        scan_f_all<NK>(P, S);
    }
    // rows 0, 2 only (row_mask 0x5); the other rows keep their pair
    if constexpr (NK == 4) {
        asm("s_nop 1\n\t"
            "v_fmac_f32_dpp %0, %8, %4 quad_perm:[0,1,2,3] row_mask:0x5 bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %1, %9, %5 quad_perm:[0,1,2,3] row_mask:0x5 bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %2, %10, %6 quad_perm:[0,1,2,3] row_mask:0x5 bank_mask:0xf\n\t"
            "v_fmac_f32_dpp %3, %11, %7 quad_perm:[0,1,2,3] row_mask:0x5 bank_mask:0xf\n\t"
            "v_mul_f32_dpp %4, %12, %4 quad_perm:[0,1,2,3] row_mask:0x5 bank_mask:0xf\n\t"
            "v_mul_f32_dpp %5, %13, %5 quad_perm:[0,1,2,3] row_mask:0x5 bank_mask:0xf\n\t"
            "v_mul_f32_dpp %6, %14, %6 quad_perm:[0,1,2,3] row_mask:0x5 bank_mask:0xf\n\t"
            "v_mul_f32_dpp %7, %15, %7 quad_perm:[0,1,2,3] row_mask:0x5 bank_mask:0xf"
            : "+v"(Sr[0]), "+v"(Sr[1]), "+v"(Sr[2]), "+v"(Sr[3]), "+v"(Pr[0]), "+v"(Pr[1]), "+v"(Pr[2]), "+v"(Pr[3])
            : "v"(Sp[0]), "v"(Sp[1]), "v"(Sp[2]), "v"(Sp[3]), "v"(Pp[0]), "v"(Pp[1]), "v"(Pp[2]), "v"(Pp[3]));
    } else {
#pragma unroll
        for (int k = 0; k < NK; ++k)
            asm("s_nop 1\n\t"
                "v_fmac_f32_dpp %0, %2, %1 quad_perm:[0,1,2,3] row_mask:0x5 bank_mask:0xf\n\t"
                "v_mul_f32_dpp %1, %3, %1 quad_perm:[0,1,2,3] row_mask:0x5 bank_mask:0xf"
                : "+v"(Sr[k]), "+v"(Pr[k]) : "v"(Sp[k]), "v"(Pp[k]));
    }
    // rows 0 and 1 take the suffix now held by lane 32: Sr += Pr * Sr[32] (the product of the multipliers is not
    // needed any more).  The value travels through a scalar register; the update runs with the upper half of the
    // wavefront switched off.  Wait states: one between the VALU write of Sr and its v_readlane, two between the
    // v_readlane and the VALU read of its scalar result.
    if constexpr (NK == 4) {
        unsigned save;
        float t0, t1, t2, t3;
        asm("s_nop 1\n\t"
            "v_readlane_b32 %4, %0, 32\n\t"
            "v_readlane_b32 %5, %1, 32\n\t"
            "v_readlane_b32 %6, %2, 32\n\t"
            "v_readlane_b32 %7, %3, 32\n\t"
            "s_mov_b32 %8, exec_hi\n\t"
            "s_mov_b32 exec_hi, 0\n\t"
            "v_fmac_f32 %0, %4, %9\n\t"
            "v_fmac_f32 %1, %5, %10\n\t"
            "v_fmac_f32 %2, %6, %11\n\t"
            "v_fmac_f32 %3, %7, %12\n\t"
            "s_mov_b32 exec_hi, %8"
            : "+v"(Sr[0]), "+v"(Sr[1]), "+v"(Sr[2]), "+v"(Sr[3]), "=&s"(t0), "=&s"(t1), "=&s"(t2), "=&s"(t3), "=&s"(save)
            : "v"(Pr[0]), "v"(Pr[1]), "v"(Pr[2]), "v"(Pr[3]));
    } else {
#pragma unroll
        for (int k = 0; k < NK; ++k) {
            unsigned save;
            float t0;
            asm("s_nop 1\n\t"
                "v_readlane_b32 %1, %0, 32\n\t"
                "s_mov_b32 %2, exec_hi\n\t"
                "s_mov_b32 exec_hi, 0\n\t"
                "v_fmac_f32 %0, %1, %3\n\t"
                "s_mov_b32 exec_hi, %2"
                : "+v"(Sr[k]), "=&s"(t0), "=&s"(save) : "v"(Pr[k]));
        }
    }
}

__device__ __forceinline__ float wave_sum(float v) {
    v += dpp<0x111>(0.0f, v);
    v += dpp<0x112>(0.0f, v);
    v += dpp<0x114>(0.0f, v);
    v += dpp<0x118>(0.0f, v);
    v += dpp<DPP_ROW_BCAST15, 0xA>(0.0f, v);
    v += dpp<DPP_ROW_BCAST31, 0xC>(0.0f, v);
    return readlane(v, 63);
}

// ---------------------------------------------------------------- I/O element access
template <typename IO> struct io_traits;
template <> struct io_traits<float> {
    static constexpr int EPC = 4;                                  // elements per 16-byte chunk
    __device__ static __forceinline__ float get(const float *p, int64_t i) { return p[i]; }
    __device__ static __forceinline__ void put(float *p, int64_t i, float v) { p[i] = v; }
    __device__ static __forceinline__ void unpack(const uint4 &r, float *o) {
        o[0] = i2f(r.x); o[1] = i2f(r.y); o[2] = i2f(r.z); o[3] = i2f(r.w);
    }
    __device__ static __forceinline__ uint4 pack(const float *v) {
        return make_uint4(f2i(v[0]), f2i(v[1]), f2i(v[2]), f2i(v[3]));
    }
};
typedef __bf16 bf16x2_native __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {   // round to nearest even
    floatx2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_native));
}
template <> struct io_traits<bf16_t> {
    static constexpr int EPC = 8;
    __device__ static __forceinline__ float get(const bf16_t *p, int64_t i) { return i2f((int)p[i].v << 16); }
    __device__ static __forceinline__ void put(bf16_t *p, int64_t i, float v) {
        p[i].v = (unsigned short)(pack_bf16x2(v, 0.0f) & 0xFFFFu);
    }
    __device__ static __forceinline__ void unpack(const uint4 &r, float *o) {
        o[0] = i2f(r.x << 16); o[1] = i2f(r.x & 0xFFFF0000u);
        o[2] = i2f(r.y << 16); o[3] = i2f(r.y & 0xFFFF0000u);
        o[4] = i2f(r.z << 16); o[5] = i2f(r.z & 0xFFFF0000u);
        o[6] = i2f(r.w << 16); o[7] = i2f(r.w & 0xFFFF0000u);
    }
    __device__ static __forceinline__ uint4 pack(const float *v) {
        return make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]),
                          pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
    }
};

// 16-, 8- and 4-byte accesses to the time axis of a [B,D,L] tensor are made at ELEMENT alignment: rows of packed
// variable-length batches start anywhere, and global memory takes unaligned vector accesses (the compiler is told
// the true alignment and still emits one instruction).  IO selects the alignment (2 or 4 bytes).
template <typename IO> struct ua;
template <> struct ua<float> {
    typedef uint4 __attribute__((aligned(4))) v4;
    typedef uint2 __attribute__((aligned(4))) v2;
    typedef uint32_t __attribute__((aligned(4))) v1;
};
template <> struct ua<bf16_t> {
    typedef uint4 __attribute__((aligned(2))) v4;
    typedef uint2 __attribute__((aligned(2))) v2;
    typedef uint32_t __attribute__((aligned(2))) v1;
};

// A lane's CNT consecutive elements row[l .. l+CNT), zero where l+i >= L.  `vec` allows vector accesses (the host
// sets it when every row pointer is element-aligned).
template <typename IO, int CNT>
__device__ __forceinline__ void load_seg(const IO *row, int64_t l, int64_t L, bool vec, float *out) {
    constexpr int EPC = io_traits<IO>::EPC;
    static_assert(CNT % EPC == 0, "segment must be whole 16-byte chunks");
#pragma unroll
    for (int c = 0; c < CNT / EPC; ++c) {
        int64_t lc = l + c * EPC;
        if (vec && lc + EPC <= L) {
            uint4 r = *reinterpret_cast<const typename ua<IO>::v4 *>(row + lc);
            io_traits<IO>::unpack(r, out + c * EPC);
        } else {
#pragma unroll
            for (int i = 0; i < EPC; ++i) out[c * EPC + i] = (lc + i < L) ? io_traits<IO>::get(row, lc + i) : 0.0f;
        }
    }
}
template <typename IO, int CNT>
__device__ __forceinline__ void store_seg(IO *row, int64_t l, int64_t L, bool vec, const float *v) {
    constexpr int EPC = io_traits<IO>::EPC;
#pragma unroll
    for (int c = 0; c < CNT / EPC; ++c) {
        int64_t lc = l + c * EPC;
        if (vec && lc + EPC <= L) {
            *reinterpret_cast<typename ua<IO>::v4 *>(row + lc) = io_traits<IO>::pack(v + c * EPC);
        } else {
#pragma unroll
            for (int i = 0; i < EPC; ++i) if (lc + i < L) io_traits<IO>::put(row, lc + i, v[c * EPC + i]);
        }
    }
}

// CNT contiguous elements starting at p, as floats.  p must be aligned to min(16, CNT*sizeof(IO)) bytes
// (CNT*sizeof(IO) is a power of two in every use).
template <typename IO, int CNT>
__device__ __forceinline__ void load_row(const IO *p, float *out) {
    constexpr int EPC = io_traits<IO>::EPC;
    constexpr int BYTES = CNT * (16 / EPC);
    if constexpr (BYTES % 16 == 0) {
#pragma unroll
        for (int c = 0; c < CNT / EPC; ++c) {
            uint4 r = reinterpret_cast<const uint4 *>(p)[c];
            io_traits<IO>::unpack(r, out + c * EPC);
        }
    } else if constexpr (BYTES == 8) {
        uint2 r = *reinterpret_cast<const uint2 *>(p);
        float tmp[EPC];
        io_traits<IO>::unpack(make_uint4(r.x, r.y, 0u, 0u), tmp);
#pragma unroll
        for (int i = 0; i < CNT; ++i) out[i] = tmp[i];
    } else if constexpr (BYTES == 4) {
        uint32_t r = *reinterpret_cast<const uint32_t *>(p);
        float tmp[EPC];
        io_traits<IO>::unpack(make_uint4(r, 0u, 0u, 0u), tmp);
#pragma unroll
        for (int i = 0; i < CNT; ++i) out[i] = tmp[i];
    } else {
#pragma unroll
        for (int i = 0; i < CNT; ++i) out[i] = io_traits<IO>::get(p, i);
    }
}

template <typename IO, int CNT, typename IDX>
__device__ __forceinline__ void store_few(IO *row, IDX l, IDX L, bool vec, const float *v) {
    constexpr int EPC = io_traits<IO>::EPC;
    constexpr int BYTES = CNT * (16 / EPC);
    if constexpr (CNT == 1) {                                   // one element: a single predicated access either way
        if (l < L) io_traits<IO>::put(row, l, v[0]);
    } else if (vec && l + CNT <= L && BYTES % 16 == 0) {
#pragma unroll
        for (int c = 0; c < BYTES / 16; ++c)
            reinterpret_cast<typename ua<IO>::v4 *>(row + l)[c] = io_traits<IO>::pack(v + c * EPC);
    } else if (vec && l + CNT <= L && (BYTES == 8 || BYTES == 4)) {
        float tmp[EPC];
#pragma unroll
        for (int i = 0; i < EPC; ++i) tmp[i] = i < CNT ? v[i] : 0.0f;
        uint4 r = io_traits<IO>::pack(tmp);
        if constexpr (BYTES == 8) *reinterpret_cast<typename ua<IO>::v2 *>(row + l) = make_uint2(r.x, r.y);
        else *reinterpret_cast<typename ua<IO>::v1 *>(row + l) = r.x;
    } else {
#pragma unroll
        for (int i = 0; i < CNT; ++i) if (l + i < L) io_traits<IO>::put(row, l + i, v[i]);
    }
}

// The same few elements as untouched 32-bit words, so that a load can be issued long before its
// data is needed (unpacking is a separate step and nothing waits on the load until then).
template <typename IO, int CNT>
struct RawFew {
    static constexpr int WORDS = (CNT * (16 / io_traits<IO>::EPC) + 3) / 4;
    uint32_t w[WORDS];
};
// One element, read without a branch and without touching the loaded register afterwards (so nothing waits for the
// load before its real use): past the end the last element is read again (L >= 1) and the CALLER discards it.
template <typename IO, typename IDX>
__device__ __forceinline__ void load_one_raw_clamped(const IO *row, IDX l, IDX L, RawFew<IO, 1> &r) {
    const IDX lc = l < L ? l : L - 1;
    if constexpr (sizeof(IO) == 4) r.w[0] = *reinterpret_cast<const uint32_t *>(row + lc);
    else r.w[0] = *reinterpret_cast<const unsigned short *>(row + lc);
}
template <typename IO, int CNT, typename IDX>
__device__ __forceinline__ void load_few_raw(const IO *row, IDX l, IDX L, bool vec, RawFew<IO, CNT> &r) {
    constexpr int BYTES = CNT * (16 / io_traits<IO>::EPC);
    constexpr int WORDS = RawFew<IO, CNT>::WORDS;
    if constexpr (CNT == 1) {
        // one element, read without a branch: past the end the last element is read again and dropped (L >= 1)
        const IDX lc = l < L ? l : L - 1;
        uint32_t v;
        if constexpr (sizeof(IO) == 4) v = *reinterpret_cast<const uint32_t *>(row + lc);
        else v = *reinterpret_cast<const unsigned short *>(row + lc);
        r.w[0] = l < L ? v : 0u;
    } else if (vec && l + CNT <= L) {
        if constexpr (BYTES % 16 == 0) {
#pragma unroll
            for (int c = 0; c < BYTES / 16; ++c) {
                const uint4 v = reinterpret_cast<const typename ua<IO>::v4 *>(row + l)[c];
                r.w[4 * c] = v.x; r.w[4 * c + 1] = v.y; r.w[4 * c + 2] = v.z; r.w[4 * c + 3] = v.w;
            }
        } else if constexpr (BYTES == 8) {
            const uint2 v = *reinterpret_cast<const typename ua<IO>::v2 *>(row + l);
            r.w[0] = v.x; r.w[1] = v.y;
        } else if constexpr (BYTES == 4) {
            r.w[0] = *reinterpret_cast<const typename ua<IO>::v1 *>(row + l);
        } else {
            r.w[0] = *reinterpret_cast<const unsigned short *>(row + l);
        }
    } else {
#pragma unroll
        for (int i = 0; i < WORDS; ++i) r.w[i] = 0u;
#pragma unroll
        for (int i = 0; i < CNT; ++i) {
            if (l + i < L) {
                if constexpr (sizeof(IO) == 4) r.w[i] = *reinterpret_cast<const uint32_t *>(row + l + i);
                else r.w[i / 2] |= (uint32_t)(*reinterpret_cast<const unsigned short *>(row + l + i)) << (16 * (i % 2));
            }
        }
    }
}
template <typename IO, int CNT>
__device__ __forceinline__ void unpack_few(const RawFew<IO, CNT> &r, float *out) {
#pragma unroll
    for (int i = 0; i < CNT; ++i) {
        if constexpr (sizeof(IO) == 4) out[i] = i2f((int)r.w[i]);
        else out[i] = (i % 2) ? i2f((int)(r.w[i / 2] & 0xFFFF0000u)) : i2f((int)(r.w[i / 2] << 16));
    }
}

}  // namespace lrnnx
