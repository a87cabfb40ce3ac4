// Complex-arithmetic building blocks shared by the forward and backward selective-scan kernels with a complex
// diagonal state matrix: the complex word of the I/O type, exp(dt A) through the hardware exp2 / sin / cos, the four
// discretisations of Sec. 3 of the paper in complex arithmetic, and one Hillis-Steele step on a complex affine pair.
#pragma once
#include "scan_common.hpp"

namespace lrnnx {

template <typename IO> struct cword;                   // one complex number in the I/O type, as stored in LDS
template <> struct cword<bf16_t> {
    using type = uint32_t;
    static __device__ __forceinline__ float2 unpack(uint32_t w) { return make_float2(i2f((int)(w << 16)), i2f((int)(w & 0xFFFF0000u))); }
};
template <> struct cword<float> {
    using type = float2;
    static __device__ __forceinline__ float2 unpack(float2 w) { return w; }
};

// NK consecutive complex words, 16 bytes at a time where they fill whole 16-byte chunks (the caller's base pointer
// is 16-byte aligned and the row pitch N * sizeof(CW) is then a multiple of 16 too)
template <typename CW, int NK>
__device__ __forceinline__ void load_cwords(const CW *p, CW *out) {
    constexpr int BYTES = NK * (int)sizeof(CW);
    if constexpr (BYTES % 16 == 0) {
        uint4 r[BYTES / 16];
#pragma unroll
        for (int c = 0; c < BYTES / 16; ++c) r[c] = reinterpret_cast<const uint4 *>(p)[c];
        __builtin_memcpy(out, r, BYTES);
    } else {
#pragma unroll
        for (int k = 0; k < NK; ++k) out[k] = p[k];
    }
}

constexpr float kInv2Pi = 0.15915494309189535f;

// a = exp(dt A) for complex A = (Ar, Ai): e^{dt Ar} (cos(dt Ai), sin(dt Ai)).  v_sin/v_cos take revolutions and are
// only valid within +-256 of them, so the whole revolutions are dropped first (v_fract_f32): any dt Im(A) is
// accepted; the phase keeps the absolute accuracy of the fp32 product, |dt Im(A) / 2 pi| * 2^-24 revolutions.
__device__ __forceinline__ float2 cexp_dt(float dt, float A2r, float Arev) {
    const float e = exp2_fast(dt * A2r);
    const float rev = __builtin_amdgcn_fractf(dt * Arev);
    return make_float2(e * __builtin_amdgcn_cosf(rev), e * __builtin_amdgcn_sinf(rev));
}

struct CCoef {
    float Ar, Ai;       // A
    float A2r, Arev;    // Ar * log2(e), Ai / (2 pi): arguments of the hardware exp2 / sin / cos
    float iAr, iAi;     // 1 / A
};
__device__ __forceinline__ CCoef make_ccoef(float Ar, float Ai) {
    CCoef c;
    c.Ar = Ar; c.Ai = Ai; c.A2r = Ar * kLog2e; c.Arev = Ai * kInv2Pi;
    const float den = Ar * Ar + Ai * Ai;
    const float r = den > 0.0f ? rcp_fast(den) : 0.0f;
    c.iAr = Ar * r; c.iAi = -Ai * r;
    return c;
}

// multiplier a and input gain g of one step (schemes of Sec. 3, complex arithmetic)
template <int DISC>
__device__ __forceinline__ void cdisc_ag(float dt, const CCoef &c, float2 &a, float2 &g) {
    if constexpr (DISC == DISC_BILINEAR) {
        const float hr = 0.5f * dt * c.Ar, hi = 0.5f * dt * c.Ai;           // dt A / 2
        const float wr = 1.0f - hr, wi = -hi;                               // 1 - dt A / 2
        const float r = rcp_fast(wr * wr + wi * wi);
        const float ir = wr * r, ii = -wi * r;                              // 1 / (1 - dt A / 2)
        a = make_float2(__builtin_fmaf(2.0f, ir, -1.0f), 2.0f * ii);        // (1 + dt A / 2) / (1 - dt A / 2) = 2 / (1 - dt A / 2) - 1
        g = make_float2(dt * ir, dt * ii);
    } else {
        a = cexp_dt(dt, c.A2r, c.Arev);
        if constexpr (DISC == DISC_ZOH_S6) g = make_float2(dt, 0.0f);
        else if constexpr (DISC == DISC_DIRAC) g = make_float2(1.0f, 0.0f);
        else {                                                              // exact ZOH: (a - 1) / A
            const float zr = dt * c.Ar, zi = dt * c.Ai;
            // small |z|: dt (1 + z/2 + z^2/6 + z^3/24), Horner in complex arithmetic
            float pr = 1.0f + zr * 0.25f, pi = zi * 0.25f;                  // 1 + z/4
            float tr = pr * zr - pi * zi, ti = pr * zi + pi * zr;           // z (1 + z/4)
            pr = 1.0f + tr * 0.33333334f; pi = ti * 0.33333334f;            // 1 + z/3 (1 + z/4)
            tr = pr * zr - pi * zi; ti = pr * zi + pi * zr;
            pr = 1.0f + tr * 0.5f; pi = ti * 0.5f;                          // 1 + z/2 (1 + z/3 (1 + z/4))
            const float sr = dt * pr, si = dt * pi;
            const float mr = a.x - 1.0f, mi = a.y;
            const float dr = mr * c.iAr - mi * c.iAi, di = mr * c.iAi + mi * c.iAr;
            const bool small = zr * zr + zi * zi < 0.015625f;
            g = make_float2(small ? sr : dr, small ? si : di);
        }
    }
}

// One Hillis-Steele step on a complex affine pair.  Lanes without a source lane (or in a masked row) read the
// identity pair, which leaves them unchanged.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void cpair_step(float2 &P, float2 &S) {
    const float qr = dpp<CTRL, ROW_MASK>(1.0f, P.x), qi = dpp<CTRL, ROW_MASK>(0.0f, P.y);
    const float tr = dpp<CTRL, ROW_MASK>(0.0f, S.x), ti = dpp<CTRL, ROW_MASK>(0.0f, S.y);
    S = make_float2(__builtin_fmaf(P.x, tr, __builtin_fmaf(-P.y, ti, S.x)),
                    __builtin_fmaf(P.x, ti, __builtin_fmaf(P.y, tr, S.y)));
    P = make_float2(P.x * qr - P.y * qi, P.x * qi + P.y * qr);
}
__device__ __forceinline__ void cwave_scan_fwd(float2 &P, float2 &S) {
    cpair_step<0x111, 0xF>(P, S);
    cpair_step<0x112, 0xF>(P, S);
    cpair_step<0x114, 0xF>(P, S);
    cpair_step<0x118, 0xF>(P, S);
    cpair_step<DPP_ROW_BCAST15, 0xA>(P, S);
    cpair_step<DPP_ROW_BCAST31, 0xC>(P, S);
}


// ---------------------------------------------------------------- complex arithmetic on float2
__device__ __forceinline__ float2 cxmul(float2 a, float2 b) {
    return make_float2(__builtin_fmaf(a.x, b.x, -a.y * b.y), __builtin_fmaf(a.x, b.y, a.y * b.x));
}
__device__ __forceinline__ float2 cxmulc(float2 a, float2 b) {        // a * conj(b)
    return make_float2(__builtin_fmaf(a.x, b.x, a.y * b.y), __builtin_fmaf(a.y, b.x, -a.x * b.y));
}
__device__ __forceinline__ float2 cxfma(float2 a, float2 b, float2 c) {   // a * b + c
    return make_float2(__builtin_fmaf(a.x, b.x, __builtin_fmaf(-a.y, b.y, c.x)),
                       __builtin_fmaf(a.x, b.y, __builtin_fmaf(a.y, b.x, c.y)));
}
__device__ __forceinline__ float2 cxcfma(float2 a, float2 b, float2 c) {  // conj(a) * b + c
    return make_float2(__builtin_fmaf(a.x, b.x, __builtin_fmaf(a.y, b.y, c.x)),
                       __builtin_fmaf(a.x, b.y, __builtin_fmaf(-a.y, b.x, c.y)));
}

// Partials (da/ddt, da/dA, dg/ddt, dg/dA) of one step given its a and g; a and g are holomorphic in A.
template <int DISC>
__device__ __forceinline__ void cdisc_partials(float dt, const CCoef &c, float2 a, float2 g,
                                               float2 &a_t, float2 &a_A, float2 &g_t, float2 &g_A) {
    const float2 Ac = make_float2(c.Ar, c.Ai);
    if constexpr (DISC == DISC_BILINEAR) {
        const float2 q = make_float2(__builtin_fmaf(a.x, 0.5f, 0.5f), 0.5f * a.y);   // 1 / (1 - dt A / 2) = (a + 1) / 2
        const float2 q2 = cxmul(q, q);
        a_t = cxmul(Ac, q2);
        a_A = make_float2(dt * q2.x, dt * q2.y);
        g_t = q2;
        const float h = 0.5f * dt * dt;
        g_A = make_float2(h * q2.x, h * q2.y);
    } else {
        a_t = cxmul(Ac, a);
        a_A = make_float2(dt * a.x, dt * a.y);
        if constexpr (DISC == DISC_ZOH_S6) { g_t = make_float2(1.0f, 0.0f); g_A = make_float2(0.0f, 0.0f); }
        else if constexpr (DISC == DISC_DIRAC) { g_t = make_float2(0.0f, 0.0f); g_A = make_float2(0.0f, 0.0f); }
        else {
            g_t = a;
            // (dt A a - (a - 1)) / A^2 = (dt a - g) / A; for small z = dt A: dt^2 (1/2 + z/3 + z^2/8 + z^3/30)
            const float2 z = make_float2(dt * c.Ar, dt * c.Ai);
            float2 s = make_float2(0.125f + z.x * 0.033333335f, z.y * 0.033333335f);
            s = cxmul(s, z); s.x += 0.33333334f;
            s = cxmul(s, z); s.x += 0.5f;
            const float d2 = dt * dt;
            const float2 big = cxmul(make_float2(__builtin_fmaf(dt, a.x, -g.x), __builtin_fmaf(dt, a.y, -g.y)),
                                     make_float2(c.iAr, c.iAi));
            const bool small = z.x * z.x + z.y * z.y < 0.015625f;
            g_A = make_float2(small ? d2 * s.x : big.x, small ? d2 * s.y : big.y);
        }
    }
}

// Both scans of the backward pass: inclusive prefix of (P,S) over the lanes (lane 0 first) and inclusive suffix of
// (Pr,Sr) (lane 63 first); the two are independent and their steps alternate.
__device__ __forceinline__ void cwave_scan_fwd_rev(float2 &P, float2 &S, float2 &Pr, float2 &Sr, int lane) {
    cpair_step<0x111, 0xF>(P, S);  cpair_step<0x101, 0xF>(Pr, Sr);      // row_shr / row_shl : 1
    cpair_step<0x112, 0xF>(P, S);  cpair_step<0x102, 0xF>(Pr, Sr);
    cpair_step<0x114, 0xF>(P, S);  cpair_step<0x104, 0xF>(Pr, Sr);
    cpair_step<0x118, 0xF>(P, S);  cpair_step<0x108, 0xF>(Pr, Sr);
    const int src = ((lane & 0x30) + 16) & 63;                          // first lane of the next row
    float2 Pp = make_float2(bpermute(src, Pr.x), bpermute(src, Pr.y));
    float2 Sp = make_float2(bpermute(src, Sr.x), bpermute(src, Sr.y));
    cpair_step<DPP_ROW_BCAST15, 0xA>(P, S);
    cpair_step<DPP_ROW_BCAST31, 0xC>(P, S);
    {   // rows 0 and 2 take the suffix held by the first lane of the next row
        const bool take = ((lane >> 4) & 1) == 0;
        Pp = take ? Pp : make_float2(1.0f, 0.0f); Sp = take ? Sp : make_float2(0.0f, 0.0f);
        Sr = cxfma(Pr, Sp, Sr); Pr = cxmul(Pr, Pp);
    }
    {   // rows 0 and 1 take the suffix held by lane 32
        float2 Pq = make_float2(bpermute(32, Pr.x), bpermute(32, Pr.y));
        float2 Sq = make_float2(bpermute(32, Sr.x), bpermute(32, Sr.y));
        const bool take = lane < 32;
        Pq = take ? Pq : make_float2(1.0f, 0.0f); Sq = take ? Sq : make_float2(0.0f, 0.0f);
        Sr = cxfma(Pr, Sq, Sr); Pr = cxmul(Pr, Pq);
    }
}

}  // namespace lrnnx
