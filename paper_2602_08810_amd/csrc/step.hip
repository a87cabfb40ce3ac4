// Single-token updates for gfx950 (the `step` method of the paper's layers, Sec. 3): one application of Eq. 2
// to a carried state, for autoregressive generation.  Both kernels are pure streaming updates of the state
// (read once, written once); the selective one fuses softplus, discretisation, output projection and gate.
#include "kernels.hpp"
#include "scan_common.hpp"
#include "cplx_common.hpp"

namespace lrnnx {

// x[b,d,:] <- a (.) x[b,d,:] + g Bm[b,:] u[b,d];  y[b,d] = Cm[b,:] . x + Dskip[d] u, gated.
// A thread owns 4 consecutive states of one (b,d) (all of them when N < 4), so that the lanes of a wavefront read and
// write the state as one contiguous run of 16-byte pieces; the N/4 lanes of a row are neighbours and sum their parts of
// y with xor-shuffles.  The per-row scalars (u, delta, z, bias) are loaded by every lane of the row (same address).
template <typename IO, int N, int DISC>
__global__ __launch_bounds__(256) void k_ss_step(const StepParams p) {
    constexpr int NPT = N >= 4 ? 4 : N;        // states per thread
    constexpr int Q = N / NPT;                 // threads per (b,d) row: a power of two, at most 64
    const int64_t i = blockIdx.x * (int64_t)256 + threadIdx.x;
    const int64_t total = (int64_t)p.B * p.D * Q;
    const bool live = i < total;               // dead lanes still take part in the shuffles below
    const int64_t row = live ? i / Q : 0;
    const int q = (int)(i % Q);
    const int b = (int)(row / p.D), d = (int)(row % p.D);
    const float uu = io_traits<IO>::get(reinterpret_cast<const IO *>(p.u), b * p.u_sb + d * p.u_sd);
    const float s = io_traits<IO>::get(reinterpret_cast<const IO *>(p.delta), b * p.dl_sb + d * p.dl_sd) +
                    (p.bias ? p.bias[d] : 0.0f);
    float dt = s, sg;
    if (p.softplus) softplus_sigmoid(s, dt, sg);
    float xs[NPT], Av[NPT], Bv[NPT], Cv[NPT];
    float *xp = p.x + row * N + q * NPT;
    const float *ap = p.A + (int64_t)d * N + q * NPT;
    if constexpr (NPT == 4) {
        const float4 vx = *reinterpret_cast<const float4 *>(xp), va = *reinterpret_cast<const float4 *>(ap);
        xs[0] = vx.x; xs[1] = vx.y; xs[2] = vx.z; xs[3] = vx.w;
        Av[0] = va.x; Av[1] = va.y; Av[2] = va.z; Av[3] = va.w;
    } else {
#pragma unroll
        for (int n = 0; n < NPT; ++n) { xs[n] = xp[n]; Av[n] = ap[n]; }
    }
    const int64_t bc = ((int64_t)b * p.bcg + d / p.dpg) * N + q * NPT;   // this channel's group of the maps
    load_row<IO, NPT>(reinterpret_cast<const IO *>(p.Bm) + bc, Bv);
    load_row<IO, NPT>(reinterpret_cast<const IO *>(p.Cm) + bc, Cv);
    float acc = 0.0f;
#pragma unroll
    for (int n = 0; n < NPT; ++n) {
        const ACoef ac = make_acoef<DISC>(Av[n]);
        float a, g;
        disc_ag<DISC>(dt, ac, a, g);
        xs[n] = __builtin_fmaf(a, xs[n], g * Bv[n] * uu);
        acc = __builtin_fmaf(Cv[n], xs[n], acc);
    }
    if (live) {
        if constexpr (NPT == 4) *reinterpret_cast<float4 *>(xp) = make_float4(xs[0], xs[1], xs[2], xs[3]);
        else {
#pragma unroll
            for (int n = 0; n < NPT; ++n) xp[n] = xs[n];
        }
    }
#pragma unroll
    for (int m = 1; m < Q; m <<= 1) acc += __shfl_xor(acc, m, 64);
    if (live && q == 0) {
        if (p.Dskip) acc = __builtin_fmaf(p.Dskip[d], uu, acc);
        if (p.z) {
            const float zz = io_traits<IO>::get(reinterpret_cast<const IO *>(p.z), b * p.z_sb + d * p.z_sd);
            acc *= zz * sigmoid_fast(zz);
        }
        io_traits<IO>::put(reinterpret_cast<IO *>(p.y), b * p.y_sb + d * p.y_sd, acc);
    }
}

// The same with a complex diagonal A: x[b,d,:] <- a (.) x[b,d,:] + g Bm[b,:] u[b,d] in complex arithmetic,
// y[b,d] = Re(Cm[b,:] . x) + Dskip[d] u, gated.  A thread owns 2 consecutive complex states (16 bytes of state).
template <typename IO, int N, int DISC>
__global__ __launch_bounds__(256) void k_ss_cstep(const CStepParams p) {
    using CW = typename cword<IO>::type;
    constexpr int NPT = N >= 2 ? 2 : 1;        // complex states per thread
    constexpr int Q = N / NPT;                 // threads per (b,d) row: a power of two, at most 64
    const int64_t i = blockIdx.x * (int64_t)256 + threadIdx.x;
    const int64_t total = (int64_t)p.B * p.D * Q;
    const bool live = i < total;               // dead lanes still take part in the shuffles below
    const int64_t row = live ? i / Q : 0;
    const int q = (int)(i % Q);
    const int b = (int)(row / p.D), d = (int)(row % p.D);
    const float uu = io_traits<IO>::get(reinterpret_cast<const IO *>(p.u), b * p.u_sb + d * p.u_sd);
    const float s = io_traits<IO>::get(reinterpret_cast<const IO *>(p.delta), b * p.dl_sb + d * p.dl_sd) +
                    (p.bias ? p.bias[d] : 0.0f);
    float dt = s, sg;
    if (p.softplus) softplus_sigmoid(s, dt, sg);
    float2 xs[NPT], Av[NPT];
    CW bw[NPT], cw[NPT];
    float2 *xp = p.x + row * N + q * NPT;
    const float2 *ap = p.A + (int64_t)d * N + q * NPT;
    load_cwords<float2, NPT>(xp, xs);
    load_cwords<float2, NPT>(ap, Av);
    const int64_t bc = ((int64_t)b * p.bcg + d / p.dpg) * N + q * NPT;   // this channel's group of the maps
    load_cwords<CW, NPT>(reinterpret_cast<const CW *>(p.Bm) + bc, bw);
    load_cwords<CW, NPT>(reinterpret_cast<const CW *>(p.Cm) + bc, cw);
    float acc = 0.0f;
#pragma unroll
    for (int n = 0; n < NPT; ++n) {
        const CCoef cc = make_ccoef(Av[n].x, Av[n].y);
        float2 a, g;
        cdisc_ag<DISC>(dt, cc, a, g);
        const float2 Bv = cword<IO>::unpack(bw[n]), Cv = cword<IO>::unpack(cw[n]);
        const float2 gu = make_float2(g.x * uu, g.y * uu);
        xs[n] = cxfma(a, xs[n], cxmul(gu, Bv));
        acc = __builtin_fmaf(Cv.x, xs[n].x, __builtin_fmaf(-Cv.y, xs[n].y, acc));
    }
    if (live) {
#pragma unroll
        for (int n = 0; n < NPT; ++n) xp[n] = xs[n];
    }
#pragma unroll
    for (int m = 1; m < Q; m <<= 1) acc += __shfl_xor(acc, m, 64);
    if (live && q == 0) {
        if (p.Dskip) acc = __builtin_fmaf(p.Dskip[d], uu, acc);
        if (p.z) {
            const float zz = io_traits<IO>::get(reinterpret_cast<const IO *>(p.z), b * p.z_sb + d * p.z_sd);
            acc *= zz * sigmoid_fast(zz);
        }
        io_traits<IO>::put(reinterpret_cast<IO *>(p.y), b * p.y_sb + d * p.y_sd, acc);
    }
}

// One thread per (b,p): x[b,p] <- lambda[p] x[b,p] + v[b,p], complex.
__global__ __launch_bounds__(256) void k_lti_step(int B, int P, const float2 *lambda, float2 *x, const float2 *v) {
    const int64_t i = blockIdx.x * (int64_t)256 + threadIdx.x;
    if (i >= (int64_t)B * P) return;
    const float2 l = lambda[i % P], xv = x[i], vv = v[i];
    x[i] = make_float2(__builtin_fmaf(l.x, xv.x, __builtin_fmaf(-l.y, xv.y, vv.x)),
                       __builtin_fmaf(l.x, xv.y, __builtin_fmaf(l.y, xv.x, vv.y)));
}

template <typename IO, int DISC>
static hipError_t launch_step_disc(const StepParams &p, hipStream_t s) {
    const int64_t threads = (int64_t)p.B * p.D * (p.N >= 4 ? p.N / 4 : 1);
    dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    switch (p.N) {
        case 1: hipLaunchKernelGGL((k_ss_step<IO, 1, DISC>), grid, block, 0, s, p); break;
        case 2: hipLaunchKernelGGL((k_ss_step<IO, 2, DISC>), grid, block, 0, s, p); break;
        case 4: hipLaunchKernelGGL((k_ss_step<IO, 4, DISC>), grid, block, 0, s, p); break;
        case 8: hipLaunchKernelGGL((k_ss_step<IO, 8, DISC>), grid, block, 0, s, p); break;
        case 16: hipLaunchKernelGGL((k_ss_step<IO, 16, DISC>), grid, block, 0, s, p); break;
        case 32: hipLaunchKernelGGL((k_ss_step<IO, 32, DISC>), grid, block, 0, s, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
template <typename IO>
static hipError_t launch_step_io(const StepParams &p, int disc, hipStream_t s) {
    switch (disc) {
        case DISC_ZOH_S6: return launch_step_disc<IO, DISC_ZOH_S6>(p, s);
        case DISC_ZOH: return launch_step_disc<IO, DISC_ZOH>(p, s);
        case DISC_BILINEAR: return launch_step_disc<IO, DISC_BILINEAR>(p, s);
        case DISC_DIRAC: return launch_step_disc<IO, DISC_DIRAC>(p, s);
    }
    return hipErrorInvalidValue;
}
hipError_t launch_ss_step(const StepParams &p, int io_dtype, int disc, hipStream_t s) {
    return io_dtype == 1 ? launch_step_io<bf16_t>(p, disc, s) : launch_step_io<float>(p, disc, s);
}
template <typename IO, int DISC>
static hipError_t launch_cstep_disc(const CStepParams &p, hipStream_t s) {
    const int64_t threads = (int64_t)p.B * p.D * (p.N >= 2 ? p.N / 2 : 1);
    dim3 grid((unsigned)((threads + 255) / 256)), block(256);
    switch (p.N) {
        case 1: hipLaunchKernelGGL((k_ss_cstep<IO, 1, DISC>), grid, block, 0, s, p); break;
        case 2: hipLaunchKernelGGL((k_ss_cstep<IO, 2, DISC>), grid, block, 0, s, p); break;
        case 4: hipLaunchKernelGGL((k_ss_cstep<IO, 4, DISC>), grid, block, 0, s, p); break;
        case 8: hipLaunchKernelGGL((k_ss_cstep<IO, 8, DISC>), grid, block, 0, s, p); break;
        case 16: hipLaunchKernelGGL((k_ss_cstep<IO, 16, DISC>), grid, block, 0, s, p); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}
template <typename IO>
static hipError_t launch_cstep_io(const CStepParams &p, int disc, hipStream_t s) {
    switch (disc) {
        case DISC_ZOH_S6: return launch_cstep_disc<IO, DISC_ZOH_S6>(p, s);
        case DISC_ZOH: return launch_cstep_disc<IO, DISC_ZOH>(p, s);
        case DISC_BILINEAR: return launch_cstep_disc<IO, DISC_BILINEAR>(p, s);
        case DISC_DIRAC: return launch_cstep_disc<IO, DISC_DIRAC>(p, s);
    }
    return hipErrorInvalidValue;
}
hipError_t launch_ss_cstep(const CStepParams &p, int io_dtype, int disc, hipStream_t s) {
    return io_dtype == 1 ? launch_cstep_io<bf16_t>(p, disc, s) : launch_cstep_io<float>(p, disc, s);
}

hipError_t launch_lti_step(int B, int P, const float2 *lambda, float2 *x, const float2 *v, hipStream_t s) {
    const int64_t n = (int64_t)B * P;
    hipLaunchKernelGGL(k_lti_step, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, B, P, lambda, x, v);
    return hipGetLastError();
}

}  // namespace lrnnx
