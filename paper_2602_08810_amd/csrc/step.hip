// Single-token updates for gfx950 (the `step` method of the paper's layers, Sec. 3): one application of Eq. 2
// to a carried state, for autoregressive generation.  Both kernels are pure streaming updates of the state
// (read once, written once); the selective one fuses softplus, discretisation, output projection and gate.
#include "kernels.hpp"
#include "scan_common.hpp"

namespace lrnnx {

// One thread per (b,d): x[b,d,:] <- a (.) x[b,d,:] + g Bm[b,:] u[b,d];  y[b,d] = Cm[b,:] . x + Dskip[d] u, gated.
template <typename IO, int N, int DISC>
__global__ __launch_bounds__(256) void k_ss_step(const StepParams p) {
    const int d = blockIdx.x * 256 + threadIdx.x;
    const int b = blockIdx.y;
    if (d >= p.D) return;
    const int64_t row = (int64_t)b * p.D + d;
    const float uu = io_traits<IO>::get(reinterpret_cast<const IO *>(p.u), b * p.u_sb + d * p.u_sd);
    const float s = io_traits<IO>::get(reinterpret_cast<const IO *>(p.delta), b * p.dl_sb + d * p.dl_sd) +
                    (p.bias ? p.bias[d] : 0.0f);
    float dt = s, sg;
    if (p.softplus) softplus_sigmoid(s, dt, sg);
    float xs[N], Av[N], Bv[N], Cv[N];
    if constexpr (N % 4 == 0) {
#pragma unroll
        for (int q = 0; q < N / 4; ++q) {
            const float4 vx = reinterpret_cast<const float4 *>(p.x + row * N)[q];
            const float4 va = reinterpret_cast<const float4 *>(p.A + (int64_t)d * N)[q];
            xs[4 * q] = vx.x; xs[4 * q + 1] = vx.y; xs[4 * q + 2] = vx.z; xs[4 * q + 3] = vx.w;
            Av[4 * q] = va.x; Av[4 * q + 1] = va.y; Av[4 * q + 2] = va.z; Av[4 * q + 3] = va.w;
        }
    } else {
#pragma unroll
        for (int n = 0; n < N; ++n) { xs[n] = p.x[row * N + n]; Av[n] = p.A[(int64_t)d * N + n]; }
    }
    load_row<IO, N>(reinterpret_cast<const IO *>(p.Bm) + (int64_t)b * N, Bv);
    load_row<IO, N>(reinterpret_cast<const IO *>(p.Cm) + (int64_t)b * N, Cv);
    float acc = p.Dskip ? p.Dskip[d] * uu : 0.0f;
#pragma unroll
    for (int n = 0; n < N; ++n) {
        const ACoef ac = make_acoef<DISC>(Av[n]);
        float a, g;
        disc_ag<DISC>(dt, ac, a, g);
        xs[n] = __builtin_fmaf(a, xs[n], g * Bv[n] * uu);
        acc = __builtin_fmaf(Cv[n], xs[n], acc);
    }
    if constexpr (N % 4 == 0) {
#pragma unroll
        for (int q = 0; q < N / 4; ++q)
            reinterpret_cast<float4 *>(p.x + row * N)[q] = make_float4(xs[4 * q], xs[4 * q + 1], xs[4 * q + 2], xs[4 * q + 3]);
    } else {
#pragma unroll
        for (int n = 0; n < N; ++n) p.x[row * N + n] = xs[n];
    }
    if (p.z) {
        const float zz = io_traits<IO>::get(reinterpret_cast<const IO *>(p.z), b * p.z_sb + d * p.z_sd);
        acc *= zz * sigmoid_fast(zz);
    }
    io_traits<IO>::put(reinterpret_cast<IO *>(p.y), b * p.y_sb + d * p.y_sd, acc);
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
    dim3 grid((p.D + 255) / 256, p.B), block(256);
    switch (p.N) {
        case 1: hipLaunchKernelGGL((k_ss_step<IO, 1, DISC>), grid, block, 0, s, p); break;
        case 2: hipLaunchKernelGGL((k_ss_step<IO, 2, DISC>), grid, block, 0, s, p); break;
        case 4: hipLaunchKernelGGL((k_ss_step<IO, 4, DISC>), grid, block, 0, s, p); break;
        case 8: hipLaunchKernelGGL((k_ss_step<IO, 8, DISC>), grid, block, 0, s, p); break;
        case 16: hipLaunchKernelGGL((k_ss_step<IO, 16, DISC>), grid, block, 0, s, p); break;
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
hipError_t launch_lti_step(int B, int P, const float2 *lambda, float2 *x, const float2 *v, hipStream_t s) {
    const int64_t n = (int64_t)B * P;
    hipLaunchKernelGGL(k_lti_step, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, B, P, lambda, x, v);
    return hipGetLastError();
}

}  // namespace lrnnx
