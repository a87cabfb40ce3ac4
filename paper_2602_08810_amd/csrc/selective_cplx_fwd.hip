// Selective scan, forward, with a COMPLEX diagonal state matrix for gfx950:
//     x_{l,n} = a(Delta_l, A[d,n]) x_{l-1,n} + g(Delta_l, A[d,n]) Bm[b,l,n] u[b,d,l]        (complex)
//     y[b,d,l] = Re( sum_n Cm[b,l,n] x_{l,n} ) + Dskip[d] u[b,d,l],  then the optional gate
// (Eq. 2 of the paper with the output taken as Re(C x): the complex-diagonal layers of Sec. 2.2.1 with an
// input-dependent step size and input-dependent maps).
//
// Same mapping as the real forward kernel: time on lanes (a lane owns T = 8 consecutive steps), one wavefront per
// channel, the 8 wavefronts of a workgroup share the staged Bm/Cm tile.  The complex maps stay in LDS in their I/O
// type (a bf16 pair is one 32-bit word, so the tile is as large as the real kernel's fp32 tile) and are copied there
// word by word.  The affine pairs are complex: one Hillis-Steele step composes (P,S) o (P',S') = (P P', P S' + S)
// with four DPP reads and eight multiply-adds.  Per-state values that are uniform over the wavefront (A, the carried
// state) live one per lane and are read with v_readlane, so the loop over states stays rolled.
#include "kernels.hpp"
#include "scan_common.hpp"
#include "cplx_common.hpp"

namespace lrnnx {


// AGG: the aggregate launch of the chunk-carry path (no y, no checkpoints; the chunk's pair instead)
template <typename IO, int N, int T, int W, int DISC, bool AGG>
__global__ __launch_bounds__(W * 64, 2) void k_ss_cfwd(const CFwdParams p) {
    using CW = typename cword<IO>::type;
    constexpr int TQ = T / 4;
    constexpr int QS = 256 + (TQ > 1 ? 32 / TQ : 0);   // words per quarter-plane, padded against bank conflicts on staging
    constexpr int PLANE = TQ * QS;                     // words per state index n
    constexpr int TILE = 64 * T;
    static_assert(T % 4 == 0, "steps per lane");
    __shared__ __attribute__((aligned(16))) CW sB[N * PLANE];
    __shared__ __attribute__((aligned(16))) CW sC[N * PLANE];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b = blockIdx.y;
    // a workgroup takes W consecutive channels of ONE Bm/Cm group (it stages that group's maps in LDS)
    const int blk_per_grp = (p.dpg + W - 1) / W;
    const int grp = blockIdx.x / blk_per_grp;
    const int d_in = (blockIdx.x % blk_per_grp) * W + w;
    const bool active = d_in < p.dpg;
    const int d = grp * p.dpg + (active ? d_in : p.dpg - 1);
    // Packed variable-length mode (p.cu != nullptr): batch entry b is the sequence of steps cu[b] .. cu[b+1]-1 of ONE
    // packed time axis of p.L steps; I/O rows have no batch stride, the maps are [G, p.L, N].  The bounds are
    // clamped to the packed axis, so no content of cu can send an access out of the buffers.
    int64_t L = p.L, toff = 0, bs = b;
    if (p.cu) {
        int64_t o = p.cu[b], e = p.cu[b + 1];
        o = o < 0 ? 0 : (o > p.L ? p.L : o);
        e = e < o ? o : (e > p.L ? p.L : e);
        toff = o; L = e - o; bs = 0;
    }
    const int64_t ntiles = (L + TILE - 1) / TILE;
    const int chunk = blockIdx.z;
    [[maybe_unused]] const int mode = p.mode;
    const int64_t tile0 = (int64_t)chunk * p.tiles_per_chunk;
    const int64_t tile1 = (tile0 + p.tiles_per_chunk < ntiles) ? tile0 + p.tiles_per_chunk : ntiles;
    const int64_t row = (int64_t)b * p.D + d;
    const bool vec = p.vec != 0;

    const IO *urow = reinterpret_cast<const IO *>(p.u) + bs * p.u_sb + d * p.u_sd + toff;
    const IO *drow = reinterpret_cast<const IO *>(p.delta) + bs * p.dl_sb + d * p.dl_sd + toff;
    const IO *zrow = p.z ? reinterpret_cast<const IO *>(p.z) + bs * p.z_sb + d * p.z_sd + toff : nullptr;
    const bool want_y = !AGG && p.y != nullptr;         // a state-only sweep (checkpoints for the backward pass) has no y
    IO *yrow = reinterpret_cast<IO *>(p.y) + bs * p.y_sb + d * p.y_sd + toff;
    // checkpoints of this row: [B,D,nck,N], or packed [D,nslots,N] with sequence b starting at slot toff/interval + b
    const int64_t ck0 = p.cu ? (int64_t)d * p.nslots + toff / kCkptInterval + b
                             : row * ((L + kCkptInterval - 1) / kCkptInterval);
    const int64_t bc0 = ((bs * p.bcg + grp) * p.L + toff) * N;       // first complex element of the maps of this sequence
    const CW *Bm = reinterpret_cast<const CW *>(p.Bm) + bc0;
    const CW *Cm = reinterpret_cast<const CW *>(p.Cm) + bc0;

    // lane n holds the constants and the carried state of state n
    float Arv = 0.0f, Aiv = 0.0f, xrv = 0.0f, xiv = 0.0f;
    float prv = 1.0f, piv = 0.0f;                       // MODE_AGG: product of the chunk's multipliers
    if (lane < N) {
        const float2 Av = p.A[d * N + lane];
        Arv = Av.x; Aiv = Av.y;
        if (!AGG && mode == MODE_APPLY) { const float2 x0 = p.ws_S[(row * p.nchunks + chunk) * N + lane]; xrv = x0.x; xiv = x0.y; }
        else if (!AGG && p.x0) { const float2 x0 = p.x0[row * N + lane]; xrv = x0.x; xiv = x0.y; }
    }
    const float Dsk = p.Dskip ? p.Dskip[d] : 0.0f;
    const float bias = p.bias ? p.bias[d] : 0.0f;

    for (int64_t tile = tile0; tile < tile1; ++tile) {
        const int64_t l0 = tile * TILE;
        const int64_t ll = l0 + lane * T;

        // ---- stage the Bm/Cm tile (all wavefronts): plain copy of complex words, layout [n][t/4][lane][t%4]
        __syncthreads();
        for (int r = threadIdx.x; r < TILE; r += W * 64) {
            const int64_t l = l0 + r;
            const int off = ((r % T) / 4) * QS + (r / T) * 4 + (r % 4);
            CW bw[N], cw[N];
            if (l < L) {
#pragma unroll
                for (int k = 0; k < N; ++k) { bw[k] = Bm[l * N + k]; cw[k] = Cm[l * N + k]; }
            } else {
#pragma unroll
                for (int k = 0; k < N; ++k) { bw[k] = CW{}; cw[k] = CW{}; }
            }
#pragma unroll
            for (int k = 0; k < N; ++k) { sB[k * PLANE + off] = bw[k]; sC[k * PLANE + off] = cw[k]; }
        }
        __syncthreads();
        if (!active) continue;

        // ---- this lane's T steps of u and Delta
        float uv[T], dl[T], yv[T];
        // (with T = 4 a lane's bfloat16 steps are less than a 16-byte chunk: one 8-byte access)
        auto load_steps = [&](const IO *r, float *out) {
            if constexpr (T % io_traits<IO>::EPC == 0) {
                load_seg<IO, T>(r, ll, L, vec, out);
            } else {
                RawFew<IO, T> raw;
                load_few_raw<IO, T>(r, ll, L, vec, raw);
                unpack_few<IO, T>(raw, out);
            }
        };
        load_steps(urow, uv);
        load_steps(drow, dl);
        float sum_dl = 0.0f;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            float s = dl[t] + bias, sp, sg;
            if (p.softplus) softplus_sigmoid<sizeof(IO) == 4>(s, sp, sg); else sp = s;
            dl[t] = (ll + t < L) ? sp : 0.0f;         // steps past the end are the identity map (a = 1, b = 0)
            uv[t] = (ll + t < L) ? uv[t] : 0.0f;
            sum_dl += dl[t];
            yv[t] = Dsk * uv[t];
        }

#pragma unroll 1
        for (int n = 0; n < N; ++n) {
            const CCoef cc = make_ccoef(readlane(Arv, n), readlane(Aiv, n));
            const float2 xc = make_float2(readlane(xrv, n), readlane(xiv, n));
            float2 a[T], bb[T];
            float2 P = make_float2(1.0f, 0.0f), S = make_float2(0.0f, 0.0f);
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const float2 Bv = cword<IO>::unpack(sB[n * PLANE + (t / 4) * QS + lane * 4 + (t % 4)]);
                float2 g;
                cdisc_ag<DISC>(dl[t], cc, a[t], g);
                if constexpr (DISC == DISC_ZOH_S6 || DISC == DISC_DIRAC) {
                    const float gu = g.x * uv[t];                         // the gain is real
                    bb[t] = make_float2(gu * Bv.x, gu * Bv.y);
                } else {
                    const float gu_r = g.x * uv[t], gu_i = g.y * uv[t];
                    bb[t] = make_float2(gu_r * Bv.x - gu_i * Bv.y, gu_r * Bv.y + gu_i * Bv.x);
                }
                S = make_float2(__builtin_fmaf(a[t].x, S.x, __builtin_fmaf(-a[t].y, S.y, bb[t].x)),
                                __builtin_fmaf(a[t].x, S.y, __builtin_fmaf(a[t].y, S.x, bb[t].y)));
                if constexpr (DISC == DISC_BILINEAR) P = make_float2(P.x * a[t].x - P.y * a[t].y, P.x * a[t].y + P.y * a[t].x);
            }
            if constexpr (DISC != DISC_BILINEAR) P = cexp_dt(sum_dl, cc.A2r, cc.Arev);   // product of the T multipliers
            if (lane == 0) {                                          // the carried state enters through lane 0
                S = make_float2(__builtin_fmaf(P.x, xc.x, __builtin_fmaf(-P.y, xc.y, S.x)),
                                __builtin_fmaf(P.x, xc.y, __builtin_fmaf(P.y, xc.x, S.y)));
            }
            cwave_scan_fwd(P, S);
            float2 x = make_float2(dpp<DPP_WAVE_SHR1>(xc.x, S.x), dpp<DPP_WAVE_SHR1>(xc.y, S.y));
            if constexpr (AGG) {                                      // lane 63: product of the tile's multipliers
                const float tr = readlane(P.x, 63), ti = readlane(P.y, 63), cr = readlane(prv, n), ci = readlane(piv, n);
                prv = writelane(prv, tr * cr - ti * ci, n);
                piv = writelane(piv, tr * ci + ti * cr, n);
            }
            // the state entering every kCkptInterval-th step is what the backward pass restarts from
            if (!AGG && p.ckpt && (lane * T) % (int)kCkptInterval == 0 && ll < L)
                p.ckpt[(ck0 + ll / kCkptInterval) * N + n] = x;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const float2 Cv = cword<IO>::unpack(sC[n * PLANE + (t / 4) * QS + lane * 4 + (t % 4)]);
                x = make_float2(__builtin_fmaf(a[t].x, x.x, __builtin_fmaf(-a[t].y, x.y, bb[t].x)),
                                __builtin_fmaf(a[t].x, x.y, __builtin_fmaf(a[t].y, x.x, bb[t].y)));
                yv[t] = __builtin_fmaf(Cv.x, x.x, __builtin_fmaf(-Cv.y, x.y, yv[t]));   // Re(C x)
            }
            xrv = writelane(xrv, readlane(x.x, 63), n);               // lane 63 ends on the tile's last step
            xiv = writelane(xiv, readlane(x.y, 63), n);
        }

        if (!want_y) continue;
        if (zrow) {
            float zv[T];
            load_steps(zrow, zv);
#pragma unroll
            for (int t = 0; t < T; ++t) yv[t] *= zv[t] * sigmoid_fast(zv[t]);
        }
        if constexpr (T % io_traits<IO>::EPC == 0) store_seg<IO, T>(yrow, ll, L, vec, yv);
        else store_few<IO, T>(yrow, ll, L, vec, yv);
    }

    if constexpr (AGG) {
        if (active && lane < N) {
            const int64_t j = (row * p.nchunks + chunk) * N + lane;
            p.ws_P[j] = make_float2(prv, piv);
            p.ws_S[j] = make_float2(xrv, xiv);
        }
        return;
    }
    if (active && lane < N && p.x_last && chunk == p.nchunks - 1) p.x_last[row * N + lane] = make_float2(xrv, xiv);
}

// Chains the chunk aggregates of one (b,d,n): carry-in of chunk c+1 = P_c * carry-in of chunk c + S_c.
// ws_S[c] is replaced by the carry-in of chunk c.
__global__ void k_ss_ccarry(const CFwdParams p) {
    const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)p.B * p.D * p.N;
    if (i >= total) return;
    const int64_t row = i / p.N;
    const int n = (int)(i % p.N);
    float2 x = p.x0 ? p.x0[i] : make_float2(0.0f, 0.0f);
    for (int c = 0; c < p.nchunks; ++c) {
        const int64_t j = (row * p.nchunks + c) * p.N + n;
        if (c + 1 == p.nchunks) { p.ws_S[j] = x; break; }     // nothing follows the last chunk: its pair was not computed
        const float2 P = p.ws_P[j], S = p.ws_S[j];
        p.ws_S[j] = x;
        x = cxfma(P, x, S);
    }
}

// ---------------------------------------------------------------- launchers
// Short tiles (4 steps per lane, 4 channels per workgroup: tiles of 256 steps) for the single pass over short rows,
// by the rule of the real forward pass (selective_fwd.hip): a tile is walked whole, so the smaller one pays when it
// wastes enough fewer steps to make up for its higher cost per step.
static bool cfwd_short_tiles(const CFwdParams &p) {
    if (p.nchunks != 1 || p.mode != MODE_FULL) return false;
    if (p.cu) return p.L < (int64_t)360 * p.B;
    const int64_t walked8 = (p.L + 511) / 512 * 512, walked4 = (p.L + 255) / 256 * 256;
    return walked4 * 125 < walked8 * 100;
}

template <typename IO, int N, int DISC>
static hipError_t launch_cfwd_n(const CFwdParams &p, hipStream_t s) {
    if (cfwd_short_tiles(p)) {
        constexpr int W = 4, T = 4;
        dim3 grid(p.bcg * ((p.dpg + W - 1) / W), p.B, 1);
        hipLaunchKernelGGL((k_ss_cfwd<IO, N, T, W, DISC, false>), grid, dim3(W * 64), 0, s, p);
        return hipGetLastError();
    }
    constexpr int W = 8, T = 8;
    // the aggregate launch skips the last chunk: nobody needs its pair
    dim3 grid(p.bcg * ((p.dpg + W - 1) / W), p.B, p.nchunks > 1 ? (p.mode == MODE_AGG ? p.nchunks - 1 : p.nchunks) : 1);
    if (p.mode == MODE_AGG) hipLaunchKernelGGL((k_ss_cfwd<IO, N, T, W, DISC, true>), grid, dim3(W * 64), 0, s, p);
    else hipLaunchKernelGGL((k_ss_cfwd<IO, N, T, W, DISC, false>), grid, dim3(W * 64), 0, s, p);
    return hipGetLastError();
}
template <typename IO, int DISC>
static hipError_t launch_cfwd_disc(const CFwdParams &p, hipStream_t s) {
    switch (p.N) {
        case 1: return launch_cfwd_n<IO, 1, DISC>(p, s);
        case 2: return launch_cfwd_n<IO, 2, DISC>(p, s);
        case 4: return launch_cfwd_n<IO, 4, DISC>(p, s);
        case 8: return launch_cfwd_n<IO, 8, DISC>(p, s);
        case 16: return launch_cfwd_n<IO, 16, DISC>(p, s);
    }
    return hipErrorInvalidValue;
}
template <typename IO>
static hipError_t launch_cfwd_io(const CFwdParams &p, int disc, hipStream_t s) {
    switch (disc) {
        case DISC_ZOH_S6: return launch_cfwd_disc<IO, DISC_ZOH_S6>(p, s);
        case DISC_ZOH: return launch_cfwd_disc<IO, DISC_ZOH>(p, s);
        case DISC_BILINEAR: return launch_cfwd_disc<IO, DISC_BILINEAR>(p, s);
        case DISC_DIRAC: return launch_cfwd_disc<IO, DISC_DIRAC>(p, s);
    }
    return hipErrorInvalidValue;
}
hipError_t launch_ss_ccarry(const CFwdParams &p, hipStream_t s) {
    const int64_t total = (int64_t)p.B * p.D * p.N;
    hipLaunchKernelGGL(k_ss_ccarry, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p);
    return hipGetLastError();
}
hipError_t launch_ss_cfwd(const CFwdParams &p, int io_dtype, int disc, hipStream_t s) {
    return io_dtype == 1 ? launch_cfwd_io<bf16_t>(p, disc, s) : launch_cfwd_io<float>(p, disc, s);
}

}  // namespace lrnnx
