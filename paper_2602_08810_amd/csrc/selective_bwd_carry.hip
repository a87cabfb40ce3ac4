// Chunked backward selective scan for gfx950, first two launches: the adjoint aggregate of every chunk of the time
// axis and the chain over them.  The backward pass of Eq. 2 of the paper runs the adjoint recurrence
//     H_l = Cm_{l,n} dypre_l + a_{l+1} H_{l+1}
// from the last step to the first; one workgroup per row group walks the whole sequence.  With few rows and a long
// sequence that leaves most of the chip idle, so the time axis is cut into chunks that run side by side (the same
// idea as the forward pass's separate chunk-carry launch for very long L).  A chunk [l0, l1] needs the adjoint
// entering it from the later side, h_in = a_{l1+1} H_{l1+1}; what it hands to the earlier side is affine in it:
//     h_out = a_{l0} H_{l0} = Q + P h_in,   P = prod_{l0 <= j <= l1} a_j,   Q = sum_{l0 <= l <= l1} (prod_{l0 <= j <= l} a_j) Cm_l dypre_l.
// k_ss_bwd_agg computes (P, Q) per (row, chunk, state); k_ss_bwd_carry chains them from the last chunk (h_in = 0) to
// the first and leaves every chunk's h_in; the backward kernel proper then starts each chunk from it.  The forward
// state needs no such chain: every tile restarts from the forward pass's checkpoint.
//
// Mapping of k_ss_bwd_agg: that of the forward kernel.  Time on lanes (a lane owns T = 8 consecutive steps), one
// wavefront per channel, the 8 wavefronts of a workgroup share the Cm tile staged in LDS as fp32.  Only the tile's
// total pair is needed, so the lanes take the tile's time slots in reverse order (lane 63 the earliest): the
// composition "earlier o later" then runs towards higher lanes and is the forward scan, all DPP steps; lane 63 ends up
// with the tile's pair, and the chunk's pair is carried from tile to tile in lane n of two registers.
#include "kernels.hpp"
#include "scan_common.hpp"
#include "cplx_common.hpp"

namespace lrnnx {

// Steps of chunk `chunk` of batch entry b: Lc steps from step s0 of the time axis on, in row bs of the [B,D,L] tensors.
// Chunks are counted from the start of the sequence, `span` steps each; the last one takes whatever is left, so a
// chunk count planned for a shorter longest sequence than the batch really has (packed mode: the lengths are on the
// device) still covers every step.  Packed mode (cu != nullptr): sequence b lies at cu[b] .. cu[b+1]-1 of ONE time
// axis of L steps (bounds clamped to it), the rows have no batch stride (bs = 0), and a sequence that ends before
// the chunk starts has Lc = 0.
__device__ __forceinline__ void chunk_span(const int64_t *cu, int b, int64_t L, int chunk, int nchunks, int64_t span,
                                           int64_t &s0, int64_t &Lc, int64_t &bs) {
    int64_t o = 0, e = L;
    bs = b;
    if (cu) {
        o = cu[b]; e = cu[b + 1];
        o = o < 0 ? 0 : (o > L ? L : o);
        e = e < o ? o : (e > L ? L : e);
        bs = 0;
    }
    const int64_t c0 = (int64_t)chunk * span;
    const int64_t left = e - o - c0;
    s0 = o + (left > 0 ? c0 : 0);
    Lc = left <= 0 ? 0 : ((chunk == nchunks - 1 || left < span) ? left : span);
}

template <typename IO, int N, int DISC>
__global__ __launch_bounds__(512, 2) void k_ss_bwd_agg(const BwdParams p) {
    constexpr int T = 8, W = 8;
    constexpr int TQ = T / 4;
    constexpr int QS = 256 + 32 / TQ;                  // floats per quarter-plane, padded against bank conflicts on staging
    constexpr int PLANE = TQ * QS;
    constexpr int TILE = 64 * T;
    __shared__ __attribute__((aligned(16))) float sC[N * PLANE];

    const int lane = threadIdx.x & 63;
    const int slot = 63 - lane;                        // this lane's time slot within a tile
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b = blockIdx.y;
    const int chunk = blockIdx.z + 1;                  // chunk 0 hands its adjoint to nobody: its pair is not needed
    // a workgroup takes W consecutive channels of ONE Bm/Cm group (it stages that group's Cm in LDS)
    const int blk_per_grp = (p.dpg + W - 1) / W;
    const int grp = blockIdx.x / blk_per_grp;
    const int d_in = (blockIdx.x % blk_per_grp) * W + w;
    const bool active = d_in < p.dpg;
    const int d = grp * p.dpg + (active ? d_in : p.dpg - 1);
    // the chunk's Lc steps of the sequence, from step s0 of the time axis on; the chunk starts a multiple of the
    // backward tile (256 steps) after the start of its sequence
    int64_t s0, Lc, bs;
    chunk_span(p.cu, b, p.L, chunk, p.nchunks, p.tiles_per_chunk * kBwdTileSteps, s0, Lc, bs);
    const int64_t ntiles = (Lc + TILE - 1) / TILE;     // none for a packed sequence that ends before this chunk: the pair stays (1, 0)
    const bool vec = p.vec != 0;
    const bool has_z = p.z != nullptr;

    const IO *drow = reinterpret_cast<const IO *>(p.delta) + bs * p.dl_sb + d * p.dl_sd + s0;
    const IO *gyrow = reinterpret_cast<const IO *>(p.dy) + bs * p.dy_sb + d * p.dy_sd + s0;
    const IO *zrow = has_z ? reinterpret_cast<const IO *>(p.z) + bs * p.z_sb + d * p.z_sd + s0 : nullptr;
    const IO *Cm = reinterpret_cast<const IO *>(p.Cm) + ((bs * p.bcg + grp) * p.L + s0) * N;

    // lane n holds A[d,n] and the chunk's pair of state n
    const float Av = (lane < N) ? p.A[d * N + lane] : 0.0f;
    const float bias = p.bias ? p.bias[d] : 0.0f;
    float pcv = 1.0f, qcv = 0.0f;

    for (int64_t tile = ntiles - 1; tile >= 0; --tile) {
        const int64_t l0 = tile * TILE;
        const int64_t ll = l0 + slot * T;

        // ---- stage the Cm tile (all wavefronts), fp32, layout [n][t/4][slot][t%4]; rows past the chunk read as zero
        __syncthreads();
        for (int r = threadIdx.x; r < TILE; r += W * 64) {
            float cv[N];
            const int64_t l = l0 + r;
            if (l < Lc) {
                load_row<IO, N>(Cm + l * N, cv);
            } else {
#pragma unroll
                for (int k = 0; k < N; ++k) cv[k] = 0.0f;
            }
            const int off = ((r % T) / 4) * QS + (r / T) * 4 + (r % 4);
#pragma unroll
            for (int k = 0; k < N; ++k) sC[k * PLANE + off] = cv[k];
        }
        __syncthreads();
        if (!active) continue;

        // ---- this lane's T steps of Delta and of the gradient reaching ypre
        float dl[T], dyp[T], zv[T];
        load_seg<IO, T>(drow, ll, Lc, vec, dl);
        load_seg<IO, T>(gyrow, ll, Lc, vec, dyp);
        if (has_z) load_seg<IO, T>(zrow, ll, Lc, vec, zv);
        float sum_dl = 0.0f;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            float sp, sg, gp, zf;
            bwd_step_inputs<sizeof(IO) == 4>(dl[t] + bias, dyp[t], has_z ? zv[t] : 0.0f, p.softplus != 0, has_z, sp, sg, gp, zf);
            dl[t] = (ll + t < Lc) ? sp : 0.0f;        // steps past the end are the identity (a = 1, no source term)
            dyp[t] = (ll + t < Lc) ? gp : 0.0f;
            sum_dl += dl[t];
        }

#pragma unroll 1
        for (int n = 0; n < N; ++n) {
            const ACoef ac = make_acoef<DISC>(readlane(Av, n));
            float4 Cc[TQ];
#pragma unroll
            for (int q = 0; q < TQ; ++q) Cc[q] = *reinterpret_cast<const float4 *>(&sC[n * PLANE + q * QS + slot * 4]);
            // the lane's pair: Q = a_0 (c_0 + a_1 (c_1 + ...)), P = a_0 a_1 ... a_{T-1}
            float P = 1.0f, Q = 0.0f;
#pragma unroll
            for (int t = T - 1; t >= 0; --t) {
                float a, g;
                disc_ag<DISC>(dl[t], ac, a, g);
                const float Ct = reinterpret_cast<const float *>(&Cc[t / 4])[t % 4];
                Q = a * __builtin_fmaf(Ct, dyp[t], Q);
                if constexpr (DISC == DISC_BILINEAR) P *= a;
            }
            if constexpr (DISC != DISC_BILINEAR) P = exp2_fast(sum_dl * ac.A2);
            wave_scan_fwd(P, Q);                                      // lane 63 (the earliest slot): the tile's pair
            const float Pt = readlane(P, 63), Qt = readlane(Q, 63);
            // this tile lies before what has been accumulated so far: (Pt, Qt) o (Pc, Qc)
            qcv = writelane(qcv, __builtin_fmaf(Pt, readlane(qcv, n), Qt), n);
            pcv = writelane(pcv, Pt * readlane(pcv, n), n);
        }
    }

    if (active && lane < N) {
        const int64_t j = (((int64_t)b * p.D + d) * p.nchunks + chunk) * N + lane;
        p.ws_P[j] = pcv;
        p.ws_Q[j] = qcv;
    }
}

// Chains the chunk aggregates of one (b,d,n) from the last chunk to the first: the adjoint entering chunk c from
// the later side is Q_{c+1} + P_{c+1} (that entering chunk c+1), zero for the last chunk.  ws_Q[c] is replaced by it.
__global__ void k_ss_bwd_carry(const BwdParams p) {
    const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)p.B * p.D * p.N;
    if (i >= total) return;
    const int64_t row = i / p.N;
    const int n = (int)(i % p.N);
    float h = 0.0f;
    for (int c = p.nchunks - 1; c >= 0; --c) {
        const int64_t j = (row * p.nchunks + c) * p.N + n;
        if (c == 0) { p.ws_Q[j] = h; break; }                // the pair of chunk 0 was not computed
        const float P = p.ws_P[j], Q = p.ws_Q[j];
        p.ws_Q[j] = h;
        h = __builtin_fmaf(P, h, Q);
    }
}

// ---------------------------------------------------------------- the same for the complex-A scan
// H_l = dypre_l conj(Cm_l) + conj(a_{l+1}) H_{l+1}: the pair of a chunk is P = prod conj(a_j),
// Q = sum_l (prod_{l0 <= j <= l} conj(a_j)) dypre_l conj(Cm_l).  Only the tile's total is needed, so the lanes take the
// tile's time slots in reverse order (lane 63 the earliest): the composition "earlier o later" then runs towards
// higher lanes and is the forward scan, all DPP steps; lane 63 ends up with the tile's pair.
template <typename IO, int N, int DISC>
__global__ __launch_bounds__(512, 2) void k_ss_cbwd_agg(const CBwdParams p) {
    using CW = typename cword<IO>::type;
    constexpr int T = 8, W = 8;
    constexpr int TQ = T / 4;
    constexpr int QS = 256 + 32 / TQ;
    constexpr int PLANE = TQ * QS;
    constexpr int TILE = 64 * T;
    __shared__ __attribute__((aligned(16))) CW sC[N * PLANE];

    const int lane = threadIdx.x & 63;
    const int slot = 63 - lane;                        // this lane's time slot within a tile
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b = blockIdx.y;
    const int chunk = blockIdx.z + 1;                  // chunk 0 hands its adjoint to nobody: its pair is not needed
    const int blk_per_grp = (p.dpg + W - 1) / W;
    const int grp = blockIdx.x / blk_per_grp;
    const int d_in = (blockIdx.x % blk_per_grp) * W + w;
    const bool active = d_in < p.dpg;
    const int d = grp * p.dpg + (active ? d_in : p.dpg - 1);
    int64_t s0, Lc, bs;                                // as in k_ss_bwd_agg
    chunk_span(p.cu, b, p.L, chunk, p.nchunks, p.tiles_per_chunk * kBwdTileSteps, s0, Lc, bs);
    const int64_t ntiles = (Lc + TILE - 1) / TILE;
    const bool vec = p.vec != 0;
    const bool has_z = p.z != nullptr;

    const IO *drow = reinterpret_cast<const IO *>(p.delta) + bs * p.dl_sb + d * p.dl_sd + s0;
    const IO *gyrow = reinterpret_cast<const IO *>(p.dy) + bs * p.dy_sb + d * p.dy_sd + s0;
    const IO *zrow = has_z ? reinterpret_cast<const IO *>(p.z) + bs * p.z_sb + d * p.z_sd + s0 : nullptr;
    const CW *Cm = reinterpret_cast<const CW *>(p.Cm) + ((bs * p.bcg + grp) * p.L + s0) * N;

    // lane n holds A[d,n] and the chunk's pair of state n
    float Arv = 0.0f, Aiv = 0.0f;
    if (lane < N) { const float2 Av = p.A[d * N + lane]; Arv = Av.x; Aiv = Av.y; }
    const float bias = p.bias ? p.bias[d] : 0.0f;
    float pr = 1.0f, pi = 0.0f, qr = 0.0f, qi = 0.0f;

    for (int64_t tile = ntiles - 1; tile >= 0; --tile) {
        const int64_t l0 = tile * TILE;
        const int64_t ll = l0 + slot * T;

        // ---- stage the Cm tile (all wavefronts): plain copy of complex words, layout [n][t/4][slot][t%4]
        __syncthreads();
        for (int r = threadIdx.x; r < TILE; r += W * 64) {
            const int64_t l = l0 + r;
            const int off = ((r % T) / 4) * QS + (r / T) * 4 + (r % 4);
            CW cw[N];
            if (l < Lc) {
#pragma unroll
                for (int k = 0; k < N; ++k) cw[k] = Cm[l * N + k];
            } else {
#pragma unroll
                for (int k = 0; k < N; ++k) cw[k] = CW{};
            }
#pragma unroll
            for (int k = 0; k < N; ++k) sC[k * PLANE + off] = cw[k];
        }
        __syncthreads();
        if (!active) continue;

        float dl[T], dyp[T], zv[T];
        load_seg<IO, T>(drow, ll, Lc, vec, dl);
        load_seg<IO, T>(gyrow, ll, Lc, vec, dyp);
        if (has_z) load_seg<IO, T>(zrow, ll, Lc, vec, zv);
        float sum_dl = 0.0f;
#pragma unroll
        for (int t = 0; t < T; ++t) {
            float sp, sg, gp, zf;
            bwd_step_inputs<sizeof(IO) == 4>(dl[t] + bias, dyp[t], has_z ? zv[t] : 0.0f, p.softplus != 0, has_z, sp, sg, gp, zf);
            dl[t] = (ll + t < Lc) ? sp : 0.0f;        // steps past the end are the identity (a = 1, no source term)
            dyp[t] = (ll + t < Lc) ? gp : 0.0f;
            sum_dl += dl[t];
        }

#pragma unroll 1
        for (int n = 0; n < N; ++n) {
            const CCoef cc = make_ccoef(readlane(Arv, n), readlane(Aiv, n));
            // the lane's pair: Q = conj(a_0) (c_0 + conj(a_1) (c_1 + ...)), P = conj(a_0 a_1 ... a_{T-1})
            float2 P = make_float2(1.0f, 0.0f), Q = make_float2(0.0f, 0.0f);
#pragma unroll
            for (int t = T - 1; t >= 0; --t) {
                float2 a, g;
                cdisc_ag<DISC>(dl[t], cc, a, g);
                const float2 Cv = cword<IO>::unpack(sC[n * PLANE + (t / 4) * QS + slot * 4 + (t % 4)]);
                const float2 tmp = make_float2(__builtin_fmaf(Cv.x, dyp[t], Q.x), __builtin_fmaf(-Cv.y, dyp[t], Q.y));
                Q = cxmulc(tmp, a);
                if constexpr (DISC == DISC_BILINEAR) P = cxmulc(P, a);
            }
            if constexpr (DISC != DISC_BILINEAR) {
                const float2 e = cexp_dt(sum_dl, cc.A2r, cc.Arev);
                P = make_float2(e.x, -e.y);
            }
            cwave_scan_fwd(P, Q);                                      // lane 63 (the earliest slot): the tile's pair
            const float Ptr = readlane(P.x, 63), Pti = readlane(P.y, 63), Qtr = readlane(Q.x, 63), Qti = readlane(Q.y, 63);
            // this tile lies before what has been accumulated so far: (Pt, Qt) o (Pc, Qc)
            const float cqr = readlane(qr, n), cqi = readlane(qi, n), cpr = readlane(pr, n), cpi = readlane(pi, n);
            qr = writelane(qr, __builtin_fmaf(Ptr, cqr, __builtin_fmaf(-Pti, cqi, Qtr)), n);
            qi = writelane(qi, __builtin_fmaf(Ptr, cqi, __builtin_fmaf(Pti, cqr, Qti)), n);
            pr = writelane(pr, Ptr * cpr - Pti * cpi, n);
            pi = writelane(pi, Ptr * cpi + Pti * cpr, n);
        }
    }

    if (active && lane < N) {
        const int64_t j = (((int64_t)b * p.D + d) * p.nchunks + chunk) * N + lane;
        p.ws_P[j] = make_float2(pr, pi);
        p.ws_Q[j] = make_float2(qr, qi);
    }
}

__global__ void k_ss_cbwd_carry(const CBwdParams p) {
    const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)p.B * p.D * p.N;
    if (i >= total) return;
    const int64_t row = i / p.N;
    const int n = (int)(i % p.N);
    float2 h = make_float2(0.0f, 0.0f);
    for (int c = p.nchunks - 1; c >= 0; --c) {
        const int64_t j = (row * p.nchunks + c) * p.N + n;
        if (c == 0) { p.ws_Q[j] = h; break; }                // the pair of chunk 0 was not computed
        const float2 P = p.ws_P[j], Q = p.ws_Q[j];
        p.ws_Q[j] = h;
        h = cxfma(P, h, Q);
    }
}

// Packed variable-length batches: order[r] = index of the sequence with the r-th largest length (ties by index).
// One small block; B is at most kMaxOrdered, the lengths sit in LDS, so the quadratic ranking is a few microseconds.
__global__ void k_seq_order(const int64_t *cu, int B, int64_t L, int *order) {
    __shared__ int64_t slen[kMaxOrdered];
    for (int j = threadIdx.x; j < B; j += blockDim.x) {
        int64_t o = cu[j], e = cu[j + 1];
        o = o < 0 ? 0 : (o > L ? L : o);
        e = e < o ? o : (e > L ? L : e);
        slen[j] = e - o;
    }
    __syncthreads();
    for (int b = threadIdx.x; b < B; b += blockDim.x) {
        const int64_t lb = slen[b];
        int rank = 0;
        for (int j = 0; j < B; ++j) {
            const int64_t lj = slen[j];
            rank += (lj > lb || (lj == lb && j < b)) ? 1 : 0;
        }
        order[rank] = b;
    }
}
hipError_t launch_seq_order(const int64_t *cu, int B, int64_t L, int *order, hipStream_t s) {
    hipLaunchKernelGGL(k_seq_order, dim3(1), dim3(256), 0, s, cu, B, L, order);
    return hipGetLastError();
}

// ---------------------------------------------------------------- launchers
template <typename IO, int N, int DISC>
static hipError_t launch_agg_n(const BwdParams &p, hipStream_t s) {
    dim3 grid(p.bcg * ((p.dpg + 7) / 8), p.B, p.nchunks - 1);
    hipLaunchKernelGGL((k_ss_bwd_agg<IO, N, DISC>), grid, dim3(512), 0, s, p);
    return hipGetLastError();
}
template <typename IO, int DISC>
static hipError_t launch_agg_disc(const BwdParams &p, hipStream_t s) {
    switch (p.N) {
        case 1: return launch_agg_n<IO, 1, DISC>(p, s);
        case 2: return launch_agg_n<IO, 2, DISC>(p, s);
        case 4: return launch_agg_n<IO, 4, DISC>(p, s);
        case 8: return launch_agg_n<IO, 8, DISC>(p, s);
        case 16: return launch_agg_n<IO, 16, DISC>(p, s);
        case 32: return launch_agg_n<IO, 32, DISC>(p, s);
    }
    return hipErrorInvalidValue;
}
template <typename IO>
static hipError_t launch_agg_io(const BwdParams &p, int disc, hipStream_t s) {
    switch (disc) {
        case DISC_ZOH_S6: return launch_agg_disc<IO, DISC_ZOH_S6>(p, s);
        case DISC_ZOH: return launch_agg_disc<IO, DISC_ZOH>(p, s);
        case DISC_BILINEAR: return launch_agg_disc<IO, DISC_BILINEAR>(p, s);
        case DISC_DIRAC: return launch_agg_disc<IO, DISC_DIRAC>(p, s);
    }
    return hipErrorInvalidValue;
}
hipError_t launch_ss_bwd_agg(const BwdParams &p, int io_dtype, int disc, hipStream_t s) {
    return io_dtype == 1 ? launch_agg_io<bf16_t>(p, disc, s) : launch_agg_io<float>(p, disc, s);
}
template <typename IO, int DISC>
static hipError_t launch_cagg_disc(const CBwdParams &p, hipStream_t s) {
    dim3 grid(p.bcg * ((p.dpg + 7) / 8), p.B, p.nchunks - 1);
#define LRNNX_CAGG(NN) hipLaunchKernelGGL((k_ss_cbwd_agg<IO, NN, DISC>), grid, dim3(512), 0, s, p); return hipGetLastError()
    switch (p.N) {
        case 1: LRNNX_CAGG(1);
        case 2: LRNNX_CAGG(2);
        case 4: LRNNX_CAGG(4);
        case 8: LRNNX_CAGG(8);
        case 16: LRNNX_CAGG(16);
    }
#undef LRNNX_CAGG
    return hipErrorInvalidValue;
}
template <typename IO>
static hipError_t launch_cagg_io(const CBwdParams &p, int disc, hipStream_t s) {
    switch (disc) {
        case DISC_ZOH_S6: return launch_cagg_disc<IO, DISC_ZOH_S6>(p, s);
        case DISC_ZOH: return launch_cagg_disc<IO, DISC_ZOH>(p, s);
        case DISC_BILINEAR: return launch_cagg_disc<IO, DISC_BILINEAR>(p, s);
        case DISC_DIRAC: return launch_cagg_disc<IO, DISC_DIRAC>(p, s);
    }
    return hipErrorInvalidValue;
}
hipError_t launch_ss_cbwd_agg(const CBwdParams &p, int io_dtype, int disc, hipStream_t s) {
    return io_dtype == 1 ? launch_cagg_io<bf16_t>(p, disc, s) : launch_cagg_io<float>(p, disc, s);
}
hipError_t launch_ss_cbwd_carry(const CBwdParams &p, hipStream_t s) {
    const int64_t total = (int64_t)p.B * p.D * p.N;
    hipLaunchKernelGGL(k_ss_cbwd_carry, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p);
    return hipGetLastError();
}
hipError_t launch_ss_bwd_carry(const BwdParams &p, hipStream_t s) {
    const int64_t total = (int64_t)p.B * p.D * p.N;
    hipLaunchKernelGGL(k_ss_bwd_carry, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p);
    return hipGetLastError();
}

}  // namespace lrnnx
