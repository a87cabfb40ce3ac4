// Forward selective scan for gfx950 (Eq. 2 of the paper with diagonal, input-dependent
// A(k), B(k), C(k); S6 row of Table 1; discretisation fused in, Sec. 3).
//
// Mapping.  Time runs along the lanes: lane i of a wavefront owns T consecutive steps
// of one (b,d) row, so the [B,D,L] tensors are read and written with 16-byte accesses
// that are contiguous across the wavefront.  One wavefront = one channel; the W
// wavefronts of a workgroup are W channels of the same batch entry walking the same
// time tile (64*T steps), so the tile of Bm/Cm (shared by all channels) is staged once
// per workgroup into LDS as fp32, in an order that makes every later read a
// conflict-free ds_read_b128.  States never leave registers (Sec. 3: no hidden-state
// materialisation): for each n the lane folds its T steps into one affine pair, the
// wavefront takes an inclusive prefix over the 64 pairs with DPP moves, and the lane
// replays its steps from the carried-in state, accumulating y = sum_n C x on the fly.
// The state after the tile is lane 63's, broadcast through a scalar register to the
// next tile of the same row.
//
// The same kernel serves the three launches of the chunk-carry path for long L / few
// rows (blockIdx.z = chunk): MODE_AGG returns each chunk's affine aggregate,
// k_ss_carry chains them, MODE_APPLY reruns the chunk from its true carry-in.
#include "kernels.hpp"
#include "scan_common.hpp"

namespace lrnnx {

// Two workgroups share a compute unit only if a wavefront stays within 128 vector registers, and with short rows
// (many workgroups per CU, one after the other) the second one is worth 20-25 %: it covers the other's start-up
// and drain (measured with a variant that needed 146 registers).  The compiler is therefore held to 128 (the exact-ZOH
// variant otherwise takes 133).  With float32 I/O the rows of Bm/Cm fetched one tile ahead would alone cost 2 N
// registers, so that prefetch is for bfloat16 only (float32: 196 -> 171 us on the Mamba-block shape).  N = 32 fills
// the LDS of a CU with one workgroup's tile and is left alone.
template <typename IO, int N, int T, int W, int DISC, bool WANT_Y, bool CKPT>
__global__ __launch_bounds__(W * 64, (N <= 16) ? 4 : 2) void k_ss_fwd(const FwdParams p) {
    constexpr int TQ = T / 4;
    constexpr int QS = 256 + (TQ > 1 ? 32 / TQ : 0);   // floats per quarter-plane, padded against bank conflicts on staging
    constexpr int PLANE = TQ * QS;                     // floats per state index n
    constexpr int TILE = 64 * T;
    __shared__ __attribute__((aligned(16))) float sB[N * PLANE];
    __shared__ __attribute__((aligned(16))) float sC[N * PLANE];

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int b = blockIdx.y;
    // a workgroup takes W consecutive channels of ONE Bm/Cm group (it stages that group's maps in LDS)
    const int blk_per_grp = (p.dpg + W - 1) / W;
    const int grp = blockIdx.x / blk_per_grp;
    const int d_in = (blockIdx.x % blk_per_grp) * W + w;
    const bool active = d_in < p.dpg;
    const int d = grp * p.dpg + (active ? d_in : p.dpg - 1);
    const int chunk = blockIdx.z;
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
    const int64_t tile0 = (int64_t)chunk * p.tiles_per_chunk;
    const int64_t tile1 = (tile0 + p.tiles_per_chunk < ntiles) ? tile0 + p.tiles_per_chunk : ntiles;
    const int64_t row = (int64_t)b * p.D + d;
    const bool vec = p.vec != 0;
    const int mode = p.mode;

    const IO *urow = reinterpret_cast<const IO *>(p.u) + bs * p.u_sb + d * p.u_sd + toff;
    const IO *drow = reinterpret_cast<const IO *>(p.delta) + bs * p.dl_sb + d * p.dl_sd + toff;
    const IO *zrow = p.z ? reinterpret_cast<const IO *>(p.z) + bs * p.z_sb + d * p.z_sd + toff : nullptr;
    IO *yrow = p.y ? reinterpret_cast<IO *>(p.y) + bs * p.y_sb + d * p.y_sd + toff : nullptr;
    const int64_t bc0 = ((bs * p.bcg + grp) * p.L + toff) * N;       // first element of the maps of this sequence
    const IO *Bm = reinterpret_cast<const IO *>(p.Bm) + bc0;
    const IO *Cm = reinterpret_cast<const IO *>(p.Cm) + bc0;

    // Per-state uniform values live one per lane (lane n holds state n) and are read with
    // v_readlane, so the loop over n stays rolled and nothing is indexed dynamically.
    float xcv = 0.0f, pcv = 1.0f;
    if (lane < N) {
        if (mode == MODE_APPLY) xcv = p.ws_S[(row * p.nchunks + chunk) * N + lane];
        else if (mode != MODE_AGG && p.x0) xcv = p.x0[row * N + lane];
    }
    const float Av = (lane < N) ? p.A[d * N + lane] : 0.0f;
    const float Dsk = p.Dskip ? p.Dskip[d] : 0.0f;
    const float bias = p.bias ? p.bias[d] : 0.0f;
    // checkpoints of this row: [B,D,nck,N], or packed [D,nslots,N] with sequence b starting at slot toff/interval + b
    const int64_t ck0 = p.cu ? (int64_t)d * p.nslots + toff / kCkptInterval + b
                             : row * ((L + kCkptInterval - 1) / kCkptInterval);

    // this lane's T steps of u, Delta and z are fetched one tile ahead (raw, converted when their tile starts), so
    // that their latency hides behind the previous tile's state loop
    RawFew<IO, T> r_u, r_dl, r_z;
    auto fetch = [&](int64_t tile) {
        const int64_t lf = tile * TILE + lane * T;
        if (vec && (tile + 1) * TILE <= L) {
            // a tile wholly inside the sequence (wave-uniform): plain vector loads, nothing to check per element
            load_few_raw<IO, T>(urow + lf, 0, T, true, r_u);
            load_few_raw<IO, T>(drow + lf, 0, T, true, r_dl);
            if constexpr (WANT_Y) { if (zrow) load_few_raw<IO, T>(zrow + lf, 0, T, true, r_z); }
        } else {
            load_few_raw<IO, T>(urow, lf, L, vec, r_u);
            load_few_raw<IO, T>(drow, lf, L, vec, r_dl);
            if constexpr (WANT_Y) { if (zrow) load_few_raw<IO, T>(zrow, lf, L, vec, r_z); }
        }
    };
    if (active && tile0 < tile1) fetch(tile0);
    // likewise the row of Bm and Cm this thread stages (one step of the tile per thread when the tile has as many
    // steps as the workgroup has threads); rows past the sequence read as zero
    constexpr bool PREFETCH_MAPS = TILE == W * 64 && sizeof(IO) == 2;   // float32 rows would cost 2 N registers
    RawFew<IO, PREFETCH_MAPS ? N : 1> r_B, r_C;
    auto fetch_maps = [&](int64_t tile) {
        const int64_t l = tile * TILE + threadIdx.x;
        if constexpr (PREFETCH_MAPS) {
            load_few_raw<IO, N>(Bm + l * N, (int64_t)0, l < L ? (int64_t)N : (int64_t)0, true, r_B);
            load_few_raw<IO, N>(Cm + l * N, (int64_t)0, l < L ? (int64_t)N : (int64_t)0, true, r_C);
        }
    };
    if constexpr (PREFETCH_MAPS) { if (tile0 < tile1) fetch_maps(tile0); }

    for (int64_t tile = tile0; tile < tile1; ++tile) {
        const int64_t l0 = tile * TILE;
        const int64_t ll = l0 + lane * T;
        static_assert(TILE % kCkptInterval == 0 && kCkptInterval % T == 0, "checkpoints fall on lane boundaries");
        const bool ck_lane = (lane % ((int)kCkptInterval / T)) == 0;     // ll is a multiple of the checkpoint interval

        // ---- stage the Bm/Cm tile (all wavefronts), fp32, layout [n][t/4][lane][t%4]; the rows were fetched (raw) one
        // tile ahead
        __syncthreads();
        if constexpr (PREFETCH_MAPS) {
            const int r = threadIdx.x;
            float bv[N], cv[N];
            unpack_few<IO, PREFETCH_MAPS ? N : 1>(r_B, bv);
            unpack_few<IO, PREFETCH_MAPS ? N : 1>(r_C, cv);
            const int off = ((r % T) / 4) * QS + (r / T) * 4 + (r % 4);
#pragma unroll
            for (int k = 0; k < N; ++k) { sB[k * PLANE + off] = bv[k]; sC[k * PLANE + off] = cv[k]; }
            if (tile + 1 < tile1) fetch_maps(tile + 1);
        } else {
            for (int r = threadIdx.x; r < TILE; r += W * 64) {
                float bv[N], cv[N];
                const int64_t l = l0 + r;
                if (l < L) {
                    load_row<IO, N>(Bm + l * N, bv);
                    load_row<IO, N>(Cm + l * N, cv);
                } else {
#pragma unroll
                    for (int k = 0; k < N; ++k) { bv[k] = 0.0f; cv[k] = 0.0f; }
                }
                const int off = ((r % T) / 4) * QS + (r / T) * 4 + (r % 4);
#pragma unroll
                for (int k = 0; k < N; ++k) { sB[k * PLANE + off] = bv[k]; sC[k * PLANE + off] = cv[k]; }
            }
        }
        __syncthreads();
        if (!active) continue;

        // ---- this lane's T steps of u and Delta
        float uv[T], dl[T], du[T], yv[T];
        unpack_few<IO, T>(r_u, uv);
        unpack_few<IO, T>(r_dl, dl);
        const RawFew<IO, T> c_z = r_z;                // this tile's gate values, needed after the state loop
        if (tile + 1 < tile1) fetch(tile + 1);
        float sum_dl = 0.0f;
        const int rem = (L - l0 < TILE) ? (int)(L - l0) : TILE;   // valid steps of this tile (wave-uniform)
#pragma unroll
        for (int t = 0; t < T; ++t) {
            float s = dl[t] + bias, sp, sg;
            if (p.softplus) softplus_sigmoid<sizeof(IO) == 4>(s, sp, sg); else sp = s;
            dl[t] = sp;
        }
        if (rem < TILE) {                             // steps past the end are the identity map (a = 1, b = 0)
#pragma unroll
            for (int t = 0; t < T; ++t) dl[t] = (lane * T + t < rem) ? dl[t] : 0.0f;
        }
#pragma unroll
        for (int t = 0; t < T; ++t) {
            sum_dl += dl[t];
            du[t] = dl[t] * uv[t];
            yv[t] = Dsk * uv[t];
        }

        // One state: fold the lane's T steps, wavefront prefix, replay.  Bc holds this state's Bm for the lane; Bn
        // receives the next state's while this one computes (ping-pong, no copies).  Cm is only needed by the
        // replay, so it is read from LDS after the fold and its latency hides behind the prefix.
        auto one_state = [&](int n, const float4 (&Bc)[TQ], float4 (&Bn)[TQ]) {
            if (n + 1 < N) {
#pragma unroll
                for (int q = 0; q < TQ; ++q)
                    Bn[q] = *reinterpret_cast<const float4 *>(&sB[(n + 1) * PLANE + q * QS + lane * 4]);
            }
            float Bv[T], a[T], bb[T];
#pragma unroll
            for (int q = 0; q < TQ; ++q) {
                Bv[4 * q] = Bc[q].x; Bv[4 * q + 1] = Bc[q].y; Bv[4 * q + 2] = Bc[q].z; Bv[4 * q + 3] = Bc[q].w;
            }
            const ACoef ac = make_acoef<DISC>(readlane(Av, n));
            const float xc = readlane(xcv, n);
            float P = 1.0f, S = 0.0f;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                float g;
                disc_ag<DISC>(dl[t], ac, a[t], g);
                if constexpr (DISC == DISC_ZOH_S6) bb[t] = du[t] * Bv[t];
                else if constexpr (DISC == DISC_DIRAC) bb[t] = uv[t] * Bv[t];
                else bb[t] = g * uv[t] * Bv[t];
                S = (t == 0) ? bb[0] : __builtin_fmaf(a[t], S, bb[t]);   // the fold starts from zero
                if constexpr (DISC == DISC_BILINEAR) P *= a[t];
            }
            float4 Cc[TQ];
            if constexpr (WANT_Y) {
#pragma unroll
                for (int q = 0; q < TQ; ++q)
                    Cc[q] = *reinterpret_cast<const float4 *>(&sC[n * PLANE + q * QS + lane * 4]);
            }
            if constexpr (DISC != DISC_BILINEAR) P = exp2_fast(sum_dl * ac.A2);   // product of the T multipliers
            if (lane == 0) S = __builtin_fmaf(P, xc, S);             // the carried state enters through lane 0
            wave_scan_fwd(P, S);
            float x = dpp<DPP_WAVE_SHR1>(xc, S);                     // state entering this lane's first step
            if constexpr (CKPT) {
                if (ck_lane && ll < L) p.ckpt[(ck0 + ll / kCkptInterval) * N + n] = x;
            }
            if constexpr (!WANT_Y) {
                xcv = writelane(xcv, readlane(S, 63), n);            // inclusive prefix at lane 63 = state after the tile
                pcv = writelane(pcv, readlane(pcv, n) * readlane(P, 63), n);
            } else {
                float Cv[T];
#pragma unroll
                for (int q = 0; q < TQ; ++q) {
                    Cv[4 * q] = Cc[q].x; Cv[4 * q + 1] = Cc[q].y; Cv[4 * q + 2] = Cc[q].z; Cv[4 * q + 3] = Cc[q].w;
                }
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    x = __builtin_fmaf(a[t], x, bb[t]);
                    yv[t] = __builtin_fmaf(Cv[t], x, yv[t]);
                }
                xcv = writelane(xcv, readlane(x, 63), n);            // lane 63 ends on the tile's last step
            }
        };
        // Two states at a time (every supported N > 1 is even): their folds and replays are independent chains and
        // their prefix scans are interleaved step by step, which fills the issue gaps a single dependent chain leaves.
        auto two_states = [&](int n) {
            float4 B0[TQ], B1[TQ];
#pragma unroll
            for (int q = 0; q < TQ; ++q) {
                B0[q] = *reinterpret_cast<const float4 *>(&sB[n * PLANE + q * QS + lane * 4]);
                B1[q] = *reinterpret_cast<const float4 *>(&sB[(n + 1) * PLANE + q * QS + lane * 4]);
            }
            const ACoef ac0 = make_acoef<DISC>(readlane(Av, n)), ac1 = make_acoef<DISC>(readlane(Av, n + 1));
            const float xc0 = readlane(xcv, n), xc1 = readlane(xcv, n + 1);
            float a0[T], b0[T], a1[T], b1[T];
            float P0 = 1.0f, S0 = 0.0f, P1 = 1.0f, S1 = 0.0f;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const float Bt0 = reinterpret_cast<const float *>(&B0[t / 4])[t % 4];
                const float Bt1 = reinterpret_cast<const float *>(&B1[t / 4])[t % 4];
                float g0, g1;
                disc_ag<DISC>(dl[t], ac0, a0[t], g0);
                disc_ag<DISC>(dl[t], ac1, a1[t], g1);
                if constexpr (DISC == DISC_ZOH_S6) { b0[t] = du[t] * Bt0; b1[t] = du[t] * Bt1; }
                else if constexpr (DISC == DISC_DIRAC) { b0[t] = uv[t] * Bt0; b1[t] = uv[t] * Bt1; }
                else { b0[t] = g0 * uv[t] * Bt0; b1[t] = g1 * uv[t] * Bt1; }
                S0 = (t == 0) ? b0[0] : __builtin_fmaf(a0[t], S0, b0[t]);   // the folds start from zero
                S1 = (t == 0) ? b1[0] : __builtin_fmaf(a1[t], S1, b1[t]);
                if constexpr (DISC == DISC_BILINEAR) { P0 *= a0[t]; P1 *= a1[t]; }
            }
            float4 C0[TQ], C1[TQ];
            if constexpr (WANT_Y) {
#pragma unroll
                for (int q = 0; q < TQ; ++q) {
                    C0[q] = *reinterpret_cast<const float4 *>(&sC[n * PLANE + q * QS + lane * 4]);
                    C1[q] = *reinterpret_cast<const float4 *>(&sC[(n + 1) * PLANE + q * QS + lane * 4]);
                }
            }
            if constexpr (DISC != DISC_BILINEAR) {                   // product of the T multipliers
                P0 = exp2_fast(sum_dl * ac0.A2);
                P1 = exp2_fast(sum_dl * ac1.A2);
            }
            if (lane == 0) {                                         // the carried states enter through lane 0
                S0 = __builtin_fmaf(P0, xc0, S0);
                S1 = __builtin_fmaf(P1, xc1, S1);
            }
            wave_scan_fwd2(P0, S0, P1, S1);
            float x0 = dpp<DPP_WAVE_SHR1>(xc0, S0);                  // states entering this lane's first step
            float x1 = dpp<DPP_WAVE_SHR1>(xc1, S1);
            if constexpr (CKPT) {
                if (ck_lane && ll < L) {
                    float *ck = p.ckpt + (ck0 + ll / kCkptInterval) * N + n;
                    ck[0] = x0; ck[1] = x1;
                }
            }
            if constexpr (!WANT_Y) {
                xcv = writelane(xcv, readlane(S0, 63), n);           // inclusive prefix at lane 63 = state after the tile
                xcv = writelane(xcv, readlane(S1, 63), n + 1);
                pcv = writelane(pcv, readlane(pcv, n) * readlane(P0, 63), n);
                pcv = writelane(pcv, readlane(pcv, n + 1) * readlane(P1, 63), n + 1);
            } else {
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    const float Ct0 = reinterpret_cast<const float *>(&C0[t / 4])[t % 4];
                    const float Ct1 = reinterpret_cast<const float *>(&C1[t / 4])[t % 4];
                    x0 = __builtin_fmaf(a0[t], x0, b0[t]);
                    x1 = __builtin_fmaf(a1[t], x1, b1[t]);
                    yv[t] = __builtin_fmaf(Ct0, x0, yv[t]);
                    yv[t] = __builtin_fmaf(Ct1, x1, yv[t]);
                }
                xcv = writelane(xcv, readlane(x0, 63), n);           // lane 63 ends on the tile's last step
                xcv = writelane(xcv, readlane(x1, 63), n + 1);
            }
        };
        if constexpr (N == 1) {
            float4 Bq0[TQ], Bq1[TQ];
#pragma unroll
            for (int q = 0; q < TQ; ++q) Bq0[q] = *reinterpret_cast<const float4 *>(&sB[q * QS + lane * 4]);
            one_state(0, Bq0, Bq1);
        } else {
            static_assert(N == 1 || N % 2 == 0, "states are processed in pairs");
#pragma unroll 1
            for (int n = 0; n < N; n += 2) two_states(n);
        }

        if constexpr (WANT_Y) {
            if (zrow) {
                float zv[T];
                unpack_few<IO, T>(c_z, zv);
#pragma unroll
                for (int t = 0; t < T; ++t) yv[t] *= zv[t] * sigmoid_fast(zv[t]);
            }
            if constexpr (T % io_traits<IO>::EPC == 0) {
                if (vec && rem == TILE) store_seg<IO, T>(yrow + ll, 0, T, true, yv);   // whole tile inside the sequence
                else store_seg<IO, T>(yrow, ll, L, vec, yv);
            } else {                                                             // less than a 16-byte chunk per lane
                store_few<IO, T>(yrow, ll, L, vec, yv);
            }
        }
    }

    if (active && lane < N) {
        if (mode == MODE_AGG) {
            p.ws_P[(row * p.nchunks + chunk) * N + lane] = pcv;
            p.ws_S[(row * p.nchunks + chunk) * N + lane] = xcv;
        } else if (p.x_last && tile1 == ntiles) {
            p.x_last[row * N + lane] = xcv;
        }
    }
}

// Chains the chunk aggregates of one (b,d,n): carry-in of chunk c+1 = P_c * carry-in of chunk c + S_c.
// ws_S[c] is replaced by the carry-in of chunk c.
__global__ void k_ss_carry(const FwdParams p) {
    const int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)p.B * p.D * p.N;
    if (i >= total) return;
    const int64_t row = i / p.N;
    const int n = (int)(i % p.N);
    float x = p.x0 ? p.x0[i] : 0.0f;
    for (int c = 0; c < p.nchunks; ++c) {
        const int64_t j = (row * p.nchunks + c) * p.N + n;
        if (c + 1 == p.nchunks) { p.ws_S[j] = x; break; }     // nothing follows the last chunk: its pair was not computed
        const float P = p.ws_P[j], S = p.ws_S[j];
        p.ws_S[j] = x;
        x = __builtin_fmaf(P, x, S);
    }
}

// Fills up to five buffers of 32-bit words, each with its own word, in one launch (a fill kernel rather than
// hipMemsetAsync, so that a caller may capture the library call in a HIP graph).
__global__ void k_fill(const FillList z) {
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
#pragma unroll
    for (int k = 0; k < FillList::kMax; ++k) {
        uint32_t *ptr = reinterpret_cast<uint32_t *>(z.ptr[k]);
        if (!ptr) continue;
        const uint32_t word = z.bits[k];
        for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < z.count[k]; i += stride) ptr[i] = word;
    }
}

// ---------------------------------------------------------------- launchers
constexpr int kFwdT = 8;
constexpr int kFwdW = 8;

int fwd_tile_steps(int) { return 64 * kFwdT; }
int fwd_channels_per_workgroup() { return kFwdW; }

// Short tiles: the single pass can also run with 4 steps per lane and 4 channels per workgroup (tiles of 256 steps).
// A tile is walked whole whether its steps are real or past the end of the sequence, so short rows and packed
// batches of short sequences waste fewer steps on the smaller tile, which costs about 25 % more per real step (the
// 64-lane prefix is shared by 4 steps instead of 8, the staged maps by 4 channels instead of 8; measured 2.6e12
// against 3.3e12 elements/s on full tiles).  Batch [B,D,L]: taken when the steps walked shrink by more than that
// (L <= 256: twice the rate; 512 < L <= 768: 9 % faster); packed batch: the lengths are on the device, so by the
// mean length (a sequence wastes half a tile on average: the smaller tile pays below about 360 steps per sequence).
constexpr int kFwdShortT = 4;
constexpr int kFwdShortW = 4;
static bool fwd_short_tiles(const FwdParams &p) {
    if (p.nchunks != 1 || (p.mode != MODE_FULL && p.mode != MODE_CKPT_ONLY)) return false;
    if (p.cu) return p.L < (int64_t)360 * p.B;
    const int64_t s8 = 64 * kFwdT, s4 = 64 * kFwdShortT;
    const int64_t walked8 = (p.L + s8 - 1) / s8 * s8, walked4 = (p.L + s4 - 1) / s4 * s4;
    return walked4 * 125 < walked8 * 100;
}

template <typename IO, int N, int DISC>
static hipError_t launch_fwd_short(FwdParams p, hipStream_t s) {
    p.tiles_per_chunk = (p.L + 64 * kFwdShortT - 1) / (64 * kFwdShortT);          // one chunk: every tile of the row
    dim3 grid(p.bcg * ((p.dpg + kFwdShortW - 1) / kFwdShortW), p.B, 1);
    const dim3 block(kFwdShortW * 64);
    if (p.mode == MODE_CKPT_ONLY) hipLaunchKernelGGL((k_ss_fwd<IO, N, kFwdShortT, kFwdShortW, DISC, false, true>), grid, block, 0, s, p);
    else if (p.ckpt) hipLaunchKernelGGL((k_ss_fwd<IO, N, kFwdShortT, kFwdShortW, DISC, true, true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((k_ss_fwd<IO, N, kFwdShortT, kFwdShortW, DISC, true, false>), grid, block, 0, s, p);
    return hipGetLastError();
}

template <typename IO, int N, int DISC>
static hipError_t launch_fwd_n(const FwdParams &p, hipStream_t s) {
    // the aggregate launch skips the last chunk: nobody needs its pair
    if (p.mode == MODE_AGG && p.nchunks < 2) return hipSuccess;
    if (fwd_short_tiles(p)) return launch_fwd_short<IO, N, DISC>(p, s);
    dim3 grid(p.bcg * ((p.dpg + kFwdW - 1) / kFwdW), p.B, p.mode == MODE_AGG ? p.nchunks - 1 : p.nchunks);
    const bool want_y = (p.mode == MODE_FULL || p.mode == MODE_APPLY);
    const dim3 block(kFwdW * 64);
    if (want_y && p.ckpt) hipLaunchKernelGGL((k_ss_fwd<IO, N, kFwdT, kFwdW, DISC, true, true>), grid, block, 0, s, p);
    else if (want_y) hipLaunchKernelGGL((k_ss_fwd<IO, N, kFwdT, kFwdW, DISC, true, false>), grid, block, 0, s, p);
    else if (p.ckpt) hipLaunchKernelGGL((k_ss_fwd<IO, N, kFwdT, kFwdW, DISC, false, true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((k_ss_fwd<IO, N, kFwdT, kFwdW, DISC, false, false>), grid, block, 0, s, p);
    return hipGetLastError();
}

template <typename IO, int DISC>
static hipError_t launch_fwd_disc(const FwdParams &p, hipStream_t s) {
    switch (p.N) {
        case 1: return launch_fwd_n<IO, 1, DISC>(p, s);
        case 2: return launch_fwd_n<IO, 2, DISC>(p, s);
        case 4: return launch_fwd_n<IO, 4, DISC>(p, s);
        case 8: return launch_fwd_n<IO, 8, DISC>(p, s);
        case 16: return launch_fwd_n<IO, 16, DISC>(p, s);
        case 32: return launch_fwd_n<IO, 32, DISC>(p, s);
    }
    return hipErrorInvalidValue;
}

template <typename IO>
static hipError_t launch_fwd_io(const FwdParams &p, int disc, hipStream_t s) {
    switch (disc) {
        case DISC_ZOH_S6: return launch_fwd_disc<IO, DISC_ZOH_S6>(p, s);
        case DISC_ZOH: return launch_fwd_disc<IO, DISC_ZOH>(p, s);
        case DISC_BILINEAR: return launch_fwd_disc<IO, DISC_BILINEAR>(p, s);
        case DISC_DIRAC: return launch_fwd_disc<IO, DISC_DIRAC>(p, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_ss_fwd(const FwdParams &p, int io_dtype, int disc, hipStream_t s) {
    return io_dtype == 1 ? launch_fwd_io<bf16_t>(p, disc, s) : launch_fwd_io<float>(p, disc, s);
}

hipError_t launch_ss_carry(const FwdParams &p, hipStream_t s) {
    const int64_t total = (int64_t)p.B * p.D * p.N;
    hipLaunchKernelGGL(k_ss_carry, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, p);
    return hipGetLastError();
}

hipError_t launch_fill(const FillList &z, hipStream_t s) {
    int64_t most = 0;
    for (int k = 0; k < FillList::kMax; ++k) if (z.ptr[k] && z.count[k] > most) most = z.count[k];
    if (most <= 0) return hipSuccess;
    int64_t blocks = (most + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_fill, dim3((unsigned)blocks), dim3(256), 0, s, z);
    return hipGetLastError();
}

}  // namespace lrnnx
