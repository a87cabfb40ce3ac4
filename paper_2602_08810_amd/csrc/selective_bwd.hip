// Backward selective scan for gfx950: reverse-mode derivative of Eq. 2 of the paper (diagonal,
// input-dependent A(k), B(k), C(k)) with the fused discretisations of Sec. 3.  The state is never
// stored per step (Sec. 3): every time tile is recomputed from the checkpoint the forward wrote.
//
// For one (b,d) row and one state n, with H_l = dLoss/dx_l:
//     H_l      = Cm_{l,n} dypre_l + a_{l+1} H_{l+1}                 (same affine scan, time reversed)
//     dCm_{l,n} += dypre_l x_l          dBm_{l,n} += H_l g_l u_l
//     du_l     += H_l g_l Bm_{l,n}      da_l = H_l x_{l-1}          dg_l = H_l Bm_{l,n} u_l
//     dDelta_l += da_l da/dDelta + dg_l dg/dDelta                    dA_n += da_l da/dA + dg_l dg/dA
//
// Mapping.  Time runs along the lanes as in the forward kernel (lane i owns T consecutive steps of
// the tile), but the N states are split over the W = N/NK wavefronts of the workgroup, which all
// work on the same channel at the same time.  A wavefront therefore keeps its NK columns of Bm/Cm
// for the tile, and the running sums of dBm/dCm over channels, in registers while the workgroup
// loops over G channels: the reduction of dBm/dCm over channels costs no memory traffic and no
// per-element atomics inside the loop (LDS float atomics are very slow on this chip when every lane
// takes part; only the few lanes that own a per-channel sum use them).  What is summed over n
// (du, dDelta, ypre for dz) is exchanged through LDS once per (channel, tile): each wavefront
// writes its partial sums, and after a barrier the threads share the epilogue of the 64*T steps
// in flat order, so u/delta/dy/z are each read once and du/ddelta/dz written once, coalesced.
// At the end of a tile the dBm/dCm sums are transposed through LDS and added to global memory
// with fully coalesced float atomics (other workgroups hold other channel groups).
#include "kernels.hpp"
#include "scan_common.hpp"

namespace lrnnx {

constexpr int kMaxG = 128;

template <typename IO, int N, int NK, int T, int DISC, bool DZ>
__global__ __launch_bounds__((N / NK) * 64, 2) void k_ss_bwd(const BwdParams p) {
    constexpr int W = N / NK;
    constexpr int NT = W * 64;
    constexpr int TILE = 64 * T;
    constexpr int TPW = TILE / NT > 0 ? TILE / NT : 1;   // flat steps per thread in prologue / epilogue
    constexpr int NA = TILE / TPW;                   // threads that take part in them: all, or (N = 32) the first 256
    constexpr int TQ = T / 4;
    constexpr int CK_PER_TILE = TILE / (int)kCkptInterval;
    // states whose scans advance together: all of the wavefront's, or two for the schemes that also keep the gains
    // g of every step (more registers)
    constexpr int JSW = (DISC == DISC_ZOH || DISC == DISC_BILINEAR) ? 2 : 4;
    constexpr int JS = NK < JSW ? NK : JSW;
    static_assert(T % 4 == 0 && (T % W == 0 || W % T == 0) && TPW <= 8 && NA % 64 == 0 && NA <= NT, "tile shape");
    static_assert(TILE % kCkptInterval == 0, "tiles must start on checkpoints");
    static_assert(TILE == kBwdTileSteps, "the chunked launch counts its chunks in tiles of this kernel");

    __shared__ __attribute__((aligned(16))) float sIn[3 * TILE];          // delta, u, dypre   [q][lane][4]
    __shared__ __attribute__((aligned(16))) float sPart[W * 3 * TILE];    // per wave: ypre, du, ddelta partials
    __shared__ __attribute__((aligned(16))) float sBt[N * TILE];          // Bm columns of the tile, fp32: [n][q][lane][4], wave-private slices
    __shared__ float sH[kMaxG * N];       // a_{l0} H_{l0} carried to the earlier tile, per (channel, n)
    __shared__ float sdA[2][kMaxG * N];   // per half-wavefront partial sums of dA (added up when they are flushed)
    __shared__ float sdD[2 * W * kMaxG];  // dD and dbias partial sums per (half-wavefront, wavefront, channel)
    __shared__ float sdb[2 * W * kMaxG];

    // Two workgroups share a compute unit, so each SIMD holds one wavefront of each.  The issue arbiter prefers the
    // older wavefront, the older workgroup finishes some 17 % earlier and the younger one then runs alone, badly
    // hiding its latencies (measured: 474 us against 570 us on the Mamba-block shape).  With four wavefronts per
    // workgroup the two wavefronts of a SIMD therefore take turns at the higher issue priority, one channel each
    // (told apart by the lowest bit of the hardware wavefront slot): 5-7 % faster on every shape tried.  Not with
    // eight wavefronts per workgroup (both wavefronts of a SIMD then belong to one workgroup and meet at its
    // barriers: 7 % slower), and of no effect with two.
    constexpr bool ALT_PRIO = (N / NK == 4);
    [[maybe_unused]] const unsigned hw_slot = ALT_PRIO ? (__builtin_amdgcn_s_getreg(6148) & 1u) : 0u;   // HW_ID.WAVE_ID, bit 0
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // packed batches: workgroups start in launch order, so the longest sequences go first and the short ones fill the
    // end of the launch instead of a long one running on alone
    const int b = p.order ? p.order[blockIdx.y] : blockIdx.y;
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
    // Chunked launch: this workgroup walks chunk blockIdx.z of its rows only, i.e. the steps toff .. toff + L - 1 of
    // the time axis, starting from that chunk's carried adjoint.  Chunks are counted from the start of the sequence;
    // the last one takes whatever is left (see chunk_span in selective_bwd_carry.hip), and the workgroups of a packed
    // sequence that ends before their chunk leave here, all threads together and before any barrier (chunk 0 stays
    // even for an empty sequence: it writes that sequence's dx0).
    const int chunk = blockIdx.z;
    if (p.nchunks > 1) {
        const int64_t span = p.tiles_per_chunk * TILE;
        const int64_t left = L - chunk * span;
        if (chunk > 0 && left <= 0) return;
        toff += chunk * span;
        L = (chunk == p.nchunks - 1 || left < span) ? left : span;
    }
    const int64_t ntiles = (L + TILE - 1) / TILE;
    // a workgroup takes up to G consecutive channels of ONE Bm/Cm group; in a packed batch with a work cap fewer when
    // its sequence is long, and the workgroups of the launch that its sequence then does not need leave here, all
    // threads together and before any barrier
    int G = p.G;
    if (p.wcap > 0) {
        const int64_t fit = p.wcap / (ntiles > 0 ? ntiles : 1);
        G = fit < p.gmin ? p.gmin : (fit < G ? (int)fit : G);
    }
    const int chunks_per_grp = (p.dpg + G - 1) / G;
    if ((int)blockIdx.x >= p.bcg * chunks_per_grp) return;
    const int grp = blockIdx.x / chunks_per_grp;
    const int din0 = (blockIdx.x % chunks_per_grp) * G;
    const int d0 = grp * p.dpg + din0;
    const int Gact = (p.dpg - din0 < G) ? p.dpg - din0 : G;
    const int bcrow = b * p.bcg + grp;                               // row of Bm, Cm, dBm, dCm (unpacked)
    // checkpoints of this workgroup's rows: [B,D,nck,N], or packed [D,nslots,N] with sequence b at slot toff/interval + b
    const int64_t nck = p.cu ? p.nslots : (p.L + kCkptInterval - 1) / kCkptInterval;
    const int64_t ck0 = p.cu ? toff / kCkptInterval + b : toff / kCkptInterval;
    const bool vec = p.vec != 0;
    const bool has_z = p.z != nullptr;

    for (int i = tid; i < kMaxG * N; i += NT) {
        float h = 0.0f;
        if (p.nchunks > 1 && i < Gact * N)
            h = p.hc[(((int64_t)b * p.D + d0 + i / N) * p.nchunks + chunk) * N + i % N];
        sH[i] = h; sdA[0][i] = 0.0f; sdA[1][i] = 0.0f;
    }
    for (int i = tid; i < 2 * W * kMaxG; i += NT) { sdD[i] = 0.0f; sdb[i] = 0.0f; }

    const int64_t bc0 = ((p.cu ? (int64_t)grp : (int64_t)bcrow) * p.L + toff) * N;   // first element of the maps of this sequence
    const IO *Bm = reinterpret_cast<const IO *>(p.Bm) + bc0;
    const IO *Cm = reinterpret_cast<const IO *>(p.Cm) + bc0;

    // flat position of this thread in prologue / epilogue, and its slot in the [q][lane][4] layout
    const int f0 = tid * TPW;
    const bool io_thread = NA == NT || tid < NA;                     // wave-uniform: NA is a multiple of 64
    auto fslot = [](int f) { return (((f % T) / 4) * 64 + f / T) * 4 + (f % 4); };

    // ---- The dBm/dCm sums of a tile (over the workgroup's channels) are added to global memory one tile late: after
    // the next tile's loads have been issued, so that those round trips run while the flush goes through LDS, and so
    // that nothing has to wait for the atomics (the memory counter is in order: a load issued after them cannot be
    // claimed before they are done, and all workgroups flush at about the same time).  The sums are transposed
    // through LDS so that consecutive threads hit consecutive addresses: two rounds of 32 lanes each, in the area of
    // the Bm columns (the tile they belonged to is finished, the next tile stages its own after the flush).
    // `mid` runs after the first round's trip through LDS, before the first atomic.
    float dBacc[NK][T], dCacc[NK][T];
    int64_t fl_l0 = 0;                                               // first step of the tile the sums belong to
    int fl_rem = 0;                                                  // its valid steps; 0: nothing to flush
    auto flush = [&](auto &&mid) {
        constexpr int FL = 32;                                           // lanes per round
        float *fbB = sBt, *fbC = sBt + FL * T * N;
        static_assert(2 * FL * T * N <= N * TILE, "flush buffer must fit in the Bm area");
#pragma unroll
        for (int j = 0; j < 64 / FL; ++j) {
            __syncthreads();
            // A lane's values of one step are NK consecutive floats of that step's row.  With NK = 4 they go out as one
            // 16-byte write; lanes are T * N floats apart, which would put all of them on the same banks (measured:
            // the 32-way conflicts of the plain layout made the flush 11 % of the kernel), so the 16-byte chunk index
            // is XORed with the lane's low bits: eight consecutive lanes then cover all banks, and a reader's 64
            // consecutive floats stay a permutation of whole chunks within the same 8-chunk block.
            constexpr bool SWZ = NK == 4;
            constexpr int CPL = T * N / 4;                               // 16-byte chunks per lane
            if (lane / FL == j) {
                // (the addresses are formed here and now: hoisted out of the tile loop they would sit in registers
                // all through the channel loop, which has none to spare)
                int lr = lane % FL;
                asm volatile("" : "+v"(lr));
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    if constexpr (SWZ) {
                        const int c4 = ((lr * T + t) * (N / 4) + w) ^ (lr & 7);
                        *reinterpret_cast<float4 *>(&fbB[c4 * 4]) = make_float4(dBacc[0][t], dBacc[1][t], dBacc[2][t], dBacc[3][t]);
                        *reinterpret_cast<float4 *>(&fbC[c4 * 4]) = make_float4(dCacc[0][t], dCacc[1][t], dCacc[2][t], dCacc[3][t]);
                    } else {
#pragma unroll
                        for (int k = 0; k < NK; ++k) {
                            fbB[(lr * T + t) * N + w * NK + k] = dBacc[k][t];
                            fbC[(lr * T + t) * N + w * NK + k] = dCacc[k][t];
                        }
                    }
                }
            }
            __syncthreads();
            const int step0 = j * FL * T;                                // within the tile
            float *gB = p.dBm + bc0 + (fl_l0 + step0) * N, *gC = p.dCm + bc0 + (fl_l0 + step0) * N;
            // each thread's values are read from LDS in one batch, then added (one round trip instead of one per value)
            constexpr int PER = FL * T * N / NT;                         // = T * NK / 2
            static_assert(PER * NT == FL * T * N, "the flush buffer is a whole number of values per thread");
            float vB[PER], vC[PER];
            int tf = tid;
            asm volatile("" : "+v"(tf));
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int idx = tf + i * NT;
                const int at = SWZ ? ((((idx >> 2) ^ (((idx >> 2) / CPL) & 7)) << 2) | (idx & 3)) : idx;
                vB[i] = fbB[at]; vC[i] = fbC[at];
            }
            if (j == 0) mid();
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int idx = tid + i * NT;
                if (step0 + idx / N < fl_rem) {
                    unsafeAtomicAdd(gB + (unsigned)idx, vB[i]);
                    unsafeAtomicAdd(gC + (unsigned)idx, vC[i]);
                }
            }
        }
        __syncthreads();
    };

    for (int64_t tile = ntiles - 1; tile >= 0; --tile) {
        const int64_t l0 = tile * TILE;
        const int rem = (L - l0 < TILE) ? (int)(L - l0) : TILE;      // valid steps of this tile
        // all global addresses below are a wave-uniform base plus a small unsigned per-lane offset, so that
        // they need one 32-bit register per lane instead of a 64-bit induction variable each
        const IO *BmT = Bm + l0 * N + w * NK, *CmT = Cm + l0 * N + w * NK;

        // ---- this wavefront's NK columns of Bm/Cm for the tile: fetched here (raw), used after the flush of the
        // tile before (below), so that the round trip runs while that flush goes through LDS.  Every row is loaded
        // without a branch (past the end of the tile the last valid row is read again and then discarded), so that
        // all 2 T loads of a lane are in flight together instead of one round trip per step.
        RawFew<IO, NK> rB[T], rC[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            const int step = lane * T + t;
            const int row = step < rem ? step : rem - 1;                  // rem >= 1: a tile has at least one step
            load_few_raw<IO, NK>(BmT + (unsigned)(row * N), 0, NK, true, rB[t]);
            load_few_raw<IO, NK>(CmT + (unsigned)(row * N), 0, NK, true, rC[t]);
        }

        // Per-channel inputs are fetched one channel ahead, so that their latency hides behind the main pass.  Every
        // memory access of the channel loop is unconditional straight-line code (rows past the end of the tile, absent
        // optional inputs and the channel past the last one read a valid address again and the value is discarded).
        // (Fetching two channels ahead into two register sets was tried: the doubled loop body costs more than the
        // longer distance gains.)
        struct Pref { RawFew<IO, TPW> u, dl, dy, z; float A[NK], ck[NK], Dsk, bias; };
        Pref S0;
        // Row pointers (wave-uniform) of the channel the next prefetch reads and of the channel the next epilogue
        // writes: set once per tile and stepped by one channel stride each time, so that the channel loop carries no
        // 64-bit multiplications.
        const int64_t tl = toff + l0;
        const IO *n_u = reinterpret_cast<const IO *>(p.u) + bs * p.u_sb + d0 * p.u_sd + tl;
        const IO *n_dl = reinterpret_cast<const IO *>(p.delta) + bs * p.dl_sb + d0 * p.dl_sd + tl;
        const IO *n_dy = reinterpret_cast<const IO *>(p.dy) + bs * p.dy_sb + d0 * p.dy_sd + tl;
        const IO *n_z = has_z ? reinterpret_cast<const IO *>(p.z) + bs * p.z_sb + d0 * p.z_sd + tl : n_dy;
        const int64_t z_step = has_z ? p.z_sd : p.dy_sd;
        IO *o_du_row = reinterpret_cast<IO *>(p.du) + bs * p.du_sb + d0 * p.du_sd + tl;
        IO *o_dd_row = reinterpret_cast<IO *>(p.ddelta) + bs * p.dd_sb + d0 * p.dd_sd + tl;
        IO *o_dz_row = DZ ? reinterpret_cast<IO *>(p.dz) + bs * p.dz_sb + d0 * p.dz_sd + tl : nullptr;
        const float *n_A = p.A + (int64_t)d0 * N + w * NK;
        const int64_t ck_stride = nck * N;                              // floats between the checkpoints of two channels
        const float *n_ck = p.ckpt + ((p.cu ? (int64_t)d0 : (int64_t)b * p.D + d0) * nck + ck0 + tile * CK_PER_TILE) * N + w * NK;
        const bool has_D = p.Dskip != nullptr, has_bias = p.bias != nullptr;
        const float *n_Dsk = has_D ? p.Dskip + d0 : p.A, *n_bias = has_bias ? p.bias + d0 : p.A;
        int n_left = Gact - 1;                                           // channels after the one the pointers are on
        auto prefetch = [&](Pref &s) {
            if (io_thread) {
                if constexpr (TPW == 1) {
                    // steps past the end of the tile read the last valid one again; the prologue discards them
                    load_one_raw_clamped<IO>(n_u, f0, rem, s.u);
                    load_one_raw_clamped<IO>(n_dl, f0, rem, s.dl);
                    load_one_raw_clamped<IO>(n_dy, f0, rem, s.dy);
                    load_one_raw_clamped<IO>(n_z, f0, rem, s.z);
                } else {
                    load_few_raw<IO, TPW>(n_u, f0, rem, vec, s.u);
                    load_few_raw<IO, TPW>(n_dl, f0, rem, vec, s.dl);
                    load_few_raw<IO, TPW>(n_dy, f0, rem, vec, s.dy);
                    load_few_raw<IO, TPW>(n_z, f0, rem, vec, s.z);
                }
            }
#pragma unroll
            for (int k = 0; k < NK; ++k) { s.A[k] = n_A[k]; s.ck[k] = n_ck[k]; }
            s.Dsk = *n_Dsk;
            s.bias = *n_bias;
            const bool more = n_left > 0;                                // else stay on the last channel
            n_left -= more ? 1 : 0;
            n_u += more ? p.u_sd : 0; n_dl += more ? p.dl_sd : 0; n_dy += more ? p.dy_sd : 0; n_z += more ? z_step : 0;
            n_A += more ? N : 0; n_ck += more ? ck_stride : 0;
            n_Dsk += (more && has_D) ? 1 : 0; n_bias += (more && has_bias) ? 1 : 0;
        };
        // The prefetched registers are claimed ("settled") at a point of the program where their loads have long
        // arrived and no store is in flight behind them: the memory counter is in order, so a wait for a load that
        // comes after younger stores (the epilogue's, issued under a branch) would wait for those stores as well.
        auto settle = [&](Pref &s) {
#pragma unroll
            for (int i = 0; i < RawFew<IO, TPW>::WORDS; ++i)
                asm volatile("" : "+v"(s.u.w[i]), "+v"(s.dl.w[i]), "+v"(s.dy.w[i]), "+v"(s.z.w[i]) : : "memory");
#pragma unroll
            for (int k = 0; k < NK; ++k) asm volatile("" : "+v"(s.A[k]), "+v"(s.ck[k]) : : "memory");
            asm volatile("" : "+v"(s.Dsk), "+v"(s.bias) : : "memory");
        };
        prefetch(S0);
        // The loads above are claimed before the first atomic of the flush is issued (the memory counter is in
        // order and the atomics sit under a branch: a wait placed after them would wait for them as well), i.e. after
        // the flush's first trip through LDS.
        auto settle_tile = [&]() {
            settle(S0);
#pragma unroll
            for (int t = 0; t < T; ++t)
#pragma unroll
                for (int i = 0; i < RawFew<IO, NK>::WORDS; ++i)
                    asm volatile("" : "+v"(rB[t].w[i]), "+v"(rC[t].w[i]) : : "memory");
        };
        if (fl_rem > 0) flush(settle_tile);          // the sums of the tile before (later in time); same branch for the whole workgroup
        settle_tile();
        // Cm and both sums stay in registers; the Bm columns go to this wavefront's own slice of LDS (read back as
        // ds_read_b128 in each pass)
        float Cv[NK][T];
        {
        float Bv[NK][T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            float tb[NK], tc[NK];
            unpack_few<IO, NK>(rB[t], tb);
            unpack_few<IO, NK>(rC[t], tc);
            const int step = lane * T + t;
#pragma unroll
            for (int k = 0; k < NK; ++k) {
                Bv[k][t] = step < rem ? tb[k] : 0.0f; Cv[k][t] = step < rem ? tc[k] : 0.0f;
                dBacc[k][t] = 0.0f; dCacc[k][t] = 0.0f;
            }
        }
#pragma unroll
        for (int k = 0; k < NK; ++k)
#pragma unroll
            for (int q = 0; q < TQ; ++q)
                *reinterpret_cast<float4 *>(&sBt[(((w * NK + k) * TQ + q) * 64 + lane) * 4]) =
                    make_float4(Bv[k][4 * q], Bv[k][4 * q + 1], Bv[k][4 * q + 2], Bv[k][4 * q + 3]);
        }

        // Order of a channel's work between the workgroup's two barriers per channel.  After the first barrier (the
        // step inputs of channel g are in LDS): the main pass, which leaves the wavefronts' partial sums in LDS.
        // After the second: the LDS reads of the epilogue of channel g are issued, the prologue of channel g+1 runs
        // while they are in flight (softplus, gate, staging of the step inputs; its inputs were fetched during the
        // main pass), then the epilogue's arithmetic and stores.  Kept in registers from a channel's prologue to its
        // epilogue: d softplus / ds, the factor that turns ypre into dz, and Dskip (n_*: of the channel after).
        float e_sg[TPW], e_zf[TPW], n_sg[TPW], n_zf[TPW];
        float Dsk = 0.0f, nDsk = 0.0f;
        float cA[NK], cck[NK];                       // A and the checkpointed state of the main pass's channel

        // ---- prologue of the channel whose inputs S0 holds: each thread prepares TPW flat steps for everybody
        auto prologue = [&]() {
            const float bias = has_bias ? S0.bias : 0.0f;
            // The values are moved out of S0 here and now (real moves, which the compiler may not turn into a renaming):
            // the fetch that follows then loads into the very registers S0 has at the top of the loop.  Left to the
            // compiler, the fetch gets fresh registers and the copies land at the end of the loop body, where they
            // wait for the loads that have just been issued.
            nDsk = has_D ? S0.Dsk : 0.0f;
            asm volatile("" : "+v"(nDsk));
#pragma unroll
            for (int k = 0; k < NK; ++k) {
                asm volatile("v_mov_b32 %0, %1" : "=v"(cA[k]) : "v"(S0.A[k]));
                asm volatile("v_mov_b32 %0, %1" : "=v"(cck[k]) : "v"(S0.ck[k]));
            }
            if (io_thread) {
                float e_u[TPW], r_d[TPW], e_dy[TPW], e_z[TPW];
                unpack_few<IO, TPW>(S0.u, e_u);
                unpack_few<IO, TPW>(S0.dl, r_d);
                unpack_few<IO, TPW>(S0.dy, e_dy);
                unpack_few<IO, TPW>(S0.z, e_z);
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
                    float sp, dyp;
                    bwd_step_inputs<sizeof(IO) == 4>(r_d[i] + bias, e_dy[i], has_z ? e_z[i] : 0.0f, p.softplus != 0, has_z, sp, n_sg[i], dyp, n_zf[i]);
                    const bool valid = f0 + i < rem;     // steps past the end: Delta = 0 (a = 1), no input, no gradient
                    sIn[0 * TILE + fslot(f0 + i)] = valid ? sp : 0.0f;
                    sIn[1 * TILE + fslot(f0 + i)] = valid ? e_u[i] : 0.0f;
                    sIn[2 * TILE + fslot(f0 + i)] = valid ? dyp : 0.0f;
                }
            }
        };
        auto rotate = [&]() {
#pragma unroll
            for (int i = 0; i < TPW; ++i) { e_sg[i] = n_sg[i]; e_zf[i] = n_zf[i]; }
            Dsk = nDsk;
        };
        prologue();                                  // channel 0
        rotate();
        prefetch(S0);                                // channel 1 (where there is none, the last channel again)

        auto channel = [&](const int g) {
            if constexpr (ALT_PRIO) {
                if ((unsigned)(g & 1) == hw_slot) __builtin_amdgcn_s_setprio(1); else __builtin_amdgcn_s_setprio(0);
            }
            __syncthreads();

            // ---- main: this lane's T steps, this wavefront's NK states
            float dl[T], dyp[T], dlu[T], ypre[T], pdu[T], pdd[T];
#pragma unroll
            for (int q = 0; q < TQ; ++q) {
                const float4 v0 = *reinterpret_cast<const float4 *>(&sIn[0 * TILE + (q * 64 + lane) * 4]);
                const float4 v1 = *reinterpret_cast<const float4 *>(&sIn[1 * TILE + (q * 64 + lane) * 4]);
                const float4 v2 = *reinterpret_cast<const float4 *>(&sIn[2 * TILE + (q * 64 + lane) * 4]);
                dl[4 * q] = v0.x; dl[4 * q + 1] = v0.y; dl[4 * q + 2] = v0.z; dl[4 * q + 3] = v0.w;
                dlu[4 * q] = v1.x; dlu[4 * q + 1] = v1.y; dlu[4 * q + 2] = v1.z; dlu[4 * q + 3] = v1.w;   // u for now
                dyp[4 * q] = v2.x; dyp[4 * q + 1] = v2.y; dyp[4 * q + 2] = v2.z; dyp[4 * q + 3] = v2.w;
            }
#pragma unroll
            for (int t = 0; t < T; ++t)
                if constexpr (DISC == DISC_ZOH_S6) dlu[t] *= dl[t];   // S6 only ever needs Delta*u; the others keep u

            float dA4[NK];
#pragma unroll
            for (int k0 = 0; k0 < NK; k0 += JS) {
            // ---- phase 1: forward fold (states) and backward fold (adjoint) of this lane's T steps, JS states at a time
            float a[NK][T + 1], gg[NK][T], x[NK][T], cdy[NK][T];
            float P[NK], S[NK], Pr[NK], Sr[NK], hcv[NK];
            ACoef acs[NK];
            // The Bm columns of all JS states are read from LDS in one batch (one round trip instead of one per state;
            // the scheduler is kept from moving the reads down to their uses)
            float Bk[NK][T];
            auto read_Bk = [&]() {
#pragma unroll
                for (int k = k0; k < k0 + JS; ++k)
#pragma unroll
                    for (int q = 0; q < TQ; ++q) {
                        const float4 vb = *reinterpret_cast<const float4 *>(&sBt[(((w * NK + k) * TQ + q) * 64 + lane) * 4]);
                        Bk[k][4 * q] = vb.x; Bk[k][4 * q + 1] = vb.y; Bk[k][4 * q + 2] = vb.z; Bk[k][4 * q + 3] = vb.w;
                    }
            };
            read_Bk();
#pragma unroll
            for (int k = k0; k < k0 + JS; ++k) hcv[k] = sH[g * N + w * NK + k];
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = k0; k < k0 + JS; ++k) {
                const ACoef ac = make_acoef<DISC>(cA[k]);
                acs[k] = ac;
                const float xck = cck[k];
                const float hc = hcv[k];
                float sx = 0.0f;
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    disc_ag<DISC>(dl[t], ac, a[k][t], gg[k][t]);
                    if constexpr (DISC == DISC_ZOH_S6) x[k][t] = dlu[t] * Bk[k][t];
                    else if constexpr (DISC == DISC_DIRAC) x[k][t] = dlu[t] * Bk[k][t];
                    else x[k][t] = gg[k][t] * dlu[t] * Bk[k][t];
                    sx = (t == 0) ? x[k][0] : __builtin_fmaf(a[k][t], sx, x[k][t]);   // the fold starts from zero
                }
                // products of the multipliers of this lane's steps (state prefix) and of the same steps shifted by one
                // (adjoint suffix: H_l = c_l + a_{l+1} H_{l+1}; the multiplier after the tile's last step is 1 because
                // the carried value is already a_{l1} H_{l1}).  The inner factors are shared.
                a[k][T] = dpp<DPP_WAVE_SHL1>(1.0f, a[k][0]);
                float inner = a[k][1];
#pragma unroll
                for (int t = 2; t < T; ++t) inner *= a[k][t];
                const float p = a[k][0] * inner, pr = inner * a[k][T];
                if (lane == 0) sx = __builtin_fmaf(p, xck, sx);             // the checkpointed state enters through lane 0
                P[k] = p; S[k] = sx;

                float sr = 0.0f;
#pragma unroll
                for (int t = T - 1; t >= 0; --t) {
                    cdy[k][t] = Cv[k][t] * dyp[t];
                    sr = (t == T - 1) ? cdy[k][t] : __builtin_fmaf(a[k][t + 1], sr, cdy[k][t]);
                }
                if (lane == 63) sr = __builtin_fmaf(pr, hc, sr);            // the carried adjoint enters through lane 63
                Pr[k] = pr; Sr[k] = sr;
            }
            // ---- phase 2: state prefixes (forward in time) and adjoint suffixes (backward in time) of these JS states;
            // the Bm columns are read again meanwhile (the fold has consumed the first copy)
            __builtin_amdgcn_sched_barrier(0);
            read_Bk();
            __builtin_amdgcn_sched_barrier(0);
            wave_scan_fwd_rev_multi<JS>(P + k0, S + k0, Pr + k0, Sr + k0, lane);
            // ---- phase 3: replay of the states and of the adjoint, gradients
#pragma unroll
            for (int k = k0; k < k0 + JS; ++k) {
                const int n = w * NK + k;
                const ACoef ac = acs[k];
                const float xin = dpp<DPP_WAVE_SHR1>(cck[k], S[k]);         // x entering this lane's first step
                {
                    float xp = xin;
#pragma unroll
                    for (int t = 0; t < T; ++t) { xp = __builtin_fmaf(a[k][t], xp, x[k][t]); x[k][t] = xp; }
                }
                const float H0 = Sr[k];                                     // H of this lane's first step
                float R = dpp<DPP_WAVE_SHL1>(hcv[k], Sr[k]);                // H of the next lane's first step (the carry itself past lane 63)
                if (lane == 0) sH[g * N + n] = a[k][0] * H0;                // carried to the earlier tile

                float dA_part = 0.0f;                                       // this lane's share of dA[d, n]
#pragma unroll
                for (int t = T - 1; t >= 0; --t) {
                    R = __builtin_fmaf(a[k][t + 1], R, cdy[k][t]);            // H_t
                    const float xprev = (t > 0) ? x[k][t - 1] : xin;
                    dCacc[k][t] = __builtin_fmaf(dyp[t], x[k][t], dCacc[k][t]);
                    if constexpr (DZ) ypre[t] = (k == 0) ? Cv[k][t] * x[k][t] : __builtin_fmaf(Cv[k][t], x[k][t], ypre[t]);
                    // the first state of the wavefront starts the sums over n (pdu, pdd), the others add to them
                    auto acc = [&](float &sum, float m1, float m2) { sum = (k == 0) ? m1 * m2 : __builtin_fmaf(m1, m2, sum); };
                    if constexpr (DISC == DISC_ZOH_S6 || DISC == DISC_DIRAC) {
                        // S6: g = Delta (du and dDelta share sum_n H B, scaled in the epilogue); dirac: g = 1, and only
                        // a = e^{Delta A} depends on Delta and A
                        acc(pdu[t], R, Bk[k][t]);
                        dBacc[k][t] = __builtin_fmaf(R, dlu[t], dBacc[k][t]);
                        const float q = R * xprev * a[k][t];
                        acc(pdd[t], q, ac.A);
                        dA_part = __builtin_fmaf(q, dl[t], dA_part);
                    } else if constexpr (DISC == DISC_ZOH) {
                        // da/dDelta = A a, da/dA = Delta a, dg/dDelta = a: the common factor a is taken out
                        float a_t, a_A, g_t, g_A;
                        disc_partials<DISC>(dl[t], ac, a[k][t], gg[k][t], a_t, a_A, g_t, g_A);
                        const float hb = R * Bk[k][t];
                        const float dg = hb * dlu[t];
                        const float dax = R * a[k][t] * xprev;               // H x_{l-1} a
                        acc(pdu[t], hb, gg[k][t]);
                        dBacc[k][t] = __builtin_fmaf(R * gg[k][t], dlu[t], dBacc[k][t]);
                        if (k == 0) pdd[t] = __builtin_fmaf(dax, ac.A, dg * a[k][t]);
                        else pdd[t] = __builtin_fmaf(dax, ac.A, __builtin_fmaf(dg, a[k][t], pdd[t]));
                        dA_part = __builtin_fmaf(dax, dl[t], __builtin_fmaf(dg, g_A, dA_part));
                    } else {
                        // bilinear: with q = 1 / (1 - Delta A / 2) all four partials are multiples of q^2, and
                        // a = (1 + Delta A / 2) q gives q = (a + 1) / 2 without a second reciprocal
                        const float q = __builtin_fmaf(a[k][t], 0.5f, 0.5f);
                        const float q2 = q * q;
                        const float da = R * xprev;
                        const float hb = R * Bk[k][t];
                        const float dg = hb * dlu[t];
                        acc(pdu[t], hb, gg[k][t]);
                        dBacc[k][t] = __builtin_fmaf(R * gg[k][t], dlu[t], dBacc[k][t]);
                        acc(pdd[t], __builtin_fmaf(da, ac.A, dg), q2);                                            // A q^2 da + q^2 dg
                        dA_part = __builtin_fmaf(__builtin_fmaf(0.5f * dl[t], dg, da) * dl[t], q2, dA_part);     // Delta q^2 da + Delta^2 q^2 dg / 2
                    }
                }
                if constexpr (NK == 4 || NK == 2) {
                    dA4[k] = dA_part;
                } else {
                    const float dA_tot = wave_sum(dA_part);
                    if (lane == 0) lds_add(&sdA[0][g * N + n], dA_tot);
                }
            }
            }   // groups of JS states
            if constexpr (NK == 4) {
                // The four per-lane partial sums are reduced together: two exchange steps leave each lane of a quad
                // with the quad's sum of ONE state (lane%4 = 0,1,2,3 -> state 0,2,1,3), two rotations sum the quads of
                // a row, one row-pair swap sums the two rows of a half-wavefront; lanes 0-3 and 32-35 own the results.
                const bool b0 = lane & 1, b1 = lane & 2;
                float kA = b0 ? dA4[2] : dA4[0], kB = b0 ? dA4[3] : dA4[1];
                const float sA = b0 ? dA4[0] : dA4[2], sB = b0 ? dA4[1] : dA4[3];
                kA += dpp<0xB1>(0.0f, sA);                                  // quad_perm [1,0,3,2]
                kB += dpp<0xB1>(0.0f, sB);
                float v = b1 ? kB : kA;
                v += dpp<0x4E>(0.0f, b1 ? kA : kB);                         // quad_perm [2,3,0,1]
                v += dpp<0x124>(0.0f, v);                                   // row_ror:4
                v += dpp<0x128>(0.0f, v);                                   // row_ror:8
                v = sum_xor16(v);
                if ((lane & 0x1C) == 0) lds_add(&sdA[lane >> 5][g * N + w * NK + ((lane & 1) << 1) + ((lane >> 1) & 1)], v);
            } else if constexpr (NK == 2) {
                // the same with two partial sums: even lanes end up with state 0, odd lanes with state 1
                const bool odd = lane & 1;
                float v = odd ? dA4[1] : dA4[0];
                v += dpp<0xB1>(0.0f, odd ? dA4[0] : dA4[1]);               // quad_perm [1,0,3,2]
                v += dpp<0x4E>(0.0f, v);                                    // quad_perm [2,3,0,1]
                v += dpp<0x124>(0.0f, v);                                   // row_ror:4
                v += dpp<0x128>(0.0f, v);                                   // row_ror:8
                v = sum_xor16(v);
                if ((lane & 0x1E) == 0) lds_add(&sdA[lane >> 5][g * N + w * NK + (lane & 1)], v);
            }
#pragma unroll
            for (int q = 0; q < TQ; ++q) {
                float *base = &sPart[(w * 3) * TILE + (q * 64 + lane) * 4];
                if constexpr (DZ) *reinterpret_cast<float4 *>(base) = make_float4(ypre[4 * q], ypre[4 * q + 1], ypre[4 * q + 2], ypre[4 * q + 3]);
                *reinterpret_cast<float4 *>(base + TILE) = make_float4(pdu[4 * q], pdu[4 * q + 1], pdu[4 * q + 2], pdu[4 * q + 3]);
                *reinterpret_cast<float4 *>(base + 2 * TILE) = make_float4(pdd[4 * q], pdd[4 * q + 1], pdd[4 * q + 2], pdd[4 * q + 3]);
            }
            __syncthreads();
            // ---- epilogue of this channel, with the prologue of the next one in its shadow
            float e_in[TPW][3], e_part[TPW][W][3];
            if (io_thread) {
                // every LDS value of the epilogue is read up front, in one round trip (left alone, the compiler moves
                // the reads that only feed the stores into the stores' own branch, one round trip after the other)
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
#pragma unroll
                    for (int j = 0; j < 3; ++j) e_in[i][j] = sIn[j * TILE + fslot(f0 + i)];
#pragma unroll
                    for (int ww = 0; ww < W; ++ww)
#pragma unroll
                        for (int j = DZ ? 0 : 1; j < 3; ++j) e_part[i][ww][j] = sPart[(ww * 3 + j) * TILE + fslot(f0 + i)];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            settle(S0);                              // the next channel's inputs: claimed before this channel's stores
            prologue();                              // (past the last channel: the last one again, unused)
            prefetch(S0);                            // the channel after the next
            __builtin_amdgcn_sched_barrier(0);
            if (io_thread) {
                float o_du[TPW], o_dd[TPW], o_dz[TPW];
                float dD_part = 0.0f, db_part = 0.0f;
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
                    const float e_u = e_in[i][1], e_dyp = e_in[i][2];
                    float yp = Dsk * e_u, s_du = 0.0f, s_dd = 0.0f;
#pragma unroll
                    for (int ww = 0; ww < W; ++ww) {
                        if constexpr (DZ) yp += e_part[i][ww][0];
                        s_du += e_part[i][ww][1];
                        s_dd += e_part[i][ww][2];
                    }
                    if constexpr (DISC == DISC_ZOH_S6) {
                        // the wavefronts' sums are sum_n H B: dDelta += u sum_n H B, du = Delta sum_n H B
                        s_dd = __builtin_fmaf(e_u, s_du, s_dd);
                        s_du *= e_in[i][0];
                    }
                    o_du[i] = __builtin_fmaf(e_dyp, Dsk, s_du);
                    o_dd[i] = s_dd * e_sg[i];
                    o_dz[i] = yp * e_zf[i];
                    dD_part = __builtin_fmaf(e_dyp, e_u, dD_part);
                    db_part += (f0 + i < rem) ? o_dd[i] : 0.0f;
                    asm volatile("" : "+v"(o_du[i]), "+v"(o_dd[i]), "+v"(o_dz[i]));   // computed here, not inside the stores' branch
                }
                store_few<IO, TPW>(o_du_row, f0, rem, vec, o_du);
                store_few<IO, TPW>(o_dd_row, f0, rem, vec, o_dd);
                if constexpr (DZ) store_few<IO, TPW>(o_dz_row, f0, rem, vec, o_dz);
                // joint reduction of the two per-lane sums: one exchange leaves even lanes with dD and odd lanes with
                // dbias pair sums, then lanes of equal parity are summed over the half-wavefront (lanes 0,1 / 32,33)
                const bool odd = lane & 1;
                float v = odd ? db_part : dD_part;
                v += dpp<0xB1>(0.0f, odd ? dD_part : db_part);             // quad_perm [1,0,3,2]
                v += dpp<0x4E>(0.0f, v);                                    // quad_perm [2,3,0,1]
                v += dpp<0x124>(0.0f, v);                                   // row_ror:4
                v += dpp<0x128>(0.0f, v);                                   // row_ror:8
                v = sum_xor16(v);
                if ((lane & 0x1E) == 0) lds_add(&(odd ? sdb : sdD)[((lane >> 5) * W + w) * kMaxG + g], v);
            }
            rotate();
            o_du_row += p.du_sd; o_dd_row += p.dd_sd;
            if constexpr (DZ) o_dz_row += p.dz_sd;
        };
        for (int g = 0; g < Gact; ++g) channel(g);
        fl_l0 = l0; fl_rem = rem;                    // flushed while the next tile's maps are on their way
    }
    if (fl_rem > 0) flush([]() {});
    // ---- per-channel results of this workgroup
    for (int i = tid; i < Gact * N; i += NT) {
        const int g = i / N, n = i % N;
        unsafeAtomicAdd(p.dA + (int64_t)(d0 + g) * N + n, sdA[0][g * N + n] + sdA[1][g * N + n]);
        if (p.dx0 && chunk == 0) p.dx0[((int64_t)b * p.D + d0 + g) * N + n] = sH[g * N + n];
    }
    for (int g = tid; g < Gact; g += NT) {
        float sD = 0.0f, sb = 0.0f;
#pragma unroll
        for (int ww = 0; ww < 2 * W; ++ww) { sD += sdD[ww * kMaxG + g]; sb += sdb[ww * kMaxG + g]; }
        if (p.dD) unsafeAtomicAdd(p.dD + d0 + g, sD);
        if (p.dbias) unsafeAtomicAdd(p.dbias + d0 + g, sb);
    }
}

// ---------------------------------------------------------------- launchers
// channels per workgroup: D here is the number of channels that share one pair of Bm/Cm maps.  `balanced` says
// that all batch entries have the same length; otherwise (packed variable-length batches) four times as many,
// smaller, workgroups let the dispatcher even out sequences of different lengths.
int bwd_waves_per_workgroup(int N) { return N >= 8 ? N / 4 : (N == 4 ? 2 : 1); }   // as dispatched in launch_bwd_disc

int bwd_channels_per_group(int B, int D, int N, int64_t, bool balanced) {
    // aim at eight wavefronts per CU (two per SIMD, what the register budget allows): a workgroup has 8, 4, 2, 2, 1, 1
    // of them for N = 32, 16, 8, 4, 2, 1, so 256, 512, 1024, 1024, 2048, 2048 workgroups
    const int waves = bwd_waves_per_workgroup(N);
    const int64_t full = 2048 / waves;                 // workgroups the chip holds at once
    int64_t G = ((int64_t)B * D) / (balanced ? full : 2048);
    // All workgroups of a balanced launch take equally long: a few more than the chip holds would run as a second,
    // almost empty round (518 instead of 512 workgroups: 40 % slower).  So as many channel blocks per row group as
    // fit into a whole number of rounds, not one more (several rounds only when a block cannot hold more channels).
    if (balanced) {
        int64_t rounds = 1;
        while ((int64_t)B * ((D + kMaxG - 1) / kMaxG) > rounds * full && rounds < 64) ++rounds;
        const int64_t nb = rounds * full / B;          // channel blocks per row group
        if (nb >= 1) G = (D + nb - 1) / nb;
    }
    if (G < 8) G = 8;
    if (G > kMaxG) G = kMaxG;
    if (G > D) G = D;
    const int64_t groups = (D + G - 1) / G;
    G = (D + groups - 1) / groups;                     // even split
    return (int)G;
}

void bwd_packed_shape(int B, int D, int64_t L, int64_t max_seqlen, int Gbal, int places, int *G, int *wcap, int *gmin) {
    *wcap = 0; *gmin = *G;
    if (max_seqlen <= 0) return;
    // what each place of the chip gets at perfect balance, in channel-tiles: D channels x the tiles of all sequences
    // (each sequence rounded up by half a tile on average), and the channels of the longest sequence that come to that
    const double tiles = (double)L / kBwdTileSteps + 0.5 * B;
    const double cap = (double)D * tiles / places;
    const int64_t longest = (max_seqlen + kBwdTileSteps - 1) / kBwdTileSteps;
    const double fit = cap / (double)longest;
    // sequences of about one length: the launch shape of a batch [B,D,L] (whole rounds of equal workgroups, as many
    // channels each as that allows) is within a tenth of perfect balance and pays staging and flush less often
    if (Gbal > *G && (double)Gbal <= 1.1 * fit) { *G = *gmin = Gbal; return; }
    if (fit >= (double)*G || *G <= kBwdMinG) return;    // the longest sequence is no longer than a fair share: no cap
    *wcap = cap < 1.0 ? 1 : (cap > 1e9 ? 1000000000 : (int)cap);
    *gmin = fit < (double)kBwdMinG ? kBwdMinG : (int)fit;
}

// launch shape incl. the chunked path for few rows and long sequences (selective_bwd_carry.hip)
BwdPlan bwd_plan(int rowsg, int dpg, int N, int64_t L, int mode, bool balanced) {
    const int G = bwd_channels_per_group(rowsg, dpg, N, L, balanced);
    // two wavefronts per SIMD are what the chip holds of this kernel: 2048 wavefronts
    return plan_time_chunks(rowsg, dpg, L, balanced ? mode : 1, G, 2048 / bwd_waves_per_workgroup(N), kMaxG);
}

// DZ (the caller wants dz) is a template parameter: without it the kernel does not rebuild ypre = sum_n C x
template <typename IO, int N, int NK, int DISC, int T = 8>
static hipError_t launch_bwd_n(const BwdParams &p, hipStream_t s) {
    const int gmin = p.wcap > 0 ? p.gmin : p.G;                       // fewest channels a workgroup may take
    dim3 grid(p.bcg * ((p.dpg + gmin - 1) / gmin), p.B, p.nchunks > 1 ? p.nchunks : 1);
    if (p.dz) hipLaunchKernelGGL((k_ss_bwd<IO, N, NK, T, DISC, true>), grid, dim3((N / NK) * 64), 0, s, p);
    else hipLaunchKernelGGL((k_ss_bwd<IO, N, NK, T, DISC, false>), grid, dim3((N / NK) * 64), 0, s, p);
    return hipGetLastError();
}

template <typename IO, int DISC>
static hipError_t launch_bwd_disc(const BwdParams &p, hipStream_t s) {
    switch (p.N) {
        // T = 4 steps per lane: with T = 8 the compiler spills to scratch, which costs far more than the
        // longer scans (measured 2.4x slower on the Mamba-block shape)
        case 1: return launch_bwd_n<IO, 1, 1, DISC, 4>(p, s);
        case 2: return launch_bwd_n<IO, 2, 2, DISC, 4>(p, s);
        case 4: return launch_bwd_n<IO, 4, 2, DISC, 4>(p, s);
        case 8: return launch_bwd_n<IO, 8, 4, DISC, 4>(p, s);
        case 16: return launch_bwd_n<IO, 16, 4, DISC, 4>(p, s);
        case 32: return launch_bwd_n<IO, 32, 4, DISC, 4>(p, s);    // eight wavefronts: one workgroup per compute unit
    }
    return hipErrorInvalidValue;
}

template <typename IO>
static hipError_t launch_bwd_io(const BwdParams &p, int disc, hipStream_t s) {
    switch (disc) {
        case DISC_ZOH_S6: return launch_bwd_disc<IO, DISC_ZOH_S6>(p, s);
        case DISC_ZOH: return launch_bwd_disc<IO, DISC_ZOH>(p, s);
        case DISC_BILINEAR: return launch_bwd_disc<IO, DISC_BILINEAR>(p, s);
        case DISC_DIRAC: return launch_bwd_disc<IO, DISC_DIRAC>(p, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_ss_bwd(const BwdParams &p, int io_dtype, int disc, hipStream_t s) {
    return io_dtype == 1 ? launch_bwd_io<bf16_t>(p, disc, s) : launch_bwd_io<float>(p, disc, s);
}

}  // namespace lrnnx
