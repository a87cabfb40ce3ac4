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
// atomics inside the loop (LDS float atomics are very slow on this chip).  What is summed over n
// (du, dDelta, ypre for dz) is exchanged through LDS once per (channel, tile): each wavefront
// writes its partial sums, and after a barrier the threads share the epilogue of the 64*T steps
// in flat order, so u/delta/dy/z are each read once and du/ddelta/dz written once, coalesced.
// At the end of a tile the dBm/dCm sums are transposed through LDS and added to global memory
// with fully coalesced float atomics (other workgroups hold other channel groups).
#include "kernels.hpp"
#include "scan_common.hpp"

namespace lrnnx {

constexpr int kMaxG = 128;

template <typename IO, int N, int NK, int T, int DISC>
__global__ __launch_bounds__((N / NK) * 64, 2) void k_ss_bwd(const BwdParams p) {
    constexpr int W = N / NK;
    constexpr int NT = W * 64;
    constexpr int TILE = 64 * T;
    constexpr int TPW = TILE / NT > 0 ? TILE / NT : 1;   // flat steps per thread in prologue / epilogue
    constexpr int NA = TILE / TPW;                   // threads that take part in them: all, or (N = 32) the first 256
    constexpr int TQ = T / 4;
    constexpr int CK_PER_TILE = TILE / (int)kCkptInterval;
    static_assert(T % 4 == 0 && (T % W == 0 || W % T == 0) && TPW <= 8 && NA % 64 == 0 && NA <= NT, "tile shape");
    static_assert(TILE % kCkptInterval == 0, "tiles must start on checkpoints");
    static_assert(TILE == kBwdTileSteps, "the chunked launch counts its chunks in tiles of this kernel");
    static_assert(W * 3 * TILE >= 2 * 16 * T * N, "flush buffer must fit in the partials area");

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
    // a workgroup takes up to G consecutive channels of ONE Bm/Cm group
    const int chunks_per_grp = (p.dpg + p.G - 1) / p.G;
    const int grp = blockIdx.x / chunks_per_grp;
    const int din0 = (blockIdx.x % chunks_per_grp) * p.G;
    const int d0 = grp * p.dpg + din0;
    const int Gact = (p.dpg - din0 < p.G) ? p.dpg - din0 : p.G;
    const int bcrow = b * p.bcg + grp;                               // row of Bm, Cm, dBm, dCm (unpacked)
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
    // the sequence, starting from that chunk's carried adjoint.
    const int chunk = blockIdx.z;
    if (p.nchunks > 1) {
        const int64_t span = p.tiles_per_chunk * TILE;
        toff = chunk * span;
        L = (p.L - toff < span) ? p.L - toff : span;
    }
    const int64_t ntiles = (L + TILE - 1) / TILE;
    // checkpoints of this workgroup's rows: [B,D,nck,N], or packed [D,nslots,N] with sequence b at slot toff/interval + b
    const int64_t nck = p.cu ? p.nslots : (p.L + kCkptInterval - 1) / kCkptInterval;
    const int64_t ck0 = p.cu ? toff / kCkptInterval + b : toff / kCkptInterval;
    const bool vec = p.vec != 0 && (toff % 8) == 0;
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

    for (int64_t tile = ntiles - 1; tile >= 0; --tile) {
        const int64_t l0 = tile * TILE;
        const int rem = (L - l0 < TILE) ? (int)(L - l0) : TILE;      // valid steps of this tile
        // all global addresses below are a wave-uniform base plus a small unsigned per-lane offset, so that
        // they need one 32-bit register per lane instead of a 64-bit induction variable each
        const IO *BmT = Bm + l0 * N + w * NK, *CmT = Cm + l0 * N + w * NK;

        // ---- this wavefront's NK columns of Bm/Cm for the tile, and zeroed dBm/dCm sums.  Cm and both sums stay in
        // registers; the Bm columns go to this wavefront's own slice of LDS (read back as ds_read_b128 in each pass)
        float Cv[NK][T], dBacc[NK][T], dCacc[NK][T];
        {
        float Bv[NK][T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            float tb[NK], tc[NK];
            if (lane * T + t < rem) {
                load_row<IO, NK>(BmT + (unsigned)((lane * T + t) * N), tb);
                load_row<IO, NK>(CmT + (unsigned)((lane * T + t) * N), tc);
            } else {
#pragma unroll
                for (int k = 0; k < NK; ++k) { tb[k] = 0.0f; tc[k] = 0.0f; }
            }
#pragma unroll
            for (int k = 0; k < NK; ++k) { Bv[k][t] = tb[k]; Cv[k][t] = tc[k]; dBacc[k][t] = 0.0f; dCacc[k][t] = 0.0f; }
        }
#pragma unroll
        for (int k = 0; k < NK; ++k)
#pragma unroll
            for (int q = 0; q < TQ; ++q)
                *reinterpret_cast<float4 *>(&sBt[(((w * NK + k) * TQ + q) * 64 + lane) * 4]) =
                    make_float4(Bv[k][4 * q], Bv[k][4 * q + 1], Bv[k][4 * q + 2], Bv[k][4 * q + 3]);
        }

        // per-channel inputs are fetched one channel ahead, so their latency hides behind the main pass
        RawFew<IO, TPW> r_u, r_dl, r_dy, r_z;
        float pA[NK], pck[NK], pDsk, pbias;
        auto prefetch = [&](int g) {
            const int d = d0 + g;
            const int64_t row = (int64_t)b * p.D + d;
            if (io_thread) {
                load_few_raw<IO, TPW>(reinterpret_cast<const IO *>(p.u) + bs * p.u_sb + d * p.u_sd + toff + l0, f0, rem, vec, r_u);
                load_few_raw<IO, TPW>(reinterpret_cast<const IO *>(p.delta) + bs * p.dl_sb + d * p.dl_sd + toff + l0, f0, rem, vec, r_dl);
                load_few_raw<IO, TPW>(reinterpret_cast<const IO *>(p.dy) + bs * p.dy_sb + d * p.dy_sd + toff + l0, f0, rem, vec, r_dy);
                if (has_z) load_few_raw<IO, TPW>(reinterpret_cast<const IO *>(p.z) + bs * p.z_sb + d * p.z_sd + toff + l0, f0, rem, vec, r_z);
            }
#pragma unroll
            for (int k = 0; k < NK; ++k) {
                pA[k] = p.A[d * N + w * NK + k];
                pck[k] = p.ckpt[((p.cu ? (int64_t)d : row) * nck + ck0 + tile * CK_PER_TILE) * N + w * NK + k];
            }
            pDsk = p.Dskip ? p.Dskip[d] : 0.0f;
            pbias = p.bias ? p.bias[d] : 0.0f;
        };
        prefetch(0);

        for (int g = 0; g < Gact; ++g) {
            if constexpr (ALT_PRIO) {
                if ((unsigned)(g & 1) == hw_slot) __builtin_amdgcn_s_setprio(1); else __builtin_amdgcn_s_setprio(0);
            }
            const int d = d0 + g;
            const float Dsk = pDsk, bias = pbias;
            float cA[NK], cck[NK];
#pragma unroll
            for (int k = 0; k < NK; ++k) { cA[k] = pA[k]; cck[k] = pck[k]; }

            // ---- prologue: each thread prepares TPW flat steps for everybody
            // kept for the epilogue: d softplus / ds, and the factor that turns ypre into dz
            float e_sg[TPW], e_zf[TPW];
            if (io_thread) {
                float e_u[TPW], r_d[TPW], e_dy[TPW], e_z[TPW];
                unpack_few<IO, TPW>(r_u, e_u);
                unpack_few<IO, TPW>(r_dl, r_d);
                unpack_few<IO, TPW>(r_dy, e_dy);
                if (has_z) unpack_few<IO, TPW>(r_z, e_z);
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
                    float sp, dyp;
                    bwd_step_inputs(r_d[i] + bias, e_dy[i], has_z ? e_z[i] : 0.0f, p.softplus != 0, has_z, sp, e_sg[i], dyp, e_zf[i]);
                    sIn[0 * TILE + fslot(f0 + i)] = (f0 + i < rem) ? sp : 0.0f;
                    sIn[1 * TILE + fslot(f0 + i)] = e_u[i];
                    sIn[2 * TILE + fslot(f0 + i)] = dyp;
                }
            }
            __syncthreads();
            if (g + 1 < Gact) prefetch(g + 1);

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
            float sum_dl = 0.0f;
#pragma unroll
            for (int t = 0; t < T; ++t) {
                sum_dl += dl[t];
                if constexpr (DISC == DISC_ZOH_S6) dlu[t] *= dl[t];   // S6 only ever needs Delta*u; the others keep u
                ypre[t] = 0.0f; pdu[t] = 0.0f; pdd[t] = 0.0f;
            }
            const float dl_next0 = dpp<DPP_WAVE_SHL1>(0.0f, dl[0]);        // first Delta of the next lane (0 past lane 63)
            const float sum_shift = sum_dl - dl[0] + dl_next0;

            float dA4[NK];
#pragma unroll
            for (int k = 0; k < NK; ++k) {
                const int n = w * NK + k;
                const ACoef ac = make_acoef<DISC>(cA[k]);
                const float xck = cck[k];
                const float hc = sH[g * N + n];
                float Bk[T];
#pragma unroll
                for (int q = 0; q < TQ; ++q) {
                    const float4 vb = *reinterpret_cast<const float4 *>(&sBt[((n * TQ + q) * 64 + lane) * 4]);
                    Bk[4 * q] = vb.x; Bk[4 * q + 1] = vb.y; Bk[4 * q + 2] = vb.z; Bk[4 * q + 3] = vb.w;
                }

                // forward recompute of the states of this tile
                float a[T + 1], gg[T], x[T];
                float P = 1.0f, S = 0.0f;
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    disc_ag<DISC>(dl[t], ac, a[t], gg[t]);
                    if constexpr (DISC == DISC_ZOH_S6) x[t] = dlu[t] * Bk[t];
                    else if constexpr (DISC == DISC_DIRAC) x[t] = dlu[t] * Bk[t];
                    else x[t] = gg[t] * dlu[t] * Bk[t];
                    S = (t == 0) ? x[0] : __builtin_fmaf(a[t], S, x[t]);     // the fold starts from zero
                    if constexpr (DISC == DISC_BILINEAR) P *= a[t];
                }
                if constexpr (DISC != DISC_BILINEAR) P = exp2_fast(sum_dl * ac.A2);
                if (lane == 0) S = __builtin_fmaf(P, xck, S);               // the checkpointed state enters through lane 0

                // lane aggregate of the adjoint H_l = c_l + a_{l+1} H_{l+1}; the multiplier of the tile's last step is 1
                // because the carried value is already a_{l1} H_{l1}
                a[T] = dpp<DPP_WAVE_SHL1>(1.0f, a[0]);
                float Pr = 1.0f, Sr = 0.0f;
#pragma unroll
                for (int t = T - 1; t >= 0; --t) {
                    Sr = (t == T - 1) ? Cv[k][t] * dyp[t] : __builtin_fmaf(a[t + 1], Sr, Cv[k][t] * dyp[t]);
                    if constexpr (DISC == DISC_BILINEAR) Pr *= a[t + 1];
                }
                if constexpr (DISC != DISC_BILINEAR) Pr = exp2_fast(sum_shift * ac.A2);
                if (lane == 63) Sr = __builtin_fmaf(Pr, hc, Sr);            // the carried adjoint enters through lane 63

                // state prefix (forward in time) and adjoint suffix (backward in time) are independent: scanned together
                wave_scan_fwd_rev(P, S, Pr, Sr, lane);
                const float xin = dpp<DPP_WAVE_SHR1>(xck, S);               // x entering this lane's first step
                {
                    float xp = xin;
#pragma unroll
                    for (int t = 0; t < T; ++t) { xp = __builtin_fmaf(a[t], xp, x[t]); x[t] = xp; }
                }
                const float H0 = Sr;                                        // H of this lane's first step
                float R = dpp<DPP_WAVE_SHL1>(hc, Sr);                       // H of the next lane's first step (the carry itself past lane 63)
                if (lane == 0) sH[g * N + n] = a[0] * H0;                   // carried to the earlier tile

                float dA_part = 0.0f;                                       // this lane's share of dA[d, n]
#pragma unroll
                for (int t = T - 1; t >= 0; --t) {
                    R = __builtin_fmaf(a[t + 1], R, Cv[k][t] * dyp[t]);       // H_t (the product is recomputed: registers are scarcer than VALU slots here)
                    const float xprev = (t > 0) ? x[t - 1] : xin;
                    dCacc[k][t] = __builtin_fmaf(dyp[t], x[t], dCacc[k][t]);
                    ypre[t] = __builtin_fmaf(Cv[k][t], x[t], ypre[t]);
                    if constexpr (DISC == DISC_ZOH_S6) {
                        pdu[t] = __builtin_fmaf(R, Bk[t], pdu[t]);       // sum_n H B; scaled by Delta resp. u in the epilogue
                        dBacc[k][t] = __builtin_fmaf(R, dlu[t], dBacc[k][t]);
                        const float q = R * xprev * a[t];
                        pdd[t] = __builtin_fmaf(q, ac.A, pdd[t]);
                        dA_part = __builtin_fmaf(q, dl[t], dA_part);
                    } else if constexpr (DISC == DISC_DIRAC) {
                        // g = 1: only a = e^{Delta A} depends on Delta and A
                        pdu[t] = __builtin_fmaf(R, Bk[t], pdu[t]);
                        dBacc[k][t] = __builtin_fmaf(R, dlu[t], dBacc[k][t]);
                        const float q = R * xprev * a[t];
                        pdd[t] = __builtin_fmaf(q, ac.A, pdd[t]);
                        dA_part = __builtin_fmaf(q, dl[t], dA_part);
                    } else if constexpr (DISC == DISC_ZOH) {
                        // da/dDelta = A a, da/dA = Delta a, dg/dDelta = a: the common factor a is taken out
                        float a_t, a_A, g_t, g_A;
                        disc_partials<DISC>(dl[t], ac, a[t], gg[t], a_t, a_A, g_t, g_A);
                        const float hb = R * Bk[t];
                        const float dg = hb * dlu[t];
                        const float dax = R * a[t] * xprev;                  // H x_{l-1} a
                        pdu[t] = __builtin_fmaf(hb, gg[t], pdu[t]);
                        dBacc[k][t] = __builtin_fmaf(R * gg[t], dlu[t], dBacc[k][t]);
                        pdd[t] = __builtin_fmaf(dax, ac.A, __builtin_fmaf(dg, a[t], pdd[t]));
                        dA_part = __builtin_fmaf(dax, dl[t], __builtin_fmaf(dg, g_A, dA_part));
                    } else {
                        // bilinear: with q = 1 / (1 - Delta A / 2) all four partials are multiples of q^2
                        const float q = rcp_fast(__builtin_fmaf(-dl[t], ac.hA, 1.0f));
                        const float q2 = q * q;
                        const float da = R * xprev;
                        const float hb = R * Bk[t];
                        const float dg = hb * dlu[t];
                        pdu[t] = __builtin_fmaf(hb, gg[t], pdu[t]);
                        dBacc[k][t] = __builtin_fmaf(R * gg[t], dlu[t], dBacc[k][t]);
                        pdd[t] = __builtin_fmaf(__builtin_fmaf(da, ac.A, dg), q2, pdd[t]);                       // A q^2 da + q^2 dg
                        dA_part = __builtin_fmaf(__builtin_fmaf(0.5f * dl[t], dg, da) * dl[t], q2, dA_part);     // Delta q^2 da + Delta^2 q^2 dg / 2
                    }
                }
                if constexpr (NK == 4 || NK == 2) {
                    dA4[k] = dA_part;
                } else {
                    const float dA_tot = wave_sum(dA_part);
                    if (lane == 0) sdA[0][g * N + n] += dA_tot;
                }
            }
            if constexpr (NK == 4) {
                // The four per-lane partial sums are reduced together: two exchange steps leave each lane of a quad
                // with the quad's sum of ONE state (lane%4 = 0,1,2,3 -> state 0,2,1,3), two rotations sum the quads of
                // a row, one swizzle sums the two rows of a half-wavefront; lanes 0-3 and 32-35 own the results.
                const bool b0 = lane & 1, b1 = lane & 2;
                float kA = b0 ? dA4[2] : dA4[0], kB = b0 ? dA4[3] : dA4[1];
                const float sA = b0 ? dA4[0] : dA4[2], sB = b0 ? dA4[1] : dA4[3];
                kA += dpp<0xB1>(0.0f, sA);                                  // quad_perm [1,0,3,2]
                kB += dpp<0xB1>(0.0f, sB);
                float v = b1 ? kB : kA;
                v += dpp<0x4E>(0.0f, b1 ? kA : kB);                         // quad_perm [2,3,0,1]
                v += dpp<0x124>(0.0f, v);                                   // row_ror:4
                v += dpp<0x128>(0.0f, v);                                   // row_ror:8
                v += i2f(__builtin_amdgcn_ds_swizzle(f2i(v), 0x401F));      // lane ^ 16
                if ((lane & 0x1C) == 0) sdA[lane >> 5][g * N + w * NK + ((lane & 1) << 1) + ((lane >> 1) & 1)] += v;
            } else if constexpr (NK == 2) {
                // the same with two partial sums: even lanes end up with state 0, odd lanes with state 1
                const bool odd = lane & 1;
                float v = odd ? dA4[1] : dA4[0];
                v += dpp<0xB1>(0.0f, odd ? dA4[0] : dA4[1]);               // quad_perm [1,0,3,2]
                v += dpp<0x4E>(0.0f, v);                                    // quad_perm [2,3,0,1]
                v += dpp<0x124>(0.0f, v);                                   // row_ror:4
                v += dpp<0x128>(0.0f, v);                                   // row_ror:8
                v += i2f(__builtin_amdgcn_ds_swizzle(f2i(v), 0x401F));      // lane ^ 16
                if ((lane & 0x1E) == 0) sdA[lane >> 5][g * N + w * NK + (lane & 1)] += v;
            }
#pragma unroll
            for (int q = 0; q < TQ; ++q) {
                float *base = &sPart[(w * 3) * TILE + (q * 64 + lane) * 4];
                *reinterpret_cast<float4 *>(base) = make_float4(ypre[4 * q], ypre[4 * q + 1], ypre[4 * q + 2], ypre[4 * q + 3]);
                *reinterpret_cast<float4 *>(base + TILE) = make_float4(pdu[4 * q], pdu[4 * q + 1], pdu[4 * q + 2], pdu[4 * q + 3]);
                *reinterpret_cast<float4 *>(base + 2 * TILE) = make_float4(pdd[4 * q], pdd[4 * q + 1], pdd[4 * q + 2], pdd[4 * q + 3]);
            }
            __syncthreads();

            // ---- epilogue: the threads share the tile in flat order
            if (io_thread) {
                float o_du[TPW], o_dd[TPW], o_dz[TPW];
                float dD_part = 0.0f, db_part = 0.0f;
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
                    const float e_u = sIn[1 * TILE + fslot(f0 + i)], e_dyp = sIn[2 * TILE + fslot(f0 + i)];
                    float yp = Dsk * e_u, s_du = 0.0f, s_dd = 0.0f;
#pragma unroll
                    for (int ww = 0; ww < W; ++ww) {
                        yp += sPart[(ww * 3 + 0) * TILE + fslot(f0 + i)];
                        s_du += sPart[(ww * 3 + 1) * TILE + fslot(f0 + i)];
                        s_dd += sPart[(ww * 3 + 2) * TILE + fslot(f0 + i)];
                    }
                    if constexpr (DISC == DISC_ZOH_S6) {
                        // the wavefronts' sums are sum_n H B: dDelta += u sum_n H B, du = Delta sum_n H B
                        s_dd = __builtin_fmaf(e_u, s_du, s_dd);
                        s_du *= sIn[0 * TILE + fslot(f0 + i)];
                    }
                    o_du[i] = __builtin_fmaf(e_dyp, Dsk, s_du);
                    o_dd[i] = s_dd * e_sg[i];
                    o_dz[i] = yp * e_zf[i];
                    dD_part = __builtin_fmaf(e_dyp, e_u, dD_part);
                    db_part += (f0 + i < rem) ? o_dd[i] : 0.0f;
                }
                store_few<IO, TPW>(reinterpret_cast<IO *>(p.du) + bs * p.du_sb + d * p.du_sd + toff + l0, f0, rem, vec, o_du);
                store_few<IO, TPW>(reinterpret_cast<IO *>(p.ddelta) + bs * p.dd_sb + d * p.dd_sd + toff + l0, f0, rem, vec, o_dd);
                if (p.dz) store_few<IO, TPW>(reinterpret_cast<IO *>(p.dz) + bs * p.dz_sb + d * p.dz_sd + toff + l0, f0, rem, vec, o_dz);
                // joint reduction of the two per-lane sums: one exchange leaves even lanes with dD and odd lanes with
                // dbias pair sums, then lanes of equal parity are summed over the half-wavefront (lanes 0,1 / 32,33)
                const bool odd = lane & 1;
                float v = odd ? db_part : dD_part;
                v += dpp<0xB1>(0.0f, odd ? dD_part : db_part);             // quad_perm [1,0,3,2]
                v += dpp<0x4E>(0.0f, v);                                    // quad_perm [2,3,0,1]
                v += dpp<0x124>(0.0f, v);                                   // row_ror:4
                v += dpp<0x128>(0.0f, v);                                   // row_ror:8
                v += i2f(__builtin_amdgcn_ds_swizzle(f2i(v), 0x401F));      // lane ^ 16
                if ((lane & 0x1E) == 0) (odd ? sdb : sdD)[((lane >> 5) * W + w) * kMaxG + g] += v;
            }
        }

        // ---- add this tile's dBm/dCm sums (over the G channels) to global memory, transposed through LDS
        // so that consecutive threads hit consecutive addresses
        float *fbB = sPart, *fbC = sPart + 16 * T * N;
        for (int j = 0; j < 4; ++j) {
            __syncthreads();
            if ((lane >> 4) == j) {
#pragma unroll
                for (int t = 0; t < T; ++t)
#pragma unroll
                    for (int k = 0; k < NK; ++k) {
                        fbB[((lane & 15) * T + t) * N + w * NK + k] = dBacc[k][t];
                        fbC[((lane & 15) * T + t) * N + w * NK + k] = dCacc[k][t];
                    }
            }
            __syncthreads();
            const int step0 = j * 16 * T;                                // within the tile
            float *gB = p.dBm + bc0 + (l0 + step0) * N, *gC = p.dCm + bc0 + (l0 + step0) * N;
            for (int idx = tid; idx < 16 * T * N; idx += NT) {
                if (step0 + idx / N < rem) {
                    unsafeAtomicAdd(gB + (unsigned)idx, fbB[idx]);
                    unsafeAtomicAdd(gC + (unsigned)idx, fbC[idx]);
                }
            }
        }
        __syncthreads();
    }

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

// launch shape incl. the chunked path for few rows and long sequences (selective_bwd_carry.hip)
BwdPlan bwd_plan(int rowsg, int dpg, int N, int64_t L, int mode, bool balanced) {
    const int G = bwd_channels_per_group(rowsg, dpg, N, L, balanced);
    // two wavefronts per SIMD are what the chip holds of this kernel: 2048 wavefronts
    return plan_time_chunks(rowsg, dpg, L, balanced ? mode : 1, G, 2048 / bwd_waves_per_workgroup(N), kMaxG);
}

template <typename IO, int N, int NK, int DISC, int T = 8>
static hipError_t launch_bwd_n(const BwdParams &p, hipStream_t s) {
    dim3 grid(p.bcg * ((p.dpg + p.G - 1) / p.G), p.B, p.nchunks > 1 ? p.nchunks : 1);
    hipLaunchKernelGGL((k_ss_bwd<IO, N, NK, T, DISC>), grid, dim3((N / NK) * 64), 0, s, p);
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
