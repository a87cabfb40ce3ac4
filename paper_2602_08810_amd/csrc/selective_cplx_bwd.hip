// Backward selective scan with a COMPLEX diagonal state matrix for gfx950: reverse-mode derivative of
//     x_{l,n} = a(Delta_l, A[d,n]) x_{l-1,n} + g(Delta_l, A[d,n]) Bm[b,l,n] u[b,d,l]        (complex)
//     y[b,d,l] = Re( sum_n Cm[b,l,n] x_{l,n} ) + Dskip[d] u[b,d,l],  then the optional gate
// (Eq. 2 of the paper with a complex diagonal A as in the layers of Sec. 2.2.1, states recomputed from checkpoints
// as Sec. 3 prescribes for the real scan).
//
// The gradient of the real loss with respect to a complex quantity q is dLoss/dRe q + i dLoss/dIm q.  With it, for
// one (b,d) row and one state n, H_l = grad x_l:
//     H_l       = dypre_l conj(Cm_l) + conj(a_{l+1}) H_{l+1}        (the same affine scan, time reversed)
//     dCm_l    += dypre_l conj(x_l)            dBm_l += H_l conj(g_l) u_l
//     du_l     += Re(H_l conj(g_l Bm_l))       grad a_l = H_l conj(x_{l-1})     grad g_l = H_l conj(Bm_l) u_l
//     dDelta_l += Re(grad a_l conj(da/dDelta) + grad g_l conj(dg/dDelta))
//     dA_n     += grad a_l conj(da/dA) + grad g_l conj(dg/dA)
//
// Mapping: that of the real backward kernel.  Time runs along the lanes (a lane owns T consecutive steps of a tile),
// the N states are split over the W = N/NK wavefronts of a workgroup, which work on the same channel at the same
// time and loop over G channels, so the sums of dBm/dCm over channels stay in registers.  Both complex maps of the
// tile live in LDS as fp32 pairs (converted once per tile), in slices private to the wavefront that owns
// the states.  What is summed over n (du, dDelta, ypre) goes through LDS once per (channel, tile).
#include "kernels.hpp"
#include "scan_common.hpp"
#include "cplx_common.hpp"

namespace lrnnx {

constexpr int kMaxGc = 64;

namespace {

// Sum over the 32 lanes of each half-wavefront of four per-lane values at once: two exchange steps leave each lane
// of a quad with the quad's sum of ONE value (lane%4 = 0,1,2,3 -> value 0,2,1,3), two rotations sum the quads of a
// row, one row-pair swap sums the two rows.  Lanes 0-3 and 32-35 own the results.
__device__ __forceinline__ float half_sum4(const float *v4, int lane) {
    const bool b0 = lane & 1, b1 = lane & 2;
    float kA = b0 ? v4[2] : v4[0], kB = b0 ? v4[3] : v4[1];
    const float sA = b0 ? v4[0] : v4[2], sB = b0 ? v4[1] : v4[3];
    kA += dpp<0xB1>(0.0f, sA);                                  // quad_perm [1,0,3,2]
    kB += dpp<0xB1>(0.0f, sB);
    float v = b1 ? kB : kA;
    v += dpp<0x4E>(0.0f, b1 ? kA : kB);                         // quad_perm [2,3,0,1]
    v += dpp<0x124>(0.0f, v);                                   // row_ror:4
    v += dpp<0x128>(0.0f, v);                                   // row_ror:8
    return sum_xor16(v);
}
__device__ __forceinline__ float half_sum(float v) {
    v += dpp<0xB1>(0.0f, v);
    v += dpp<0x4E>(0.0f, v);
    v += dpp<0x124>(0.0f, v);
    v += dpp<0x128>(0.0f, v);
    return sum_xor16(v);
}

}  // namespace

template <typename IO, int N, int NK, int T, int DISC>
__global__ __launch_bounds__((N / NK) * 64, 2) void k_ss_cbwd(const CBwdParams p) {
    using CW = typename cword<IO>::type;
    constexpr int W = N / NK;
    constexpr int NT = W * 64;
    constexpr int TILE = 64 * T;
    constexpr int TPW = TILE / NT > 0 ? TILE / NT : 1;   // flat steps per thread in prologue / epilogue
    constexpr int NA = TILE / TPW;                   // threads that take part in them (all, or the first wavefronts)
    constexpr int TQ = T / 4;
    constexpr int CK_PER_TILE = TILE / (int)kCkptInterval;
    constexpr int FL = 16;                           // lanes whose dBm/dCm sums are flushed together
    static_assert(T % 4 == 0 && (T % W == 0 || W % T == 0) && TPW <= 8 && NA % 64 == 0 && NA <= NT, "tile shape");
    static_assert(TILE % kCkptInterval == 0, "tiles must start on checkpoints");
    static_assert(TILE == kBwdTileSteps, "the chunked launch counts its chunks in tiles of this kernel");
    static_assert(W * 3 * TILE >= 2 * FL * T * N * 2, "flush buffer must fit in the partials area");

    __shared__ __attribute__((aligned(16))) float sIn[2][5 * TILE];       // two channels in flight: delta, u, dypre, d softplus, dz factor; [q][lane][4]
    __shared__ __attribute__((aligned(16))) float sPart[W * 3 * TILE];    // per wave: ypre, du, ddelta partials
    // maps of the tile as fp32 pairs: [n][t/2][lane][t%2], wave-private slices (converted once per tile; every channel
    // of the workgroup then reads them five times)
    __shared__ __attribute__((aligned(16))) float2 sB[N * TILE];
    __shared__ __attribute__((aligned(16))) float2 sC[N * TILE];
    __shared__ float2 sH[kMaxGc * N];     // conj(a_{l0}) H_{l0} carried to the earlier tile, per (channel, n)
    __shared__ float sdA[2][kMaxGc * N * 2];   // per half-wavefront partial sums of dA, (re, im) pairs
    __shared__ float sdD[2 * W * kMaxGc]; // dD and dbias partial sums per (half-wavefront, wavefront, channel)
    __shared__ float sdb[2 * W * kMaxGc];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = p.order ? p.order[blockIdx.y] : blockIdx.y;   // packed batches: the longest sequences start first
    // Packed variable-length mode (p.cu != nullptr): batch entry b is the sequence of steps cu[b] .. cu[b+1]-1 of ONE
    // packed time axis of p.L steps; I/O rows have no batch stride, the maps and their gradients are [G, p.L, N].
    // The bounds are clamped to the packed axis, so no content of cu can send an access out of the buffers.
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
    // checkpoints of this workgroup's rows: [B,D,nck,N], or packed [D,nslots,N] with sequence b at slot toff/interval + b
    const int64_t nck = p.cu ? p.nslots : (p.L + kCkptInterval - 1) / kCkptInterval;
    const int64_t ck0 = p.cu ? toff / kCkptInterval + b : toff / kCkptInterval;
    const bool vec = p.vec != 0;
    const bool has_z = p.z != nullptr;

    for (int i = tid; i < kMaxGc * N; i += NT) {
        float2 h = make_float2(0.0f, 0.0f);
        if (p.nchunks > 1 && i < Gact * N)
            h = p.hc[(((int64_t)b * p.D + d0 + i / N) * p.nchunks + chunk) * N + i % N];
        sH[i] = h;
        sdA[0][2 * i] = 0.0f; sdA[0][2 * i + 1] = 0.0f; sdA[1][2 * i] = 0.0f; sdA[1][2 * i + 1] = 0.0f;
    }
    for (int i = tid; i < 2 * W * kMaxGc; i += NT) { sdD[i] = 0.0f; sdb[i] = 0.0f; }

    const int64_t bc0 = ((bs * p.bcg + grp) * p.L + toff) * N;       // first complex element of the maps of this sequence and group
    const CW *Bm = reinterpret_cast<const CW *>(p.Bm) + bc0;
    const CW *Cm = reinterpret_cast<const CW *>(p.Cm) + bc0;

    // The flat prologue (inputs of a channel -> LDS) and epilogue (partials -> outputs) need NA threads each.  A
    // workgroup of 2 NA threads gives the prologue to its first half and the epilogue to its second half, which then
    // run side by side (epilogue of channel g, prologue of channel g + 1); otherwise the same threads do both.
    constexpr bool SPLIT = NT == 2 * NA;
    const bool pro_thread = NA == NT || tid < NA;                     // wave-uniform: NA is a multiple of 64
    const bool epi_thread = SPLIT ? tid >= NA : pro_thread;
    const int f0 = tid * TPW;                                         // first flat step of a prologue thread
    const int f0e = (SPLIT ? tid - NA : tid) * TPW;                   // ... of an epilogue thread
    auto fslot = [](int f) { return (((f % T) / 4) * 64 + f / T) * 4 + (f % 4); };

    for (int64_t tile = ntiles - 1; tile >= 0; --tile) {
        const int64_t l0 = tile * TILE;
        const int rem = (L - l0 < TILE) ? (int)(L - l0) : TILE;      // valid steps of this tile

        // ---- this wavefront's NK columns of both maps into its own slices of LDS; zeroed dBm/dCm sums
        float2 dBacc[NK][T], dCacc[NK][T];
        {
            const CW *BmT = Bm + l0 * N + w * NK, *CmT = Cm + l0 * N + w * NK;
            CW tb[T][NK], tc[T][NK];
#pragma unroll
            for (int t = 0; t < T; ++t) {
                if (lane * T + t < rem) {
                    load_cwords<CW, NK>(BmT + (unsigned)((lane * T + t) * N), tb[t]);
                    load_cwords<CW, NK>(CmT + (unsigned)((lane * T + t) * N), tc[t]);
                } else {
#pragma unroll
                    for (int k = 0; k < NK; ++k) { tb[t][k] = CW{}; tc[t][k] = CW{}; }
                }
#pragma unroll
                for (int k = 0; k < NK; ++k) { dBacc[k][t] = make_float2(0.0f, 0.0f); dCacc[k][t] = make_float2(0.0f, 0.0f); }
            }
#pragma unroll
            for (int k = 0; k < NK; ++k)
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    sB[(((w * NK + k) * (T / 2) + t / 2) * 64 + lane) * 2 + (t % 2)] = cword<IO>::unpack(tb[t][k]);
                    sC[(((w * NK + k) * (T / 2) + t / 2) * 64 + lane) * 2 + (t % 2)] = cword<IO>::unpack(tc[t][k]);
                }
        }

        // per-channel inputs are fetched one channel ahead
        RawFew<IO, TPW> r_u, r_dl, r_dy, r_z;
        float2 pA[NK], pck[NK];
        float pDsk, pbias;
        auto prefetch = [&](int g) {
            const int d = d0 + g;
            const int64_t row = (int64_t)b * p.D + d;
            if (pro_thread) {
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

        // ---- prologue of channel g: each prologue thread prepares TPW flat steps for everybody
        auto prologue = [&](int g) {
            float *in = sIn[g & 1];
            const float bias = pbias;
            float e_u[TPW], r_d[TPW], e_dy[TPW], e_z[TPW];
            unpack_few<IO, TPW>(r_u, e_u);
            unpack_few<IO, TPW>(r_dl, r_d);
            unpack_few<IO, TPW>(r_dy, e_dy);
            if (has_z) unpack_few<IO, TPW>(r_z, e_z);
#pragma unroll
            for (int i = 0; i < TPW; ++i) {
                float sp, sg, dyp, zf;
                bwd_step_inputs<sizeof(IO) == 4>(r_d[i] + bias, e_dy[i], has_z ? e_z[i] : 0.0f, p.softplus != 0, has_z, sp, sg, dyp, zf);
                in[0 * TILE + fslot(f0 + i)] = (f0 + i < rem) ? sp : 0.0f;
                in[1 * TILE + fslot(f0 + i)] = e_u[i];
                in[2 * TILE + fslot(f0 + i)] = dyp;
                in[3 * TILE + fslot(f0 + i)] = sg;
                in[4 * TILE + fslot(f0 + i)] = zf;
            }
        };
        if (pro_thread) prologue(0);

        for (int g = 0; g < Gact; ++g) {
            const int d = d0 + g;
            const float Dsk = pDsk;
            const float *in = sIn[g & 1];
            float2 cA[NK], cck[NK];
#pragma unroll
            for (int k = 0; k < NK; ++k) { cA[k] = pA[k]; cck[k] = pck[k]; }

            __syncthreads();
            if (g + 1 < Gact) prefetch(g + 1);

            // ---- main: this lane's T steps, this wavefront's NK states
            float dl[T], dyp[T], uv[T], ypre[T], pdu[T], pdd[T];
#pragma unroll
            for (int q = 0; q < TQ; ++q) {
                const float4 v0 = *reinterpret_cast<const float4 *>(&in[0 * TILE + (q * 64 + lane) * 4]);
                const float4 v1 = *reinterpret_cast<const float4 *>(&in[1 * TILE + (q * 64 + lane) * 4]);
                const float4 v2 = *reinterpret_cast<const float4 *>(&in[2 * TILE + (q * 64 + lane) * 4]);
                dl[4 * q] = v0.x; dl[4 * q + 1] = v0.y; dl[4 * q + 2] = v0.z; dl[4 * q + 3] = v0.w;
                uv[4 * q] = v1.x; uv[4 * q + 1] = v1.y; uv[4 * q + 2] = v1.z; uv[4 * q + 3] = v1.w;
                dyp[4 * q] = v2.x; dyp[4 * q + 1] = v2.y; dyp[4 * q + 2] = v2.z; dyp[4 * q + 3] = v2.w;
            }
            float sum_dl = 0.0f;
#pragma unroll
            for (int t = 0; t < T; ++t) { sum_dl += dl[t]; ypre[t] = 0.0f; pdu[t] = 0.0f; pdd[t] = 0.0f; }
            const float dl_next0 = dpp<DPP_WAVE_SHL1>(0.0f, dl[0]);        // first Delta of the next lane (0 past lane 63)
            const float sum_shift = sum_dl - dl[0] + dl_next0;

            float dAr4[NK], dAi4[NK];
#pragma unroll
            for (int k = 0; k < NK; ++k) {
                const int n = w * NK + k;
                const CCoef cc = make_ccoef(cA[k].x, cA[k].y);
                const float2 xck = cck[k];
                const float2 hc = sH[g * N + n];
                // [n][t/2][lane][t%2]: two steps of a lane are one 16-byte chunk and neighbouring lanes neighbouring
                // chunks, so a ds_read_b128 touches every bank once (with the lane's four steps side by side, 32 bytes
                // per lane, each such read hit half the banks twice: a quarter of this kernel's LDS cycles)
                const float2 *sBn = &sB[(n * (T / 2) * 64 + lane) * 2], *sCn = &sC[(n * (T / 2) * 64 + lane) * 2];
                auto mapB = [&](int t) { return sBn[(t / 2) * 128 + (t % 2)]; };
                auto mapC = [&](int t) { return sCn[(t / 2) * 128 + (t % 2)]; };

                // forward recompute of the states of this tile
                float2 a[T + 1], gg[T], x[T];
                float2 P = make_float2(1.0f, 0.0f), S = make_float2(0.0f, 0.0f);
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    cdisc_ag<DISC>(dl[t], cc, a[t], gg[t]);
                    const float2 Bv = mapB(t);
                    if constexpr (DISC == DISC_ZOH_S6 || DISC == DISC_DIRAC) {
                        const float gu = gg[t].x * uv[t];                  // the gain is real
                        x[t] = make_float2(gu * Bv.x, gu * Bv.y);
                    } else {
                        x[t] = cxmul(make_float2(gg[t].x * uv[t], gg[t].y * uv[t]), Bv);
                    }
                    S = (t == 0) ? x[0] : cxfma(a[t], S, x[t]);           // the fold starts from zero
                    if constexpr (DISC == DISC_BILINEAR) P = cxmul(P, a[t]);
                }
                if constexpr (DISC != DISC_BILINEAR) P = cexp_dt(sum_dl, cc.A2r, cc.Arev);
                if (lane == 0) S = cxfma(P, xck, S);                       // the checkpointed state enters through lane 0

                // lane aggregate of the adjoint H_l = c_l + conj(a_{l+1}) H_{l+1}; the multiplier of the tile's last
                // step is 1 because the carried value is already conj(a_{l1}) H_{l1}
                a[T] = make_float2(dpp<DPP_WAVE_SHL1>(1.0f, a[0].x), dpp<DPP_WAVE_SHL1>(0.0f, a[0].y));
                float2 Pr = make_float2(1.0f, 0.0f), Sr = make_float2(0.0f, 0.0f);
#pragma unroll
                for (int t = T - 1; t >= 0; --t) {
                    const float2 Cv = mapC(t);
                    const float2 c = make_float2(Cv.x * dyp[t], -Cv.y * dyp[t]);
                    Sr = (t == T - 1) ? c : cxcfma(a[t + 1], Sr, c);
                    if constexpr (DISC == DISC_BILINEAR) Pr = cxmulc(Pr, a[t + 1]);
                }
                if constexpr (DISC != DISC_BILINEAR) {
                    const float2 e = cexp_dt(sum_shift, cc.A2r, cc.Arev);
                    Pr = make_float2(e.x, -e.y);
                }
                if (lane == 63) Sr = cxfma(Pr, hc, Sr);                    // the carried adjoint enters through lane 63

                cwave_scan_fwd_rev(P, S, Pr, Sr, lane);
                const float2 xin = make_float2(dpp<DPP_WAVE_SHR1>(xck.x, S.x), dpp<DPP_WAVE_SHR1>(xck.y, S.y));
                {
                    float2 xp = xin;
#pragma unroll
                    for (int t = 0; t < T; ++t) { xp = cxfma(a[t], xp, x[t]); x[t] = xp; }
                }
                const float2 H0 = Sr;                                       // H of this lane's first step
                float2 R = make_float2(dpp<DPP_WAVE_SHL1>(hc.x, Sr.x), dpp<DPP_WAVE_SHL1>(hc.y, Sr.y));   // H of the next lane's first step
                if (lane == 0) sH[g * N + n] = cxcfma(a[0], H0, make_float2(0.0f, 0.0f));   // carried to the earlier tile

                float2 dA_part = make_float2(0.0f, 0.0f);
#pragma unroll
                for (int t = T - 1; t >= 0; --t) {
                    const float2 Cv = mapC(t), Bv = mapB(t);
                    R = cxcfma(a[t + 1], R, make_float2(Cv.x * dyp[t], -Cv.y * dyp[t]));   // H_t
                    [[maybe_unused]] const float2 xprev = (t > 0) ? x[t - 1] : xin;
                    dCacc[k][t].x = __builtin_fmaf(dyp[t], x[t].x, dCacc[k][t].x);        // dypre conj(x)
                    dCacc[k][t].y = __builtin_fmaf(-dyp[t], x[t].y, dCacc[k][t].y);
                    ypre[t] = __builtin_fmaf(Cv.x, x[t].x, __builtin_fmaf(-Cv.y, x[t].y, ypre[t]));   // Re(C x)
                    const float2 hb = cxmulc(R, Bv);                        // H conj(B)
                    if constexpr (DISC == DISC_ZOH_S6) {
                        pdu[t] += hb.x;                                      // sum_n Re(H conj(B)); scaled by Delta resp. u in the epilogue
                        const float du_ = dl[t] * uv[t];
                        dBacc[k][t].x = __builtin_fmaf(R.x, du_, dBacc[k][t].x);
                        dBacc[k][t].y = __builtin_fmaf(R.y, du_, dBacc[k][t].y);
                        // grad a conj(a) = H conj(a x_{l-1}), and a x_{l-1} = x_l - Delta u B
                        const float2 ax = make_float2(__builtin_fmaf(-du_, Bv.x, x[t].x), __builtin_fmaf(-du_, Bv.y, x[t].y));
                        const float2 q = cxmulc(R, ax);
                        pdd[t] = __builtin_fmaf(q.x, cc.Ar, __builtin_fmaf(q.y, cc.Ai, pdd[t]));   // Re(q conj(A))
                        dA_part.x = __builtin_fmaf(q.x, dl[t], dA_part.x);
                        dA_part.y = __builtin_fmaf(q.y, dl[t], dA_part.y);
                    } else if constexpr (DISC == DISC_DIRAC) {
                        // g = 1: the S6 expressions with u in place of Delta u
                        pdu[t] += hb.x;
                        dBacc[k][t].x = __builtin_fmaf(R.x, uv[t], dBacc[k][t].x);
                        dBacc[k][t].y = __builtin_fmaf(R.y, uv[t], dBacc[k][t].y);
                        const float2 ax = make_float2(__builtin_fmaf(-uv[t], Bv.x, x[t].x), __builtin_fmaf(-uv[t], Bv.y, x[t].y));
                        const float2 q = cxmulc(R, ax);                      // grad a conj(a)
                        pdd[t] = __builtin_fmaf(q.x, cc.Ar, __builtin_fmaf(q.y, cc.Ai, pdd[t]));
                        dA_part.x = __builtin_fmaf(q.x, dl[t], dA_part.x);
                        dA_part.y = __builtin_fmaf(q.y, dl[t], dA_part.y);
                    } else {
                        const float2 ga = cxmulc(R, xprev);                 // grad a
                        const float2 gq = make_float2(hb.x * uv[t], hb.y * uv[t]);      // grad g
                        pdu[t] += cxmulc(hb, gg[t]).x;                                     // Re(H conj(B) conj(g))
                        const float2 rg = cxmulc(R, gg[t]);
                        dBacc[k][t].x = __builtin_fmaf(rg.x, uv[t], dBacc[k][t].x);
                        dBacc[k][t].y = __builtin_fmaf(rg.y, uv[t], dBacc[k][t].y);
                        if constexpr (DISC == DISC_ZOH) {
                            // da/dDelta = A a, da/dA = Delta a, dg/dDelta = a: with q = grad a conj(a),
                            // dDelta += Re(q conj(A) + grad g conj(a)), dA += Delta q + grad g conj(dg/dA)
                            float2 a_t, a_A, g_t, g_A;
                            cdisc_partials<DISC>(dl[t], cc, a[t], gg[t], a_t, a_A, g_t, g_A);
                            const float2 q = cxmulc(ga, a[t]);
                            pdd[t] = __builtin_fmaf(q.x, cc.Ar, __builtin_fmaf(q.y, cc.Ai, pdd[t])) + cxmulc(gq, a[t]).x;
                            const float2 s2 = cxmulc(gq, g_A);
                            dA_part.x = __builtin_fmaf(q.x, dl[t], dA_part.x) + s2.x;
                            dA_part.y = __builtin_fmaf(q.y, dl[t], dA_part.y) + s2.y;
                        } else {
                            // bilinear: with q = 1 / (1 - Delta A / 2) all four partials are multiples of q^2:
                            // dDelta += Re((grad a conj(A) + grad g) conj(q^2)),
                            // dA += Delta (grad a + grad g Delta / 2) conj(q^2)
                            const float r = (dl[t] != 0.0f) ? rcp_fast(dl[t]) : 0.0f;
                            const float2 q = (dl[t] != 0.0f) ? make_float2(gg[t].x * r, gg[t].y * r) : make_float2(1.0f, 0.0f);
                            const float2 q2 = cxmul(q, q);
                            const float2 t1 = make_float2(__builtin_fmaf(ga.x, cc.Ar, __builtin_fmaf(ga.y, cc.Ai, gq.x)),
                                                          __builtin_fmaf(ga.y, cc.Ar, __builtin_fmaf(-ga.x, cc.Ai, gq.y)));
                            pdd[t] += cxmulc(t1, q2).x;
                            const float hd = 0.5f * dl[t];
                            const float2 t2 = make_float2(__builtin_fmaf(gq.x, hd, ga.x) * dl[t], __builtin_fmaf(gq.y, hd, ga.y) * dl[t]);
                            const float2 s = cxmulc(t2, q2);
                            dA_part.x += s.x;
                            dA_part.y += s.y;
                        }
                    }
                }
                dAr4[k] = dA_part.x; dAi4[k] = dA_part.y;
                __builtin_amdgcn_sched_barrier(0);   // keep the states apart: interleaving them costs more registers than there are
            }
            // the per-lane sums of dA: four real values (two states) per joint reduction; lanes 0-3 and 32-35 own them
            if constexpr (NK % 2 == 0) {
#pragma unroll
                for (int k2 = 0; k2 < NK; k2 += 2) {
                    const float v4[4] = {dAr4[k2], dAr4[k2 + 1], dAi4[k2], dAi4[k2 + 1]};
                    const float v = half_sum4(v4, lane);       // lane % 4 = 0,1,2,3 holds value 0,2,1,3
                    if ((lane & 0x1C) == 0)
                        lds_add(&sdA[lane >> 5][((g * N + w * NK + k2 + ((lane >> 1) & 1)) << 1) + (lane & 1)], v);
                }
            } else {
                const float vr = half_sum(dAr4[0]), vi = half_sum(dAi4[0]);
                if ((lane & 31) == 0) { lds_add(&sdA[lane >> 5][(g * N + w) << 1], vr); lds_add(&sdA[lane >> 5][((g * N + w) << 1) + 1], vi); }
            }
#pragma unroll
            for (int q = 0; q < TQ; ++q) {
                float *base = &sPart[(w * 3) * TILE + (q * 64 + lane) * 4];
                *reinterpret_cast<float4 *>(base) = make_float4(ypre[4 * q], ypre[4 * q + 1], ypre[4 * q + 2], ypre[4 * q + 3]);
                *reinterpret_cast<float4 *>(base + TILE) = make_float4(pdu[4 * q], pdu[4 * q + 1], pdu[4 * q + 2], pdu[4 * q + 3]);
                *reinterpret_cast<float4 *>(base + 2 * TILE) = make_float4(pdd[4 * q], pdd[4 * q + 1], pdd[4 * q + 2], pdd[4 * q + 3]);
            }
            __syncthreads();

            // ---- epilogue: the epilogue threads share the tile in flat order
            if (epi_thread) {
                float o_du[TPW], o_dd[TPW], o_dz[TPW];
                float dD_part = 0.0f, db_part = 0.0f;
                // every LDS value of the epilogue is read up front, in one round trip (left alone, the compiler moves
                // the reads that only feed the stores into the stores' own branch, one round trip after the other)
                float e_in[TPW][5], e_part[TPW][W][3];
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
                    const int fs = fslot(f0e + i);
#pragma unroll
                    for (int j = 0; j < 5; ++j) e_in[i][j] = in[j * TILE + fs];
#pragma unroll
                    for (int ww = 0; ww < W; ++ww)
#pragma unroll
                        for (int j = 0; j < 3; ++j) e_part[i][ww][j] = sPart[(ww * 3 + j) * TILE + fs];
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < TPW; ++i) {
                    const float e_u = e_in[i][1], e_dyp = e_in[i][2];
                    float yp = Dsk * e_u, s_du = 0.0f, s_dd = 0.0f;
#pragma unroll
                    for (int ww = 0; ww < W; ++ww) {
                        yp += e_part[i][ww][0];
                        s_du += e_part[i][ww][1];
                        s_dd += e_part[i][ww][2];
                    }
                    if constexpr (DISC == DISC_ZOH_S6) {
                        // the wavefronts' sums are sum_n Re(H conj(B)): dDelta += u times it, du = Delta times it
                        s_dd = __builtin_fmaf(e_u, s_du, s_dd);
                        s_du *= e_in[i][0];
                    }
                    o_du[i] = __builtin_fmaf(e_dyp, Dsk, s_du);
                    o_dd[i] = s_dd * e_in[i][3];
                    o_dz[i] = yp * e_in[i][4];
                    dD_part = __builtin_fmaf(e_dyp, e_u, dD_part);
                    db_part += (f0e + i < rem) ? o_dd[i] : 0.0f;
                    asm volatile("" : "+v"(o_du[i]), "+v"(o_dd[i]), "+v"(o_dz[i]));   // computed here, not inside the stores' branch
                }
                store_few<IO, TPW>(reinterpret_cast<IO *>(p.du) + bs * p.du_sb + d * p.du_sd + toff + l0, f0e, rem, vec, o_du);
                store_few<IO, TPW>(reinterpret_cast<IO *>(p.ddelta) + bs * p.dd_sb + d * p.dd_sd + toff + l0, f0e, rem, vec, o_dd);
                if (p.dz) store_few<IO, TPW>(reinterpret_cast<IO *>(p.dz) + bs * p.dz_sb + d * p.dz_sd + toff + l0, f0e, rem, vec, o_dz);
                const float vD = half_sum(dD_part), vb = half_sum(db_part);
                if ((lane & 31) == 0) {
                    lds_add(&sdD[((lane >> 5) * W + w) * kMaxGc + g], vD);
                    lds_add(&sdb[((lane >> 5) * W + w) * kMaxGc + g], vb);
                }
            }
            // the next channel's prologue fills the other half of sIn (the prefetch that feeds it was issued before
            // the main pass)
            if (pro_thread && g + 1 < Gact) prologue(g + 1);
        }

        // ---- add this tile's dBm/dCm sums (over the G channels) to global memory, transposed through LDS so that
        // consecutive threads hit consecutive addresses; FL lanes (FL * T time steps) at a time
        // A lane's two states of a step are one 16-byte chunk of that step's row; lanes are T * N pairs apart, which
        // would put all of them on the same banks, so the chunk index is XORed with the lane's low bits (eight
        // consecutive lanes then cover all banks; a reader's consecutive floats stay a permutation of whole chunks
        // within one 8-chunk block).  A thread reads all its values in one batch before it issues its atomics.
        float2 *fbB = reinterpret_cast<float2 *>(sPart), *fbC = fbB + FL * T * N;
        constexpr int CPL = T * N / 2;                                   // 16-byte chunks per lane
        constexpr bool SWZ = NK == 2 && CPL >= 8;
        for (int j = 0; j < 64 / FL; ++j) {
            __syncthreads();
            if (lane / FL == j) {
                // (addresses formed here and now: hoisted out of the tile loop they would cost the channel loop registers)
                int lr = lane % FL;
                asm volatile("" : "+v"(lr));
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    if constexpr (SWZ) {
                        const int c4 = ((lr * T + t) * (N / 2) + w) ^ (lr & 7);
                        *reinterpret_cast<float4 *>(&fbB[c4 * 2]) = make_float4(dBacc[0][t].x, dBacc[0][t].y, dBacc[1][t].x, dBacc[1][t].y);
                        *reinterpret_cast<float4 *>(&fbC[c4 * 2]) = make_float4(dCacc[0][t].x, dCacc[0][t].y, dCacc[1][t].x, dCacc[1][t].y);
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
            float *gB = reinterpret_cast<float *>(p.dBm + bc0 + (l0 + step0) * N);
            float *gC = reinterpret_cast<float *>(p.dCm + bc0 + (l0 + step0) * N);
            const float *lB = reinterpret_cast<const float *>(fbB), *lC = reinterpret_cast<const float *>(fbC);
            constexpr int TOTAL = FL * T * N * 2;                        // floats per array and round
            constexpr int PER = (TOTAL + NT - 1) / NT;
            float vB[PER], vC[PER];
            int tf = tid;
            asm volatile("" : "+v"(tf));
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int idx = tf + i * NT;
                const int at = SWZ ? ((((idx >> 2) ^ (((idx >> 2) / CPL) & 7)) << 2) | (idx & 3)) : idx;
                const bool in = TOTAL % NT == 0 || idx < TOTAL;
                vB[i] = in ? lB[at] : 0.0f; vC[i] = in ? lC[at] : 0.0f;
            }
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int idx = tf + i * NT;
                if ((TOTAL % NT == 0 || idx < TOTAL) && step0 + idx / (2 * N) < rem) {
                    unsafeAtomicAdd(gB + (unsigned)idx, vB[i]);
                    unsafeAtomicAdd(gC + (unsigned)idx, vC[i]);
                }
            }
        }
        __syncthreads();
    }

    // ---- per-channel results of this workgroup
    for (int i = tid; i < Gact * N; i += NT) {
        const int g = i / N, n = i % N;
        float *dst = reinterpret_cast<float *>(p.dA + (int64_t)(d0 + g) * N + n);
        unsafeAtomicAdd(dst, sdA[0][2 * (g * N + n)] + sdA[1][2 * (g * N + n)]);
        unsafeAtomicAdd(dst + 1, sdA[0][2 * (g * N + n) + 1] + sdA[1][2 * (g * N + n) + 1]);
        if (p.dx0 && chunk == 0) p.dx0[((int64_t)b * p.D + d0 + g) * N + n] = sH[g * N + n];
    }
    for (int g = tid; g < Gact; g += NT) {
        float sD = 0.0f, sb = 0.0f;
#pragma unroll
        for (int ww = 0; ww < 2 * W; ++ww) { sD += sdD[ww * kMaxGc + g]; sb += sdb[ww * kMaxGc + g]; }
        if (p.dD) unsafeAtomicAdd(p.dD + d0 + g, sD);
        if (p.dbias) unsafeAtomicAdd(p.dbias + d0 + g, sb);
    }
}

// ---------------------------------------------------------------- launchers
// channels per workgroup: aim at one workgroup per CU (256), as many channels each as fit: the staging of the maps
// and the flush of dBm/dCm are paid once per (workgroup, tile).  Measured on B=8, D=1536, N=16, L=2048: 1.69 ms with
// 256 workgroups, 1.76 ms with 512, 1.90 ms with 1024.
int cbwd_channels_per_group(int B, int D, int, bool balanced) {
    // packed sequences of unknown lengths: four times as many workgroups, so that the short ones fill in beside the long
    int64_t G = ((int64_t)B * D) / (balanced ? 256 : 1024);
    if (balanced) {
        // never a few workgroups more than a whole number of rounds of 256 (see bwd_channels_per_group)
        int64_t rounds = 1;
        while ((int64_t)B * ((D + kMaxGc - 1) / kMaxGc) > rounds * 256 && rounds < 64) ++rounds;
        const int64_t nb = rounds * 256 / B;
        if (nb >= 1) G = (D + nb - 1) / nb;
    }
    if (G < 8) G = 8;
    if (G > kMaxGc) G = kMaxGc;
    if (G > D) G = D;
    const int64_t groups = (D + G - 1) / G;
    G = (D + groups - 1) / groups;                     // even split
    return (int)G;
}

// launch shape incl. the chunked path for few rows and long sequences (selective_bwd_carry.hip): the chip holds one
// 512-thread workgroup per CU for N = 16, two smaller ones below
BwdPlan cbwd_plan(int rowsg, int dpg, int N, int64_t L, int mode, bool balanced) {
    const int G = cbwd_channels_per_group(rowsg, dpg, N, balanced);
    return plan_time_chunks(rowsg, dpg, L, balanced ? mode : 1, G, N >= 16 ? 256 : 512, kMaxGc);
}

template <typename IO, int N, int NK, int DISC>
static hipError_t launch_cbwd_n(const CBwdParams &p, hipStream_t s) {
    const int gmin = p.wcap > 0 ? p.gmin : p.G;                       // fewest channels a workgroup may take
    dim3 grid(p.bcg * ((p.dpg + gmin - 1) / gmin), p.B, p.nchunks > 1 ? p.nchunks : 1);
    hipLaunchKernelGGL((k_ss_cbwd<IO, N, NK, 4, DISC>), grid, dim3((N / NK) * 64), 0, s, p);
    return hipGetLastError();
}

template <typename IO, int DISC>
static hipError_t launch_cbwd_disc(const CBwdParams &p, hipStream_t s) {
    switch (p.N) {
        case 1: return launch_cbwd_n<IO, 1, 1, DISC>(p, s);
        case 2: return launch_cbwd_n<IO, 2, 2, DISC>(p, s);
        // two states per wavefront: with four, the complex sums of dBm/dCm alone take 64 registers and the
        // compiler spills to scratch memory (measured 1.9x slower on the Mamba-block shape)
        case 4: return launch_cbwd_n<IO, 4, 2, DISC>(p, s);
        case 8: return launch_cbwd_n<IO, 8, 2, DISC>(p, s);
        case 16: return launch_cbwd_n<IO, 16, 2, DISC>(p, s);
    }
    return hipErrorInvalidValue;
}

template <typename IO>
static hipError_t launch_cbwd_io(const CBwdParams &p, int disc, hipStream_t s) {
    switch (disc) {
        case DISC_ZOH_S6: return launch_cbwd_disc<IO, DISC_ZOH_S6>(p, s);
        case DISC_ZOH: return launch_cbwd_disc<IO, DISC_ZOH>(p, s);
        case DISC_BILINEAR: return launch_cbwd_disc<IO, DISC_BILINEAR>(p, s);
        case DISC_DIRAC: return launch_cbwd_disc<IO, DISC_DIRAC>(p, s);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_ss_cbwd(const CBwdParams &p, int io_dtype, int disc, hipStream_t s) {
    return io_dtype == 1 ? launch_cbwd_io<bf16_t>(p, disc, s) : launch_cbwd_io<float>(p, disc, s);
}

}  // namespace lrnnx
