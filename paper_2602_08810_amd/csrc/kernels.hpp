// Host-visible parameter blocks and launcher declarations of the scan kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lrnnx {

constexpr int64_t kCkptInterval = 256;   // steps between state checkpoints (public: lrnnx_ckpt_interval)

enum : int { MODE_FULL = 0, MODE_AGG = 1, MODE_APPLY = 2, MODE_CKPT_ONLY = 3 };

struct FwdParams {
    int B, D, N;
    int64_t L;
    int softplus, mode, vec;
    int bcg, dpg;            // number of Bm/Cm groups and channels per group (D = bcg * dpg)
    const int64_t *cu;       // packed variable-length mode: [B+1] sequence boundaries on the packed axis of L steps
    int64_t nslots;          // packed mode: checkpoint slots per channel
    int nchunks;
    int64_t tiles_per_chunk;
    const void *u, *delta, *z;
    void *y;
    int64_t u_sb, u_sd, dl_sb, dl_sd, z_sb, z_sd, y_sb, y_sd;
    const float *A, *Dskip, *bias, *x0;
    const void *Bm, *Cm;
    float *x_last, *ckpt;
    float *ws_P, *ws_S;      // [B,D,nchunks,N] chunk aggregates; ws_S is overwritten with the chunk carry-in
};

// forward selective scan with a complex diagonal A and complex maps (single pass)
struct CFwdParams {
    int B, D, N;
    int64_t L;
    int softplus, vec;
    int bcg, dpg;            // number of Bm/Cm groups and channels per group (D = bcg * dpg)
    const int64_t *cu;       // packed variable-length mode: [B+1] sequence boundaries on the packed axis of L steps
    int64_t nslots;          // packed mode: checkpoint slots per channel
    const void *u, *delta, *z;
    void *y;
    int64_t u_sb, u_sd, dl_sb, dl_sd, z_sb, z_sd, y_sb, y_sd;
    const float2 *A;         // [D,N] complex
    const float *Dskip, *bias;
    const float2 *x0;        // [B,D,N] complex
    const void *Bm, *Cm;     // [B,L,N] complex in the I/O type
    float2 *x_last;
    float2 *ckpt;            // [B,D,ceil(L/kCkptInterval),N] complex: state entering every kCkptInterval-th step, or null
    // chunk-carry path (blockIdx.z = chunk), as for the real forward: MODE_AGG writes each chunk's pair (product of
    // the multipliers, end state from zero) to ws_P, ws_S [B,D,nchunks,N]; the carry kernel turns ws_S into each
    // chunk's true carry-in; MODE_APPLY reruns the chunk from it.  MODE_FULL: one pass, nchunks = 1.
    int mode, nchunks;
    int64_t tiles_per_chunk;
    float2 *ws_P, *ws_S;
};

// backward of the same
struct CBwdParams {
    int B, D, N;
    int64_t L;
    int softplus, vec;
    int G;                   // channels per workgroup
    int bcg, dpg;            // number of Bm/Cm groups and channels per group (D = bcg * dpg)
    const int64_t *cu;       // packed variable-length mode: [B+1] sequence boundaries on the packed axis of L steps
    int64_t nslots;          // packed mode: checkpoint slots per channel
    const void *u, *delta, *z, *dy;
    void *du, *ddelta, *dz;
    int64_t u_sb, u_sd, dl_sb, dl_sd, z_sb, z_sd, dy_sb, dy_sd, du_sb, du_sd, dd_sb, dd_sd, dz_sb, dz_sd;
    const float2 *A, *ckpt;
    const float *Dskip, *bias;
    const void *Bm, *Cm;     // [B,L,N] complex in the I/O type
    float2 *dA, *dBm, *dCm, *dx0;
    float *dD, *dbias;
    // chunked backward, as in BwdParams below (complex aggregates and carries)
    int nchunks;
    int64_t tiles_per_chunk;
    float2 *ws_P, *ws_Q;
    const float2 *hc;
    const int *order;        // packed mode: sequences in the order the launch should start them, or null
    int wcap, gmin;          // packed mode with a known longest sequence: as in BwdParams
};

struct BwdParams {
    int B, D, N;
    int64_t L;
    int softplus, vec;
    int G;                   // channels per workgroup
    int bcg, dpg;            // number of Bm/Cm groups and channels per group (D = bcg * dpg)
    const int64_t *cu;       // packed variable-length mode: [B+1] sequence boundaries on the packed axis of L steps
    int64_t nslots;          // packed mode: checkpoint slots per channel
    const void *u, *delta, *z, *dy;
    void *du, *ddelta, *dz;
    int64_t u_sb, u_sd, dl_sb, dl_sd, z_sb, z_sd, dy_sb, dy_sd, du_sb, du_sd, dd_sb, dd_sd, dz_sb, dz_sd;
    const float *A, *Dskip, *bias, *x0, *ckpt;
    const void *Bm, *Cm;
    float *dA, *dBm, *dCm, *dD, *dbias, *dx0;
    // Chunked backward for long sequences with few rows: the time axis is cut into nchunks chunks of
    // tiles_per_chunk backward tiles (kBwdTileSteps steps each), one workgroup per (channel group, batch entry, chunk).
    // ws_P, ws_Q [B,D,nchunks,N] receive each chunk's adjoint aggregate; the carry kernel turns ws_Q into `hc`, the
    // adjoint carry a_{l1+1} H_{l1+1} entering each chunk from the later side.  nchunks <= 1: no chunking, hc unused.
    int nchunks;
    int64_t tiles_per_chunk;
    float *ws_P, *ws_Q;
    const float *hc;
    // packed mode: sequences in the order the launch should start them (longest first), or null for 0, 1, 2, ...
    const int *order;
    // packed mode with a known longest sequence: cap on the channel-tiles (channels x 256-step tiles) one workgroup
    // walks, and the fewest channels a workgroup may take (the grid is sized for that; 0: no cap, always G).  A
    // workgroup of a long sequence then takes wcap / tiles channels, between gmin and G, and the workgroups of the
    // launch that its sequence does not need leave at once.
    int wcap, gmin;
};
constexpr int kBwdTileSteps = 256;
constexpr int kBwdMinG = 4;
// launch shape of a packed batch of B sequences on L steps, D channels, whose longest has max_seqlen steps (0: not
// known, nothing changes): *G comes in as the channels per workgroup of a batch of unknown lengths and may be raised
// to Gbal, those of a batch [B,D,L] of equal lengths; else cap and fewest channels as in BwdParams.  `places` =
// workgroups the chip holds at once.
void bwd_packed_shape(int B, int D, int64_t L, int64_t max_seqlen, int Gbal, int places, int *G, int *wcap, int *gmin);
constexpr int kMaxOrdered = 256;     // packed batches of more sequences than this are not reordered
hipError_t launch_seq_order(const int64_t *cu, int B, int64_t L, int *order, hipStream_t s);

struct LtiParams {
    int B, P;
    int64_t L;
    int nchunks, ngroups;    // chunks, and groups of 4 consecutive chunks
    int64_t chunk;           // time steps per chunk
    const float2 *lambda, *v, *x0;
    float2 *x, *x_last;
    float2 *ws_S;            // [B,nchunks,P] state entering each chunk if its group had started from zero
    float2 *ws_G;            // [B,ngroups,P] end state of each group started from zero
    // single-pass path
    float2 *ws_T;            // [B,ngroups,P] group end state from zero; all-ones words = not published yet
    float2 *ws_X;            // [B,ngroups/16+1,P] true end state of every 16th group; all-ones = not published
    int *err;                // set to 1 if a bounded wait ran out
    int *status;             // the caller's word for the same, or null
    // adjoint (single-pass only): v = gx, x = dv, x_last = dx0, x0 = the forward pass's x0
    const float2 *xs;        // [B,L,P] states saved by the forward scan
    float *dlambda;          // [P] complex as float pairs, accumulated with atomics (zero it first)
};

// scan with caller-supplied coefficients (single launch, chained groups)
struct DiagParams {
    int B, P;
    int64_t L;
    int is_complex, ngroups;
    const void *a, *b, *x0;  // [B,L,P], [B,L,P], [B,P] of float or float2
    void *x, *x_last;
    float2 *ws_T;            // [B,ngroups,slots,P] group aggregates (slots: 1 real = (A,S); 2 complex = A, S)
    float2 *ws_X;            // [B,ngroups/anchor+1,P] true end state of every anchor group
    int *err;
    int *status;             // the caller's word for a bounded wait that ran out, or null
    // adjoint only: b = gx, x = db, x_last = dx0, x0 = the forward pass's x0
    const void *xs;          // [B,L,P] states saved by the forward scan
    void *da;                // [B,L,P] out
};

struct StepParams {
    int B, D, N;
    int softplus;
    int bcg, dpg;                              // number of Bm/Cm groups and channels per group
    float *x;                                  // [B,D,N] in/out
    const void *u, *delta, *z, *Bm, *Cm;       // u, delta, z: [B,D] with strides; Bm, Cm: [B,N]
    void *y;
    int64_t u_sb, u_sd, dl_sb, dl_sd, z_sb, z_sd, y_sb, y_sd;
    const float *A, *Dskip, *bias;
};

struct CStepParams {
    int B, D, N;
    int softplus;
    int bcg, dpg;                              // number of Bm/Cm groups and channels per group
    float2 *x;                                 // [B,D,N] complex, in/out
    const void *u, *delta, *z, *Bm, *Cm;       // u, delta, z: [B,D] with strides; Bm, Cm: [B,N] complex in the I/O type
    void *y;
    int64_t u_sb, u_sd, dl_sb, dl_sd, z_sb, z_sd, y_sb, y_sd;
    const float2 *A;
    const float *Dskip, *bias;
};

// Each launcher returns hipSuccess or the launch error; it validates nothing.
hipError_t launch_ss_step(const StepParams &p, int io_dtype, int disc, hipStream_t s);
hipError_t launch_ss_cstep(const CStepParams &p, int io_dtype, int disc, hipStream_t s);
hipError_t launch_lti_step(int B, int P, const float2 *lambda, float2 *x, const float2 *v, hipStream_t s);
hipError_t launch_ss_fwd(const FwdParams &p, int io_dtype, int disc, hipStream_t s);
hipError_t launch_ss_carry(const FwdParams &p, hipStream_t s);
hipError_t launch_ss_cfwd(const CFwdParams &p, int io_dtype, int disc, hipStream_t s);
hipError_t launch_ss_cbwd(const CBwdParams &p, int io_dtype, int disc, hipStream_t s);
int cbwd_channels_per_group(int B, int D, int N, bool balanced);
hipError_t launch_ss_bwd(const BwdParams &p, int io_dtype, int disc, hipStream_t s);
hipError_t launch_ss_bwd_agg(const BwdParams &p, int io_dtype, int disc, hipStream_t s);   // chunk aggregates -> ws_P, ws_Q
hipError_t launch_ss_bwd_carry(const BwdParams &p, hipStream_t s);                         // ws_Q -> carries, in place
// Launch shape of the backward pass: channels per workgroup, and (chunks > 1) the chunked path's cut of the time axis
struct BwdPlan { int G, nchunks; int64_t tiles_per_chunk; };
// rowsg = B * (number of Bm/Cm groups), dpg = channels per group; mode 0: automatic, 1: single pass, 2: chunked asked for
BwdPlan bwd_plan(int rowsg, int dpg, int N, int64_t L, int mode, bool balanced);
BwdPlan cbwd_plan(int rowsg, int dpg, int N, int64_t L, int mode, bool balanced);          // the complex-A backward
hipError_t launch_ss_ccarry(const CFwdParams &p, hipStream_t s);
hipError_t launch_ss_cbwd_agg(const CBwdParams &p, int io_dtype, int disc, hipStream_t s);
hipError_t launch_ss_cbwd_carry(const CBwdParams &p, hipStream_t s);

// Few rows and a long sequence: one workgroup per row group would leave most of the chip idle, so the time axis is cut
// into chunks that run side by side.  Measured with the real kernel on one batch entry of 512-2048 channels and
// 16k-64k steps: what counts is to have as many workgroups as the chip holds at once (`full`) and not more (1.5 x
// full: a second, half-empty round, 20-30 % slower), with as many channels each as that allows (staging of the maps
// and flush of dBm/dCm are paid per workgroup and tile: G = 8 -> 64 is 25 % faster at equal workgroup count).  So:
// the largest G <= maxG for which some chunk count fills the chip without exceeding it; baseG is the single pass's G.
inline BwdPlan plan_time_chunks(int rowsg, int dpg, int64_t L, int mode, int baseG, int64_t full, int maxG) {
    BwdPlan pl;
    pl.G = baseG;
    pl.nchunks = 1;
    pl.tiles_per_chunk = (L + kBwdTileSteps - 1) / kBwdTileSteps;
    if (mode == 1) return pl;
    const int64_t ntiles = pl.tiles_per_chunk;
    const int64_t single = (int64_t)rowsg * ((dpg + pl.G - 1) / pl.G);
    // enough rows already, unless they come as many small workgroups (G at its minimum) that leave room on the chip
    if (mode == 0 && single * 4 >= full * 3 && (pl.G >= 16 || single >= full)) return pl;
    int64_t cmax = ntiles;                                                     // asked for: down to one tile per chunk
    if (mode == 0) {                                                           // automatic: four tiles or more per chunk,
        cmax = ntiles / 4;                                                     // two when the sequence is short
        if (cmax < 4) cmax = ntiles / 2 < 4 ? ntiles / 2 : 4;
    }
    if (cmax > 64) cmax = 64;
    int bestG = 0, bestC = 1;
    int64_t bestW = 0;
    for (int64_t c = 2; c <= cmax; ++c) {
        const int64_t nb = full / ((int64_t)rowsg * c);                        // channel blocks per row group that fit
        if (nb < 1) break;
        int64_t g = (dpg + nb - 1) / nb;
        if (g < 8) g = 8;
        if (g > maxG) continue;                                                // would need more blocks than fit
        if (g > dpg) g = dpg;
        const int64_t blocks = (dpg + g - 1) / g;
        g = (dpg + blocks - 1) / blocks;                                       // even split
        const int64_t wgs = (int64_t)rowsg * blocks * c;
        // fuller chip first; among equally full ones more channels per workgroup
        if (wgs > bestW || (wgs == bestW && g > bestG)) { bestW = wgs; bestG = (int)g; bestC = (int)c; }
    }
    if (bestC < 2) {
        if (mode != 2 || ntiles < 2) return pl;
        bestC = 2; bestG = pl.G;                                               // asked for: two chunks at least
    } else if (mode == 0 && bestW <= single) {
        return pl;                                                             // chunking would not fill the chip better
    }
    pl.G = bestG;
    pl.tiles_per_chunk = (ntiles + bestC - 1) / bestC;
    pl.nchunks = (int)((ntiles + pl.tiles_per_chunk - 1) / pl.tiles_per_chunk);   // no empty trailing chunk
    return pl;
}
hipError_t launch_lti(const LtiParams &p, hipStream_t s);
hipError_t launch_lti_onepass(const LtiParams &p, hipStream_t s);
int lti_onepass_group_steps(int64_t B, int64_t P);   // time steps per chained group for this shape
int lti_onepass_min_group_steps();                   // the smallest it can be (sizes the workspace)
hipError_t launch_lti_onepass_bwd(const LtiParams &p, hipStream_t s);
hipError_t launch_diag_scan(const DiagParams &p, hipStream_t s);
int diag_scan_group_steps(int64_t B, int64_t P, int is_complex);
int diag_scan_min_group_steps(int is_complex);
int diag_scan_anchor(int is_complex);
hipError_t launch_diag_scan_bwd(const DiagParams &p, hipStream_t s);
int diag_scan_bwd_group_steps(int is_complex);
int lti_onepass_bwd_group_steps();
struct FillList {
    static constexpr int kMax = 5;
    float *ptr[kMax];
    int64_t count[kMax];     // 32-bit words
    uint32_t bits[kMax];     // the word written (0 = 0.0f)
};
hipError_t launch_fill(const FillList &z, hipStream_t s);

// Tile geometry the host needs for grids, workspaces and the choice of path (each constant lives beside its kernel).
int fwd_channels_per_workgroup();            // wavefronts (= channels) of one forward workgroup
int lti_chunk_group();                       // chunks (wavefronts) of one workgroup of the two-launch LTI path
int lti_onepass_anchor();                    // every how many groups the single-launch LTI scan publishes a true state
int fwd_tile_steps(int io_dtype);            // time steps one workgroup covers per tile
int bwd_channels_per_group(int B, int D, int N, int64_t L, bool balanced);
int bwd_waves_per_workgroup(int N);

}  // namespace lrnnx
