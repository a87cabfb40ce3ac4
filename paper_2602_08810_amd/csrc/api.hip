// C ABI of the scan library: argument checks, choice of path, workspace layout, launches.
// Nothing here allocates, frees or synchronises; see include/lrnnx.h for the contract.
#include "../../include/lrnnx.h"
#include "kernels.hpp"
#include <atomic>
#include <cstddef>

using namespace lrnnx;

namespace {

constexpr int kNumCU = 256;              // MI355X

inline bool supported_n(int n) { return n == 1 || n == 2 || n == 4 || n == 8 || n == 16 || n == 32; }
inline bool supported_n_complex(int n) { return n <= 16 && supported_n(n); }   // complex-A entry points
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t elem_size(int io) { return io == LRNNX_BF16 ? 2 : 4; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Vector access to the time axis of a [B,D,L] tensor needs element alignment only (the kernels tell the compiler so
// and global memory takes unaligned vector accesses); strides are counted in elements, so the base decides.
inline bool row_vec_ok(const void *p, int64_t, int64_t, size_t es) {
    return (reinterpret_cast<uintptr_t>(p) & (es - 1)) == 0;
}

// Number of time chunks of the chunk-carry forward path.
int fwd_chunks(int64_t B, int64_t D, int64_t L, int io, bool forced) {
    const int64_t wgs = B * cdiv(D, fwd_channels_per_workgroup());
    const int64_t ntiles = cdiv(L, fwd_tile_steps(io));
    // eight workgroups per compute unit in all: measured on 256-1024 rows x 8k-64k steps, many short chunks beat the
    // two per compute unit an earlier rule aimed at by 5-10 % (the launch evens out better)
    int64_t n = cdiv(8 * kNumCU, wgs);
    if (forced && n < 2) n = 2;
    if (n > ntiles) n = ntiles;
    if (n < 1) n = 1;
    return (int)n;
}

// the complex forward kernel: 8 channels per workgroup, tiles of 512 steps for both I/O types
constexpr int kCfwdTile = 512;
int cfwd_chunks(int64_t wgs, int64_t L, bool forced) {
    const int64_t ntiles = cdiv(L, kCfwdTile);
    int64_t n = cdiv(forced ? 8 * kNumCU : 2 * kNumCU, wgs);
    if (forced && n < 2) n = 2;
    if (n > ntiles) n = ntiles;
    return n < 1 ? 1 : (int)n;
}
// one pass over whole rows (also what the backward entry point's recompute sweep runs)
void set_cfwd_single_pass(CFwdParams &p) {
    p.mode = MODE_FULL; p.nchunks = 1; p.tiles_per_chunk = (int64_t)1 << 40;
}

int lti_chunks(int64_t B, int64_t P, int64_t L) {
    const int64_t waves_per_chunk = B * cdiv(P, 64);
    int64_t n = cdiv(8 * kNumCU, waves_per_chunk);
    const int64_t max_n = cdiv(L, 16);                 // at least 16 steps per chunk
    if (n > max_n) n = max_n;
    if (n > 512) n = 512;                               // each workgroup walks the end states of the groups before it
    if (n < 1) n = 1;
    return (int)n;
}

// single-pass LTI workspace: T [B,ngroups,P] and X [B,ngroups/16+1,P] complex, then the error word
size_t onepass_bytes(int64_t B, int64_t P, int64_t ng) {
    return (size_t)(B * (ng + ng / lti_onepass_anchor() + 1) * P * 2 * sizeof(float)) + 64 * sizeof(int);
}
size_t lti_onepass_bytes(int64_t B, int64_t P, int64_t L) { return onepass_bytes(B, P, cdiv(L, lti_onepass_min_group_steps())); }
size_t lti_onepass_bwd_bytes(int64_t B, int64_t P, int64_t L) {
    return onepass_bytes(B, P, cdiv(L, lti_onepass_bwd_group_steps()));
}
size_t diag_scan_bytes(int64_t B, int64_t P, int64_t L, int is_complex) {
    const int64_t ng = cdiv(L, diag_scan_min_group_steps(is_complex));
    const int64_t slots = ng * (is_complex ? 2 : 1) + ng / diag_scan_anchor(is_complex) + 1;
    return (size_t)(B * slots * P * 2 * sizeof(float)) + 64 * sizeof(int);
}
size_t diag_scan_bwd_bytes(int64_t B, int64_t P, int64_t L, int is_complex) {
    const int64_t ng = cdiv(L, diag_scan_bwd_group_steps(is_complex));
    const int64_t slots = ng * (is_complex ? 2 : 1) + ng / diag_scan_anchor(is_complex) + 1;
    return (size_t)(B * slots * P * 2 * sizeof(float)) + 64 * sizeof(int);
}
// lays the chain workspace of a caller-coefficient scan out and returns the fill list that arms it
FillList set_diag_workspace(DiagParams &p, void *ws) {
    const int cplx = p.is_complex;
    const int64_t nT = (int64_t)p.B * p.ngroups * (cplx ? 2 : 1) * p.P;
    const int64_t nX = (int64_t)p.B * (p.ngroups / diag_scan_anchor(cplx) + 1) * p.P;
    p.ws_T = reinterpret_cast<float2 *>(ws);
    p.ws_X = p.ws_T + nT;
    p.err = reinterpret_cast<int *>(p.ws_X + nX);
    FillList z{};                                  // every slot starts as "not published", the error word as zero
    z.ptr[0] = reinterpret_cast<float *>(p.ws_T); z.count[0] = 2 * (nT + nX); z.bits[0] = 0xffffffffu;
    z.ptr[1] = reinterpret_cast<float *>(p.err);  z.count[1] = 1;
    return z;
}
void set_onepass_workspace(LtiParams &p, void *ws) {
    p.ws_T = reinterpret_cast<float2 *>(ws);
    p.ws_X = p.ws_T + (size_t)p.B * p.ngroups * p.P;
    p.err = reinterpret_cast<int *>(p.ws_X + (size_t)p.B * (p.ngroups / lti_onepass_anchor() + 1) * p.P);
}
// every slot starts as "not published" (all-ones words), the error word as zero
FillList onepass_fill(const LtiParams &p) {
    FillList z{};
    z.ptr[0] = reinterpret_cast<float *>(p.ws_T);
    z.count[0] = 2 * (int64_t)p.B * (p.ngroups + p.ngroups / lti_onepass_anchor() + 1) * p.P;
    z.bits[0] = 0xffffffffu;
    z.ptr[1] = reinterpret_cast<float *>(p.err); z.count[1] = 1;
    return z;
}

// bytes of the two aggregate arrays [B,D,nchunks,N] of the chunked backward: the larger of what the automatic choice
// and an explicit request for that path take
size_t bwd_carry_bytes(int64_t B, int64_t D, int64_t N, int64_t L) {
    const int a = bwd_plan((int)B, (int)D, (int)N, L, 0, true).nchunks, f = bwd_plan((int)B, (int)D, (int)N, L, 2, true).nchunks;
    const int nch = a > f ? a : f;
    return nch > 1 ? (size_t)2 * B * D * nch * N * sizeof(float) : 0;
}
size_t cbwd_carry_bytes(int64_t B, int64_t D, int64_t N, int64_t L) {    // the same for the complex-A backward
    const int a = cbwd_plan((int)B, (int)D, (int)N, L, 0, true).nchunks, f = cbwd_plan((int)B, (int)D, (int)N, L, 2, true).nchunks;
    const int nch = a > f ? a : f;
    return nch > 1 ? (size_t)2 * B * D * nch * N * sizeof(float2) : 0;
}
size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

// Launch plan of a backward call.  A batch [B,D,L] is planned as it is.  Of a packed batch the host knows the number of
// sequences and the length of the time axis, and max_seqlen if the caller gave it (else 0): the single pass is planned
// for sequences of unknown, unequal lengths; chunks of the time axis are planned for B sequences of max_seqlen steps
// (of the whole axis without it) when the caller asks for them, and on its own account only when max_seqlen is known.
// Every chunk but the last of a sequence has the planned number of steps and the last takes what is left, so a
// max_seqlen that is too small costs balance, never steps.
template <typename Plan>
BwdPlan packed_bwd_plan(Plan plan, int rowsg, int dpg, int N, int64_t L, int path, bool packed, int64_t max_seqlen) {
    if (!packed) return plan(rowsg, dpg, N, L, path, true);
    const bool known = max_seqlen > 0;
    if (path == LRNNX_PATH_CHUNK_CARRY || (path == LRNNX_PATH_AUTO && known)) {
        const BwdPlan pc = plan(rowsg, dpg, N, known && max_seqlen < L ? max_seqlen : L, path, true);
        if (pc.nchunks > 1) return pc;
    }
    return plan(rowsg, dpg, N, L, LRNNX_PATH_SINGLE_PASS, false);
}
// at most `nfit` chunks (what the workspace holds): fewer, longer chunks of whole tiles
void fit_chunks(BwdPlan &pl, size_t nfit) {
    if (nfit >= (size_t)pl.nchunks || nfit < 2) return;
    const int64_t ntiles = pl.tiles_per_chunk * pl.nchunks;          // an upper bound of the planned tiles
    pl.tiles_per_chunk = (ntiles + (int64_t)nfit - 1) / (int64_t)nfit;
    pl.nchunks = (int)nfit;
}

// The real and the complex backward entry points take the same per-row tensors (same field names in both argument
// structs and both parameter blocks): checks and marshalling are written once.
template <typename Args>
bool bwd_rows_valid(const Args *a) {
    if (!a->u || !a->delta || !a->A || !a->Bm || !a->Cm || !a->dy) return false;
    if (!a->du || !a->ddelta || !a->dA || !a->dBm || !a->dCm) return false;
    if ((a->dz && !a->z) || (a->dD && !a->Dskip) || (a->dbias && !a->delta_bias)) return false;
    return !(a->u_stride_b < 0 || a->u_stride_d < 0 || a->delta_stride_b < 0 || a->delta_stride_d < 0 ||
             a->dy_stride_b < 0 || a->dy_stride_d < 0 || (a->z && (a->z_stride_b < 0 || a->z_stride_d < 0)) ||
             a->du_stride_b < 0 || a->du_stride_d < a->L || a->ddelta_stride_b < 0 || a->ddelta_stride_d < a->L ||
             (a->dz && (a->dz_stride_b < 0 || a->dz_stride_d < a->L)));
}
template <typename Params, typename Args>
void set_bwd_rows(Params &p, const Args *a) {
    const size_t es = elem_size(a->io_dtype);
    p.B = a->B; p.D = a->D; p.N = a->N; p.L = a->L;
    p.softplus = a->delta_softplus ? 1 : 0;
    p.u = a->u; p.delta = a->delta; p.z = a->z; p.dy = a->dy;
    p.du = a->du; p.ddelta = a->ddelta; p.dz = a->dz;
    p.u_sb = a->u_stride_b; p.u_sd = a->u_stride_d; p.dl_sb = a->delta_stride_b; p.dl_sd = a->delta_stride_d;
    p.z_sb = a->z_stride_b; p.z_sd = a->z_stride_d; p.dy_sb = a->dy_stride_b; p.dy_sd = a->dy_stride_d;
    p.du_sb = a->du_stride_b; p.du_sd = a->du_stride_d; p.dd_sb = a->ddelta_stride_b; p.dd_sd = a->ddelta_stride_d;
    p.dz_sb = a->dz_stride_b; p.dz_sd = a->dz_stride_d;
    p.Dskip = a->Dskip; p.bias = a->delta_bias;
    p.Bm = a->Bm; p.Cm = a->Cm;
    p.dD = a->dD; p.dbias = a->dbias;
    p.vec = row_vec_ok(a->u, p.u_sb, p.u_sd, es) && row_vec_ok(a->delta, p.dl_sb, p.dl_sd, es) &&
            row_vec_ok(a->dy, p.dy_sb, p.dy_sd, es) && (!a->z || row_vec_ok(a->z, p.z_sb, p.z_sd, es)) &&
            row_vec_ok(a->du, p.du_sb, p.du_sd, es) && row_vec_ok(a->ddelta, p.dd_sb, p.dd_sd, es) &&
            (!a->dz || row_vec_ok(a->dz, p.dz_sb, p.dz_sd, es));
}

}  // namespace

extern "C" {

int64_t lrnnx_ckpt_interval(void) { return kCkptInterval; }
int64_t lrnnx_packed_ckpt_slots(int64_t L, int64_t B) { return (L < 0 || B < 0) ? 0 : L / kCkptInterval + B; }
int lrnnx_version(void) { return 300; }   // major * 100 + minor; the major number changes with any struct layout

int lrnnx_selective_scan_bwd_chunks(int64_t B, int64_t D, int64_t N, int64_t L, int bc_groups, int path, int complex_a) {
    const int bcg = bc_groups > 1 ? bc_groups : 1;
    if (B < 1 || D < 1 || L < 1 || B > 65535 || D > INT32_MAX || D % bcg) return 0;
    if (!(complex_a ? supported_n_complex((int)N) : supported_n((int)N))) return 0;
    if (path < LRNNX_PATH_AUTO || path > LRNNX_PATH_CHUNK_CARRY) return 0;
    if (path == LRNNX_PATH_SINGLE_PASS) return 1;
    return complex_a ? cbwd_plan((int)B * bcg, (int)(D / bcg), (int)N, L, path, true).nchunks
                     : bwd_plan((int)B * bcg, (int)(D / bcg), (int)N, L, path, true).nchunks;
}

int lrnnx_selective_scan_fwd_complex_chunks(int64_t B, int64_t D, int64_t N, int64_t L, int bc_groups, int path) {
    const int bcg = bc_groups > 1 ? bc_groups : 1;
    if (B < 1 || D < 1 || L < 1 || B > 65535 || D > INT32_MAX || D % bcg || !supported_n_complex((int)N)) return 0;
    if (path < LRNNX_PATH_AUTO || path > LRNNX_PATH_CHUNK_CARRY) return 0;
    const int64_t wgs = B * bcg * cdiv(D / bcg, 8);
    if (path == LRNNX_PATH_CHUNK_CARRY) return cfwd_chunks(wgs, L, true);
    if (path == LRNNX_PATH_AUTO && wgs <= kNumCU / 2 && cdiv(L, kCfwdTile) >= 4) return cfwd_chunks(wgs, L, false);
    return 1;
}

const char *lrnnx_status_string(int status) {
    switch (status) {
        case LRNNX_OK: return "ok";
        case LRNNX_ERR_INVALID_ARG: return "invalid argument";
        case LRNNX_ERR_UNSUPPORTED: return "unsupported configuration";
        case LRNNX_ERR_WORKSPACE: return "workspace missing or too small";
        case LRNNX_ERR_LAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

size_t lrnnx_workspace_bytes(int which, int64_t B, int64_t D, int64_t N, int64_t L, int io_dtype, int bc_groups,
                             int packed) {
    if (B < 1 || D < 1 || L < 1 || bc_groups < 0 || B > 65535 || D > INT32_MAX) return 0;
    const int64_t bcg = bc_groups > 1 ? bc_groups : 1;
    const bool selective = which == LRNNX_WS_FWD || which == LRNNX_WS_BWD || which == LRNNX_WS_BWD_CARRY ||
                           which == LRNNX_WS_FWD_COMPLEX || which == LRNNX_WS_BWD_COMPLEX;
    if (selective) {
        const bool cplx = which == LRNNX_WS_FWD_COMPLEX || which == LRNNX_WS_BWD_COMPLEX;
        if (!(cplx ? supported_n_complex((int)N) : supported_n((int)N)) || D % bcg) return 0;
        const size_t es = cplx ? sizeof(float2) : sizeof(float);
        if (which == LRNNX_WS_FWD) return packed ? 0 : (size_t)2 * B * D * fwd_chunks(B, D, L, io_dtype, true) * N * es;
        if (which == LRNNX_WS_FWD_COMPLEX)
            return packed ? 0 : (size_t)2 * B * D * cfwd_chunks(B * bcg * cdiv(D / bcg, 8), L, true) * N * es;
        // backward: the checkpoints of the recompute sweep (not LRNNX_WS_BWD_CARRY: the caller has the forward's), then
        // the chunk aggregates, or for a packed batch the launch order
        size_t ck = 0;
        if (which != LRNNX_WS_BWD_CARRY)
            ck = align256((size_t)(packed ? D * lrnnx_packed_ckpt_slots(L, B) : B * D * cdiv(L, kCkptInterval)) * N * es);
        const size_t carry = cplx ? cbwd_carry_bytes(B * bcg, D / bcg, N, L) : bwd_carry_bytes(B * bcg, D / bcg, N, L);
        const size_t order = packed ? sizeof(int) * (size_t)B : 0;
        return ck + (carry > order ? carry : order);
    }
    if (which == LRNNX_WS_LTI) {
        const int nch = lti_chunks(B, D, L);
        const size_t two = nch > 1 ? (size_t)B * (nch + cdiv(nch, lti_chunk_group())) * D * 2 * sizeof(float) : 0;
        const size_t one = lti_onepass_bytes(B, D, L);
        return two > one ? two : one;
    }
    if (which == LRNNX_WS_LTI_BWD) return lti_onepass_bwd_bytes(B, D, L);
    if (which == LRNNX_WS_DIAG || which == LRNNX_WS_DIAG_BWD) {
        if (io_dtype != LRNNX_F32 && io_dtype != LRNNX_C64) return 0;
        return which == LRNNX_WS_DIAG ? diag_scan_bytes(B, D, L, io_dtype == LRNNX_C64)
                                      : diag_scan_bwd_bytes(B, D, L, io_dtype == LRNNX_C64);
    }
    return 0;
}

int lrnnx_selective_scan_fwd(const lrnnx_ss_fwd_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_ss_fwd_args)) return LRNNX_ERR_INVALID_ARG;
    if (a->bc_groups < 0) return LRNNX_ERR_INVALID_ARG;
    const int bcg = a->bc_groups > 1 ? a->bc_groups : 1;
    const int64_t *cu = a->cu_seqlens;
    if (cu && (reinterpret_cast<uintptr_t>(cu) & 7u)) return LRNNX_ERR_INVALID_ARG;
    if (cu && a->path == LRNNX_PATH_CHUNK_CARRY) return LRNNX_ERR_UNSUPPORTED;
    if (a->B < 1 || a->D < 1 || a->N < 1 || a->L < 1) return LRNNX_ERR_INVALID_ARG;
    if (a->io_dtype != LRNNX_F32 && a->io_dtype != LRNNX_BF16) return LRNNX_ERR_INVALID_ARG;
    if (a->disc < 0 || a->disc > LRNNX_DISC_DIRAC) return LRNNX_ERR_INVALID_ARG;
    if (a->path < LRNNX_PATH_AUTO || a->path > LRNNX_PATH_CHUNK_CARRY) return LRNNX_ERR_INVALID_ARG;
    if (!a->u || !a->delta || !a->A || !a->Bm || !a->Cm || !a->y) return LRNNX_ERR_INVALID_ARG;
    if (a->u_stride_b < 0 || a->u_stride_d < 0 || a->delta_stride_b < 0 || a->delta_stride_d < 0 ||
        a->y_stride_b < 0 || a->y_stride_d < a->L || (a->z && (a->z_stride_b < 0 || a->z_stride_d < 0)))
        return LRNNX_ERR_INVALID_ARG;
    if (!supported_n(a->N)) return LRNNX_ERR_UNSUPPORTED;
    if (a->B > 65535) return LRNNX_ERR_UNSUPPORTED;
    if (a->D % bcg) return LRNNX_ERR_INVALID_ARG;
    const size_t es = elem_size(a->io_dtype);
    if (!aligned16(a->Bm) || !aligned16(a->Cm)) return LRNNX_ERR_INVALID_ARG;

    FwdParams p{};
    p.B = a->B; p.D = a->D; p.N = a->N; p.L = a->L;
    p.bcg = bcg; p.dpg = a->D / bcg;
    p.cu = cu; p.nslots = lrnnx_packed_ckpt_slots(a->L, a->B);
    p.softplus = a->delta_softplus ? 1 : 0;
    p.u = a->u; p.delta = a->delta; p.z = a->z; p.y = a->y;
    p.u_sb = a->u_stride_b; p.u_sd = a->u_stride_d;
    p.dl_sb = a->delta_stride_b; p.dl_sd = a->delta_stride_d;
    p.z_sb = a->z_stride_b; p.z_sd = a->z_stride_d;
    p.y_sb = a->y_stride_b; p.y_sd = a->y_stride_d;
    p.A = a->A; p.Dskip = a->Dskip; p.bias = a->delta_bias; p.x0 = a->x0;
    p.Bm = a->Bm; p.Cm = a->Cm; p.x_last = a->x_last; p.ckpt = a->ckpt;
    p.vec = row_vec_ok(a->u, p.u_sb, p.u_sd, es) && row_vec_ok(a->delta, p.dl_sb, p.dl_sd, es) &&
            row_vec_ok(a->y, p.y_sb, p.y_sd, es) && (!a->z || row_vec_ok(a->z, p.z_sb, p.z_sd, es));

    const int64_t ntiles = cdiv(a->L, fwd_tile_steps(a->io_dtype));
    const int64_t wgs = (int64_t)a->B * cdiv(a->D, fwd_channels_per_workgroup());
    bool chunked = false;
    int nch = 1;
    if (a->path == LRNNX_PATH_CHUNK_CARRY) {
        nch = fwd_chunks(a->B, a->D, a->L, a->io_dtype, true);
        const size_t need = (size_t)2 * a->B * a->D * nch * a->N * sizeof(float);
        if (!a->workspace || a->workspace_bytes < need) return LRNNX_ERR_WORKSPACE;
        chunked = true;
    } else if (a->path == LRNNX_PATH_AUTO && !cu && wgs <= kNumCU / 2 && ntiles >= 4) {
        nch = fwd_chunks(a->B, a->D, a->L, a->io_dtype, false);
        const size_t need = (size_t)2 * a->B * a->D * nch * a->N * sizeof(float);
        chunked = nch > 1 && a->workspace && a->workspace_bytes >= need;
        if (!chunked) nch = 1;
    }
    hipStream_t s = reinterpret_cast<hipStream_t>(a->stream);
    if (!chunked) {
        p.mode = MODE_FULL; p.nchunks = 1; p.tiles_per_chunk = ntiles;
        return launch_ss_fwd(p, a->io_dtype, a->disc, s) == hipSuccess ? LRNNX_OK : LRNNX_ERR_LAUNCH;
    }
    p.nchunks = nch;
    p.tiles_per_chunk = cdiv(ntiles, nch);
    p.nchunks = (int)cdiv(ntiles, p.tiles_per_chunk);      // no empty trailing chunk
    p.ws_P = reinterpret_cast<float *>(a->workspace);
    p.ws_S = p.ws_P + (size_t)a->B * a->D * p.nchunks * a->N;
    FwdParams pa = p;
    pa.mode = MODE_AGG; pa.ckpt = nullptr; pa.x_last = nullptr;
    if (launch_ss_fwd(pa, a->io_dtype, a->disc, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    if (launch_ss_carry(p, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    p.mode = MODE_APPLY;
    return launch_ss_fwd(p, a->io_dtype, a->disc, s) == hipSuccess ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

int lrnnx_selective_scan_fwd_complex(const lrnnx_ss_fwd_complex_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_ss_fwd_complex_args)) return LRNNX_ERR_INVALID_ARG;
    void *ckpt = a->ckpt;
    if (a->bc_groups < 0) return LRNNX_ERR_INVALID_ARG;
    const int bcg = a->bc_groups > 1 ? a->bc_groups : 1;
    const int64_t *cu = a->cu_seqlens;
    if (cu && (reinterpret_cast<uintptr_t>(cu) & 7u)) return LRNNX_ERR_INVALID_ARG;
    const int path = a->path;
    void *ws = a->workspace;
    const size_t ws_bytes = a->workspace_bytes;
    if (path < LRNNX_PATH_AUTO || path > LRNNX_PATH_CHUNK_CARRY) return LRNNX_ERR_INVALID_ARG;
    if (cu && path == LRNNX_PATH_CHUNK_CARRY) return LRNNX_ERR_UNSUPPORTED;
    if (reinterpret_cast<uintptr_t>(ws) & 7u) return LRNNX_ERR_INVALID_ARG;
    if (a->B < 1 || a->D < 1 || a->N < 1 || a->L < 1) return LRNNX_ERR_INVALID_ARG;
    if (a->io_dtype != LRNNX_F32 && a->io_dtype != LRNNX_BF16) return LRNNX_ERR_INVALID_ARG;
    if (a->disc < 0 || a->disc > LRNNX_DISC_DIRAC) return LRNNX_ERR_INVALID_ARG;
    if (!a->u || !a->delta || !a->A || !a->Bm || !a->Cm) return LRNNX_ERR_INVALID_ARG;
    if (!a->y && !ckpt && !a->x_last) return LRNNX_ERR_INVALID_ARG;          // nothing to compute
    if (reinterpret_cast<uintptr_t>(ckpt) & 7u) return LRNNX_ERR_INVALID_ARG;
    if (a->u_stride_b < 0 || a->u_stride_d < 0 || a->delta_stride_b < 0 || a->delta_stride_d < 0 ||
        (a->y && (a->y_stride_b < 0 || a->y_stride_d < a->L)) || (a->z && (a->z_stride_b < 0 || a->z_stride_d < 0)))
        return LRNNX_ERR_INVALID_ARG;
    if (!supported_n_complex(a->N)) return LRNNX_ERR_UNSUPPORTED;
    if (a->B > 65535) return LRNNX_ERR_UNSUPPORTED;
    if (a->D % bcg) return LRNNX_ERR_INVALID_ARG;
    if (!aligned16(a->Bm) || !aligned16(a->Cm)) return LRNNX_ERR_INVALID_ARG;
    for (const void *q : {a->A, a->x0, (const void *)a->x_last})
        if (reinterpret_cast<uintptr_t>(q) & 7u) return LRNNX_ERR_INVALID_ARG;
    const size_t es = elem_size(a->io_dtype);
    CFwdParams p{};
    p.B = a->B; p.D = a->D; p.N = a->N; p.L = a->L;
    p.bcg = bcg; p.dpg = a->D / bcg;
    p.cu = cu; p.nslots = lrnnx_packed_ckpt_slots(a->L, a->B);
    p.softplus = a->delta_softplus ? 1 : 0;
    p.u = a->u; p.delta = a->delta; p.z = a->z; p.y = a->y;
    p.u_sb = a->u_stride_b; p.u_sd = a->u_stride_d;
    p.dl_sb = a->delta_stride_b; p.dl_sd = a->delta_stride_d;
    p.z_sb = a->z_stride_b; p.z_sd = a->z_stride_d;
    p.y_sb = a->y_stride_b; p.y_sd = a->y_stride_d;
    p.A = reinterpret_cast<const float2 *>(a->A);
    p.Dskip = a->Dskip; p.bias = a->delta_bias;
    p.x0 = reinterpret_cast<const float2 *>(a->x0);
    p.Bm = a->Bm; p.Cm = a->Cm;
    p.x_last = reinterpret_cast<float2 *>(a->x_last);
    p.ckpt = reinterpret_cast<float2 *>(ckpt);
    p.vec = row_vec_ok(a->u, p.u_sb, p.u_sd, es) && row_vec_ok(a->delta, p.dl_sb, p.dl_sd, es) &&
            (!a->y || row_vec_ok(a->y, p.y_sb, p.y_sd, es)) && (!a->z || row_vec_ok(a->z, p.z_sb, p.z_sd, es));
    hipStream_t s = reinterpret_cast<hipStream_t>(a->stream);

    // chunk-carry path: asked for, or (automatic) few rows and a sequence of four tiles or more
    const int64_t ntiles = cdiv(a->L, kCfwdTile);
    const int64_t wgs = (int64_t)a->B * bcg * cdiv(a->D / bcg, 8);
    int nch = cu ? 1 : lrnnx_selective_scan_fwd_complex_chunks(a->B, a->D, a->N, a->L, bcg, path);
    if (nch > 1 && (!ws || ws_bytes < (size_t)2 * a->B * a->D * nch * a->N * sizeof(float2))) {
        if (path == LRNNX_PATH_CHUNK_CARRY) return LRNNX_ERR_WORKSPACE;
        nch = 1;
    }
    if (nch < 2) {
        set_cfwd_single_pass(p);
        return launch_ss_cfwd(p, a->io_dtype, a->disc, s) == hipSuccess ? LRNNX_OK : LRNNX_ERR_LAUNCH;
    }
    p.tiles_per_chunk = cdiv(ntiles, nch);
    p.nchunks = (int)cdiv(ntiles, p.tiles_per_chunk);          // no empty trailing chunk
    p.ws_P = reinterpret_cast<float2 *>(ws);
    p.ws_S = p.ws_P + (size_t)a->B * a->D * p.nchunks * a->N;
    CFwdParams pa = p;
    pa.mode = MODE_AGG; pa.ckpt = nullptr; pa.x_last = nullptr; pa.y = nullptr;
    if (launch_ss_cfwd(pa, a->io_dtype, a->disc, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    if (launch_ss_ccarry(p, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    p.mode = MODE_APPLY;
    return launch_ss_cfwd(p, a->io_dtype, a->disc, s) == hipSuccess ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

int lrnnx_selective_scan_bwd_complex(const lrnnx_ss_bwd_complex_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_ss_bwd_complex_args)) return LRNNX_ERR_INVALID_ARG;
    const int64_t *cu = a->cu_seqlens;
    const int path = a->path;
    if (cu && (reinterpret_cast<uintptr_t>(cu) & 7u)) return LRNNX_ERR_INVALID_ARG;
    if (path < LRNNX_PATH_AUTO || path > LRNNX_PATH_CHUNK_CARRY) return LRNNX_ERR_INVALID_ARG;
    if (a->max_seqlen < 0) return LRNNX_ERR_INVALID_ARG;
    if (a->B < 1 || a->D < 1 || a->N < 1 || a->L < 1) return LRNNX_ERR_INVALID_ARG;
    if (a->io_dtype != LRNNX_F32 && a->io_dtype != LRNNX_BF16) return LRNNX_ERR_INVALID_ARG;
    if (a->disc < 0 || a->disc > LRNNX_DISC_DIRAC) return LRNNX_ERR_INVALID_ARG;
    if (!bwd_rows_valid(a)) return LRNNX_ERR_INVALID_ARG;
    if (!supported_n_complex(a->N)) return LRNNX_ERR_UNSUPPORTED;
    if (a->B > 65535) return LRNNX_ERR_UNSUPPORTED;
    if (a->bc_groups < 0) return LRNNX_ERR_INVALID_ARG;
    const int bcg = a->bc_groups > 1 ? a->bc_groups : 1;
    if (a->D % bcg) return LRNNX_ERR_INVALID_ARG;
    if (!aligned16(a->Bm) || !aligned16(a->Cm) || !aligned16(a->dBm) || !aligned16(a->dCm)) return LRNNX_ERR_INVALID_ARG;
    for (const void *q : {a->A, a->x0, a->ckpt, (const void *)a->dA, (const void *)a->dx0, (const void *)a->workspace})
        if (reinterpret_cast<uintptr_t>(q) & 7u) return LRNNX_ERR_INVALID_ARG;
    const size_t es = elem_size(a->io_dtype);
    const int64_t nslots = lrnnx_packed_ckpt_slots(a->L, a->B);
    const size_t ck_bytes = cu ? (size_t)a->D * nslots * a->N * sizeof(float2)
                               : (size_t)a->B * a->D * cdiv(a->L, kCkptInterval) * a->N * sizeof(float2);
    if (!a->ckpt && (!a->workspace || a->workspace_bytes < ck_bytes)) return LRNNX_ERR_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(a->stream);

    // chunked path: the aggregates live in the workspace, after the checkpoints of the recompute sweep if there are any
    BwdPlan pl = packed_bwd_plan(cbwd_plan, a->B * bcg, a->D / bcg, a->N, a->L, path, cu != nullptr, a->max_seqlen);
    const size_t carry_off = a->ckpt ? 0 : align256(ck_bytes);
    if (pl.nchunks > 1) {
        const size_t per_chunk = (size_t)2 * a->B * a->D * a->N * sizeof(float2);
        const size_t room = (a->workspace && a->workspace_bytes > carry_off) ? a->workspace_bytes - carry_off : 0;
        if (cu) fit_chunks(pl, room / per_chunk);
        if (pl.nchunks > 1 && room < per_chunk * pl.nchunks) {
            if (path == LRNNX_PATH_CHUNK_CARRY) return LRNNX_ERR_WORKSPACE;
            pl = cbwd_plan(a->B * bcg, a->D / bcg, a->N, a->L, LRNNX_PATH_SINGLE_PASS, cu == nullptr);
        }
    }

    const float2 *ckpt = reinterpret_cast<const float2 *>(a->ckpt);
    if (!ckpt) {                                   // state-only forward sweep: writes the checkpoints
        CFwdParams f{};
        f.B = a->B; f.D = a->D; f.N = a->N; f.L = a->L;
        f.bcg = bcg; f.dpg = a->D / bcg;
        f.cu = cu; f.nslots = nslots;
        f.softplus = a->delta_softplus ? 1 : 0;
        f.u = a->u; f.delta = a->delta;
        f.u_sb = a->u_stride_b; f.u_sd = a->u_stride_d; f.dl_sb = a->delta_stride_b; f.dl_sd = a->delta_stride_d;
        f.A = reinterpret_cast<const float2 *>(a->A); f.bias = a->delta_bias;
        f.x0 = reinterpret_cast<const float2 *>(a->x0);
        f.Bm = a->Bm; f.Cm = a->Cm;
        f.ckpt = reinterpret_cast<float2 *>(a->workspace);
        f.vec = row_vec_ok(a->u, f.u_sb, f.u_sd, es) && row_vec_ok(a->delta, f.dl_sb, f.dl_sd, es);
        set_cfwd_single_pass(f);
        if (launch_ss_cfwd(f, a->io_dtype, a->disc, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
        ckpt = f.ckpt;
    }

    CBwdParams p{};
    set_bwd_rows(p, a);
    p.bcg = bcg; p.dpg = a->D / bcg;
    p.cu = cu; p.nslots = nslots;
    p.A = reinterpret_cast<const float2 *>(a->A); p.ckpt = ckpt;
    p.dA = reinterpret_cast<float2 *>(a->dA); p.dBm = reinterpret_cast<float2 *>(a->dBm);
    p.dCm = reinterpret_cast<float2 *>(a->dCm); p.dx0 = reinterpret_cast<float2 *>(a->dx0);
    p.G = pl.G;
    p.nchunks = pl.nchunks;
    p.tiles_per_chunk = pl.tiles_per_chunk;
    if (cu && pl.nchunks == 1)
        bwd_packed_shape(a->B, a->D, a->L, a->max_seqlen, cbwd_channels_per_group(a->B * bcg, a->D / bcg, a->N, true),
                         a->N >= 16 ? 256 : 512, &p.G, &p.wcap, &p.gmin);
    if (pl.nchunks > 1) {
        p.ws_P = reinterpret_cast<float2 *>(static_cast<char *>(a->workspace) + carry_off);
        p.ws_Q = p.ws_P + (size_t)a->B * a->D * p.nchunks * a->N;
        p.hc = p.ws_Q;
        if (launch_ss_cbwd_agg(p, a->io_dtype, a->disc, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
        if (launch_ss_cbwd_carry(p, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    }
    // packed batches: longest sequences first, if the workspace has room for the order (as in the real backward)
    if (cu && pl.nchunks == 1 && a->B > 1 && a->B <= kMaxOrdered && a->workspace &&
        a->workspace_bytes >= carry_off + sizeof(int) * (size_t)a->B) {
        int *order = reinterpret_cast<int *>(static_cast<char *>(a->workspace) + carry_off);
        if (launch_seq_order(cu, a->B, a->L, order, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
        p.order = order;
    }

    const int64_t nbc = (cu ? 1 : (int64_t)a->B) * bcg * a->L * a->N * 2;   // floats; packed mode: one time axis for all sequences
    FillList z{};
    z.ptr[0] = reinterpret_cast<float *>(a->dBm); z.count[0] = nbc;
    z.ptr[1] = reinterpret_cast<float *>(a->dCm); z.count[1] = nbc;
    z.ptr[2] = reinterpret_cast<float *>(a->dA); z.count[2] = (int64_t)a->D * a->N * 2;
    z.ptr[3] = a->dD; z.count[3] = a->D;
    z.ptr[4] = a->dbias; z.count[4] = a->D;
    if (launch_fill(z, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    return launch_ss_cbwd(p, a->io_dtype, a->disc, s) == hipSuccess ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

int lrnnx_selective_scan_bwd(const lrnnx_ss_bwd_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_ss_bwd_args)) return LRNNX_ERR_INVALID_ARG;
    const int64_t *cu = a->cu_seqlens;
    const int path = a->path;
    if (cu && (reinterpret_cast<uintptr_t>(cu) & 7u)) return LRNNX_ERR_INVALID_ARG;
    if (path < LRNNX_PATH_AUTO || path > LRNNX_PATH_CHUNK_CARRY) return LRNNX_ERR_INVALID_ARG;
    if (a->max_seqlen < 0) return LRNNX_ERR_INVALID_ARG;
    if (a->B < 1 || a->D < 1 || a->N < 1 || a->L < 1) return LRNNX_ERR_INVALID_ARG;
    if (a->io_dtype != LRNNX_F32 && a->io_dtype != LRNNX_BF16) return LRNNX_ERR_INVALID_ARG;
    if (a->disc < 0 || a->disc > LRNNX_DISC_DIRAC) return LRNNX_ERR_INVALID_ARG;
    if (!bwd_rows_valid(a)) return LRNNX_ERR_INVALID_ARG;
    if (!supported_n(a->N)) return LRNNX_ERR_UNSUPPORTED;
    if (a->B > 65535) return LRNNX_ERR_UNSUPPORTED;
    if (a->bc_groups < 0) return LRNNX_ERR_INVALID_ARG;
    const int bcg = a->bc_groups > 1 ? a->bc_groups : 1;
    if (a->D % bcg) return LRNNX_ERR_INVALID_ARG;
    if (!aligned16(a->Bm) || !aligned16(a->Cm) || !aligned16(a->dBm) || !aligned16(a->dCm)) return LRNNX_ERR_INVALID_ARG;
    const size_t es = elem_size(a->io_dtype);
    const int64_t nck = cdiv(a->L, kCkptInterval);
    const int64_t nslots = lrnnx_packed_ckpt_slots(a->L, a->B);
    const size_t ck_bytes = cu ? (size_t)a->D * nslots * a->N * sizeof(float)
                               : (size_t)a->B * a->D * nck * a->N * sizeof(float);
    if (!a->ckpt && (!a->workspace || a->workspace_bytes < ck_bytes)) return LRNNX_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(a->workspace) & 3u) return LRNNX_ERR_INVALID_ARG;
    hipStream_t s = reinterpret_cast<hipStream_t>(a->stream);

    // chunked path: the aggregates live in the workspace, after the checkpoints of the recompute sweep if there are any
    BwdPlan pl = packed_bwd_plan(bwd_plan, a->B * bcg, a->D / bcg, a->N, a->L, path, cu != nullptr, a->max_seqlen);
    const size_t carry_off = a->ckpt ? 0 : align256(ck_bytes);
    if (pl.nchunks > 1) {
        const size_t per_chunk = (size_t)2 * a->B * a->D * a->N * sizeof(float);
        const size_t room = (a->workspace && a->workspace_bytes > carry_off) ? a->workspace_bytes - carry_off : 0;
        if (cu) fit_chunks(pl, room / per_chunk);
        if (pl.nchunks > 1 && room < per_chunk * pl.nchunks) {
            if (path == LRNNX_PATH_CHUNK_CARRY) return LRNNX_ERR_WORKSPACE;
            pl = bwd_plan(a->B * bcg, a->D / bcg, a->N, a->L, LRNNX_PATH_SINGLE_PASS, cu == nullptr);
        }
    }

    const float *ckpt = a->ckpt;
    if (!ckpt) {                                   // state-only forward sweep: writes the checkpoints
        FwdParams f{};
        f.B = a->B; f.D = a->D; f.N = a->N; f.L = a->L;
        f.bcg = bcg; f.dpg = a->D / bcg;
        f.cu = cu; f.nslots = nslots;
        f.softplus = a->delta_softplus ? 1 : 0;
        f.u = a->u; f.delta = a->delta;
        f.u_sb = a->u_stride_b; f.u_sd = a->u_stride_d; f.dl_sb = a->delta_stride_b; f.dl_sd = a->delta_stride_d;
        f.A = a->A; f.bias = a->delta_bias; f.x0 = a->x0; f.Bm = a->Bm; f.Cm = a->Cm;
        f.ckpt = reinterpret_cast<float *>(a->workspace);
        f.vec = row_vec_ok(a->u, f.u_sb, f.u_sd, es) && row_vec_ok(a->delta, f.dl_sb, f.dl_sd, es);
        f.mode = MODE_CKPT_ONLY; f.nchunks = 1; f.tiles_per_chunk = cdiv(a->L, fwd_tile_steps(a->io_dtype));
        if (launch_ss_fwd(f, a->io_dtype, a->disc, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
        ckpt = f.ckpt;
    }

    BwdParams p{};
    set_bwd_rows(p, a);
    p.bcg = bcg; p.dpg = a->D / bcg;
    p.cu = cu; p.nslots = lrnnx_packed_ckpt_slots(a->L, a->B);
    p.A = a->A; p.x0 = a->x0; p.ckpt = ckpt;
    p.dA = a->dA; p.dBm = a->dBm; p.dCm = a->dCm; p.dx0 = a->dx0;
    p.G = pl.G;
    p.nchunks = pl.nchunks;
    p.tiles_per_chunk = pl.tiles_per_chunk;
    if (cu && pl.nchunks == 1)
        bwd_packed_shape(a->B, a->D, a->L, a->max_seqlen, bwd_channels_per_group(a->B * bcg, a->D / bcg, a->N, a->L, true),
                         2048 / bwd_waves_per_workgroup(a->N), &p.G, &p.wcap, &p.gmin);
    if (pl.nchunks > 1) {
        p.ws_P = reinterpret_cast<float *>(static_cast<char *>(a->workspace) + carry_off);
        p.ws_Q = p.ws_P + (size_t)a->B * a->D * p.nchunks * a->N;
        p.hc = p.ws_Q;
        if (launch_ss_bwd_agg(p, a->io_dtype, a->disc, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
        if (launch_ss_bwd_carry(p, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    }
    // packed batches: longest sequences first, if the workspace has room for the order (B ints, after the checkpoints
    // of the recompute sweep if there are any)
    if (cu && pl.nchunks == 1 && a->B > 1 && a->B <= kMaxOrdered && a->workspace &&
        a->workspace_bytes >= carry_off + sizeof(int) * (size_t)a->B) {
        int *order = reinterpret_cast<int *>(static_cast<char *>(a->workspace) + carry_off);
        if (launch_seq_order(cu, a->B, a->L, order, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
        p.order = order;
    }

    // reduced outputs are accumulated with atomics: clear them on the stream first
    const int64_t nbc = (cu ? 1 : (int64_t)a->B) * bcg * a->L * a->N;   // packed mode: one time axis for all sequences
    FillList z{};
    z.ptr[0] = a->dBm; z.count[0] = nbc;
    z.ptr[1] = a->dCm; z.count[1] = nbc;
    z.ptr[2] = a->dA; z.count[2] = (int64_t)a->D * a->N;
    z.ptr[3] = a->dD; z.count[3] = a->D;
    z.ptr[4] = a->dbias; z.count[4] = a->D;
    if (launch_fill(z, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    return launch_ss_bwd(p, a->io_dtype, a->disc, s) == hipSuccess ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

// the single-launch path on a chain workspace of at least lti_onepass_bytes(B, P, L) bytes (checked by the callers)
static int lti_onepass_run(const lrnnx_lti_args *a, void *ws, hipStream_t s) {
    const int64_t ng = cdiv(a->L, lti_onepass_group_steps(a->B, a->P));
    const int64_t wgx = (int64_t)a->B * cdiv(a->P, 64);
    if (ng > 65535 || wgx > 0x7fffffff) return LRNNX_ERR_UNSUPPORTED;
    LtiParams p{};
    p.B = a->B; p.P = a->P; p.L = a->L;
    p.lambda = reinterpret_cast<const float2 *>(a->lambda);
    p.v = reinterpret_cast<const float2 *>(a->v);
    p.x0 = reinterpret_cast<const float2 *>(a->x0);
    p.x = reinterpret_cast<float2 *>(a->x);
    p.x_last = reinterpret_cast<float2 *>(a->x_last);
    p.ngroups = (int)ng;
    p.status = a->chain_status;
    set_onepass_workspace(p, ws);
    if (launch_fill(onepass_fill(p), s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    return launch_lti_onepass(p, s) == hipSuccess ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

static int lti_args_valid(const lrnnx_lti_args *a) {
    if (a->B < 1 || a->P < 1 || a->L < 1) return LRNNX_ERR_INVALID_ARG;
    if (!a->lambda || !a->v || !a->x) return LRNNX_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(a->v) & 7u) || (reinterpret_cast<uintptr_t>(a->x) & 7u) ||
        (reinterpret_cast<uintptr_t>(a->lambda) & 7u) || (reinterpret_cast<uintptr_t>(a->x0) & 7u) ||
        (reinterpret_cast<uintptr_t>(a->x_last) & 7u) || (reinterpret_cast<uintptr_t>(a->chain_status) & 3u))
        return LRNNX_ERR_INVALID_ARG;
    if (a->B > 65535) return LRNNX_ERR_UNSUPPORTED;
    return LRNNX_OK;
}

int lrnnx_lti_diag_scan(const lrnnx_lti_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_lti_args)) return LRNNX_ERR_INVALID_ARG;
    const int path = a->path;
    if (path < LRNNX_PATH_AUTO || path > LRNNX_PATH_CHUNK_CARRY) return LRNNX_ERR_INVALID_ARG;
    if (const int st = lti_args_valid(a)) return st;
    hipStream_t s = reinterpret_cast<hipStream_t>(a->stream);

    if (path != LRNNX_PATH_CHUNK_CARRY) {
        if (!a->workspace || a->workspace_bytes < lti_onepass_bytes(a->B, a->P, a->L) ||
            (reinterpret_cast<uintptr_t>(a->workspace) & 7u))
            return LRNNX_ERR_WORKSPACE;
        return lti_onepass_run(a, a->workspace, s);
    }

    LtiParams p{};
    p.B = a->B; p.P = a->P; p.L = a->L;
    p.lambda = reinterpret_cast<const float2 *>(a->lambda);
    p.v = reinterpret_cast<const float2 *>(a->v);
    p.x0 = reinterpret_cast<const float2 *>(a->x0);
    p.x = reinterpret_cast<float2 *>(a->x);
    p.x_last = reinterpret_cast<float2 *>(a->x_last);
    int nch = lti_chunks(a->B, a->P, a->L);
    p.chunk = cdiv(a->L, nch);
    p.nchunks = (int)cdiv(a->L, p.chunk);
    p.ngroups = (int)cdiv(p.nchunks, lti_chunk_group());
    if (p.ngroups > 65535) return LRNNX_ERR_UNSUPPORTED;
    if (p.nchunks > 1) {
        const size_t need = (size_t)a->B * (p.nchunks + p.ngroups) * a->P * 2 * sizeof(float);
        if (!a->workspace || a->workspace_bytes < need) return LRNNX_ERR_WORKSPACE;
        p.ws_S = reinterpret_cast<float2 *>(a->workspace);
        p.ws_G = p.ws_S + (size_t)a->B * p.nchunks * a->P;
    }
    return launch_lti(p, s) == hipSuccess ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

// ---------------------------------------------------------------- the entry point that allocates nothing
// lrnnx_lti_diag_scan needs a chain workspace from its caller.  Callers that cannot allocate device memory (code
// under HIP graph capture, serving loops, harnesses that forbid allocation) get the same scan on a scratch array that
// is part of the library's device image: every GPU the library runs on holds its own copy until the process ends.
static __device__ __align__(256) unsigned char scratch[LRNNX_STATIC_SCRATCH_BYTES];

// Device address of `scratch` on the current device, looked up once per device (the name itself is only a host-side
// stand-in for the symbol: it must never reach a kernel, a fill or a copy).  NULL if the runtime refuses.
static void *static_scratch_ptr() {
    constexpr int kMaxDevices = 64;
    static std::atomic<void *> ptrs[kMaxDevices];
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *ptr = ptrs[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        ptrs[dev].store(ptr, std::memory_order_release);      // every thread that races here finds the same address
    }
    return ptr;
}

size_t lrnnx_static_scratch_bytes(void) { return LRNNX_STATIC_SCRATCH_BYTES; }

int lrnnx_lti_diag_scan_static(const lrnnx_lti_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_lti_args)) return LRNNX_ERR_INVALID_ARG;
    if (a->path != LRNNX_PATH_AUTO && a->path != LRNNX_PATH_SINGLE_PASS) return LRNNX_ERR_INVALID_ARG;
    if (const int st = lti_args_valid(a)) return st;
    if (lti_onepass_bytes(a->B, a->P, a->L) > LRNNX_STATIC_SCRATCH_BYTES) return LRNNX_ERR_WORKSPACE;
    void *ws = static_scratch_ptr();
    if (!ws) return LRNNX_ERR_LAUNCH;
    return lti_onepass_run(a, ws, reinterpret_cast<hipStream_t>(a->stream));
}

int lrnnx_lti_diag_scan_bwd(const lrnnx_lti_bwd_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_lti_bwd_args)) return LRNNX_ERR_INVALID_ARG;
    if (a->B < 1 || a->P < 1 || a->L < 1) return LRNNX_ERR_INVALID_ARG;
    if (!a->lambda || !a->x || !a->gx || !a->dv || !a->dlambda) return LRNNX_ERR_INVALID_ARG;
    for (const void *q : {a->lambda, a->x, a->x0, a->gx, (const void *)a->dv, (const void *)a->dlambda,
                          (const void *)a->dx0})
        if (reinterpret_cast<uintptr_t>(q) & 7u) return LRNNX_ERR_INVALID_ARG;
    const int64_t ng = cdiv(a->L, lti_onepass_bwd_group_steps());
    const int64_t wgx = (int64_t)a->B * cdiv(a->P, 64);
    if (a->B > 65535 || ng > 65535 || wgx > 0x7fffffff) return LRNNX_ERR_UNSUPPORTED;
    if (!a->workspace || a->workspace_bytes < lti_onepass_bwd_bytes(a->B, a->P, a->L) ||
        (reinterpret_cast<uintptr_t>(a->workspace) & 7u))
        return LRNNX_ERR_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(a->stream);
    LtiParams p{};
    p.B = a->B; p.P = a->P; p.L = a->L;
    p.lambda = reinterpret_cast<const float2 *>(a->lambda);
    p.v = reinterpret_cast<const float2 *>(a->gx);
    p.xs = reinterpret_cast<const float2 *>(a->x);
    p.x0 = reinterpret_cast<const float2 *>(a->x0);
    p.x = reinterpret_cast<float2 *>(a->dv);
    p.x_last = reinterpret_cast<float2 *>(a->dx0);
    p.dlambda = reinterpret_cast<float *>(a->dlambda);
    p.ngroups = (int)ng;
    p.status = a->chain_status;
    set_onepass_workspace(p, a->workspace);
    FillList z = onepass_fill(p);
    z.ptr[2] = p.dlambda; z.count[2] = 2 * (int64_t)a->P;
    if (launch_fill(z, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    return launch_lti_onepass_bwd(p, s) == hipSuccess ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

int lrnnx_diag_scan(const lrnnx_diag_scan_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_diag_scan_args)) return LRNNX_ERR_INVALID_ARG;
    if (a->B < 1 || a->P < 1 || a->L < 1) return LRNNX_ERR_INVALID_ARG;
    if (a->dtype != LRNNX_F32 && a->dtype != LRNNX_C64) return LRNNX_ERR_INVALID_ARG;
    if (!a->a || !a->b || !a->x) return LRNNX_ERR_INVALID_ARG;
    const int cplx = a->dtype == LRNNX_C64;
    const uintptr_t mask = cplx ? 7u : 3u;
    for (const void *q : {a->a, a->b, a->x0, (const void *)a->x, (const void *)a->x_last})
        if (reinterpret_cast<uintptr_t>(q) & mask) return LRNNX_ERR_INVALID_ARG;
    if ((int64_t)a->P * (cplx ? 8 : 4) > 0x7fffffff) return LRNNX_ERR_UNSUPPORTED;   // 32-bit byte offsets in a row
    const int64_t ng = cdiv(a->L, diag_scan_group_steps(a->B, a->P, cplx));
    const int64_t wgx = (int64_t)a->B * cdiv(a->P, 64);
    if (a->B > 65535 || ng > 65535 || wgx > 0x7fffffff) return LRNNX_ERR_UNSUPPORTED;
    if (!a->workspace || a->workspace_bytes < diag_scan_bytes(a->B, a->P, a->L, cplx) ||
        (reinterpret_cast<uintptr_t>(a->workspace) & 7u))
        return LRNNX_ERR_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(a->stream);
    DiagParams p{};
    p.B = a->B; p.P = a->P; p.L = a->L;
    p.is_complex = cplx; p.ngroups = (int)ng;
    p.a = a->a; p.b = a->b; p.x0 = a->x0; p.x = a->x; p.x_last = a->x_last;
    p.status = a->chain_status;
    const FillList z = set_diag_workspace(p, a->workspace);
    if (launch_fill(z, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    return launch_diag_scan(p, s) == hipSuccess ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

int lrnnx_diag_scan_bwd(const lrnnx_diag_scan_bwd_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_diag_scan_bwd_args)) return LRNNX_ERR_INVALID_ARG;
    if (a->B < 1 || a->P < 1 || a->L < 1) return LRNNX_ERR_INVALID_ARG;
    if (a->dtype != LRNNX_F32 && a->dtype != LRNNX_C64) return LRNNX_ERR_INVALID_ARG;
    if (!a->a || !a->x || !a->gx || !a->da || !a->db) return LRNNX_ERR_INVALID_ARG;
    if (a->da == a->a || a->da == a->x || a->da == a->gx || a->da == a->db) return LRNNX_ERR_INVALID_ARG;
    const int cplx = a->dtype == LRNNX_C64;
    const uintptr_t mask = cplx ? 7u : 3u;
    for (const void *q : {a->a, a->x, a->x0, a->gx, (const void *)a->da, (const void *)a->db, (const void *)a->dx0})
        if (reinterpret_cast<uintptr_t>(q) & mask) return LRNNX_ERR_INVALID_ARG;
    if ((int64_t)a->P * (cplx ? 8 : 4) > 0x7fffffff) return LRNNX_ERR_UNSUPPORTED;   // 32-bit byte offsets in a row
    const int64_t ng = cdiv(a->L, diag_scan_bwd_group_steps(cplx));
    const int64_t wgx = (int64_t)a->B * cdiv(a->P, 64);
    if (a->B > 65535 || ng > 65535 || wgx > 0x7fffffff) return LRNNX_ERR_UNSUPPORTED;
    if (!a->workspace || a->workspace_bytes < diag_scan_bwd_bytes(a->B, a->P, a->L, cplx) ||
        (reinterpret_cast<uintptr_t>(a->workspace) & 7u))
        return LRNNX_ERR_WORKSPACE;
    hipStream_t s = reinterpret_cast<hipStream_t>(a->stream);
    DiagParams p{};
    p.B = a->B; p.P = a->P; p.L = a->L;
    p.is_complex = cplx; p.ngroups = (int)ng;
    p.a = a->a; p.b = a->gx; p.xs = a->x; p.x0 = a->x0;
    p.x = a->db; p.da = a->da; p.x_last = a->dx0;
    p.status = a->chain_status;
    const FillList z = set_diag_workspace(p, a->workspace);
    if (launch_fill(z, s) != hipSuccess) return LRNNX_ERR_LAUNCH;
    return launch_diag_scan_bwd(p, s) == hipSuccess ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

int lrnnx_selective_step(const lrnnx_ss_step_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_ss_step_args)) return LRNNX_ERR_INVALID_ARG;
    if (a->bc_groups < 0) return LRNNX_ERR_INVALID_ARG;
    const int bcg = a->bc_groups > 1 ? a->bc_groups : 1;
    if (a->D % bcg) return LRNNX_ERR_INVALID_ARG;
    if (a->B < 1 || a->D < 1 || a->N < 1) return LRNNX_ERR_INVALID_ARG;
    if (a->io_dtype != LRNNX_F32 && a->io_dtype != LRNNX_BF16) return LRNNX_ERR_INVALID_ARG;
    if (a->disc < 0 || a->disc > LRNNX_DISC_DIRAC) return LRNNX_ERR_INVALID_ARG;
    if (!a->x || !a->u || !a->delta || !a->A || !a->Bm || !a->Cm || !a->y) return LRNNX_ERR_INVALID_ARG;
    if (!supported_n(a->N)) return LRNNX_ERR_UNSUPPORTED;
    if (a->B > 65535) return LRNNX_ERR_UNSUPPORTED;
    if (!aligned16(a->x) || !aligned16(a->A) || !aligned16(a->Bm) || !aligned16(a->Cm)) return LRNNX_ERR_INVALID_ARG;
    StepParams p{};
    p.B = a->B; p.D = a->D; p.N = a->N; p.softplus = a->delta_softplus ? 1 : 0;
    p.bcg = bcg; p.dpg = a->D / bcg;
    p.x = a->x; p.u = a->u; p.delta = a->delta; p.z = a->z; p.Bm = a->Bm; p.Cm = a->Cm; p.y = a->y;
    p.u_sb = a->u_stride_b; p.u_sd = a->u_stride_d; p.dl_sb = a->delta_stride_b; p.dl_sd = a->delta_stride_d;
    p.z_sb = a->z_stride_b; p.z_sd = a->z_stride_d; p.y_sb = a->y_stride_b; p.y_sd = a->y_stride_d;
    p.A = a->A; p.Dskip = a->Dskip; p.bias = a->delta_bias;
    return launch_ss_step(p, a->io_dtype, a->disc, reinterpret_cast<hipStream_t>(a->stream)) == hipSuccess
               ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

int lrnnx_selective_step_complex(const lrnnx_ss_step_complex_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_ss_step_complex_args)) return LRNNX_ERR_INVALID_ARG;
    if (a->bc_groups < 0) return LRNNX_ERR_INVALID_ARG;
    const int bcg = a->bc_groups > 1 ? a->bc_groups : 1;
    if (a->B < 1 || a->D < 1 || a->N < 1 || a->D % bcg) return LRNNX_ERR_INVALID_ARG;
    if (a->io_dtype != LRNNX_F32 && a->io_dtype != LRNNX_BF16) return LRNNX_ERR_INVALID_ARG;
    if (a->disc < 0 || a->disc > LRNNX_DISC_DIRAC) return LRNNX_ERR_INVALID_ARG;
    if (!a->x || !a->u || !a->delta || !a->A || !a->Bm || !a->Cm || !a->y) return LRNNX_ERR_INVALID_ARG;
    if (!supported_n_complex(a->N)) return LRNNX_ERR_UNSUPPORTED;
    if (a->B > 65535) return LRNNX_ERR_UNSUPPORTED;
    if (!aligned16(a->x) || !aligned16(a->A) || !aligned16(a->Bm) || !aligned16(a->Cm)) return LRNNX_ERR_INVALID_ARG;
    CStepParams p{};
    p.B = a->B; p.D = a->D; p.N = a->N; p.softplus = a->delta_softplus ? 1 : 0;
    p.bcg = bcg; p.dpg = a->D / bcg;
    p.x = reinterpret_cast<float2 *>(a->x); p.u = a->u; p.delta = a->delta; p.z = a->z; p.Bm = a->Bm; p.Cm = a->Cm; p.y = a->y;
    p.u_sb = a->u_stride_b; p.u_sd = a->u_stride_d; p.dl_sb = a->delta_stride_b; p.dl_sd = a->delta_stride_d;
    p.z_sb = a->z_stride_b; p.z_sd = a->z_stride_d; p.y_sb = a->y_stride_b; p.y_sd = a->y_stride_d;
    p.A = reinterpret_cast<const float2 *>(a->A); p.Dskip = a->Dskip; p.bias = a->delta_bias;
    return launch_ss_cstep(p, a->io_dtype, a->disc, reinterpret_cast<hipStream_t>(a->stream)) == hipSuccess
               ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

int lrnnx_lti_step(const lrnnx_lti_step_args *a) {
    if (!a || a->struct_size != sizeof(lrnnx_lti_step_args)) return LRNNX_ERR_INVALID_ARG;
    if (a->B < 1 || a->P < 1 || !a->lambda || !a->x || !a->v) return LRNNX_ERR_INVALID_ARG;
    if (a->B > 65535) return LRNNX_ERR_UNSUPPORTED;
    if ((reinterpret_cast<uintptr_t>(a->v) & 7u) || (reinterpret_cast<uintptr_t>(a->x) & 7u) ||
        (reinterpret_cast<uintptr_t>(a->lambda) & 7u))
        return LRNNX_ERR_INVALID_ARG;
    return launch_lti_step(a->B, a->P, reinterpret_cast<const float2 *>(a->lambda), reinterpret_cast<float2 *>(a->x),
                           reinterpret_cast<const float2 *>(a->v), reinterpret_cast<hipStream_t>(a->stream)) == hipSuccess
               ? LRNNX_OK : LRNNX_ERR_LAUNCH;
}

}  // extern "C"
