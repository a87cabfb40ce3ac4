// Driver for the sanitizer build of the C ABI's host code (tests/test_sanitizers.py).  It only walks paths that end
// on the host: the size queries and launch plans over a sweep of shapes, and calls that must be refused before
// anything is launched (the pointers are fake, aligned, and never dereferenced).  Runs without a GPU.
#include "../include/lrnnx.h"

#include <cstdio>
#include <cstring>
#include <initializer_list>

#define CHECK(x) do { if (!(x)) { std::fprintf(stderr, "failed: %s (line %d)\n", #x, __LINE__); return 1; } } while (0)

static void *const kFake = reinterpret_cast<void *>(0x10000);

template <typename T> static T blank() { T a; std::memset(&a, 0, sizeof(a)); a.struct_size = sizeof(T); return a; }

static lrnnx_ss_fwd_args fwd_args() {
    lrnnx_ss_fwd_args a = blank<lrnnx_ss_fwd_args>();
    a.B = 2; a.D = 8; a.N = 16; a.L = 100; a.io_dtype = LRNNX_BF16;
    a.u = a.delta = a.Bm = a.Cm = kFake; a.A = static_cast<const float *>(kFake); a.y = kFake;
    a.u_stride_b = a.delta_stride_b = a.y_stride_b = 800;
    a.u_stride_d = a.delta_stride_d = a.y_stride_d = 100;
    return a;
}

static lrnnx_ss_bwd_args bwd_args() {
    lrnnx_ss_bwd_args a = blank<lrnnx_ss_bwd_args>();
    a.B = 2; a.D = 8; a.N = 16; a.L = 100; a.io_dtype = LRNNX_BF16;
    a.u = a.delta = a.Bm = a.Cm = a.dy = kFake; a.A = static_cast<const float *>(kFake);
    a.du = a.ddelta = kFake; a.dA = a.dBm = a.dCm = static_cast<float *>(kFake);
    a.u_stride_b = a.delta_stride_b = a.dy_stride_b = a.du_stride_b = a.ddelta_stride_b = 800;
    a.u_stride_d = a.delta_stride_d = a.dy_stride_d = a.du_stride_d = a.ddelta_stride_d = 100;
    return a;
}

int main() {
    // ---- queries over a sweep of sizes, including degenerate and huge ones
    size_t total = 0;
    for (int which = -1; which <= 9; ++which)
        for (int64_t B : {0, 1, 3, 16, 65535, 65536})
            for (int64_t D : {0, 1, 7, 2560, 1 << 20})
                for (int64_t N : {0, 1, 3, 16, 32, 64})
                    for (int64_t L : {0, 1, 255, 256, 4097, 1 << 22})
                        for (int groups : {-1, 0, 1, 7})
                            for (int packed : {0, 1})
                                total += lrnnx_workspace_bytes(which, B, D, N, L, which & 1, groups, packed) & 0xff;
    for (int64_t B : {0, 1, 8, 70000})
        for (int64_t D : {1, 12, 1536, 4096})
            for (int64_t L : {1, 300, 2048, 65536, 1 << 24})
                for (int path = -1; path <= 3; ++path)
                    for (int cplx = 0; cplx < 2; ++cplx) {
                        total += lrnnx_selective_scan_bwd_chunks(B, D, 16, L, 1, path, cplx);
                        total += lrnnx_selective_scan_bwd_chunks(B, D, 8, L, 4, path, cplx);
                        total += lrnnx_selective_scan_fwd_complex_chunks(B, D, 16, L, 2, path);
                    }
    CHECK(lrnnx_ckpt_interval() > 0 && lrnnx_packed_ckpt_slots(1024, 3) > 0 && lrnnx_packed_ckpt_slots(-1, 3) == 0);
    CHECK(lrnnx_static_scratch_bytes() == LRNNX_STATIC_SCRATCH_BYTES && lrnnx_version() >= 200);
    for (int st = -1; st <= 6; ++st) CHECK(lrnnx_status_string(st) != nullptr);

    // ---- refusals of the forward call
    CHECK(lrnnx_selective_scan_fwd(nullptr) == LRNNX_ERR_INVALID_ARG);
    { auto a = fwd_args(); a.struct_size -= 8; CHECK(lrnnx_selective_scan_fwd(&a) == LRNNX_ERR_INVALID_ARG); }
    { auto a = fwd_args(); a.N = 3; CHECK(lrnnx_selective_scan_fwd(&a) == LRNNX_ERR_UNSUPPORTED); }
    { auto a = fwd_args(); a.B = 65536; CHECK(lrnnx_selective_scan_fwd(&a) == LRNNX_ERR_UNSUPPORTED); }
    { auto a = fwd_args(); a.L = 0; CHECK(lrnnx_selective_scan_fwd(&a) == LRNNX_ERR_INVALID_ARG); }
    { auto a = fwd_args(); a.bc_groups = 3; CHECK(lrnnx_selective_scan_fwd(&a) == LRNNX_ERR_INVALID_ARG); }
    { auto a = fwd_args(); a.y_stride_d = 50; CHECK(lrnnx_selective_scan_fwd(&a) == LRNNX_ERR_INVALID_ARG); }
    { auto a = fwd_args(); a.path = LRNNX_PATH_CHUNK_CARRY; CHECK(lrnnx_selective_scan_fwd(&a) == LRNNX_ERR_WORKSPACE); }
    { auto a = fwd_args(); a.path = LRNNX_PATH_CHUNK_CARRY; a.cu_seqlens = static_cast<const int64_t *>(kFake);
      CHECK(lrnnx_selective_scan_fwd(&a) == LRNNX_ERR_UNSUPPORTED); }

    // ---- refusals of the backward call (real and complex share their checks)
    CHECK(lrnnx_selective_scan_bwd(nullptr) == LRNNX_ERR_INVALID_ARG);
    { auto a = bwd_args(); CHECK(lrnnx_selective_scan_bwd(&a) == LRNNX_ERR_WORKSPACE); }           // no ckpt, no workspace
    { auto a = bwd_args(); a.workspace = kFake; a.workspace_bytes = 16; CHECK(lrnnx_selective_scan_bwd(&a) == LRNNX_ERR_WORKSPACE); }
    { auto a = bwd_args(); a.ckpt = static_cast<const float *>(kFake); a.dz = kFake; CHECK(lrnnx_selective_scan_bwd(&a) == LRNNX_ERR_INVALID_ARG); }
    { auto a = bwd_args(); a.ckpt = static_cast<const float *>(kFake); a.L = 2000; a.du_stride_d = a.ddelta_stride_d = 2000;
      a.path = LRNNX_PATH_CHUNK_CARRY; CHECK(lrnnx_selective_scan_bwd(&a) == LRNNX_ERR_WORKSPACE); }
    { auto a = bwd_args(); a.N = 5; CHECK(lrnnx_selective_scan_bwd(&a) == LRNNX_ERR_UNSUPPORTED); }
    {
        lrnnx_ss_bwd_complex_args c = blank<lrnnx_ss_bwd_complex_args>();
        CHECK(lrnnx_selective_scan_bwd_complex(&c) == LRNNX_ERR_INVALID_ARG);
        lrnnx_ss_fwd_complex_args f = blank<lrnnx_ss_fwd_complex_args>();
        CHECK(lrnnx_selective_scan_fwd_complex(&f) == LRNNX_ERR_INVALID_ARG);
    }

    // ---- the chained scans and the single-token updates
    {
        lrnnx_lti_args a = blank<lrnnx_lti_args>();
        a.B = 2; a.P = 64; a.L = 100; a.lambda = a.v = kFake; a.x = kFake;
        CHECK(lrnnx_lti_diag_scan(&a) == LRNNX_ERR_WORKSPACE);
        a.path = LRNNX_PATH_CHUNK_CARRY; CHECK(lrnnx_lti_diag_scan(&a) == LRNNX_ERR_WORKSPACE);
        CHECK(lrnnx_lti_diag_scan_static(&a) == LRNNX_ERR_INVALID_ARG);       // the two-launch path is not offered there
        a.path = LRNNX_PATH_AUTO; a.B = 8; a.P = 1024; a.L = 8192;
        CHECK(lrnnx_lti_diag_scan_static(&a) == LRNNX_ERR_WORKSPACE);         // beyond the static array
        a.B = 70000; CHECK(lrnnx_lti_diag_scan(&a) == LRNNX_ERR_UNSUPPORTED);
        lrnnx_lti_bwd_args b = blank<lrnnx_lti_bwd_args>();
        CHECK(lrnnx_lti_diag_scan_bwd(&b) == LRNNX_ERR_INVALID_ARG);
        b.B = 1; b.P = 4; b.L = 9; b.lambda = b.x = b.gx = kFake; b.dv = b.dlambda = kFake;
        CHECK(lrnnx_lti_diag_scan_bwd(&b) == LRNNX_ERR_WORKSPACE);
        lrnnx_diag_scan_args d = blank<lrnnx_diag_scan_args>();
        d.B = 1; d.P = 4; d.L = 9; d.dtype = LRNNX_C64; d.a = d.b = kFake; d.x = kFake;
        CHECK(lrnnx_diag_scan(&d) == LRNNX_ERR_WORKSPACE);
        d.dtype = LRNNX_BF16; CHECK(lrnnx_diag_scan(&d) == LRNNX_ERR_INVALID_ARG);
        lrnnx_diag_scan_bwd_args e = blank<lrnnx_diag_scan_bwd_args>();
        e.B = 1; e.P = 4; e.L = 9; e.a = e.x = e.gx = kFake; e.da = reinterpret_cast<void *>(0x20000); e.db = reinterpret_cast<void *>(0x30000);
        CHECK(lrnnx_diag_scan_bwd(&e) == LRNNX_ERR_WORKSPACE);
        e.da = kFake; CHECK(lrnnx_diag_scan_bwd(&e) == LRNNX_ERR_INVALID_ARG);   // da aliases an input
        lrnnx_ss_step_args s = blank<lrnnx_ss_step_args>();
        CHECK(lrnnx_selective_step(&s) == LRNNX_ERR_INVALID_ARG);
        lrnnx_ss_step_complex_args sc = blank<lrnnx_ss_step_complex_args>();
        CHECK(lrnnx_selective_step_complex(&sc) == LRNNX_ERR_INVALID_ARG);
        lrnnx_lti_step_args ls = blank<lrnnx_lti_step_args>();
        CHECK(lrnnx_lti_step(&ls) == LRNNX_ERR_INVALID_ARG);
    }
    std::printf("sanitized C ABI run ok (%zu)\n", total);
    return 0;
}
