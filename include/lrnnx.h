/*
 * lrnnx.h -- C ABI of the MI355X (gfx950) diagonal linear-recurrence scan library.
 *
 * The library computes the linear RNN recurrence of the lrnnx paper (Sec. 2.2, Eq. 2)
 *
 *     x_k = A(k) x_{k-1} + B(k) u_k,        y_k = C(k) x_k + D(k) u_k
 *
 * for a diagonal state matrix, in three forms:
 *   - time-varying, input-dependent ("selective", the S6 row of Table 1; Sec. 2.2.2),
 *     forward and backward (also with a complex diagonal A and complex maps, y = Re(C x) + D u),
 *     with the discretisation fused into the scan (Sec. 3: ZOH,
 *     bilinear, dirac; the asynchronous / event-driven scheme is served by
 *     delta_softplus = 0 with the caller's own per-step Delta) and with the output
 *     projection fused in; also as a single-token update (the `step` method, Sec. 3);
 *   - time-invariant complex-diagonal (the S5 / LRU rows of Table 1; Sec. 2.2.1),
 *     forward, backward and single-token update;
 *   - time-varying with the per-step coefficients a_k, b_k supplied by the caller, real or
 *     complex (the time-varying S5-style and gated layers of Sec. 2.2.2), forward and backward.
 * The hidden state x[B,D,L,N] is never written to memory (Sec. 3, the stated
 * advantage of the fused kernels); the backward pass recomputes it.
 *
 * General rules for every entry point
 *   - Every pointer is a DEVICE pointer unless stated otherwise.  The caller owns all
 *     buffers; the library allocates nothing, frees nothing and never synchronises.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream) and the call returns at once.
 *   - The return value is an lrnnx_status.  On any status other than LRNNX_OK nothing
 *     has been launched and no output has been touched.  No C++ exception crosses the
 *     ABI and the library never aborts.
 *   - `struct_size` must be set to sizeof(the struct) of the header the caller was built with; any other
 *     value is rejected (lrnnx_version() tells which layout a library build expects).
 *   - Tensors named [B,D,L] have the time axis contiguous (stride 1) and explicit
 *     batch / channel strides counted in ELEMENTS; a channel stride of 0 broadcasts
 *     one row over all channels (inputs only).  Tensors [B,L,N], [D,N], [D], [B,D,N]
 *     are contiguous.  io_dtype selects the element type of u, delta, z, Bm, Cm, y, dy,
 *     du, ddelta, dz (float or bfloat16); the state, all accumulation, A, Dskip,
 *     delta_bias, x0, x_last, checkpoints and the reduced gradients are float.
 *   - Supported: N in {1,2,4,8,16,32} (the complex-A entry points: up to 16); 1 <= B <= 65535 (a launch grid
 *     dimension; more batch entries are refused with LRNNX_ERR_UNSUPPORTED); any D >= 1; any L >= 1
 *     (B*D*L must fit int64).
 */
#ifndef LRNNX_H
#define LRNNX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LRNNX_OK = 0,
    LRNNX_ERR_INVALID_ARG = 1,   /* NULL required pointer, bad size, bad enum, bad stride */
    LRNNX_ERR_UNSUPPORTED = 2,   /* valid request the library has no kernel for (e.g. N = 3) */
    LRNNX_ERR_WORKSPACE = 3,     /* workspace missing or smaller than lrnnx_workspace_bytes() */
    LRNNX_ERR_LAUNCH = 4         /* the HIP runtime refused a launch; hipGetLastError has details */
} lrnnx_status;

typedef enum { LRNNX_F32 = 0, LRNNX_BF16 = 1, LRNNX_C64 = 2 /* complex, two floats; lrnnx_diag_scan only */ } lrnnx_dtype;

/* Discretisation of x' = A x + B u with step Delta (schemes named in Sec. 3).
 * a is the state multiplier, g the input gain (Bbar = g * B).                */
typedef enum {
    LRNNX_DISC_ZOH_S6 = 0,    /* a = exp(Delta A), g = Delta               (S6's simplified ZOH) */
    LRNNX_DISC_ZOH = 1,       /* a = exp(Delta A), g = (a - 1) / A         (exact zero-order hold) */
    LRNNX_DISC_BILINEAR = 2,  /* a = (1 + Delta A/2)/(1 - Delta A/2), g = Delta/(1 - Delta A/2) */
    LRNNX_DISC_DIRAC = 3      /* a = exp(Delta A), g = 1 */
} lrnnx_disc;

/* How the forward pass covers the time axis. */
typedef enum {
    LRNNX_PATH_AUTO = 0,         /* library chooses from B*D and L */
    LRNNX_PATH_SINGLE_PASS = 1,  /* one launch; each row walks its tiles in order, carrying the state */
    LRNNX_PATH_CHUNK_CARRY = 2   /* three launches: per-chunk aggregates, carry over chunks, apply; needs workspace */
} lrnnx_path;

/* State checkpoints: ckpt[b,d,c,n] (float, [B,D,ceil(L/interval),N]) is the state
 * x entering time step c*interval, i.e. x_{c*interval-1} (x0 or 0 for c = 0).
 * The forward pass can write them; the backward pass restarts its recomputation
 * from them.  The interval is a constant of the build.                        */
int64_t lrnnx_ckpt_interval(void);
/* Checkpoint slots per channel in packed variable-length mode: L / interval + B. */
int64_t lrnnx_packed_ckpt_slots(int64_t L, int64_t B);

/* ------------------------------------------------------------------ selective scan, forward
 * For every row (b,d), with s_l = delta[b,d,l] + delta_bias[d],
 * Delta_l = softplus(s_l) if delta_softplus else s_l, and (a,g) from `disc`:
 *     x_{l,n} = a(Delta_l, A[d,n]) x_{l-1,n} + g(Delta_l, A[d,n]) Bm[b,l,n] u[b,d,l]     (Eq. 2, line 1)
 *     ypre_l  = sum_n Cm[b,l,n] x_{l,n} + Dskip[d] u[b,d,l]                            (Eq. 2, line 2)
 *     y[b,d,l] = ypre_l * z[b,d,l] * sigmoid(z[b,d,l])   if z != NULL, else ypre_l
 * x_{-1} = x0[b,d,:] or 0.  Optional (NULL allowed): Dskip, delta_bias, z, x0, x_last, ckpt.
 * Grouped maps: with bc_groups = G > 1, Bm and Cm are [B,G,L,N] and channel d reads group d / (D/G)
 * (D must be a multiple of G); G = 0 or 1 is the plain [B,L,N] case.
 * Packed variable-length sequences: with cu_seqlens != NULL, B independent sequences lie one after the other on
 * ONE time axis of L steps, sequence b being steps cu_seqlens[b] .. cu_seqlens[b+1]-1 (each starts from x0[b] or 0,
 * nothing crosses a boundary; steps outside every sequence are not touched).  u, delta, z, y are then [D,L] (the
 * batch strides are ignored), Bm and Cm [G,L,N], x0 and x_last [B,D,N], and ckpt is
 * [D, lrnnx_packed_ckpt_slots(L,B), N].  Boundaries are clamped to [0,L] on the device; the single-pass path
 * is used (LRNNX_PATH_CHUNK_CARRY is refused).  Sequences may start anywhere: rows are read and written with vector
 * accesses at element alignment.
 * workspace is needed only by LRNNX_PATH_CHUNK_CARRY (AUTO falls back to the single
 * pass when it is missing or too small).                                              */
typedef struct lrnnx_ss_fwd_args {
    size_t struct_size;
    int32_t B, D, N;
    int32_t bc_groups;       /* number of Bm/Cm groups G; 0 or 1: none */
    int64_t L;
    int32_t io_dtype;        /* lrnnx_dtype */
    int32_t disc;            /* lrnnx_disc */
    int32_t delta_softplus;  /* 0 or 1 */
    int32_t path;            /* lrnnx_path */
    const int64_t *cu_seqlens;   /* packed variable-length mode: device memory [B+1], 8-byte aligned; or NULL */
    const void *u;      int64_t u_stride_b, u_stride_d;            /* [B,D,L] io */
    const void *delta;  int64_t delta_stride_b, delta_stride_d;    /* [B,D,L] io, raw (pre-bias, pre-softplus) */
    const float *A;                                                /* [D,N] */
    const void *Bm;                                                /* [B,L,N] io */
    const void *Cm;                                                /* [B,L,N] io */
    const float *Dskip;                                            /* [D] or NULL */
    const float *delta_bias;                                       /* [D] or NULL */
    const void *z;      int64_t z_stride_b, z_stride_d;            /* [B,D,L] io or NULL */
    const float *x0;                                               /* [B,D,N] or NULL */
    void *y;            int64_t y_stride_b, y_stride_d;            /* [B,D,L] io, out */
    float *x_last;                                                 /* [B,D,N] out or NULL: x_{L-1} */
    float *ckpt;                                                   /* [B,D,ceil(L/interval),N] out or NULL */
    void *workspace;    size_t workspace_bytes;
    void *stream;
} lrnnx_ss_fwd_args;

int lrnnx_selective_scan_fwd(const lrnnx_ss_fwd_args *args);

/* ------------------------------------------------------------------ selective scan, forward, complex diagonal A
 * The same recurrence with a complex diagonal state matrix and complex maps, the output taken as the real part:
 *     x_{l,n} = a(Delta_l, A[d,n]) x_{l-1,n} + g(Delta_l, A[d,n]) Bm[b,l,n] u[b,d,l]      (complex)
 *     ypre_l  = Re( sum_n Cm[b,l,n] x_{l,n} ) + Dskip[d] u[b,d,l],   then the optional gate as above
 * (Eq. 2 with y = Re(C x) + D u: the complex-diagonal layers of Sec. 2.2.1 with an input-dependent step size and
 * input-dependent maps; time-invariant maps are passed with every row equal).  u, delta, z, y, Dskip, delta_bias are
 * real as above.  A [D,N] complex float pairs; Bm, Cm [B,L,N] complex in io_dtype (interleaved re, im: bfloat16
 * pairs or float pairs), contiguous, 16-byte aligned ([B,G,L,N] with bc_groups = G > 1, as for the real scan);
 * x0, x_last [B,D,N] complex float pairs (optional).
 * a and g are the four schemes of lrnnx_disc in complex arithmetic.  Any Delta * Im(A) is accepted (whole
 * revolutions are dropped before the hardware sine and cosine); the phase of a step is as accurate as its fp32
 * product, |Delta Im(A)| * 2^-24 radians.
 * ckpt (optional): [B,D,ceil(L/lrnnx_ckpt_interval()),N] complex float pairs, the state entering every
 * lrnnx_ckpt_interval()-th step, for lrnnx_selective_scan_bwd_complex.  y may be NULL when only the checkpoints
 * (and x_last) are wanted.
 * Packed variable-length sequences (cu_seqlens != NULL) work as in lrnnx_selective_scan_fwd: u, delta, z, y are
 * [D,L], Bm and Cm [G,L,N], x0 and x_last [B,D,N], ckpt [D, lrnnx_packed_ckpt_slots(L,B), N]; boundaries are
 * clamped to [0,L] on the device.                                                                              */
typedef struct lrnnx_ss_fwd_complex_args {
    size_t struct_size;
    int32_t B, D, N;
    int32_t bc_groups;       /* number of Bm/Cm groups G (maps [B,G,L,N], channel d reads group d / (D/G), D a multiple of
                                G); 0 or 1: none */
    int64_t L;
    int32_t io_dtype, disc, delta_softplus;
    int32_t path;            /* lrnnx_path as in lrnnx_ss_fwd_args: CHUNK_CARRY = aggregate per chunk of the time axis,
                                chain, rerun from the true carry-in (three launches, for few rows and long sequences);
                                AUTO picks it then if the workspace allows; not with cu_seqlens */
    const int64_t *cu_seqlens;   /* packed variable-length mode, device memory [B+1], or NULL */
    const void *u;      int64_t u_stride_b, u_stride_d;
    const void *delta;  int64_t delta_stride_b, delta_stride_d;
    const void *A;                                                 /* [D,N] complex float */
    const void *Bm;                                                /* [B,L,N] complex io */
    const void *Cm;                                                /* [B,L,N] complex io */
    const float *Dskip;
    const float *delta_bias;
    const void *z;      int64_t z_stride_b, z_stride_d;
    const void *x0;                                                /* [B,D,N] complex float or NULL */
    void *y;            int64_t y_stride_b, y_stride_d;
    void *x_last;                                                  /* [B,D,N] complex float, out or NULL */
    void *ckpt;                                                    /* out or NULL */
    void *workspace;    size_t workspace_bytes;   /* needed by LRNNX_PATH_CHUNK_CARRY only: LRNNX_WS_FWD_COMPLEX */
    void *stream;
} lrnnx_ss_fwd_complex_args;

int lrnnx_selective_scan_fwd_complex(const lrnnx_ss_fwd_complex_args *args);

/* ------------------------------------------------------------------ selective scan, backward, complex diagonal A
 * Reverse-mode derivative of lrnnx_selective_scan_fwd_complex for an upstream gradient dy[B,D,L] (real): the
 * gradients of sum(dy * y).  The gradient with respect to a complex input q is dLoss/dRe q + i dLoss/dIm q (the
 * convention of complex automatic differentiation), stored as float pairs: dA [D,N], dBm, dCm [B,L,N],
 * dx0 [B,D,N].  du, ddelta, dz [B,D,L] in io_dtype and dD, dbias [D] float are real.  The states are recomputed
 * tile by tile from checkpoints (Sec. 3): `ckpt` is the array a forward call wrote for the same inputs; if NULL the
 * library first runs a state-only forward sweep into `workspace`
 * (lrnnx_workspace_bytes(LRNNX_WS_BWD_COMPLEX, B, D, N, L, io_dtype), which also covers the chunked path's
 * aggregates).  dA, dBm, dCm, dD, dbias are OVERWRITTEN (cleared on the stream, then accumulated with atomics: their
 * last bits may differ from run to run).
 * Optional (NULL allowed): Dskip, delta_bias, z, x0, ckpt, dD, dbias, dz, dx0.  dD requires Dskip, dbias requires
 * delta_bias, dz requires z.  Alignment: Bm, Cm, dBm, dCm 16 bytes; A, x0, ckpt, dA, dx0 8 bytes.              */
typedef struct lrnnx_ss_bwd_complex_args {
    size_t struct_size;
    int32_t B, D, N;
    int32_t bc_groups;                                             /* as in the forward call (then dBm, dCm are [B,G,L,N]); 0 or 1: none */
    int64_t L;
    int32_t io_dtype, disc, delta_softplus;
    int32_t path;                /* lrnnx_path, as in lrnnx_ss_bwd_args: CHUNK_CARRY cuts the time axis into chunks
                                    that run side by side; its aggregates (2 * B * D * chunks * N float pairs) go into
                                    the workspace, after the 256-byte-aligned checkpoints of the recompute sweep if
                                    ckpt == NULL */
    const int64_t *cu_seqlens;   /* packed mode as in the forward call (then du, ddelta, dz are [D,L], dBm, dCm
                                    [G,L,N], ckpt [D, lrnnx_packed_ckpt_slots(L,B), N]), or NULL */
    int64_t max_seqlen;          /* packed mode: the longest sequence of the batch if the caller knows it, else 0; as
                                    in lrnnx_ss_bwd_args */
    const void *u;      int64_t u_stride_b, u_stride_d;
    const void *delta;  int64_t delta_stride_b, delta_stride_d;
    const void *A;                                                 /* [D,N] complex float */
    const void *Bm;                                                /* [B,L,N] complex io */
    const void *Cm;                                                /* [B,L,N] complex io */
    const float *Dskip;
    const float *delta_bias;
    const void *z;      int64_t z_stride_b, z_stride_d;
    const void *x0;                                                /* [B,D,N] complex float or NULL */
    const void *dy;     int64_t dy_stride_b, dy_stride_d;          /* [B,D,L] io */
    const void *ckpt;                                              /* from the forward call, or NULL */
    void *du;           int64_t du_stride_b, du_stride_d;          /* [B,D,L] io, out */
    void *ddelta;       int64_t ddelta_stride_b, ddelta_stride_d;  /* [B,D,L] io, out */
    void *dz;           int64_t dz_stride_b, dz_stride_d;          /* [B,D,L] io, out or NULL */
    void *dA;                                                      /* [D,N] complex float, out */
    void *dBm;                                                     /* [B,L,N] complex float, out */
    void *dCm;                                                     /* [B,L,N] complex float, out */
    float *dD;                                                     /* [D] out or NULL */
    float *dbias;                                                  /* [D] out or NULL */
    void *dx0;                                                     /* [B,D,N] complex float, out or NULL */
    void *workspace;    size_t workspace_bytes;                    /* LRNNX_WS_BWD_COMPLEX */
    void *stream;
} lrnnx_ss_bwd_complex_args;

int lrnnx_selective_scan_bwd_complex(const lrnnx_ss_bwd_complex_args *args);

/* ------------------------------------------------------------------ selective scan, backward
 * Reverse-mode derivative of lrnnx_selective_scan_fwd (real A) for an upstream gradient dy[B,D,L]:
 * the gradients of sum(dy * y) with respect to u, the raw delta, A, Bm, Cm, Dskip,
 * delta_bias, z and x0.  The state is recomputed tile by tile from checkpoints and
 * never stored per step (Sec. 3).  `ckpt` is the array a forward call wrote for the
 * same inputs; if NULL the library first runs a state-only forward sweep into
 * `workspace`.  lrnnx_workspace_bytes(LRNNX_WS_BWD, ...) covers that sweep and the chunk aggregates of the
 * chunked path (`path`); with `ckpt` given, LRNNX_WS_BWD_CARRY bytes are enough for the latter, and with a
 * workspace too small for it (or none) the call runs as a single pass.
 * Outputs du, ddelta, dz: io_dtype, written once each.  dA[D,N], dBm, dCm[B,L,N],
 * dD[D], dbias[D]: float, OVERWRITTEN (the library clears them on the stream, then
 * accumulates with atomics: their last bits may differ from run to run).
 * dx0[B,D,N] float.  Optional (NULL allowed): Dskip, delta_bias, z, x0, ckpt, dD,
 * dbias, dz, dx0.  dD requires Dskip, dbias requires delta_bias, dz requires z.    */
typedef struct lrnnx_ss_bwd_args {
    size_t struct_size;
    int32_t B, D, N;
    int32_t bc_groups;                                             /* as in the forward call; 0 or 1: none */
    int64_t L;
    int32_t io_dtype, disc, delta_softplus;
    int32_t path;                /* lrnnx_path.  CHUNK_CARRY: the time axis is cut into chunks that run side by side
                                    (three launches: adjoint aggregate per chunk, chain, backward per chunk), for long
                                    sequences with few rows; needs the workspace.  SINGLE_PASS: one workgroup walks a
                                    whole row.  AUTO picks CHUNK_CARRY when a single pass would leave most of the chip
                                    idle and the workspace allows it.  With cu_seqlens every sequence is cut into
                                    chunks of one size counted from its own start (the last chunk of a sequence takes
                                    what is left), planned for B sequences of max_seqlen steps (of L steps if that is
                                    0) and for no more chunks than the workspace holds; AUTO then picks CHUNK_CARRY
                                    only when max_seqlen is given. */
    const int64_t *cu_seqlens;   /* as in the forward call (then dBm, dCm are [G,L,N]), or NULL.  In packed mode the
                                    workspace also holds B ints that let the launch start the longest sequences first
                                    (batches of up to 256 sequences), which shortens its tail; a workspace without
                                    room for them is accepted and the launch keeps the caller's order. */
    int64_t max_seqlen;          /* packed mode: the longest sequence of the batch (steps) if the caller knows it,
                                    else 0.  A hint for the launch shape only, never for addressing: with it the
                                    workgroups of sequences much longer than the average take fewer channels each, so
                                    that one long sequence does not set the time of the whole launch; a value that is
                                    too small only loses that balance, a value that is too large costs some idle
                                    workgroups.  The chunks of CHUNK_CARRY are planned from it as well (see path).
                                    Ignored without cu_seqlens. */
    const void *u;      int64_t u_stride_b, u_stride_d;
    const void *delta;  int64_t delta_stride_b, delta_stride_d;
    const float *A;
    const void *Bm;
    const void *Cm;
    const float *Dskip;
    const float *delta_bias;
    const void *z;      int64_t z_stride_b, z_stride_d;
    const float *x0;
    const void *dy;     int64_t dy_stride_b, dy_stride_d;          /* [B,D,L] io */
    const float *ckpt;                                             /* from the forward call, or NULL */
    void *du;           int64_t du_stride_b, du_stride_d;          /* [B,D,L] io, out */
    void *ddelta;       int64_t ddelta_stride_b, ddelta_stride_d;  /* [B,D,L] io, out */
    void *dz;           int64_t dz_stride_b, dz_stride_d;          /* [B,D,L] io, out or NULL */
    float *dA;                                                     /* [D,N] out */
    float *dBm;                                                    /* [B,L,N] ([B,G,L,N] if grouped) out */
    float *dCm;                                                    /* same shape as dBm, out */
    float *dD;                                                     /* [D] out or NULL */
    float *dbias;                                                  /* [D] out or NULL */
    float *dx0;                                                    /* [B,D,N] out or NULL */
    void *workspace;    size_t workspace_bytes;                    /* LRNNX_WS_BWD, or LRNNX_WS_BWD_CARRY with ckpt */
    void *stream;
} lrnnx_ss_bwd_args;

int lrnnx_selective_scan_bwd(const lrnnx_ss_bwd_args *args);

/* ------------------------------------------------------------------ LTI complex-diagonal scan
 *     x[b,k,p] = lambda[p] * x[b,k-1,p] + v[b,k,p]        (Eq. 2 with constant diagonal A; Sec. 2.2.1)
 * for complex numbers stored as interleaved (re, im) float pairs.  v_k = Bbar u_k is
 * the caller's (a dense projection); the call returns the state at every step.
 * lambda[P], v and x [B,L,P] (P contiguous), x0 and x_last [B,P] (optional, NULL
 * allowed).  x may alias v.  workspace: lrnnx_workspace_bytes(LRNNX_WS_LTI, B, P, 0, L, 0); its contents on entry
 * do not matter (the library clears what it uses on the stream).  The single-launch path chains workgroups
 * through values published in global memory, with bounded waits; should a wait ever run out, the states from that point of
 * that sequence on are written as NaN rather than left plausible, and *chain_status (if given) is set to 1.  */
typedef struct lrnnx_lti_args {
    size_t struct_size;
    int32_t B, P;
    int64_t L;
    int32_t path;            /* lrnnx_path: AUTO / SINGLE_PASS = one launch with look-back between time groups;
                                CHUNK_CARRY = two launches */
    int32_t reserved;
    const void *lambda;
    const void *v;
    const void *x0;
    void *x;
    void *x_last;
    int32_t *chain_status;   /* device memory or NULL: set to 1 if a bounded wait of the single-launch path ran out
                                (never cleared by the library: clear it before the call) */
    void *workspace;    size_t workspace_bytes;
    void *stream;
} lrnnx_lti_args;

int lrnnx_lti_diag_scan(const lrnnx_lti_args *args);

/* ------------------------------------------------------------------ LTI scan without a caller's workspace
 * For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation): the single-launch scan of lrnnx_lti_diag_scan with its chain workspace taken from a
 * scratch array of LRNNX_STATIC_SCRATCH_BYTES bytes that is part of the library's device image (every GPU the
 * library runs on holds its own copy until the process ends).  Same struct, same results bit for bit; `workspace`
 * and `workspace_bytes` are ignored, `path` must be AUTO or SINGLE_PASS.  The call allocates and frees nothing
 * (neither does any other entry point; this one also needs no buffer beyond inputs and outputs).  Shapes whose
 * chain needs more than the array (lrnnx_workspace_bytes(LRNNX_WS_LTI, B, P, 0, L, 0) is an upper bound of the
 * need; roughly B * P * L / 15 bytes) are refused with LRNNX_ERR_WORKSPACE and nothing is launched.  All calls on
 * one GPU share that GPU's array: the library re-arms it on the stream at the start of every call, and two calls
 * whose execution overlaps on one GPU (different streams) race on it; calls on one stream are safe.              */
#define LRNNX_STATIC_SCRATCH_BYTES (4u << 20)
size_t lrnnx_static_scratch_bytes(void);
int lrnnx_lti_diag_scan_static(const lrnnx_lti_args *args);

/* ------------------------------------------------------------------ diagonal scan with caller-supplied coefficients
 *     x[b,k,p] = a[b,k,p] * x[b,k-1,p] + b[b,k,p]
 * Eq. 2 with A(k) = diag(a_k) and the input term b_k = B(k) u_k already formed: the recurrence of the
 * time-varying S5-style layers (Sec. 2.2.2), of gated real recurrences, and of event-driven discretisation
 * (Sec. 3), whose gates, step sizes and projections are the caller's.  dtype LRNNX_F32: real floats;
 * LRNNX_C64: complex numbers as interleaved (re, im) float pairs.  a, b, x: [B,L,P], P contiguous, device memory
 * aligned to the element size; x may alias b (not a).  x0, x_last: [B,P] or NULL.  Results are bitwise
 * reproducible.  workspace: lrnnx_workspace_bytes(LRNNX_WS_DIAG, B, P, 0, L, dtype), contents on entry
 * irrelevant.  Like the LTI scan, a bounded wait that runs out yields NaN states, never plausible wrong ones. */
typedef struct lrnnx_diag_scan_args {
    size_t struct_size;
    int32_t B, P;
    int64_t L;
    int32_t dtype, reserved;    /* LRNNX_F32 or LRNNX_C64 */
    const void *a;
    const void *b;
    const void *x0;
    void *x;
    void *x_last;
    int32_t *chain_status;      /* as in lrnnx_lti_args, or NULL */
    void *workspace;    size_t workspace_bytes;
    void *stream;
} lrnnx_diag_scan_args;

int lrnnx_diag_scan(const lrnnx_diag_scan_args *args);

/* ------------------------------------------------------------------ backward of lrnnx_diag_scan
 * For a real loss, with gx[b,k,p] the gradient reaching x[b,k,p] (complex data: dLoss/dRe + i dLoss/dIm, the chain
 * rule then multiplies by conjugates; real data: no conjugates):
 *     g_k  = gx_k + conj(a_{k+1}) g_{k+1}   (g beyond the last step is 0),
 *     db_k = g_k,    da_k = conj(x_{k-1}) g_k   (x_{-1} = x0),    dx0 = conj(a_0) g_0.
 * x is the array the forward call wrote, a and x0 the forward call's.  All of a, x, gx, da, db are [B,L,P] of
 * `dtype` (LRNNX_F32 or LRNNX_C64), contiguous, aligned to the element size; db may alias gx; da must not alias an
 * input.  dx0 [B,P] or NULL.  Results are bitwise reproducible.  workspace:
 * lrnnx_workspace_bytes(LRNNX_WS_DIAG_BWD, B, P, 0, L, dtype), contents on entry irrelevant.                  */
typedef struct lrnnx_diag_scan_bwd_args {
    size_t struct_size;
    int32_t B, P;
    int64_t L;
    int32_t dtype, reserved;
    const void *a;          /* [B,L,P] */
    const void *x;          /* [B,L,P] forward states */
    const void *x0;         /* [B,P] or NULL */
    const void *gx;         /* [B,L,P] */
    void *da;               /* [B,L,P] out */
    void *db;               /* [B,L,P] out */
    void *dx0;              /* [B,P] out or NULL */
    int32_t *chain_status;  /* as in lrnnx_lti_args, or NULL */
    void *workspace;    size_t workspace_bytes;
    void *stream;
} lrnnx_diag_scan_bwd_args;

int lrnnx_diag_scan_bwd(const lrnnx_diag_scan_bwd_args *args);

/* ------------------------------------------------------------------ backward of the LTI scan
 * Adjoint of the recurrence above (Sec. 2.2.1; the paper trains these layers through the same scan).  For a real
 * loss, the gradient of a complex quantity q is dLoss/dRe(q) + i dLoss/dIm(q) (the convention of complex
 * autograd).  With gx[b,k,p] the gradient reaching x[b,k,p] from the layers above:
 *     g_k  = gx_k + conj(lambda) g_{k+1}  (g beyond the last step is 0),   dv_k = g_k,
 *     dx0  = conj(lambda) g_first,        dlambda[p] = sum_b sum_k conj(x[b,k-1,p]) g[b,k,p]   (x[b,-1] = x0).
 * x is the array the forward call wrote (states are not recomputed), x0 the forward call's (NULL = zero).
 * gx and dv [B,L,P], dv may alias gx; dlambda[P] is OVERWRITTEN (cleared on the stream, then accumulated with
 * float atomics: its last bits may differ from run to run; dv and dx0 are bitwise reproducible); dx0 [B,P] or NULL.
 * All arrays device memory, 8-byte aligned, contiguous.  workspace:
 * lrnnx_workspace_bytes(LRNNX_WS_LTI_BWD, B, P, 0, L, 0), contents on entry irrelevant.                          */
typedef struct lrnnx_lti_bwd_args {
    size_t struct_size;
    int32_t B, P;
    int64_t L;
    const void *lambda;     /* [P] */
    const void *x;          /* [B,L,P] forward states */
    const void *x0;         /* [B,P] or NULL */
    const void *gx;         /* [B,L,P] */
    void *dv;               /* [B,L,P] out */
    void *dlambda;          /* [P] out */
    void *dx0;              /* [B,P] out or NULL */
    int32_t *chain_status;  /* as in lrnnx_lti_args, or NULL */
    void *workspace;    size_t workspace_bytes;
    void *stream;
} lrnnx_lti_bwd_args;

int lrnnx_lti_diag_scan_bwd(const lrnnx_lti_bwd_args *args);

/* ------------------------------------------------------------------ single-token updates
 * The `step` method of the paper's layers (Sec. 3, "Library Design": every layer implements a step for
 * autoregressive generation): one application of Eq. 2 to a carried state.
 *
 * lrnnx_selective_step: x[B,D,N] (float, updated IN PLACE) <- a (.) x + g Bm[b,:] u[b,d], and
 * y[b,d] = Cm[b,:] . x[b,d,:] + Dskip[d] u[b,d], times z sigmoid(z) if z != NULL; same Delta transform and
 * discretisations as the scan.  u, delta, z, y are [B,D] in io_dtype with element strides (so a time slice
 * of a [B,D,L] tensor can be passed); Bm, Cm are contiguous [B,N] in io_dtype.  L calls reproduce
 * lrnnx_selective_scan_fwd on L steps up to fp32 rounding.  Optional: Dskip, delta_bias, z.
 * With bc_groups = G > 1, Bm and Cm are [B,G,N] and channel d reads group d / (D/G), as in the scan. */
typedef struct lrnnx_ss_step_args {
    size_t struct_size;
    int32_t B, D, N;
    int32_t bc_groups;      /* G > 1: Bm, Cm are [B,G,N] and channel d reads group d / (D/G); 0 or 1: none */
    int32_t io_dtype, disc, delta_softplus, reserved;
    float *x;
    const void *u;      int64_t u_stride_b, u_stride_d;
    const void *delta;  int64_t delta_stride_b, delta_stride_d;
    const float *A;
    const void *Bm;
    const void *Cm;
    const float *Dskip;
    const float *delta_bias;
    const void *z;      int64_t z_stride_b, z_stride_d;
    void *y;            int64_t y_stride_b, y_stride_d;
    void *stream;
} lrnnx_ss_step_args;

int lrnnx_selective_step(const lrnnx_ss_step_args *args);

/* lrnnx_selective_step_complex: the same single-token update for the scan with a complex diagonal A
 * (lrnnx_selective_scan_fwd_complex): x[B,D,N] complex float pairs, updated IN PLACE; A [D,N] complex float pairs;
 * Bm, Cm contiguous [B,N] complex in io_dtype (interleaved re, im); y[b,d] = Re(Cm[b,:] . x[b,d,:]) + Dskip[d] u[b,d],
 * gated as above.  x, A, Bm, Cm must be 16-byte aligned.  L calls reproduce the scan on L steps up to fp32
 * rounding.  Optional: Dskip, delta_bias, z.                                                                     */
typedef struct lrnnx_ss_step_complex_args {
    size_t struct_size;
    int32_t B, D, N;
    int32_t bc_groups;      /* G > 1: Bm, Cm are [B,G,N] and channel d reads group d / (D/G); 0 or 1: none */
    int32_t io_dtype, disc, delta_softplus, reserved;
    void *x;                                                       /* [B,D,N] complex float, in/out */
    const void *u;      int64_t u_stride_b, u_stride_d;
    const void *delta;  int64_t delta_stride_b, delta_stride_d;
    const void *A;                                                 /* [D,N] complex float */
    const void *Bm;                                                /* [B,N] complex io */
    const void *Cm;                                                /* [B,N] complex io */
    const float *Dskip;
    const float *delta_bias;
    const void *z;      int64_t z_stride_b, z_stride_d;
    void *y;            int64_t y_stride_b, y_stride_d;
    void *stream;
} lrnnx_ss_step_complex_args;

int lrnnx_selective_step_complex(const lrnnx_ss_step_complex_args *args);

/* lrnnx_lti_step: x[B,P] (complex64, IN PLACE) <- lambda[P] (.) x + v[B,P]. */
typedef struct lrnnx_lti_step_args {
    size_t struct_size;
    int32_t B, P;
    const void *lambda;
    void *x;
    const void *v;
    void *stream;
} lrnnx_lti_step_args;

int lrnnx_lti_step(const lrnnx_lti_step_args *args);

/* ------------------------------------------------------------------ queries (host only, no GPU needed) */
typedef enum { LRNNX_WS_FWD = 0, LRNNX_WS_BWD = 1, LRNNX_WS_LTI = 2, LRNNX_WS_LTI_BWD = 3, LRNNX_WS_DIAG = 4,
               LRNNX_WS_DIAG_BWD = 5, LRNNX_WS_BWD_COMPLEX = 6,
               LRNNX_WS_BWD_CARRY = 7,  /* the chunk aggregates of lrnnx_selective_scan_bwd alone (ckpt supplied) */
               LRNNX_WS_FWD_COMPLEX = 8
             } lrnnx_ws_kind;

/* Bytes of device scratch the call may need (the largest over its paths).  bc_groups as in the call's struct (0 or 1:
 * none); packed != 0: the call will be given cu_seqlens (B sequences on one time axis of L steps; the backward kinds
 * then cover the checkpoints of the recompute sweep in the packed layout, and the larger of the B ints of the launch
 * order and the chunk aggregates as planned for sequences of L steps).
 * For LRNNX_WS_LTI, LRNNX_WS_LTI_BWD, LRNNX_WS_DIAG and LRNNX_WS_DIAG_BWD pass P as D and 0 for N, bc_groups and packed
 * (the DIAG kinds: io_dtype is LRNNX_F32 or LRNNX_C64).  Returns 0 for invalid sizes and for calls that need none.   */
size_t lrnnx_workspace_bytes(int which, int64_t B, int64_t D, int64_t N, int64_t L, int io_dtype, int bc_groups,
                             int packed);

/* Number of chunks lrnnx_selective_scan_bwd (complex_a = 0) or lrnnx_selective_scan_bwd_complex (complex_a = 1) cuts
 * the time axis into for these sizes and this `path` when its workspace allows it (1: single pass); the aggregates
 * then take 2 * B * D * chunks * N floats (float pairs for the complex scan) of the workspace.  0 for invalid sizes. */
int lrnnx_selective_scan_bwd_chunks(int64_t B, int64_t D, int64_t N, int64_t L, int bc_groups, int path, int complex_a);

/* The same for lrnnx_selective_scan_fwd_complex: chunks of its chunk-carry path (1: single pass); the aggregates take
 * 2 * B * D * chunks * N float pairs of the workspace.                                                          */
int lrnnx_selective_scan_fwd_complex_chunks(int64_t B, int64_t D, int64_t N, int64_t L, int bc_groups, int path);

const char *lrnnx_status_string(int status);
int lrnnx_version(void);   /* major * 100 + minor; the major number changes with any struct layout */

#ifdef __cplusplus
}
#endif
#endif /* LRNNX_H */
