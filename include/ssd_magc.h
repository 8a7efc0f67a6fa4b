/*
 * ssd_magc.h -- C ABI of the MI355X (gfx950) selective state-space scan with Multi-Axis
 * Gradient Checkpointing.
 *
 * One SSD layer computes, for every (batch b, head h) with g the B/C group of h
 * (paper Sec. 3.1, Eq. 1, in the Mamba-2 form: the transition is exp(dt_t*A_h) times the
 * identity, the input matrix is dt_t*B_t, and the output carries a skip term D_h*x_t):
 *
 *     h_t[p,n]   = exp(dt[b,t,h]*A[h]) * h_{t-1}[p,n] + dt[b,t,h] * x[b,t,h,p] * B[b,t,g,n]
 *     y[b,t,h,p] = sum_n C[b,t,g,n] * h_t[p,n] + D[h] * x[b,t,h,p]
 *
 * The sequence is cut into segments of `segment` tokens (the last one shorter when seqlen is not a
 * multiple of segment; nseg = ceil(seqlen / segment) below).  The forward pass keeps only the
 * state entering each segment (the sequence-axis checkpoints of Sec. 3.2/3.3, Alg. 1); the
 * backward pass walks the segments right to left, restores each segment's per-chunk states
 * from its checkpoint and back-propagates through it, handing the state adjoint to the segment
 * on its left (Alg. 2).  Because a state depends only on its predecessor (Sec. 3.2) this is
 * exact: results do not depend on `segment` beyond floating-point summation order.
 *
 * General conventions
 *   - Every data pointer is a DEVICE pointer unless its comment says "host".  The caller owns
 *     all buffers; the library never allocates or frees device memory and never blocks the host.
 *     All work is ordered after what is already in `hip_stream` (a hipStream_t passed as void*;
 *     NULL = the default stream) and before anything enqueued there after the call returns; with
 *     more than one segment part of it runs on a library-owned stream of default priority, forked
 *     from and joined back into `hip_stream` with events (created, under a lock, on the first such call
 *     on a device or by ssd_init; make that first call outside stream capture).
 *     Setting SSD_MAGC_SERIAL=1 in the environment keeps everything on `hip_stream` (diagnostics).
 *     Those streams and events exist once per device: calls on one device must not overlap in time
 *     across host threads (calls on different devices, or one after the other, are fine).
 *   - Tensors are dense row-major with the index order written in brackets; the batch stride
 *     may be overridden through ssd_shape_t (elements, 0 = dense) so that a token range of a
 *     longer sequence can be passed as a pointer offset.
 *   - `dtype` is the storage type of x, dt, B, C, y and of dy, dx, ddt, dB, dC.  A, D, every
 *     state and state adjoint, dA and dD are always fp32 (App. C keeps SSM states in fp32).
 *     Arithmetic accumulates in fp32; outputs are rounded once (nearest-even).
 *   - Every entry point returns 0 on success or a negative ssd_status_t.  Arguments are
 *     validated before anything is launched; on a validation error nothing was enqueued and no
 *     output was touched.  SSD_ERR_LAUNCH reports a failed HIP call (outputs undefined; work already
 *     enqueued, possibly on a library stream, may still be running: synchronise the device before
 *     releasing the buffers of that call).
 *     No C++ exception crosses this boundary.
 */
#ifndef SSD_MAGC_H
#define SSD_MAGC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum ssd_dtype_t { SSD_F32 = 0, SSD_BF16 = 1 } ssd_dtype_t;

typedef enum ssd_status_t {
    SSD_OK = 0,
    SSD_ERR_NULL = -1,         /* a required pointer is NULL */
    SSD_ERR_SHAPE = -2,        /* a dimension is non-positive or exceeds a kernel limit */
    SSD_ERR_DIVISIBILITY = -3, /* nheads % ngroups or segment % chunk is not 0 (stack: seqlen % segment) */
    SSD_ERR_DTYPE = -4,        /* unknown dtype */
    SSD_ERR_WORKSPACE = -5,    /* workspace NULL, misaligned (256 B) or smaller than ssd_workspace_bytes */
    SSD_ERR_LAUNCH = -6,       /* a HIP call failed; see hipGetLastError */
    SSD_ERR_BUDGET = -7,       /* magc_plan: no admissible (l, s) fits the budget (min-memory plan returned) */
    SSD_ERR_ARG = -8           /* any other invalid argument */
} ssd_status_t;

/* Shape of one SSD layer call.  Limits: chunk in [1, 1024]; headdim, dstate in [1, 256]. */
typedef struct ssd_shape_t {
    int32_t dtype;            /* ssd_dtype_t */
    int32_t nheads;           /* H */
    int32_t headdim;          /* P */
    int32_t ngroups;          /* G; H % G == 0; head h uses group h / (H/G) */
    int32_t dstate;           /* N */
    int32_t chunk;            /* Q: block length of the dual (quadratic) form; segment % Q == 0 */
    int64_t batch;            /* Bt */
    int64_t seqlen;           /* L (the paper's S), any length >= 0: a short last segment (and a short last chunk
                                 inside it) is run on zero-padded copies kept in the workspace; the stack driver
                                 needs L % segment == 0 */
    int64_t segment;          /* s: sequence-axis checkpoint interval; s >= L means no checkpoints */
    int64_t x_batch_stride;   /* elements between batches of x, y, dy, dx      (0 = L*H*P) */
    int64_t dt_batch_stride;  /* elements between batches of dt, ddt           (0 = L*H)   */
    int64_t bc_batch_stride;  /* elements between batches of B, C, dB, dC      (0 = L*G*N) */
    const uint8_t* seq_reset; /* optional, device, [Bt, L] (dense): packed sequences.  A token with a non-zero
                                 flag starts a new sequence: its decay factor exp(dt A) carries an extra
                                 exp(-100) (< 4e-44), i.e. the state from the tokens before it is cut off --
                                 in y, in the states and in every gradient.  NULL: one sequence per batch row.
                                 Not used by the stack driver. */
} ssd_shape_t;

/* Flags for ssd_fwd / ssd_bwd. */
enum {
    SSD_FLAG_RESIDUAL = 1,        /* fwd: y = x + SSD(x);  bwd: dx = dy + VJP(dy)  (the residual stack's layer) */
    SSD_FLAG_ACCUM_PARAM = 2,     /* bwd: dA, dD are added to instead of overwritten */
    SSD_FLAG_GENERIC_KERNELS = 4, /* force the shape-generic fp32-FMA kernels even where the MFMA path applies */
    SSD_FLAG_BF16_CHECKPOINTS = 8, /* boundary_states holds bf16 instead of fp32 elements: half the S-checkpoint
                                     term of App. C (Tab. 7 counts an fp32 state element as two); see ssd_fwd */
    SSD_FLAG_FP32_CHUNK_STATES = 16 /* matrix-core kernels only (ignored by the shape-generic ones, which always do):
                                     the per-chunk states and local state adjoints that feed the two state scans
                                     are kept in fp32 inside the workspace (App. C: SSM states in fp32).  Default:
                                     bf16, rounded once from the fp32 accumulators -- the running state of a scan
                                     is fp32 in registers either way, and the states the contractions read are
                                     bf16 matrix-core operands either way.  Costs 4 more bytes per state element
                                     and chunk in each direction; ssd_workspace_bytes_flags accounts for it. */
};

/* Bytes of scratch the call needs for this shape (device memory, 256-byte aligned, contents
 * undefined before and after).  It scales with `segment`, not with `seqlen`: this is the
 * per-segment recomputation store (the M_state term of App. C) -- one per segment in flight, up
 * to four when the sequence has that many segments -- plus, for the backward pass, eight
 * bytes per (chunk, head) of the whole sequence for the partial sums of dA and dD.
 * Returns 0 for an invalid shape.  The figure is for flags = 0; a call that passes
 * SSD_FLAG_GENERIC_KERNELS needs ssd_workspace_bytes_flags (the shape-generic kernels keep their
 * chunk states in fp32 and lay the scratch out differently). */
size_t ssd_workspace_bytes(const ssd_shape_t* shape, int32_t is_backward);
/* The same for a call made with `flags` (SSD_FLAG_GENERIC_KERNELS and SSD_FLAG_FP32_CHUNK_STATES change the result). */
size_t ssd_workspace_bytes_flags(const ssd_shape_t* shape, int32_t is_backward, uint32_t flags);

/*
 * Forward (Layer_j(x, h) -> (x, h) of Alg. 1, for one layer over the whole sequence).
 *   x  [Bt,L,H,P] dtype      dt [Bt,L,H] dtype (already positive; no bias or softplus is applied)
 *   A  [H] fp32              B, C [Bt,L,G,N] dtype          D [H] fp32
 *   init_state      [Bt,H,P,N] fp32, or NULL for zeros
 *   y               [Bt,L,H,P] dtype, overwritten
 *   final_state     [Bt,H,P,N] fp32, overwritten; may be NULL
 *   boundary_states [Bt, nseg, H, P, N] fp32, overwritten; slot k holds the state entering
 *                   segment k (slot 0 = init_state or zeros).  NULL: forward only (prefill) -- no
 *                   checkpoint is kept, the state travels from segment to segment inside the
 *                   workspace and memory use is independent of L; a later ssd_bwd is then possible
 *                   only with segment >= L.
 *                   Under SSD_FLAG_BF16_CHECKPOINTS the buffer holds [Bt, nseg, H, P, N] bf16 elements:
 *                   each checkpoint is the fp32 state rounded once (to nearest even).  The forward
 *                   pass itself still hands the fp32 state from segment to segment, so y and
 *                   final_state do not depend on the flag; ssd_bwd, given the same flag, restarts
 *                   every segment but the first from the rounded state (segment 0 from init_state).
 */
int ssd_fwd(const ssd_shape_t* shape, const void* x, const void* dt, const float* A, const void* B,
            const void* C, const float* D, const float* init_state, void* y, float* final_state,
            void* boundary_states, void* workspace, size_t workspace_bytes, uint32_t flags,
            void* hip_stream);

/*
 * ssd_fwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as ssd_fwd
 * minus the workspace: the per-segment scratch is a device array inside the library,
 * SSD_STATIC_SCRATCH_MIB MiB per GPU, held by every GPU the library runs on until the process ends.
 *   - A shape whose scratch (ssd_fwd_static_bytes; one segment at a time) exceeds the array is rejected
 *     with SSD_ERR_WORKSPACE before anything is launched: use ssd_fwd with a workspace instead.  The
 *     2.7B layer shape with 4096-token segments fits.
 *   - The call allocates nothing, frees nothing, creates no stream or event and never synchronises; every
 *     kernel is enqueued on hip_stream, one segment after the other.  The array's device address is
 *     looked up on the first call on each device (or by ssd_init with that device current); make that
 *     first call, or ssd_init, outside graph capture.
 *   - All calls on one GPU share that GPU's array, which keeps the previous call's contents (nothing in it
 *     has to start at zero: each part is written before it is read within a call).  Calls that overlap
 *     in time on one GPU -- from different streams or host threads -- race on it and give wrong results;
 *     calls ordered on one stream, or on different GPUs, are fine.
 * ssd_init: optional, idempotent, thread-safe set-up for the current device (the array's address and the
 * library's own streams and events); returns SSD_OK or SSD_ERR_LAUNCH.
 */
#define SSD_STATIC_SCRATCH_MIB 40
int ssd_init(void);
size_t ssd_fwd_static_bytes(const ssd_shape_t* shape, uint32_t flags); /* 0 for an invalid shape */
int ssd_fwd_static(const ssd_shape_t* shape, const void* x, const void* dt, const float* A, const void* B,
                   const void* C, const float* D, const float* init_state, void* y, float* final_state,
                   void* boundary_states, uint32_t flags, void* hip_stream);

/*
 * Recurrent form (Sec. 3.1, Eq. 1, token by token): for t = 0 .. seqlen-1
 *     state <- exp(dt_t A) state + dt_t x_t (x) B_t ;   y_t = C_t state + D x_t
 * The constant-memory step that continues a sequence after a prefill by ssd_fwd (whose
 * final_state is this call's state); seqlen = 1 is single-token generation.
 *   shape: dtype, batch, seqlen (tokens in this call, >= 0), nheads, headdim, ngroups, dstate and
 *          the batch strides are used; chunk and segment are ignored
 *   x, y [Bt,T,H,P] dtype; dt [Bt,T,H] dtype; B, C [Bt,T,G,N] dtype; A, D [H] fp32 (all device)
 *   state [Bt,H,P,N] fp32, device, updated in place (never NULL)
 *   flags: SSD_FLAG_RESIDUAL only (y = x + layer(x))
 * Needs no workspace and allocates nothing; work is enqueued on hip_stream.  Errors as elsewhere.
 */
int ssd_decode(const ssd_shape_t* shape, const void* x, const void* dt, const float* A, const void* B,
               const void* C, const float* D, float* state, void* y, uint32_t flags, void* hip_stream);

/*
 * The block's causal depthwise convolution (kernel 4) + bias + SiLU in front of the scan, with the
 * three-token state that a sequence checkpoint holds next to the SSM state (App. C, Tab. 7: the
 * per-checkpoint constant is the SSM state plus three tokens of the convolution's channels).  Like the
 * scan, a segment restarts exactly from its stored state:
 *     pre[t,c] = bias[c] + sum_{k=0..3} w[c,k] u[t-3+k, c],   u[-3..-1] = state_in (zeros if NULL)
 *     out[t,c] = pre / (1 + exp(-pre));    state_out = the last three rows of [state_in ; u]
 *   u, out, dout, du [Bt,L,C] dtype (batch stride overridable, 0 = L*C); w [C,4] fp32; bias [C] fp32 or NULL
 *   state_in, state_out [Bt,3,C] dtype (oldest row first), either may be NULL
 * Backward: gradients of <dout, out> + <dstate_out, state_out>.
 *   dstate_out, dstate_in [Bt,3,C] fp32, either may be NULL; dw [C,4], dbias [C] (may be NULL) fp32,
 *   overwritten, or added to under SSD_FLAG_ACCUM_PARAM (the only flag); du must not alias dout.
 *   workspace: ssd_conv1d_workspace_bytes bytes, 256-byte aligned (partial sums of dw and dbias).
 * All pointers are device pointers; nothing is allocated; work is enqueued on hip_stream.
 */
typedef struct ssd_conv_shape_t {
    int32_t dtype;         /* ssd_dtype_t of u, out, dout, du and the states */
    int32_t channels;      /* C */
    int64_t batch;         /* Bt */
    int64_t seqlen;        /* L >= 0 (an empty segment hands the state on) */
    int64_t batch_stride;  /* elements between batches of u, out, dout, du (0 = dense) */
    int64_t u_row_stride;  /* elements between tokens of u and du (0 = C): u may be a column slice of a wider
                              tensor (the input projection's output); out and dout are always dense */
} ssd_conv_shape_t;

size_t ssd_conv1d_workspace_bytes(const ssd_conv_shape_t* shape);
int ssd_conv1d_fwd(const ssd_conv_shape_t* shape, const void* u, const float* w, const float* bias,
                   const void* state_in, void* out, void* state_out, void* hip_stream);
int ssd_conv1d_bwd(const ssd_conv_shape_t* shape, const void* u, const float* w, const float* bias,
                   const void* state_in, const void* dout, const float* dstate_out, void* du, float* dw,
                   float* dbias, float* dstate_in, void* workspace, size_t workspace_bytes, uint32_t flags,
                   void* hip_stream);

/*
 * Gated RMS normalisation of the block (between the SSD output and the output projection of the
 * Mamba-2 backbone of Sec. 3.1), token by token:
 *     g = y * z * sigmoid(z);   out[t,c] = g[t,c] / sqrt(mean over c's group of g[t,.]^2 + eps) * w[c]
 * The channels form `ngroups` contiguous groups of dim / ngroups channels, each normalised on its own.
 * y and z are what a grid cell keeps per token (App. C, Tab. 7: C_grid = the input projection's
 * output, which holds z, plus the d_inner values of y); the backward call recomputes the rest from them.
 *   y, z   [rows, dim] dtype, rows `y_row_stride` / `z_row_stride` elements apart (0 = dense): z may
 *          be a column slice of the input projection's output
 *   w      [dim] fp32                     out, dout [rows, dim] dtype, dense
 *   dy, dz as y and z (same strides), overwritten;  dw [dim] fp32, overwritten, or added to under
 *          SSD_FLAG_ACCUM_PARAM (the only flag)
 *   workspace: ssd_gated_norm_workspace_bytes(shape) bytes of device scratch, 256-byte aligned
 *          (partial sums of dw; backward only)
 * z == NULL: no gate -- the plain RMS normalisation out = y / sqrt(mean y^2 + eps) * w (the layer's
 * pre-norm); dz is then not written and may be NULL.
 * Tokens are independent: a segment of the sequence is a row range, no state is carried.  Inputs and
 * outputs must not overlap.  rows == 0 is allowed.
 * Errors: SSD_ERR_NULL, SSD_ERR_DTYPE, SSD_ERR_SHAPE (sizes, strides below dim), SSD_ERR_DIVISIBILITY
 * (dim % ngroups), SSD_ERR_ARG (negative eps, unknown flag), SSD_ERR_WORKSPACE, SSD_ERR_LAUNCH.
 */
typedef struct {
    int32_t dtype;   /* ssd_dtype_t of y, z, out and their gradients */
    int32_t dim;     /* channels (d_inner) */
    int32_t ngroups; /* normalisation groups */
    float eps;
    int64_t rows;    /* tokens, batch folded in */
    int64_t y_row_stride, z_row_stride;
} ssd_norm_shape_t;
size_t ssd_gated_norm_workspace_bytes(const ssd_norm_shape_t* shape);
int ssd_gated_norm_fwd(const ssd_norm_shape_t* shape, const void* y, const void* z, const float* w, void* out,
                       void* hip_stream);
int ssd_gated_norm_bwd(const ssd_norm_shape_t* shape, const void* y, const void* z, const float* w,
                       const void* dout, void* dy, void* dz, float* dw, void* workspace, size_t workspace_bytes,
                       uint32_t flags, void* hip_stream);

/*
 * The block's projections (dense layers without bias in the Mamba-2 backbone of Sec. 3.1: the input
 * projection, whose output width is the larger part of C_grid in App. C, Tab. 7, and the output
 * projection), bf16 storage, fp32 accumulation on the matrix cores:
 *     out[t,o] = sum_i x[t,i] w[o,i]
 *     dx[t,i]  = sum_o dout[t,o] w[o,i]        dw[o,i] = sum_t dout[t,o] x[t,i]
 *   x    [rows, in_dim] bf16, rows x_row_stride elements apart (0 = dense); likewise out / dout
 *        [rows, out_dim] and dx [rows, in_dim] with their strides: any of them may be a column slice
 *   w    [out_dim, in_dim] bf16, dense         dw [out_dim, in_dim] fp32, dense, overwritten or added
 *        to under SSD_FLAG_ACCUM_PARAM (the only flag)
 *   dx or dw may be NULL (that product is skipped; w resp. x may then be NULL too).
 * in_dim, out_dim and the strides must be multiples of 8, all pointers 16-byte aligned (SSD_ERR_ARG);
 * rows is arbitrary (rows == 0: dw is zeroed or left).  No workspace.  Tokens are independent: a segment
 * is a row range.  Up to 16 rows ssd_linear_fwd runs as a product that streams w once (generation).
 * When ssd_linear_bwd computes both gradients, dw runs on a library-owned stream of default priority
 * beside dx, forked from and joined into hip_stream with events like the segments of ssd_fwd (one per
 * device: calls on one device must not overlap in time; SSD_MAGC_SERIAL=1 keeps both on hip_stream);
 * dx and dw must not overlap x, w or dout.
 * Errors: SSD_ERR_NULL, SSD_ERR_SHAPE, SSD_ERR_DIVISIBILITY, SSD_ERR_ARG, SSD_ERR_LAUNCH.
 */
int ssd_linear_fwd(int64_t rows, int32_t in_dim, int32_t out_dim, const void* x, int64_t x_row_stride,
                   const void* w, void* out, int64_t out_row_stride, void* hip_stream);
int ssd_linear_bwd(int64_t rows, int32_t in_dim, int32_t out_dim, const void* x, int64_t x_row_stride,
                   const void* w, const void* dout, int64_t dout_row_stride, void* dx, int64_t dx_row_stride,
                   float* dw, uint32_t flags, void* hip_stream);

/*
 * Backward (Recompute_Forward + Backward of Alg. 2 over every segment, right to left).
 * Gradients of  <dy, y> + <dfinal_state, final_state>.
 *   inputs as in ssd_fwd, plus
 *   dy              [Bt,L,H,P] dtype
 *   dfinal_state    [Bt,H,P,N] fp32, or NULL for zeros
 *   boundary_states as written by ssd_fwd with the same shape and the same SSD_FLAG_BF16_CHECKPOINTS
 *                   (read only); may be NULL only if segment >= L (then the single segment restarts
 *                   from init_state)
 *   dx [Bt,L,H,P], ddt [Bt,L,H], dB, dC [Bt,L,G,N] dtype, overwritten
 *   dA, dD [H] fp32, overwritten (added to under SSD_FLAG_ACCUM_PARAM)
 *   dinit_state     [Bt,H,P,N] fp32, overwritten; may be NULL
 * dx must not alias dy (SSD_ERR_ARG): several kernels read dy after dx has been written.
 */
int ssd_bwd(const ssd_shape_t* shape, const void* x, const void* dt, const float* A, const void* B,
            const void* C, const float* D, const float* init_state, const void* dy,
            const float* dfinal_state, const void* boundary_states, void* dx, void* ddt, float* dA,
            void* dB, void* dC, float* dD, float* dinit_state, void* workspace,
            size_t workspace_bytes, uint32_t flags, void* hip_stream);

/*
 * One whole Mamba-2 block (the backbone layer of Sec. 3.1) under the sequence-axis checkpoints of MA-GC
 * (Sec. 3.2; Alg. 1 and 2 with a single layer), bf16 storage, one sequence:
 *     zxbcdt = u W_in^T = (z | xBC | dt_raw)          [L, 2 d_inner + 2 G N + H],  d_inner = H P
 *     xBC = silu(conv4(xBC) + conv_b);   dt = softplus(dt_raw + dt_bias);   (x | B | C) = xBC
 *     y = SSD(x, dt, A, B, C, D);        out = RMSNorm_G(y silu(z)) norm_w  W_out^T
 * Forward: segment by segment; what is kept per segment is exactly a sequence checkpoint of App. C,
 * Tab. 7 -- the SSM state and the three-token convolution state entering the segment.  Backward:
 * segments right to left, each recomputed from its two states into the workspace (zxbcdt and y, the
 * activations C_grid counts, live there for one segment at a time), then differentiated step by
 * step; the adjoints of the two states travel left.
 *   u, out, dout, du [L, d_model] bf16, dense
 *   init_ssm [H,P,N] fp32, init_conv [3, d_inner + 2 G N] bf16: the states entering the sequence, NULL = zeros
 *   final_ssm, final_conv: the states leaving it (same shapes), may be NULL; must not alias the initial ones
 *   ssm_ckpt  [nseg, H, P, N] fp32 and conv_ckpt [nseg, 3, d_inner + 2 G N] bf16: slot k = the states
 *             entering segment k (slot 0 is not used); written by magc_block_fwd, read by magc_block_bwd.
 *             Both NULL in magc_block_fwd: no checkpoint is kept (inference; the states travel from segment
 *             to segment inside the workspace, memory does not grow with seqlen) -- prefill of a long
 *             sequence, and with seqlen of a few tokens and init = the previous call's final states,
 *             generation (such calls of at most 16 tokens run on kernels of their own: the scan as the plain
 *             recurrence of Eq. 1, the projections as products that stream the weights once; with a checkpoint
 *             store every call, however short, takes the chunked path that magc_block_bwd recomputes).
 *             magc_block_bwd needs them unless nseg == 1.
 *   dfinal_ssm [H,P,N], dfinal_conv [3, d_inner + 2 G N] fp32: adjoints of the final states, NULL = zeros;
 *   dinit_ssm, dinit_conv: adjoints of the initial states (same shapes, fp32), may be NULL.  With them a
 *             caller can cut a sequence into pieces of its own and chain the calls, as the block does inside.
 *   params: W_in [d_in_proj, d_model] bf16, conv_w [conv_dim, 4], conv_b [conv_dim], dt_bias [H], A [H],
 *           D [H], norm_w [d_inner] fp32, W_out [d_model, d_inner] bf16;
 *           pre_norm_w [d_model] fp32 or NULL.  Not NULL: the block starts with the RMS normalisation that a
 *           language-model layer puts in front of its mixer (same eps, one group), zxbcdt = RMSNorm(u) pre_norm_w
 *           W_in^T; the normalised input is recomputed per segment, never kept.  grads.dpre_norm_w is then needed.
 *   grads:  the same shapes, all fp32, overwritten or added to under SSD_FLAG_ACCUM_PARAM (the only flag)
 *   workspace: magc_block_workspace_bytes bytes, 256-byte aligned; scales with `segment`, not seqlen
 * d_model, d_inner, G N and H must be multiples of 8 (SSD_ERR_DIVISIBILITY), segment a multiple of chunk,
 * headdim and dstate at most 256, chunk at most 1024 (SSD_ERR_SHAPE: the scan's limits);
 * seqlen is arbitrary.  Everything is enqueued on hip_stream; nothing is allocated.  Errors as elsewhere.
 */
typedef struct {
    int32_t d_model, nheads, headdim, ngroups, dstate, chunk;
    float eps;          /* of the gated normalisation */
    int64_t seqlen, segment;
} magc_block_shape_t;
typedef struct {
    const void* W_in;
    const float* conv_w;
    const float* conv_b;
    const float* dt_bias;
    const float* A;
    const float* D;
    const float* norm_w;
    const void* W_out;
    const float* pre_norm_w;   /* may be NULL */
} magc_block_params_t;
typedef struct {
    float* dW_in;
    float* dconv_w;
    float* dconv_b;
    float* ddt_bias;
    float* dA;
    float* dD;
    float* dnorm_w;
    float* dW_out;
    float* dpre_norm_w;        /* used only when params.pre_norm_w is given */
} magc_block_grads_t;
size_t magc_block_workspace_bytes(const magc_block_shape_t* shape, int32_t is_backward);
int magc_block_fwd(const magc_block_shape_t* shape, const magc_block_params_t* params, const void* u,
                   const float* init_ssm, const void* init_conv, void* out, float* ssm_ckpt, void* conv_ckpt,
                   float* final_ssm, void* final_conv, void* workspace, size_t workspace_bytes, void* hip_stream);
int magc_block_bwd(const magc_block_shape_t* shape, const magc_block_params_t* params, const void* u,
                   const float* init_ssm, const void* init_conv, const void* dout, const float* dfinal_ssm,
                   const float* dfinal_conv, const float* ssm_ckpt, const void* conv_ckpt, void* du,
                   const magc_block_grads_t* grads, float* dinit_ssm, float* dinit_conv, void* workspace,
                   size_t workspace_bytes, uint32_t flags, void* hip_stream);

/*
 * A stack of whole blocks with residual adds, x_{j+1} = x_j + Block_j(x_j) (with pre_norm_w: the pre-norm
 * residual layer of the language model), on the two-axis grid of MA-GC (Sec. 3.2 / 3.3, Alg. 1 and 2): the
 * input of every `layer_interval`-th layer is kept for the whole sequence, the SSM and convolution states of
 * every layer every `segment` tokens (block.seqlen, block.segment);
 * the backward pass walks the grid cell by cell, restores a cell's layer inputs from its two kinds of
 * checkpoint and back-propagates through it.
 *   params, grads: host arrays of `nlayers` structs of device pointers (one per layer)
 *   x0, out, dout, dx0 [L, d_model] bf16
 *   l_ckpt   [ceil(nlayers / layer_interval) - 1, L, d_model] bf16: slot m - 1 = the input of layer
 *            m * layer_interval (the first group restarts from x0); may be NULL if there is one group
 *   ssm_ckpt [nlayers, nseg, H, P, N] fp32, conv_ckpt [nlayers, nseg, 3, d_inner + 2 G N] bf16 (slot 0 of
 *            every layer unused: zero initial states); may be NULL if nseg == 1
 *   workspace: magc_blockstack_workspace_bytes bytes, 256-byte aligned: the activations of one cell
 * The sequence starts from zero states in every layer; parameter gradients are overwritten or added to under
 * SSD_FLAG_ACCUM_PARAM.  Errors as for magc_block_*; layer_interval must lie in 1 .. nlayers.
 */
typedef struct {
    magc_block_shape_t block;
    int32_t nlayers, layer_interval;
} magc_blockstack_shape_t;
size_t magc_blockstack_workspace_bytes(const magc_blockstack_shape_t* shape, int32_t is_backward);
int magc_blockstack_fwd(const magc_blockstack_shape_t* shape, const magc_block_params_t* params, const void* x0, void* out,
                        void* l_ckpt, float* ssm_ckpt, void* conv_ckpt, void* workspace, size_t workspace_bytes,
                        void* hip_stream);
int magc_blockstack_bwd(const magc_blockstack_shape_t* shape, const magc_block_params_t* params, const void* x0,
                        const void* dout, const void* l_ckpt, const float* ssm_ckpt, const void* conv_ckpt, void* dx0,
                        const magc_block_grads_t* grads, void* workspace, size_t workspace_bytes, uint32_t flags,
                        void* hip_stream);

/*
 * The same stack, forward only and with nothing kept (inference over long inputs, Sec. 4: the memory taken
 * does not depend on the length; then generation with the recurrence of Eq. 1).  The states of every layer
 * live in two caller-owned device arrays,
 *   ssm_state [nlayers, H, P, N] fp32 and conv_state [nlayers, 3, d_inner + 2 G N] bf16,
 * which the call reads (fresh != 0: takes as zeros without reading them) and replaces by the states behind its
 * last token: a prompt of any length (walked in pieces of block.segment tokens through all layers), then calls
 * of one or a few tokens, continue one sequence.  x0, out [block.seqlen, d_model] bf16 (may be the same
 * buffer); layer_interval is ignored (give any value in 1 .. nlayers).
 *   workspace: magc_blockstack_workspace_bytes(shape, 0) bytes, 256-byte aligned
 * Enqueued on hip_stream in order, nothing allocated, no other stream used.  Errors as for magc_blockstack_fwd.
 */
int magc_blockstack_infer(const magc_blockstack_shape_t* shape, const magc_block_params_t* params, const void* x0, void* out,
                          float* ssm_state, void* conv_state, int32_t fresh, void* workspace, size_t workspace_bytes,
                          void* hip_stream);

/*
 * One generation step (Eq. 1) for `nseq` independent sequences at once, 0 <= nseq <= 16: every parameter is read
 * once for all of them, which is what bounds generation.  x0, out [nseq, d_model] bf16: one token per sequence.
 *   ssm_state [nseq, nlayers, H, P, N] fp32, conv_state [nseq, nlayers, 3, d_inner + 2 G N] bf16: sequence-major,
 *   so the slice of one sequence is exactly what magc_blockstack_infer keeps for it (prefill each sequence with
 *   that call, or start from zeros); read and replaced in place.
 * block.seqlen and layer_interval are ignored; workspace: magc_blockstack_workspace_bytes(shape, 0) of the shape
 * with block.seqlen = 1, 256-byte aligned.  Same stream rules as magc_blockstack_infer.
 */
int magc_blockstack_decode(const magc_blockstack_shape_t* shape, const magc_block_params_t* params, int32_t nseq,
                           const void* x0, void* out, float* ssm_state, void* conv_state, void* workspace,
                           size_t workspace_bytes, void* hip_stream);

/*
 * A stack of `nlayers` SSD layers with residual adds, x_{j+1} = x_j + SSD_j(x_j), run on the
 * MA-GC grid of Sec. 3.2/3.3: layer-axis checkpoints every `layer_interval` layers (l) and
 * sequence-axis checkpoints every shape->segment tokens (s).
 *
 * Per-layer parameters are stacked along a leading layer axis:
 *   dt [nl,Bt,L,H], A [nl,H], B, C [nl,Bt,L,G,N], D [nl,H]   (batch-stride overrides must be 0)
 * Checkpoint stores (device, caller-owned):
 *   s_ckpt [nl, Bt, L/s, H, P, N] fp32 : state of layer j entering segment k          (Alg. 1)
 *   l_ckpt [ceil(nl/l) - 1, Bt, L, H, P] dtype : input of layers l, 2l, ... ; the input of layer 0
 *          is x0 itself and is not copied.  May be NULL when layer_interval >= nlayers.
 * Forward order is segment-major (outer loop over segments, inner loop over layers) as in Alg. 1.
 */
size_t magc_stack_workspace_bytes(const ssd_shape_t* shape, int32_t nlayers, int32_t layer_interval,
                                  int32_t is_backward);

int magc_stack_fwd(const ssd_shape_t* shape, int32_t nlayers, int32_t layer_interval, const void* x0,
                   const void* dt, const float* A, const void* B, const void* C, const float* D,
                   void* out /*[Bt,L,H,P] dtype*/, float* final_states /*[nl,Bt,H,P,N] or NULL*/,
                   float* s_ckpt, void* l_ckpt, void* workspace, size_t workspace_bytes,
                   void* hip_stream);

/*
 * Backward over the grid (Alg. 2): segments right to left; inside a segment, layer blocks top to
 * bottom; each cell restores its activations from (l_ckpt, s_ckpt), then back-propagates layer by
 * layer, carrying grad-x down and the per-layer state adjoints left.
 *   dout [Bt,L,H,P] dtype : gradient w.r.t. `out`
 *   dx0  [Bt,L,H,P] dtype, overwritten
 *   ddt [nl,Bt,L,H], dB, dC [nl,Bt,L,G,N] dtype; dA, dD [nl,H] fp32 : overwritten
 * Final-state adjoints are taken as zero (the stack's loss depends on `out` only).
 */
int magc_stack_bwd(const ssd_shape_t* shape, int32_t nlayers, int32_t layer_interval, const void* x0,
                   const void* dt, const float* A, const void* B, const void* C, const float* D,
                   const void* dout, const float* s_ckpt, const void* l_ckpt, void* dx0, void* ddt,
                   float* dA, void* dB, void* dC, float* dD, void* workspace, size_t workspace_bytes,
                   void* hip_stream);

/*
 * Checkpoint-interval planner (host only; no device work).  Memory model of App. C:
 *     M(l, s) = (L*S/l)*C_Lckpt + (L*S/s)*C_Sckpt + l*s*C_grid + s*C_state
 * (all constants 1 and C_state 0 give the model of Sec. 3.3).  The search is exhaustive over
 * l in [1, L] and s in the multiples of s_multiple within [s_multiple, S] when S >= s_multiple
 * (Sec. 4 keeps s a multiple of 256 once S >= 256), else s in [1, S].  Ties: larger s, then
 * smaller l.  With budget > 0 the plan with the least recomputation (largest s, then largest l)
 * among those with M <= budget is returned; if none fits, the minimum-memory plan is filled in
 * and SSD_ERR_BUDGET returned.  Constants are in whatever unit the caller likes (bytes,
 * elements); M comes back in the same unit.
 */
typedef struct magc_model_t {
    int64_t n_layers;        /* L */
    int64_t seqlen;          /* S */
    double c_lckpt;          /* per layer-checkpointed token */
    double c_sckpt;          /* per sequence-checkpointed layer state */
    double c_grid;           /* per (layer, token) alive inside a grid cell */
    double c_state;          /* per token of the segment being restored */
    int64_t s_multiple;      /* 256 in the paper; <= 1 disables the rule */
    double budget;           /* <= 0: minimise M */
    int32_t integer_counts;  /* 0: L/l and S/s as real quotients (the paper's formula); 1: ceil() of each */
} magc_model_t;

typedef struct magc_plan_t {
    int64_t l, s;
    double m_lckpt, m_sckpt, m_grid, m_state, m_total;
    int32_t regime;          /* of the unweighted analysis, Sec. 3.3: 0 interior (L <= S^2 and S <= L^2),
                                1 sequence-dominated (L^2 <= S), 2 layer-dominated (S^2 <= L) */
    int32_t fits;            /* 1 if budget <= 0 or m_total <= budget */
} magc_plan_t;

int magc_plan(const magc_model_t* model /*host*/, magc_plan_t* out /*host*/);

/*
 * Per-kernel timing for benchmarks (diagnostics; not part of the method).  While enabled, every
 * kernel launch of this library is bracketed by two HIP events recorded on the launch stream.
 * Not thread-safe; leave it off in production.
 *   ssd_prof_enable(on)      : drops earlier records, then switches recording off (0), on for every
 *                              kernel (1), or on for kernel id `on - 2` only (on >= 2)
 *   ssd_prof_read(id, ...)   : waits for the recorded events of kernel `id`, returns the sum of
 *                              their durations in milliseconds and the number of launches (host pointers)
 *   ssd_prof_kernel_name(id) : static name of kernel `id`, NULL once id is past the last kernel
 *   ssd_prof_serialize(on)   : on = 1 keeps every segment on the caller's stream (kernels then never overlap,
 *                              which is what per-kernel durations need to mean something); 0 restores the
 *                              default.  The workspace size does not change.
 */
int ssd_prof_enable(int32_t on);
int ssd_prof_serialize(int32_t on);
int ssd_prof_read(int32_t kernel_id, double* total_ms /*host*/, int64_t* launches /*host*/);
const char* ssd_prof_kernel_name(int32_t kernel_id);
/* Calibration of the matrix cores: `workgroups` workgroups of four waves, each wave `iters` rounds of sixteen
 * independent 32 x 32 x 16 bf16 MFMAs on registers (no memory traffic): 16 * 32768 flop per wave and round.
 * `sink` is one float of device memory (never written).  The caller times the launch. */
int ssd_prof_mfma_peak(int32_t iters, int32_t workgroups, float* sink, void* hip_stream);
/* Clock probe: a single wave that waits until the constant 100 MHz counter has advanced by `ticks` (at most 1e8:
 * one second) and then writes out[0] = ticks elapsed, out[1] = shader-clock cycles elapsed (device memory, two
 * 64-bit words).  Launched on a second stream of default priority beside the work under test it measures the
 * clock that work runs at: out[1] / out[0] * 100 MHz. */
int ssd_prof_clock_probe(uint64_t ticks, uint64_t* out, void* hip_stream);

/* Static, human-readable text for a status code (host pointer, never NULL). */
const char* ssd_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* SSD_MAGC_H */
