// Internal declarations shared by the translation units of libssd_magc (not part of the ABI).
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "ssd_magc.h"

namespace ssdk {

// Internal flag (never accepted from callers): the gradient of cum arrives in three pieces,
// gterm - sterm + gintra (matrix-core path).
constexpr uint32_t SSD_INTERNAL_SPLIT_GTERM = 1u << 31;

// bf16 storage as raw bits; conversion is round-to-nearest-even.
struct bf16_t {
    uint16_t v;
};

__host__ __device__ inline float bf16_to_float(bf16_t b) {
    union {
        uint32_t u;
        float f;
    } c;
    c.u = (uint32_t)b.v << 16;
    return c.f;
}

__host__ __device__ inline bf16_t float_to_bf16(float f) {
    union {
        uint32_t u;
        float f;
    } c;
    c.f = f;
    bf16_t o;
    if ((c.u & 0x7fffffffu) > 0x7f800000u) {  // NaN stays NaN
        o.v = (uint16_t)((c.u >> 16) | 0x40u);
    } else {
        o.v = (uint16_t)((c.u + 0x7fffu + ((c.u >> 16) & 1u)) >> 16);
    }
    return o;
}

// One segment of one layer, as the kernels see it.  Tensor pointers are already offset to the
// first token of the segment; batch strides are those of the full tensors (elements).
struct SegParams {
    int Bt, H, P, G, N, Q, nc, hpg;
    int64_t xs_b, ys_b, dys_b, dxs_b;  // batch strides of x, y, dy, dx
    int64_t dts_b, bcs_b;              // of dt/ddt and of B/C/dB/dC
    const uint8_t* reset;              // optional [Bt][tokens of the segment]: non-zero = a packed sequence starts here
    int64_t reset_bs;                  // its batch stride
    uint32_t flags;
    // inputs / outputs
    const void* x;
    const void* dt;
    const void* Bm;
    const void* Cm;
    const void* dy;
    const float* A;
    const float* D;
    void* y;
    void* dx;
    void* ddt;
    void* dB;
    void* dC;
    // per-segment workspace (fp32)
    float* cum;        // [Bt][H][nc][Q]  chunk-local inclusive cumsum of dt*A
    float* dtf;        // [Bt][H][nc][Q]  dt as fp32, head-major
    float* states;     // generic path only: [Bt][nc+1][H][P][N]  slot c: state entering chunk c; slot nc: state leaving the segment
    float* dstates;    // generic path only: [Bt][nc][H][P][N]    slot c: adjoint of the state leaving chunk c
    float* Gm;         // [Bt][nc][G][Q][Q]    C_i . B_j   (generic path: fp32)
    float* dG;         // generic path: [Bt][nc][G][Q][Q] fp32 head-summed masked dY X^T; MFMA path: [Bt][nc][G][dg_split][Q/32][Q/32][32][32] bf16 per-slice sums, tile by tile
    float* gterm;      // [Bt][H][nc][Q]  gradient of cum, per token (MFMA path: the part through the entering state)
    float* sterm;      // [Bt][H][nc][Q]  MFMA path: dt_j x_j . (part of u_j through the leaving adjoint); subtracted
    float* gintra;     // [Bt][H][nc][Q]  MFMA path: chunk-local part (row sums minus column sums of E); added
    float* fterm;      // [Bt][H][nc][Q]
    float* dDrow;      // [Bt][H][nc][Q]
    float* tail_part;  // [Bt][H][nc][nslice]
    float* dA_part;    // [Bt][nc][H]
    float* dD_part;    // [Bt][nc][H]
    float* dcarry;     // [Bt][H][P][N] adjoint of the state entering the segment to the right of the current one
    int nslice;
    // extra scratch of the MFMA path
    float* ein;        // [Bt][H][nc][Q] exp(cum_i - cum at the start of i's 64-token block)
    float* eout;       // [Bt][H][nc][Q] exp(cum at the end of j's 64-token block - cum_j)
    bf16_t* states_bf;   // [Bt][nc][H][P][N] chunk states, replaced in place by the states entering the chunks (bf16 only)
    bf16_t* dstates_bf;  // [Bt][nc][H][P][N] local state adjoints, replaced in place by the adjoints of the leaving states
    int dg_split;        // number of head slices whose dG / dB / dC partial sums are kept apart
    int dual_split;      // number of head slices per (batch, chunk, group) in the dual-form kernels
    int part_split;      // number of head slices of the dB / dC head sums
    int outer_split;     // number of head slices of the chunk-state / local-adjoint kernel
    int part_alternate;  // the head-sum pass alternates between the halves of its slice (see part_body)
    int wg_target;       // least number of workgroups a persistent-over-heads launch should have
    float* dbc_part;     // [Bt][nc][G][part_split][2][Q][N] per-slice head terms of dC (0) and dB (1)
    // state plumbing for the scans (all fp32, element strides between batches)
    const float* state_in;   // state entering the segment, or NULL for zeros
    int64_t state_in_bs;
    float* bnd_write;        // where to store that entering state (checkpoint slot), or NULL
    int64_t bnd_write_bs;
    float* state_out;        // where to store the state leaving the segment, or NULL
    int64_t state_out_bs;
    float* state_out2;       // second copy (final_state when the last segment also has no slot), or NULL
    int64_t state_out2_bs;
    // bf16 checkpoints: the entering state comes from (state_in16, used when state_in is NULL) or goes to
    // (bnd_write16, state_out16) a bf16 slot; strides as for their fp32 counterparts
    const bf16_t* state_in16;
    bf16_t* bnd_write16;
    bf16_t* state_out16;
    int64_t state_out16_bs;
    float* dinit_out;        // bwd: where the adjoint of the entering state goes at segment 0, or NULL
    float* dA;
    float* dD;
    int accumulate;          // bwd: 1 = add this segment's dA/dD to what is there
    // dA / dD partial sums: slot (b, chunk0 + c, h) of an array with nc_total chunks per batch.  The
    // defaults (chunk0 = 0, nc_total = nc) keep them per segment; defer_param = 1 leaves the final
    // reduction over all chunks to the caller (launch_param_reduce), so segments may run concurrently.
    int chunk0, nc_total, defer_param;
    // optional cross-stream ordering of the state scans (consecutive segments run on different streams):
    // the scan waits for ev_wait and records ev_record when it has been enqueued
    hipEvent_t ev_wait, ev_record;
#ifdef SSDK_STAMPS
    unsigned long long* stamps;  // diagnostics build: cycle stamps of the head loops (see SSDK_STAMP)
#endif
};

// Diagnostics build (-DSSDK_STAMPS): wave 0 of the first eight workgroups of a head-walking kernel writes the
// shader cycle counter at six points of every head iteration, slot (body, workgroup, head, point).
#ifdef SSDK_STAMPS
extern unsigned long long* g_stamps;
#define SSDK_STAMP(body, id)                                                                              \
    do {                                                                                                  \
        if (sp.stamps && lane == 0 && w == 0 && zlog < 8 && hh < 64)                                      \
            sp.stamps[((((body)) * 8 + zlog) * 64 + hh) * 16 + (id)] = __builtin_readcyclecounter();      \
    } while (0)
#else
#define SSDK_STAMP(body, id) \
    do {                     \
    } while (0)
#endif

// Validated dimensions of one call.
struct Dims {
    int64_t Bt, L, s;
    int H, P, G, N, Q, nc, hpg;
    int64_t nseg;       // segments, the last one possibly short
    int64_t tail;       // tokens of a short last segment (0: every segment is full)
    int nc_tail;        // chunks of that segment (the last one padded with identity tokens)
    size_t esz;
    bool bf16;
    int64_t xs_b, dts_b, bcs_b;
    const uint8_t* reset;  // optional packed-sequence flags [Bt][L]
};

// What a packed-sequence start adds to the token's log-decay dt*A: exp(-100) < 4e-44 cuts the state off
// (and with it every gradient path through it) while every decay factor stays a product of factors <= 1.
constexpr float RESET_LOG_DECAY = -100.f;

// Byte offsets of the per-segment scratch arrays inside the caller's workspace (WS_NONE: the array
// does not exist on the chosen kernel path and its pointer stays null).
constexpr size_t WS_NONE = ~(size_t)0;
struct WsLayout {
    size_t cum, dtf, states, Gm, dstates, dG, gterm, fterm, dDrow, tail_part, dA_part, dD_part, dcarry, total;
    size_t ein, eout, states_bf, dstates_bf, dbc_part, sterm, gintra;
    int nslice, dg_split, part_split;
};

int check_shape(const ssd_shape_t* sh, Dims* d);
// mfma: the layout for the matrix-core kernels, which keep the chunk states and their adjoints in
// bf16 only (the fp32 arrays of the shape-generic kernels are left out).
// fp32cs: the matrix-core layout keeps fp32 chunk states / local adjoints beside the bf16 operand copies.
WsLayout ws_layout(const Dims& d, bool bwd, bool mfma, int wg_target = 256, bool fp32cs = false);
void bind_workspace(SegParams& sp, const WsLayout& w, void* workspace, bool bwd);
void base_params(SegParams& sp, const Dims& d, uint32_t flags);
bool use_mfma(const ssd_shape_t& sh, uint32_t flags);

// Kernel ids for the optional event timing (see prof.hip).
enum KernelId {
    K_CUMSUM, K_CB, K_CHUNK_STATE, K_SCAN_FWD, K_CHUNK_OUT, K_DSTATE, K_SCAN_BWD, K_BWD_MAIN, K_DDT, K_PARAM, K_DG, K_DBC,
    K_FILL, K_COPY, K_MFMA_CB, K_MFMA_CHUNK_STATE, K_MFMA_CHUNK_OUT, K_MFMA_DSTATE, K_MFMA_BWD_MAIN, K_MFMA_DG,
    K_MFMA_DBC, K_MFMA_DBC_FINAL, K_MFMA_BWD_TRIO, K_MFMA_PREP_CB, K_MFMA_FINAL_DDT, K_COUNT
};
// When timing of kernel `kid` is enabled: a pair of events for the launch to fill in (kernel start
// and end, as the command processor stamps them -- the time the launch waits behind other work is
// not part of it); otherwise false.
bool prof_events(int kid, hipEvent_t* start, hipEvent_t* stop);

// Launch on `st`, timed when enabled; returns the launch error from the enclosing function.
#define SSDK_LAUNCH(kid, st, kernel, grid, block, ...)                                        \
    do {                                                                                      \
        hipEvent_t ea_ = nullptr, eb_ = nullptr;                                              \
        if (::ssdk::prof_events(kid, &ea_, &eb_))                                             \
            hipExtLaunchKernelGGL(kernel, grid, block, 0, st, ea_, eb_, 0, __VA_ARGS__);      \
        else                                                                                  \
            hipLaunchKernelGGL(kernel, grid, block, 0, st, __VA_ARGS__);                      \
        hipError_t e_ = hipGetLastError();                                                    \
        if (e_ != hipSuccess) return e_;                                                      \
    } while (0)

// Launchers.  Each returns hipSuccess or the launch error.  is_bf16 selects the storage type.
hipError_t launch_fill_zero(float* p, size_t n, hipStream_t st);
hipError_t launch_copy_f32(float* dst, const float* src, size_t n, hipStream_t st);
// dst[b][row][:] = row < rows_valid ? src[b][row][:] : 0 for row < rows_dst (batch strides in elements of esz bytes).
hipError_t launch_stage_rows(void* dst, int64_t dst_bs, const void* src, int64_t src_bs, int rows_valid, int rows_dst,
                             int row_elems, int Bt, size_t esz, hipStream_t st);
hipError_t generic_forward_segment(const SegParams& sp, bool is_bf16, bool need_y, hipStream_t st);
hipError_t generic_backward_segment(const SegParams& sp, bool is_bf16, hipStream_t st);
hipError_t generic_backward_scalars(const SegParams& sp, hipStream_t st);
// dA, dD = (or +=, under sp.accumulate) the sum of the partial sums of all sp.nc_total chunks.
hipError_t launch_param_reduce(const SegParams& sp, hipStream_t st);

// MFMA path (bf16, P = 64, N = 128, Q in {64, 128, 256}).
bool mfma_path_supported(const ssd_shape_t& s);
hipError_t mfma_forward_segment(const SegParams& sp, bool need_y, hipStream_t st);
hipError_t mfma_backward_segment(const SegParams& sp, hipStream_t st);
// One dual-form pass over a segment: epi 0 = forward output, 2 = the backward pass.
hipError_t mfma_launch_dual(const SegParams& sp, int epi, hipStream_t st);
// dG, the head sums and the final contraction that give dB and dC of one segment.
hipError_t mfma_launch_grad_bc(const SegParams& sp, bool with_dual, hipStream_t st);
// Smallest divisor ns of heads_per_group with base * ns >= target workgroups (else heads_per_group).
int pick_split(int heads_per_group, int64_t base, int target);

// The block's convolution with its output (forward) or the gradient of its output (backward) given as three
// dense tensors side by side -- channels [0, c1), [c1, c2), [c2, C) with rows c1, c2 - c1, C - c2 apart: the
// x | B | C operands of the scan and their gradients -- instead of one [L, C] tensor.  Otherwise as
// ssd_conv1d_fwd / ssd_conv1d_bwd.
struct ConvSplit {
    void* p[3];
    int c1, c2;
};
int conv1d_fwd_split(const ssd_conv_shape_t* sh, const void* u, const float* w, const float* bias, const void* state_in,
                     const ConvSplit& out, void* state_out, hipStream_t st);
int conv1d_bwd_split(const ssd_conv_shape_t* sh, const void* u, const float* w, const float* bias, const void* state_in,
                     const ConvSplit& dout, const float* dstate_out, void* du, float* dw, float* dbias, float* dstate_in,
                     void* workspace, size_t workspace_bytes, uint32_t flags, hipStream_t st);

// True when everything is to stay on the caller's stream (SSD_MAGC_SERIAL=1 in the environment, or ssd_prof_serialize).
bool serial_mode();

// The library's side stream of the current device (default priority, created on first use) with a pair of
// events for the caller to fork it from and join it into its own stream; NULL in serial mode or on failure.
// ssd_linear_bwd enqueues on the same stream with events of its own, so work given to it here and the
// products of such a call run in the order they were enqueued.
struct SideStream {
    hipStream_t st;
    hipEvent_t fork, join;
};
SideStream* side_stream();

// Generation (few_rows.hip): products and the block's middle steps for at most FEW_ROWS tokens, bf16 storage.
constexpr int FEW_ROWS = 16;
// Up to this many rows the product runs on the vector ALUs with an optional normalisation of the rows folded in;
// above, on the matrix cores (mode 0 only: the caller normalises first).
constexpr int FEW_ROWS_VALU = 4;
// out[r, n] = sum_k f(x)[r, k] w[n, k] (+ res[r, n]); w [N, K] dense.  mode 0: f = identity; 1: RMS normalisation
// over all of K times in_w; 2: the same of x z sigmoid(z).  Row strides in elements.
struct FewRowsJob {
    int rows, K, N, mode;
    const void* x;
    int64_t ldx;
    const void* w;
    void* out;
    int64_t ldo;
    const float* in_w;
    const void* z;
    int64_t ldz;
    float eps;
    const void* res;
    int64_t ldres;
    // optional: copy_chunks (0 = 1) pieces of copy_bytes bytes (a multiple of 16; at most 16 N vectors in all), the
    // pieces copy_src_stride / copy_dst_stride bytes apart, moved from copy_src to copy_dst by the same launch
    const void* copy_src;
    void* copy_dst;
    size_t copy_bytes;
    int copy_chunks;
    size_t copy_src_stride, copy_dst_stride;
};
bool few_rows_supported(const FewRowsJob& j);  // sizes, strides and 16-byte alignment the kernel relies on
hipError_t launch_linear_few_rows(const FewRowsJob& j, hipStream_t st);
// zx [T, ld] = (z | xBC | dt_raw) of T tokens -> y [T, H P]; state [H, P, N] in place; cs_in / cs_out [3, H P + 2 G N]
// (either may be null; never the same buffer).  nb > 1: that many independent sequences of T tokens each (nb T <=
// FEW_ROWS), sequence b in rows b T .. of zx and y, its states state_bs / cs_in_bs / cs_out_bs elements further on.
struct DecodeMidJob {
    int nb;
    int64_t state_bs, cs_in_bs, cs_out_bs;
    int T, H, P, G, N;
    const void* zx;
    int64_t ld;
    const float *conv_w, *conv_b, *dt_bias, *A, *D;
    const void* cs_in;
    void* cs_out;
    float* state;
    void* y;
};
hipError_t launch_decode_mid(const DecodeMidJob& j, hipStream_t st);
// The same for one token of each of nb sequences as two kernels (many sequences: a convolution per workgroup of
// the recurrence kernel costs more than a launch): convolution + SiLU and softplus(dt) into dense x [nb, H P],
// B, C [nb, G N], dt [nb, H], the convolution state cs (sequence b: cs_bs elements further on) replaced in place;
// then the recurrence on states state_bs floats apart.
struct ConvStepJob {
    int nb, H, P, G, N;
    const void* zx;
    int64_t ld;
    const float *conv_w, *conv_b, *dt_bias;
    void* cs;
    int64_t cs_bs;
    void *x, *B, *C, *dt;
};
hipError_t launch_conv_step(const ConvStepJob& j, hipStream_t st);
hipError_t launch_decode_strided(int nb, int H, int P, int G, int N, const void* x, const void* dt, const float* A, const void* B,
                                 const void* C, const float* D, float* state, int64_t state_bs, void* y, hipStream_t st);

}  // namespace ssdk
