// One Mamba-2 block (the backbone layer of Sec. 3.1) under MA-GC's sequence-axis checkpoints (Sec. 3.2,
// Alg. 1/2 with one layer): per segment of `segment` tokens
//     zxbcdt = u W_in^T = (z | xBC | dt_raw);   xBC = silu(conv4(xBC) + b);   dt = softplus(dt_raw + dt_bias)
//     y = SSD(x, dt, A, B, C, D) with (x | B | C) = xBC;   out = RMSNorm_G(y silu(z)) norm_w  W_out^T
// (with pre_norm_w the projection reads RMSNorm(u) pre_norm_w instead of u: the pre-norm of a language-model layer)
// The forward pass keeps, per segment, only what a sequence checkpoint holds in App. C, Tab. 7: the SSM
// state and the three-token convolution state entering the segment.  The backward pass walks the segments
// right to left, redoes a segment's forward from its two states (Recompute_Forward of Alg. 2) into the
// workspace -- zxbcdt and y are the per-token activations C_grid counts -- and then runs the reverse of
// every step, handing the two state adjoints to the segment on the left.
// Everything is a sequence of calls to the library's own entry points plus small kernels for softplus of dt
// (the convolution writes x, B and C as the three dense tensors the scan reads, and reads their gradients
// the same way); all on the caller's stream.
#include <string.h>

#include "ssd_internal.h"

namespace ssdk {
namespace {

typedef __bf16 b8 __attribute__((ext_vector_type(8)));

constexpr int DECODE_ROWS = 16;  // calls of at most this many tokens run the scan as the plain recurrence
constexpr int DT_ROWS = 16;  // rows per workgroup of the dt kernels (granularity of the ddt_bias partial sums)

// dt[r,h] = softplus(raw[r,h] + bias[h]); raw is a column slice (rows raw_rs apart), dt dense
__global__ __launch_bounds__(256) void k_dt_fwd(const bf16_t* raw, int64_t raw_rs, const float* bias, bf16_t* dt, int64_t rows, int H) {
    const int64_t r0 = (int64_t)blockIdx.x * DT_ROWS;
    for (int i = threadIdx.x; i < DT_ROWS * H; i += 256) {
        const int64_t r = r0 + i / H;
        const int h = i % H;
        if (r < rows) {
            const float v = bf16_to_float(raw[r * raw_rs + h]) + bias[h];
            // log(1 + e^v) without overflow: max(v, 0) + log1p(e^-|v|)
            dt[r * H + h] = float_to_bf16(fmaxf(v, 0.f) + log1pf(__expf(-fabsf(v))));
        }
    }
}

// draw[r,h] = ddt[r,h] sigmoid(raw[r,h] + bias[h]) into a column slice; part[tile][h] = sum over the tile's rows
__global__ __launch_bounds__(256) void k_dt_bwd(const bf16_t* raw, int64_t raw_rs, const float* bias, const bf16_t* ddt, bf16_t* draw,
                                               int64_t draw_rs, float* part, int64_t rows, int H) {
    const int64_t r0 = (int64_t)blockIdx.x * DT_ROWS;
    for (int h = threadIdx.x; h < H; h += 256) {
        const float bh = bias[h];
        float s = 0.f;
        for (int rr = 0; rr < DT_ROWS; ++rr) {
            const int64_t r = r0 + rr;
            if (r >= rows) break;
            const float v = bf16_to_float(raw[r * raw_rs + h]) + bh;
            const float g = bf16_to_float(ddt[r * H + h]) * __builtin_amdgcn_rcpf(1.f + __expf(-v));
            draw[r * draw_rs + h] = float_to_bf16(g);
            s += g;
        }
        part[(int64_t)blockIdx.x * H + h] = s;
    }
}

// out[h] (+)= sum_p part[p][h], in a fixed order: a workgroup owns 64 columns, its four waves sum every
// fourth part each, wave 0 adds the four results
__global__ __launch_bounds__(256) void k_colsum(const float* part, int64_t nparts, int H, float* out, int accumulate) {
    __shared__ float red[4][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int h = blockIdx.x * 64 + lane;
    float s = 0.f;
    if (h < H)
        for (int64_t p = wv; p < nparts; p += 4) s += part[p * H + h];
    red[wv][lane] = s;
    __syncthreads();
    if (wv == 0 && h < H) {
        s = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
        out[h] = accumulate ? out[h] + s : s;
    }
}

struct BlockDims {
    int64_t L, s, nseg;
    int dm, H, P, G, N, Q, d_inner, conv_dim, gn, d_in_proj, off_xbc, off_dt;
    size_t HPN;
};

int check(const magc_block_shape_t* sh, BlockDims* d) {
    if (!sh) return SSD_ERR_NULL;
    if (sh->d_model <= 0 || sh->nheads <= 0 || sh->headdim <= 0 || sh->ngroups <= 0 || sh->dstate <= 0 || sh->chunk <= 0 ||
        sh->seqlen < 0 || sh->segment <= 0)
        return SSD_ERR_SHAPE;
    if (sh->nheads % sh->ngroups) return SSD_ERR_DIVISIBILITY;
    if (sh->segment % sh->chunk) return SSD_ERR_DIVISIBILITY;
    if (!(sh->eps >= 0.f)) return SSD_ERR_ARG;
    if (sh->chunk > 1024 || sh->headdim > 256 || sh->dstate > 256) return SSD_ERR_SHAPE;  // the limits of the scan
    d->L = sh->seqlen;
    d->s = sh->segment;
    d->nseg = sh->seqlen > 0 ? (sh->seqlen + sh->segment - 1) / sh->segment : 0;
    d->dm = sh->d_model;
    d->H = sh->nheads;
    d->P = sh->headdim;
    d->G = sh->ngroups;
    d->N = sh->dstate;
    d->Q = sh->chunk;
    d->d_inner = d->H * d->P;
    d->gn = d->G * d->N;
    d->conv_dim = d->d_inner + 2 * d->gn;
    d->d_in_proj = 2 * d->d_inner + 2 * d->gn + d->H;
    d->off_xbc = d->d_inner;
    d->off_dt = d->d_inner + d->conv_dim;
    d->HPN = (size_t)d->H * d->P * d->N;
    // 16-byte vectors of bf16 everywhere: every column range starts and ends on a multiple of 8
    if ((d->dm | d->d_inner | d->gn | d->H) & 7) return SSD_ERR_DIVISIBILITY;
    return SSD_OK;
}

ssd_shape_t seg_shape(const BlockDims& d, int64_t rows) {
    ssd_shape_t sh;
    memset(&sh, 0, sizeof(sh));
    sh.dtype = SSD_BF16;
    sh.nheads = d.H;
    sh.headdim = d.P;
    sh.ngroups = d.G;
    sh.dstate = d.N;
    sh.chunk = d.Q;
    sh.batch = 1;
    sh.seqlen = rows;
    sh.segment = d.s;  // one segment per call: the block's own loop is the sequence axis
    return sh;
}

ssd_conv_shape_t conv_shape(const BlockDims& d, int64_t rows) {
    ssd_conv_shape_t c;
    memset(&c, 0, sizeof(c));
    c.dtype = SSD_BF16;
    c.channels = d.conv_dim;
    c.batch = 1;
    c.seqlen = rows;
    c.u_row_stride = d.d_in_proj;
    return c;
}

ssd_norm_shape_t norm_shape(const BlockDims& d, int64_t rows, float eps) {
    ssd_norm_shape_t n;
    memset(&n, 0, sizeof(n));
    n.dtype = SSD_BF16;
    n.dim = d.d_inner;
    n.ngroups = d.G;
    n.eps = eps;
    n.rows = rows;
    n.z_row_stride = d.d_in_proj;
    return n;
}

// the normalisation in front of the input projection: all of d_model is one group, dense rows
ssd_norm_shape_t pre_norm_shape(const BlockDims& d, int64_t rows, float eps) {
    ssd_norm_shape_t n;
    memset(&n, 0, sizeof(n));
    n.dtype = SSD_BF16;
    n.dim = d.dm;
    n.ngroups = 1;
    n.eps = eps;
    n.rows = rows;
    return n;
}

size_t al(size_t n) { return (n + 255) & ~(size_t)255; }

// Workspace: one segment's activations (and, backward, their gradients), the scratch of the inner calls.
struct BlockWs {
    size_t un, zx, x, B, C, dt, y, yn;                      // forward activations of the segment
    size_t dun, dyn, dy, dzx, dx, dB, dC, ddt;              // backward
    size_t dssm[2], dconv[2], dtpart, inner, total;
    size_t cssm[2], cconv[2];                               // states handed from segment to segment when no checkpoints are kept
    size_t inner_bytes;
};

BlockWs layout(const BlockDims& d, bool bwd) {
    BlockWs w;
    memset(&w, 0, sizeof(w));
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += al(bytes);
        return o;
    };
    const size_t s = (size_t)d.s;
    w.un = take(s * d.dm * 2);
    w.zx = take(s * d.d_in_proj * 2);
    w.x = take(s * d.d_inner * 2);
    w.B = take(s * d.gn * 2);
    w.C = take(s * d.gn * 2);
    w.dt = take(s * d.H * 2);
    w.y = take(s * d.d_inner * 2);
    w.yn = take(s * d.d_inner * 2);
    // scratch of the inner calls: for a whole segment and for the short last one (which the scan pads)
    const ssd_shape_t ss = seg_shape(d, d.s);
    const ssd_shape_t st = seg_shape(d, d.L % d.s ? d.L % d.s : d.s);
    size_t inner = 0;  // the backward pass also runs the forward scan (recomputation)
    for (int pass = 0; pass <= (bwd ? 1 : 0); ++pass) {
        const size_t a = ssd_workspace_bytes(&ss, pass), b = ssd_workspace_bytes(&st, pass);
        inner = a > inner ? a : inner;
        inner = b > inner ? b : inner;
    }
    if (bwd) {
        w.dun = take(s * d.dm * 2);
        w.dyn = take(s * d.d_inner * 2);
        w.dy = take(s * d.d_inner * 2);
        w.dzx = take(s * d.d_in_proj * 2);
        w.dx = take(s * d.d_inner * 2);
        w.dB = take(s * d.gn * 2);
        w.dC = take(s * d.gn * 2);
        w.ddt = take(s * d.H * 2);
        for (int i = 0; i < 2; ++i) w.dssm[i] = take(d.HPN * 4);
        for (int i = 0; i < 2; ++i) w.dconv[i] = take((size_t)3 * d.conv_dim * 4);
        w.dtpart = take(((s + DT_ROWS - 1) / DT_ROWS) * d.H * 4);
        const ssd_conv_shape_t cs = conv_shape(d, d.s);
        const ssd_norm_shape_t ns = norm_shape(d, d.s, 0.f);
        const ssd_norm_shape_t ps = pre_norm_shape(d, d.s, 0.f);
        const size_t b = ssd_conv1d_workspace_bytes(&cs), c = ssd_gated_norm_workspace_bytes(&ns), e = ssd_gated_norm_workspace_bytes(&ps);
        inner = b > inner ? b : inner;
        inner = c > inner ? c : inner;
        inner = e > inner ? e : inner;
    }
    for (int i = 0; i < 2; ++i) w.cssm[i] = take(d.HPN * 4);
    for (int i = 0; i < 2; ++i) w.cconv[i] = take((size_t)3 * d.conv_dim * 2);
    w.inner = take(inner);
    w.inner_bytes = inner;
    w.total = off;
    return w;
}

#define BLK_TRY(expr)                   \
    do {                                \
        const int rc_ = (expr);         \
        if (rc_ != SSD_OK) return rc_;  \
    } while (0)
#define BLK_HIP(expr)                                   \
    do {                                                \
        if ((expr) != hipSuccess) return SSD_ERR_LAUNCH; \
    } while (0)

// The forward steps of a segment.  zx [rows, d_in_proj] and y [rows, d_inner] are given by the caller (the
// block's own workspace, or the per-layer slots a grid cell keeps: they are the activations C_grid of App. C,
// Tab. 7 counts); everything else lives in the workspace `ws` laid out by `w`.
// the input of the projection: u itself, or (pre_norm_w given) its RMS normalisation, written to the workspace
int seg_pre_norm(const BlockDims& d, float eps, const magc_block_params_t* p, char* ws, const BlockWs& w, const void* u_seg,
                 int64_t rows, const void** proj_in, hipStream_t st) {
    *proj_in = u_seg;
    if (!p->pre_norm_w) return SSD_OK;
    const ssd_norm_shape_t ps = pre_norm_shape(d, rows, eps);
    *proj_in = ws + w.un;
    return ssd_gated_norm_fwd(&ps, u_seg, nullptr, p->pre_norm_w, ws + w.un, st);
}

int seg_in_proj(const BlockDims& d, float eps, const magc_block_params_t* p, char* ws, const BlockWs& w, const void* u_seg, int64_t rows,
                char* zx, hipStream_t st) {
    const void* in;
    BLK_TRY(seg_pre_norm(d, eps, p, ws, w, u_seg, rows, &in, st));
    return ssd_linear_fwd(rows, d.dm, d.d_in_proj, in, 0, p->W_in, zx, 0, st);
}

// convolution + SiLU of the xBC columns into dense x / B / C, softplus of the dt columns
int seg_mid(const BlockDims& d, const magc_block_params_t* p, char* ws, const BlockWs& w, const char* zx, int64_t rows,
            const void* conv_in, void* conv_out, hipStream_t st) {
    const ssd_conv_shape_t cs = conv_shape(d, rows);
    const ConvSplit xbc = {{ws + w.x, ws + w.B, ws + w.C}, d.d_inner, d.d_inner + d.gn};  // each part dense, as the scan reads it
    BLK_TRY(conv1d_fwd_split(&cs, zx + (size_t)d.off_xbc * 2, p->conv_w, p->conv_b, conv_in, xbc, conv_out, st));
    hipLaunchKernelGGL(k_dt_fwd, dim3((unsigned)((rows + DT_ROWS - 1) / DT_ROWS)), dim3(256), 0, st,
                       (const bf16_t*)(zx + (size_t)d.off_dt * 2), (int64_t)d.d_in_proj, p->dt_bias, (bf16_t*)(ws + w.dt), rows, d.H);
    BLK_HIP(hipGetLastError());
    return SSD_OK;
}

int seg_scan(const BlockDims& d, const magc_block_params_t* p, char* ws, const BlockWs& w, int64_t rows, const float* ssm_in,
             float* ssm_out, char* y, hipStream_t st, bool recur_ok = false) {
    const ssd_shape_t ss = seg_shape(d, rows);
    if (recur_ok && rows <= DECODE_ROWS && ssm_out) {
        // a few tokens (inference only: see block_fwd): the recurrence token by token on the state itself instead of a padded chunk
        if (ssm_in != ssm_out)
            BLK_HIP(ssm_in ? launch_copy_f32(ssm_out, ssm_in, d.HPN, st) : launch_fill_zero(ssm_out, d.HPN, st));
        return ssd_decode(&ss, ws + w.x, ws + w.dt, p->A, ws + w.B, ws + w.C, p->D, ssm_out, y, 0, st);
    }
    return ssd_fwd(&ss, ws + w.x, ws + w.dt, p->A, ws + w.B, ws + w.C, p->D, ssm_in, y, ssm_out, nullptr, ws + w.inner, w.inner_bytes, 0, st);
}

int seg_norm(const BlockDims& d, const magc_block_shape_t* sh, const magc_block_params_t* p, char* ws, const BlockWs& w, const char* zx,
             const char* y, int64_t rows, hipStream_t st) {
    const ssd_norm_shape_t ns = norm_shape(d, rows, sh->eps);
    return ssd_gated_norm_fwd(&ns, y, zx, p->norm_w, ws + w.yn, st);
}

// All of them: everything up to y and the normalised y, from the two states entering the segment.
int forward_segment(const BlockDims& d, const magc_block_shape_t* sh, const magc_block_params_t* p, char* ws, const BlockWs& w,
                    char* zx, char* y, const void* u_seg, int64_t rows, const float* ssm_in, const void* conv_in, float* ssm_out,
                    void* conv_out, hipStream_t st, bool recur_ok = false) {
    BLK_TRY(seg_in_proj(d, sh->eps, p, ws, w, u_seg, rows, zx, st));
    BLK_TRY(seg_mid(d, p, ws, w, zx, rows, conv_in, conv_out, st));
    BLK_TRY(seg_scan(d, p, ws, w, rows, ssm_in, ssm_out, y, st, recur_ok));
    BLK_TRY(seg_norm(d, sh, p, ws, w, zx, y, rows, st));
    return SSD_OK;
}

// A few tokens with both states handed on (generation): the whole block in three launches, the steps folded into
// the two products and the recurrence kernel (few_rows.hip).  `res`, if given, is added to the output.
bool few_path(const BlockDims& d, const magc_block_params_t* p, int64_t rows, const float* ssm_out, const void* u, const void* out) {
    if (rows < 1 || rows > FEW_ROWS || !ssm_out || d.N > 512 || d.P > 256) return false;
    const void* ptrs[] = {u, out, p->W_in, p->W_out, p->norm_w, p->pre_norm_w};
    for (const void* q : ptrs)
        if ((uintptr_t)q & 15) return false;
    return true;
}

// Where the states of the sequences of a few-token call live.  One sequence: the strides are not used.  Several
// (one token each, or a few): sequence b's SSM state is ssm + b ssm_bs floats (updated in place: ssm_in == ssm_out),
// its convolution states conv_in + b conv_in_bs and conv_out + b conv_out_bs elements; conv_final, if given, is
// where conv_out is moved to once the call's last kernel runs (sequence b: conv_final_bs bytes further on).
struct FewSeqs {
    int nb = 1;
    int64_t ssm_bs = 0, conv_in_bs = 0, conv_out_bs = 0;
    void* conv_final = nullptr;
    size_t conv_final_bs = 0;
};

int forward_few(const BlockDims& d, const magc_block_shape_t* sh, const magc_block_params_t* p, char* ws, const BlockWs& w,
                const void* u, int64_t tokens, const float* ssm_in, const void* conv_in, float* ssm_out, void* conv_out, void* out,
                const void* res, const FewSeqs& sq, hipStream_t st) {
    const int rows = (int)tokens * sq.nb;  // rows of every product: sequence-major, the tokens of a sequence in order
    if (sq.nb > 1 && ssm_in != ssm_out) return SSD_ERR_ARG;
    const bool fold = rows <= FEW_ROWS_VALU;  // few enough rows for the normalisations to ride on the products
    FewRowsJob in;
    memset(&in, 0, sizeof(in));
    in.rows = rows;
    in.K = d.dm;
    in.N = d.d_in_proj;
    in.mode = p->pre_norm_w && fold ? 1 : 0;
    in.x = u;
    if (p->pre_norm_w && !fold) {
        const void* un;
        BLK_TRY(seg_pre_norm(d, sh->eps, p, ws, w, u, rows, &un, st));
        in.x = un;
    }
    in.ldx = d.dm;
    in.w = p->W_in;
    in.out = ws + w.zx;
    in.ldo = d.d_in_proj;
    in.in_w = p->pre_norm_w;
    in.eps = sh->eps;
    BLK_HIP(launch_linear_few_rows(in, st));
    if (ssm_in != ssm_out) BLK_HIP(ssm_in ? launch_copy_f32(ssm_out, ssm_in, d.HPN, st) : launch_fill_zero(ssm_out, d.HPN, st));
    // many sequences, a token each, their convolution states updated where they are: two kernels (see ConvStepJob)
    const bool split_mid = sq.nb > FEW_ROWS_VALU && tokens == 1 && conv_in && sq.conv_final == conv_in && sq.conv_final_bs == (size_t)sq.conv_in_bs * 2;
    if (split_mid) {
        ConvStepJob cj;
        memset(&cj, 0, sizeof(cj));
        cj.nb = sq.nb;
        cj.H = d.H;
        cj.P = d.P;
        cj.G = d.G;
        cj.N = d.N;
        cj.zx = ws + w.zx;
        cj.ld = d.d_in_proj;
        cj.conv_w = p->conv_w;
        cj.conv_b = p->conv_b;
        cj.dt_bias = p->dt_bias;
        cj.cs = sq.conv_final;
        cj.cs_bs = sq.conv_in_bs;
        cj.x = ws + w.x;
        cj.B = ws + w.B;
        cj.C = ws + w.C;
        cj.dt = ws + w.dt;
        BLK_HIP(launch_conv_step(cj, st));
        BLK_HIP(launch_decode_strided(sq.nb, d.H, d.P, d.G, d.N, ws + w.x, ws + w.dt, p->A, ws + w.B, ws + w.C, p->D, ssm_out, sq.ssm_bs,
                                      ws + w.y, st));
    }
    DecodeMidJob mid;
    memset(&mid, 0, sizeof(mid));
    mid.nb = sq.nb;
    mid.state_bs = sq.ssm_bs;
    mid.cs_in_bs = sq.conv_in_bs;
    mid.cs_out_bs = sq.conv_out_bs;
    mid.T = (int)tokens;
    mid.H = d.H;
    mid.P = d.P;
    mid.G = d.G;
    mid.N = d.N;
    mid.zx = ws + w.zx;
    mid.ld = d.d_in_proj;
    mid.conv_w = p->conv_w;
    mid.conv_b = p->conv_b;
    mid.dt_bias = p->dt_bias;
    mid.A = p->A;
    mid.D = p->D;
    mid.cs_in = conv_in;
    mid.cs_out = conv_out;
    mid.state = ssm_out;
    mid.y = ws + w.y;
    if (!split_mid) BLK_HIP(launch_decode_mid(mid, st));
    FewRowsJob o;
    memset(&o, 0, sizeof(o));
    o.rows = rows;
    o.K = d.d_inner;
    o.N = d.dm;
    o.w = p->W_out;
    o.out = out;
    o.ldo = d.dm;
    o.ldx = d.d_inner;
    o.res = res;
    o.ldres = d.dm;
    if (d.G == 1 && fold) {  // one group: the gated normalisation rides on the product
        o.mode = 2;
        o.x = ws + w.y;
        o.in_w = p->norm_w;
        o.z = ws + w.zx;
        o.ldz = d.d_in_proj;
        o.eps = sh->eps;
    } else {
        BLK_TRY(seg_norm(d, sh, p, ws, w, ws + w.zx, ws + w.y, rows, st));
        o.x = ws + w.yn;
    }
    // the new convolution states move to their place on the back of the last launch where its threads suffice
    const size_t cs_bytes = (size_t)3 * d.conv_dim * 2;
    bool moved = false;
    if (sq.conv_final && !split_mid) {
        o.copy_src = conv_out;
        o.copy_dst = sq.conv_final;
        o.copy_bytes = cs_bytes;
        o.copy_chunks = sq.nb;
        o.copy_src_stride = (size_t)sq.conv_out_bs * 2;
        o.copy_dst_stride = sq.conv_final_bs;
        moved = few_rows_supported(o);
        if (!moved) {
            o.copy_src = o.copy_dst = nullptr;
            o.copy_bytes = 0;
            o.copy_chunks = 0;
        }
    }
    BLK_HIP(launch_linear_few_rows(o, st));
    if (sq.conv_final && !moved && !split_mid)
        for (int b = 0; b < sq.nb; ++b)  // bf16 pairs as words
            BLK_HIP(launch_copy_f32((float*)((char*)sq.conv_final + b * sq.conv_final_bs),
                                    (const float*)((const char*)conv_out + (size_t)b * sq.conv_out_bs * 2), cs_bytes / 4, st));
    return SSD_OK;
}

// The reverse of every step of a segment, given its forward activations (zx, y from the caller; x / B / C,
// dt and the normalised y in the workspace): du of the segment, parameter gradients added to `g`, the
// adjoints of the two states entering the segment.
int backward_segment(const BlockDims& d, const magc_block_shape_t* sh, const magc_block_params_t* p, const magc_block_grads_t* g,
                     char* ws, const BlockWs& w, const char* zx, const char* y, const void* u_seg, const void* dout_seg, void* du_seg,
                     int64_t rows, const float* ssm_in, const void* conv_in, const float* dssm_out, const float* dconv_out,
                     float* dssm_in, float* dconv_in, hipStream_t st) {
    const uint32_t acc = SSD_FLAG_ACCUM_PARAM;
    char* dzx = ws + w.dzx;
    // output projection
    BLK_TRY(ssd_linear_bwd(rows, d.d_inner, d.dm, ws + w.yn, 0, p->W_out, dout_seg, 0, ws + w.dyn, 0, g->dW_out, acc, st));
    // gated normalisation: dy, and dz straight into its columns of d zxbcdt
    const ssd_norm_shape_t ns = norm_shape(d, rows, sh->eps);
    BLK_TRY(ssd_gated_norm_bwd(&ns, y, zx, p->norm_w, ws + w.dyn, ws + w.dy, dzx, g->dnorm_w, ws + w.inner, w.inner_bytes, acc, st));
    // scan
    const ssd_shape_t ss = seg_shape(d, rows);
    BLK_TRY(ssd_bwd(&ss, ws + w.x, ws + w.dt, p->A, ws + w.B, ws + w.C, p->D, ssm_in, ws + w.dy, dssm_out, nullptr, ws + w.dx, ws + w.ddt,
                    g->dA, ws + w.dB, ws + w.dC, g->dD, dssm_in, ws + w.inner, w.inner_bytes, acc, st));
    // softplus of dt: into the dt columns of d zxbcdt
    const int ntile = (int)((rows + DT_ROWS - 1) / DT_ROWS);
    hipLaunchKernelGGL(k_dt_bwd, dim3(ntile), dim3(256), 0, st, (const bf16_t*)(zx + (size_t)d.off_dt * 2), (int64_t)d.d_in_proj,
                       p->dt_bias, (const bf16_t*)(ws + w.ddt), (bf16_t*)(dzx + (size_t)d.off_dt * 2), (int64_t)d.d_in_proj,
                       (float*)(ws + w.dtpart), rows, d.H);
    BLK_HIP(hipGetLastError());
    hipLaunchKernelGGL(k_colsum, dim3((d.H + 63) / 64), dim3(256), 0, st, (const float*)(ws + w.dtpart), (int64_t)ntile, d.H, g->ddt_bias, 1);
    BLK_HIP(hipGetLastError());
    // convolution: reads dx, dB, dC where the scan left them, du into the xBC columns of d zxbcdt
    const ssd_conv_shape_t cs = conv_shape(d, rows);
    const ConvSplit dxbc = {{ws + w.dx, ws + w.dB, ws + w.dC}, d.d_inner, d.d_inner + d.gn};
    BLK_TRY(conv1d_bwd_split(&cs, zx + (size_t)d.off_xbc * 2, p->conv_w, p->conv_b, conv_in, dxbc, dconv_out,
                             dzx + (size_t)d.off_xbc * 2, g->dconv_w, g->dconv_b, dconv_in, ws + w.inner, w.inner_bytes, acc, st));
    // input projection, and the normalisation in front of it (its output is cheap to redo and other layers of
    // a grid cell may have used the buffer since this layer's forward steps)
    if (!p->pre_norm_w) return ssd_linear_bwd(rows, d.dm, d.d_in_proj, u_seg, 0, p->W_in, dzx, 0, du_seg, 0, g->dW_in, acc, st);
    const void* un;
    BLK_TRY(seg_pre_norm(d, sh->eps, p, ws, w, u_seg, rows, &un, st));
    BLK_TRY(ssd_linear_bwd(rows, d.dm, d.d_in_proj, un, 0, p->W_in, dzx, 0, ws + w.dun, 0, g->dW_in, acc, st));
    const ssd_norm_shape_t ps = pre_norm_shape(d, rows, sh->eps);
    BLK_TRY(ssd_gated_norm_bwd(&ps, u_seg, nullptr, p->pre_norm_w, ws + w.dun, du_seg, nullptr, g->dpre_norm_w, ws + w.inner, w.inner_bytes,
                               acc, st));
    return SSD_OK;
}

}  // namespace
}  // namespace ssdk

using namespace ssdk;

extern "C" size_t magc_block_workspace_bytes(const magc_block_shape_t* sh, int32_t is_backward) {
    BlockDims d;
    if (check(sh, &d) != SSD_OK) return 0;
    const ssd_shape_t ss = seg_shape(d, d.s);
    if (ssd_workspace_bytes(&ss, is_backward) == 0) return 0;
    return layout(d, is_backward != 0).total;
}

// few_ok: calls of a few tokens may take the generation kernels.  Not while a training pass records checkpoints:
// those kernels round at other places than the chunked path that the backward pass recomputes the segment with,
// and the result would depend (in its last bits) on how the sequence is cut into segments.
static int block_fwd(const magc_block_shape_t* sh, const magc_block_params_t* p, const void* u, const float* init_ssm,
                     const void* init_conv, void* out, float* ssm_ckpt, void* conv_ckpt, float* final_ssm, void* final_conv,
                     void* workspace, size_t workspace_bytes, bool few_ok, void* hip_stream) {
    BlockDims d;
    BLK_TRY(check(sh, &d));
    if (!p || !p->W_in || !p->conv_w || !p->conv_b || !p->dt_bias || !p->A || !p->D || !p->norm_w || !p->W_out) return SSD_ERR_NULL;
    if ((ssm_ckpt == nullptr) != (conv_ckpt == nullptr)) return SSD_ERR_NULL;  // both kinds of checkpoint or none
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t conv_state_bytes = (size_t)3 * d.conv_dim * 2;
    if (d.L == 0) {  // nothing to do: the states pass through
        if (final_ssm) BLK_HIP(init_ssm ? launch_copy_f32(final_ssm, init_ssm, d.HPN, st) : launch_fill_zero(final_ssm, d.HPN, st));
        if (final_conv)  // bf16 values moved as 32-bit words
            BLK_HIP(init_conv ? launch_copy_f32((float*)final_conv, (const float*)init_conv, conv_state_bytes / 4, st)
                              : launch_fill_zero((float*)final_conv, conv_state_bytes / 4, st));
        return SSD_OK;
    }
    if (!u || !out) return SSD_ERR_NULL;
    const BlockWs w = layout(d, false);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return SSD_ERR_WORKSPACE;
    char* ws = (char*)workspace;
    // Several segments: a segment's output projection and the next segment's input projection do not depend on
    // each other, and either alone leaves compute units idle (4096 rows: 160 and 672 tiles for 256 units), so
    // the output projection goes to the library's side stream while the caller's stream runs ahead.
    const int64_t tail_rows = d.L - (d.nseg - 1) * d.s;
    SideStream* side = d.nseg > 1 && (tail_rows > FEW_ROWS || !few_ok) ? side_stream() : nullptr;
    bool side_busy = false;
    auto join_side = [&]() -> bool {  // the caller's stream waits for what the side stream was given
        if (!side_busy) return true;
        side_busy = false;
        return hipStreamWaitEvent(st, side->join, 0) == hipSuccess;
    };
    for (int64_t k = 0; k < d.nseg; ++k) {
        const int64_t t0 = k * d.s, rows = d.L - t0 < d.s ? d.L - t0 : d.s;
        const bool last = k + 1 == d.nseg;
        // entering states: the caller's for segment 0, else the checkpoint, or (none kept) what the last segment left
        const float* ssm_in = k == 0 ? init_ssm : ssm_ckpt ? ssm_ckpt + (size_t)k * d.HPN : (const float*)(ws + w.cssm[k & 1]);
        const void* conv_in = k == 0 ? init_conv : conv_ckpt ? (const char*)conv_ckpt + (size_t)k * conv_state_bytes : ws + w.cconv[k & 1];
        float* ssm_out = last ? final_ssm : ssm_ckpt ? ssm_ckpt + (size_t)(k + 1) * d.HPN : (float*)(ws + w.cssm[(k + 1) & 1]);
        void* conv_out = last ? final_conv : conv_ckpt ? (char*)conv_ckpt + (size_t)(k + 1) * conv_state_bytes : ws + w.cconv[(k + 1) & 1];
        const char* u_seg = (const char*)u + (size_t)t0 * d.dm * 2;
        char* out_seg = (char*)out + (size_t)t0 * d.dm * 2;
        if (few_ok && few_path(d, p, rows, ssm_out, u_seg, out_seg) && (!conv_out || conv_out != conv_in)) {
            BLK_TRY(forward_few(d, sh, p, ws, w, u_seg, rows, ssm_in, conv_in, ssm_out, conv_out, out_seg, nullptr, FewSeqs(), st));
            continue;
        }
        if (!side) {
            BLK_TRY(forward_segment(d, sh, p, ws, w, ws + w.zx, ws + w.y, u_seg, rows, ssm_in, conv_in, ssm_out, conv_out, st, few_ok));
            BLK_TRY(ssd_linear_fwd(rows, d.d_inner, d.dm, ws + w.yn, 0, p->W_out, out_seg, 0, st));
            continue;
        }
        int rc = SSD_OK;
        if (k == 0) rc = seg_in_proj(d, sh->eps, p, ws, w, u_seg, rows, ws + w.zx, st);  // later ones were issued a segment ahead
        if (rc == SSD_OK) rc = seg_mid(d, p, ws, w, ws + w.zx, rows, conv_in, conv_out, st);
        if (rc == SSD_OK) rc = seg_scan(d, p, ws, w, rows, ssm_in, ssm_out, ws + w.y, st, few_ok);
        if (!join_side() && rc == SSD_OK) rc = SSD_ERR_LAUNCH;  // the last output projection has read the normalised y
        if (rc == SSD_OK) rc = seg_norm(d, sh, p, ws, w, ws + w.zx, ws + w.y, rows, st);
        if (rc != SSD_OK) return rc;
        BLK_HIP(hipEventRecord(side->fork, st));
        BLK_HIP(hipStreamWaitEvent(side->st, side->fork, 0));
        rc = ssd_linear_fwd(rows, d.d_inner, d.dm, ws + w.yn, 0, p->W_out, out_seg, 0, side->st);
        side_busy = hipEventRecord(side->join, side->st) == hipSuccess;  // joined below whatever the product returned
        if (!side_busy) return SSD_ERR_LAUNCH;  // no event to wait for: the host is not blocked, the error is reported
        if (rc == SSD_OK && !last) {
            // every reader of this segment's zxbcdt is already in the stream: the next one may replace it
            const int64_t t1 = t0 + d.s, rows1 = d.L - t1 < d.s ? d.L - t1 : d.s;
            rc = seg_in_proj(d, sh->eps, p, ws, w, (const char*)u + (size_t)t1 * d.dm * 2, rows1, ws + w.zx, st);
        }
        if (rc != SSD_OK) {
            (void)join_side();
            return rc;
        }
    }
    if (!join_side()) return SSD_ERR_LAUNCH;
    return SSD_OK;
}

extern "C" int magc_block_fwd(const magc_block_shape_t* sh, const magc_block_params_t* p, const void* u, const float* init_ssm,
                              const void* init_conv, void* out, float* ssm_ckpt, void* conv_ckpt, float* final_ssm, void* final_conv,
                              void* workspace, size_t workspace_bytes, void* hip_stream) {
    // no checkpoint store: inference (prefill, generation)
    return block_fwd(sh, p, u, init_ssm, init_conv, out, ssm_ckpt, conv_ckpt, final_ssm, final_conv, workspace, workspace_bytes,
                     ssm_ckpt == nullptr, hip_stream);
}

extern "C" int magc_block_bwd(const magc_block_shape_t* sh, const magc_block_params_t* p, const void* u, const float* init_ssm,
                              const void* init_conv, const void* dout, const float* dfinal_ssm, const float* dfinal_conv,
                              const float* ssm_ckpt, const void* conv_ckpt, void* du, const magc_block_grads_t* g, float* dinit_ssm,
                              float* dinit_conv, void* workspace, size_t workspace_bytes, uint32_t flags, void* hip_stream) {
    BlockDims d;
    BLK_TRY(check(sh, &d));
    if (flags & ~(uint32_t)SSD_FLAG_ACCUM_PARAM) return SSD_ERR_ARG;
    if (!p || !p->W_in || !p->conv_w || !p->conv_b || !p->dt_bias || !p->A || !p->D || !p->norm_w || !p->W_out) return SSD_ERR_NULL;
    if (!g || !g->dW_in || !g->dconv_w || !g->dconv_b || !g->ddt_bias || !g->dA || !g->dD || !g->dnorm_w || !g->dW_out) return SSD_ERR_NULL;
    if (p->pre_norm_w && !g->dpre_norm_w) return SSD_ERR_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    if (!(flags & SSD_FLAG_ACCUM_PARAM)) {  // every segment adds to the parameter gradients
        BLK_HIP(launch_fill_zero(g->dW_in, (size_t)d.d_in_proj * d.dm, st));
        BLK_HIP(launch_fill_zero(g->dconv_w, (size_t)d.conv_dim * 4, st));
        BLK_HIP(launch_fill_zero(g->dconv_b, (size_t)d.conv_dim, st));
        BLK_HIP(launch_fill_zero(g->ddt_bias, (size_t)d.H, st));
        BLK_HIP(launch_fill_zero(g->dA, (size_t)d.H, st));
        BLK_HIP(launch_fill_zero(g->dD, (size_t)d.H, st));
        BLK_HIP(launch_fill_zero(g->dnorm_w, (size_t)d.d_inner, st));
        BLK_HIP(launch_fill_zero(g->dW_out, (size_t)d.dm * d.d_inner, st));
        if (p->pre_norm_w) BLK_HIP(launch_fill_zero(g->dpre_norm_w, (size_t)d.dm, st));
    }
    if (d.L == 0) {  // the state adjoints pass through
        if (dinit_ssm) BLK_HIP(dfinal_ssm ? launch_copy_f32(dinit_ssm, dfinal_ssm, d.HPN, st) : launch_fill_zero(dinit_ssm, d.HPN, st));
        if (dinit_conv)
            BLK_HIP(dfinal_conv ? launch_copy_f32(dinit_conv, dfinal_conv, (size_t)3 * d.conv_dim, st)
                                : launch_fill_zero(dinit_conv, (size_t)3 * d.conv_dim, st));
        return SSD_OK;
    }
    if (!u || !dout || !du || (d.nseg > 1 && (!ssm_ckpt || !conv_ckpt))) return SSD_ERR_NULL;
    const BlockWs w = layout(d, true);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return SSD_ERR_WORKSPACE;
    char* ws = (char*)workspace;
    const size_t conv_state_bytes = (size_t)3 * d.conv_dim * 2;
    for (int64_t k = d.nseg - 1; k >= 0; --k) {
        const int64_t t0 = k * d.s, rows = d.L - t0 < d.s ? d.L - t0 : d.s;
        const bool last = k + 1 == d.nseg;
        const float* ssm_in = k ? ssm_ckpt + (size_t)k * d.HPN : init_ssm;
        const void* conv_in = k ? (const char*)conv_ckpt + (size_t)k * conv_state_bytes : init_conv;
        // adjoints of the states leaving this segment (the caller's behind the last one) / entering it
        const float* dssm_out = last ? dfinal_ssm : (const float*)(ws + w.dssm[(k + 1) & 1]);
        const float* dconv_out = last ? dfinal_conv : (const float*)(ws + w.dconv[(k + 1) & 1]);
        float* dssm_in = k ? (float*)(ws + w.dssm[k & 1]) : dinit_ssm;
        float* dconv_in = k ? (float*)(ws + w.dconv[k & 1]) : dinit_conv;
        const void* u_seg = (const char*)u + (size_t)t0 * d.dm * 2;
        // Recompute_Forward: zxbcdt, (x | B | C), dt, y, normalised y of this segment
        BLK_TRY(forward_segment(d, sh, p, ws, w, ws + w.zx, ws + w.y, u_seg, rows, ssm_in, conv_in, nullptr, nullptr, st));
        BLK_TRY(backward_segment(d, sh, p, g, ws, w, ws + w.zx, ws + w.y, u_seg, (const char*)dout + (size_t)t0 * d.dm * 2,
                                 (char*)du + (size_t)t0 * d.dm * 2, rows, ssm_in, conv_in, dssm_out, dconv_out, dssm_in, dconv_in, st));
    }
    return SSD_OK;
}

// ---------------------------------------------------------------------------------------------------
// A stack of whole blocks with residual adds, x_{j+1} = x_j + Block_j(x_j), on the two-axis grid of MA-GC
// (Sec. 3.2/3.3, Alg. 1 and 2): the input of every `layer_interval`-th layer is kept for the whole sequence
// (layer-axis checkpoints), the SSM and convolution states of every layer are kept every `segment` tokens
// (sequence-axis checkpoints).  The backward pass walks the cells right to left and top to bottom: inside a
// cell it first restores, from the layer checkpoint and the cell's state checkpoints, the input of every layer
// of the cell together with its zxbcdt and y (the per-token activations C_grid of App. C, Tab. 7 counts), then
// back-propagates through the layers top down -- redoing only the cheap streaming steps of a layer -- each
// layer's two state adjoints being handed to the cell on its left.
namespace ssdk {
namespace {

// dst = a + b, bf16, 16-byte vectors (n a multiple of 8)
__global__ __launch_bounds__(256) void k_add_bf16(bf16_t* dst, const bf16_t* a, const bf16_t* b, int64_t n8) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (int64_t)gridDim.x * 256) {
        const b8 x = *(const b8*)((const __bf16*)a + i * 8), y = *(const b8*)((const __bf16*)b + i * 8);
        b8 o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (__bf16)((float)x[e] + (float)y[e]);
        *(b8*)((__bf16*)dst + i * 8) = o;
    }
}

hipError_t add_bf16(void* dst, const void* a, const void* b, int64_t n, hipStream_t st) {
    if (n == 0) return hipSuccess;
    const int64_t n8 = n / 8, blocks = (n8 + 255) / 256;
    hipLaunchKernelGGL(k_add_bf16, dim3((unsigned)(blocks < 8192 ? blocks : 8192)), dim3(256), 0, st, (bf16_t*)dst, (const bf16_t*)a,
                       (const bf16_t*)b, n8);
    return hipGetLastError();
}

struct StackDims {
    BlockDims b;
    int NL, l, ngl;  // layers, layer interval, layer groups
    size_t act, conv_state, conv_adj;
};

int check_stack(const magc_blockstack_shape_t* sh, StackDims* d) {
    if (!sh) return SSD_ERR_NULL;
    const int rc = check(&sh->block, &d->b);
    if (rc != SSD_OK) return rc;
    if (sh->nlayers <= 0 || sh->layer_interval <= 0 || sh->layer_interval > sh->nlayers) return SSD_ERR_SHAPE;
    d->NL = sh->nlayers;
    d->l = sh->layer_interval;
    d->ngl = (d->NL + d->l - 1) / d->l;
    d->act = (size_t)d->b.s * d->b.dm * 2;
    d->conv_state = (size_t)3 * d->b.conv_dim * 2;
    d->conv_adj = (size_t)3 * d->b.conv_dim * 4;
    return SSD_OK;
}

magc_block_shape_t cell_shape(const magc_blockstack_shape_t* sh, int64_t rows) {
    magc_block_shape_t c = sh->block;
    c.seqlen = rows;  // one segment: the cell
    return c;
}

struct StackWs {
    size_t act[2], xs, zx, y, dcur, du, dssm, dconv, fin_ssm, fin_conv, inner, inner_bytes, total;
    size_t zx_bytes, y_bytes;  // per layer of a cell
};

StackWs stack_layout(const magc_blockstack_shape_t* sh, const StackDims& d, bool bwd) {
    StackWs w;
    memset(&w, 0, sizeof(w));
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += al(bytes);
        return o;
    };
    w.act[0] = take(d.act);
    w.act[1] = take(d.act);
    w.fin_ssm = take(d.b.HPN * 4);
    w.fin_conv = take((size_t)FEW_ROWS * d.conv_state);  // one per sequence of a batched generation step
    w.zx_bytes = al((size_t)d.b.s * d.b.d_in_proj * 2);
    w.y_bytes = al((size_t)d.b.s * d.b.d_inner * 2);
    if (bwd) {
        w.xs = take((size_t)d.l * d.act);
        // what a cell keeps per layer and token besides the layer inputs: zxbcdt and y (C_grid of App. C, Tab. 7)
        w.zx = take((size_t)d.l * w.zx_bytes);
        w.y = take((size_t)d.l * w.y_bytes);
        w.dcur = take(d.act);
        w.du = take(d.act);
        w.dssm = take((size_t)d.NL * 2 * d.b.HPN * 4);      // per layer, two buffers used alternately
        w.dconv = take((size_t)d.NL * 2 * d.conv_adj);
    }
    const magc_block_shape_t c = cell_shape(sh, d.b.s);
    size_t inner = magc_block_workspace_bytes(&c, bwd ? 1 : 0);
    if (d.b.L % d.b.s) {  // the short last segment pads the scan: its scratch may differ
        const magc_block_shape_t ct = cell_shape(sh, d.b.L % d.b.s);
        const size_t t = magc_block_workspace_bytes(&ct, bwd ? 1 : 0);
        inner = t > inner ? t : inner;
    }
    const size_t f = magc_block_workspace_bytes(&c, 0);  // the forward pass calls the block's forward entry point
    inner = f > inner ? f : inner;
    if (bwd) {  // the backward pass lays a block workspace out in this region itself
        const size_t own = layout(d.b, true).total;
        inner = own > inner ? own : inner;
    }
    w.inner = take(inner);
    w.inner_bytes = inner;
    w.total = off;
    return w;
}

bool params_ok(const magc_block_params_t* p, int n) {
    if (!p) return false;
    for (int j = 0; j < n; ++j)
        if (!p[j].W_in || !p[j].conv_w || !p[j].conv_b || !p[j].dt_bias || !p[j].A || !p[j].D || !p[j].norm_w || !p[j].W_out) return false;
    return true;
}

}  // namespace
}  // namespace ssdk

extern "C" size_t magc_blockstack_workspace_bytes(const magc_blockstack_shape_t* sh, int32_t is_backward) {
    StackDims d;
    if (check_stack(sh, &d) != SSD_OK) return 0;
    const magc_block_shape_t c = cell_shape(sh, d.b.s);
    if (magc_block_workspace_bytes(&c, is_backward) == 0) return 0;
    return stack_layout(sh, d, is_backward != 0).total;
}

extern "C" int magc_blockstack_fwd(const magc_blockstack_shape_t* sh, const magc_block_params_t* params, const void* x0, void* out,
                                   void* l_ckpt, float* ssm_ckpt, void* conv_ckpt, void* workspace, size_t workspace_bytes,
                                   void* hip_stream) {
    StackDims d;
    BLK_TRY(check_stack(sh, &d));
    if (!params_ok(params, d.NL)) return SSD_ERR_NULL;
    if (d.b.L == 0) return SSD_OK;
    if (!x0 || !out || (d.ngl > 1 && !l_ckpt) || (d.b.nseg > 1 && (!ssm_ckpt || !conv_ckpt))) return SSD_ERR_NULL;
    const StackWs w = stack_layout(sh, d, false);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return SSD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    const size_t row = (size_t)d.b.dm * 2;
    for (int64_t k = 0; k < d.b.nseg; ++k) {
        const int64_t t0 = k * d.b.s, rows = d.b.L - t0 < d.b.s ? d.b.L - t0 : d.b.s;
        const magc_block_shape_t c = cell_shape(sh, rows);
        const bool last = k + 1 == d.b.nseg;
        const char* cur = (const char*)x0 + (size_t)t0 * row;
        for (int j = 0; j < d.NL; ++j) {
            if (j && j % d.l == 0) {  // layer-axis checkpoint: the input of layer j for these tokens
                char* slot = (char*)l_ckpt + ((size_t)(j / d.l - 1) * d.b.L + t0) * row;
                BLK_HIP(launch_copy_f32((float*)slot, (const float*)cur, (size_t)rows * d.b.dm / 2, st));  // bf16 pairs as words
                cur = slot;
            }
            // sequence-axis checkpoints of layer j: slot k = the states entering segment k (slot 0 unused: zeros)
            float* sj = ssm_ckpt ? ssm_ckpt + (size_t)j * d.b.nseg * d.b.HPN : nullptr;
            char* cj = conv_ckpt ? (char*)conv_ckpt + (size_t)j * d.b.nseg * d.conv_state : nullptr;
            const float* ssm_in = k ? sj + (size_t)k * d.b.HPN : nullptr;
            const void* conv_in = k ? cj + (size_t)k * d.conv_state : nullptr;
            float* ssm_out = last ? (float*)(ws + w.fin_ssm) : sj + (size_t)(k + 1) * d.b.HPN;
            void* conv_out = last ? (void*)(ws + w.fin_conv) : (void*)(cj + (size_t)(k + 1) * d.conv_state);
            char* y = ws + w.act[j & 1];
            BLK_TRY(block_fwd(&c, &params[j], cur, ssm_in, conv_in, y, nullptr, nullptr, ssm_out, conv_out, ws + w.inner, w.inner_bytes,
                              false, st));
            char* nxt = j + 1 == d.NL ? (char*)out + (size_t)t0 * row : y;  // x_{j+1} = x_j + Block_j(x_j)
            BLK_HIP(add_bf16(nxt, cur, y, rows * d.b.dm, st));
            cur = nxt;
        }
    }
    return SSD_OK;
}

extern "C" int magc_blockstack_bwd(const magc_blockstack_shape_t* sh, const magc_block_params_t* params, const void* x0, const void* dout,
                                   const void* l_ckpt, const float* ssm_ckpt, const void* conv_ckpt, void* dx0,
                                   const magc_block_grads_t* grads, void* workspace, size_t workspace_bytes, uint32_t flags,
                                   void* hip_stream) {
    StackDims d;
    BLK_TRY(check_stack(sh, &d));
    if (flags & ~(uint32_t)SSD_FLAG_ACCUM_PARAM) return SSD_ERR_ARG;
    if (!params_ok(params, d.NL) || !grads) return SSD_ERR_NULL;
    for (int j = 0; j < d.NL; ++j)
        if (!grads[j].dW_in || !grads[j].dconv_w || !grads[j].dconv_b || !grads[j].ddt_bias || !grads[j].dA || !grads[j].dD ||
            !grads[j].dnorm_w || !grads[j].dW_out || (params[j].pre_norm_w && !grads[j].dpre_norm_w))
            return SSD_ERR_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t row = (size_t)d.b.dm * 2;
    if (!(flags & SSD_FLAG_ACCUM_PARAM)) {  // every cell adds to the parameter gradients of its layers
        for (int j = 0; j < d.NL; ++j) {
            BLK_HIP(launch_fill_zero(grads[j].dW_in, (size_t)d.b.d_in_proj * d.b.dm, st));
            BLK_HIP(launch_fill_zero(grads[j].dconv_w, (size_t)d.b.conv_dim * 4, st));
            BLK_HIP(launch_fill_zero(grads[j].dconv_b, (size_t)d.b.conv_dim, st));
            BLK_HIP(launch_fill_zero(grads[j].ddt_bias, (size_t)d.b.H, st));
            BLK_HIP(launch_fill_zero(grads[j].dA, (size_t)d.b.H, st));
            BLK_HIP(launch_fill_zero(grads[j].dD, (size_t)d.b.H, st));
            BLK_HIP(launch_fill_zero(grads[j].dnorm_w, (size_t)d.b.d_inner, st));
            BLK_HIP(launch_fill_zero(grads[j].dW_out, (size_t)d.b.dm * d.b.d_inner, st));
            if (params[j].pre_norm_w) BLK_HIP(launch_fill_zero(grads[j].dpre_norm_w, (size_t)d.b.dm, st));
        }
    }
    if (d.b.L == 0) return SSD_OK;
    if (!x0 || !dout || !dx0 || (d.ngl > 1 && !l_ckpt) || (d.b.nseg > 1 && (!ssm_ckpt || !conv_ckpt))) return SSD_ERR_NULL;
    const StackWs w = stack_layout(sh, d, true);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return SSD_ERR_WORKSPACE;
    char* ws = (char*)workspace;
    // a cell's layer uses the block's own workspace layout inside the inner region (buffers of one segment;
    // its scan scratch covers both a whole segment and the short last one)
    const BlockWs bw = layout(d.b, true);
    if (bw.total > w.inner_bytes) return SSD_ERR_WORKSPACE;
    char* bws = ws + w.inner;
    for (int64_t k = d.b.nseg - 1; k >= 0; --k) {
        const int64_t t0 = k * d.b.s, rows = d.b.L - t0 < d.b.s ? d.b.L - t0 : d.b.s;
        const magc_block_shape_t c = cell_shape(sh, rows);
        BlockDims dc;
        BLK_TRY(check(&c, &dc));
        const bool last = k + 1 == d.b.nseg;
        const char* dcur = (const char*)dout + (size_t)t0 * row;  // gradient of the stack output for these tokens
        for (int m = d.ngl - 1; m >= 0; --m) {
            const int j0 = m * d.l, j1 = (j0 + d.l < d.NL ? j0 + d.l : d.NL) - 1;
            // Recompute_Forward of Alg. 2: from the cell's layer checkpoint and its layers' state checkpoints,
            // the input x_j, zxbcdt_j and y_j of every layer of the cell
            const char* xin = m ? (const char*)l_ckpt + ((size_t)(m - 1) * d.b.L + t0) * row : (const char*)x0 + (size_t)t0 * row;
            for (int j = j0; j <= j1; ++j) {
                const float* ssm_in = k ? ssm_ckpt + ((size_t)j * d.b.nseg + k) * d.b.HPN : nullptr;
                const void* conv_in = k ? (const char*)conv_ckpt + ((size_t)j * d.b.nseg + k) * d.conv_state : nullptr;
                char* zx = ws + w.zx + (size_t)(j - j0) * w.zx_bytes;
                char* y = ws + w.y + (size_t)(j - j0) * w.y_bytes;
                BLK_TRY(seg_in_proj(dc, c.eps, &params[j], bws, bw, xin, rows, zx, st));
                BLK_TRY(seg_mid(dc, &params[j], bws, bw, zx, rows, conv_in, nullptr, st));
                BLK_TRY(seg_scan(dc, &params[j], bws, bw, rows, ssm_in, nullptr, y, st));
                if (j < j1) {  // the next layer's input
                    BLK_TRY(seg_norm(dc, &c, &params[j], bws, bw, zx, y, rows, st));
                    char* out = ws + w.act[0];
                    BLK_TRY(ssd_linear_fwd(rows, d.b.d_inner, d.b.dm, bws + bw.yn, 0, params[j].W_out, out, 0, st));
                    char* nxt = ws + w.xs + (size_t)(j - j0 + 1) * d.act;
                    BLK_HIP(add_bf16(nxt, xin, out, rows * d.b.dm, st));
                    xin = nxt;
                }
            }
            // back through the layers, top down: dx_j = dx_{j+1} + Block_j^T(dx_{j+1})
            for (int j = j1; j >= j0; --j) {
                const char* xj = j == j0 ? (m ? (const char*)l_ckpt + ((size_t)(m - 1) * d.b.L + t0) * row : (const char*)x0 + (size_t)t0 * row)
                                         : ws + w.xs + (size_t)(j - j0) * d.act;
                const float* ssm_in = k ? ssm_ckpt + ((size_t)j * d.b.nseg + k) * d.b.HPN : nullptr;
                const void* conv_in = k ? (const char*)conv_ckpt + ((size_t)j * d.b.nseg + k) * d.conv_state : nullptr;
                const char* zx = ws + w.zx + (size_t)(j - j0) * w.zx_bytes;
                const char* y = ws + w.y + (size_t)(j - j0) * w.y_bytes;
                // the cheap steps again from zxbcdt_j and y_j: (x | B | C), dt, the normalised y
                BLK_TRY(seg_mid(dc, &params[j], bws, bw, zx, rows, conv_in, nullptr, st));
                BLK_TRY(seg_norm(dc, &c, &params[j], bws, bw, zx, y, rows, st));
                // this layer's state adjoints: written for segment k into buffer k % 2, read by segment k - 1 from it
                float* dssm_w = (float*)(ws + w.dssm + ((size_t)j * 2 + (k & 1)) * d.b.HPN * 4);
                float* dconv_w = (float*)(ws + w.dconv + ((size_t)j * 2 + (k & 1)) * d.conv_adj);
                const float* dssm_r = last ? nullptr : (const float*)(ws + w.dssm + ((size_t)j * 2 + ((k + 1) & 1)) * d.b.HPN * 4);
                const float* dconv_r = last ? nullptr : (const float*)(ws + w.dconv + ((size_t)j * 2 + ((k + 1) & 1)) * d.conv_adj);
                BLK_TRY(backward_segment(dc, &c, &params[j], &grads[j], bws, bw, zx, y, xj, dcur, ws + w.du, rows, ssm_in, conv_in, dssm_r,
                                         dconv_r, k ? dssm_w : nullptr, k ? dconv_w : nullptr, st));
                char* dnext = (j == 0) ? (char*)dx0 + (size_t)t0 * row : ws + w.dcur;
                BLK_HIP(add_bf16(dnext, dcur, ws + w.du, rows * d.b.dm, st));
                dcur = dnext;
            }
        }
    }
    return SSD_OK;
}

// Forward only, nothing kept: the stack as a language model runs it at inference.  The states of every layer
// live in two caller-owned arrays and are replaced by the states behind the last token of the call, so a
// prompt of any length (in segments: memory does not grow with it) and then single tokens are the same call.
extern "C" int magc_blockstack_infer(const magc_blockstack_shape_t* sh, const magc_block_params_t* params, const void* x0, void* out,
                                     float* ssm_state, void* conv_state, int32_t fresh, void* workspace, size_t workspace_bytes,
                                     void* hip_stream) {
    StackDims d;
    BLK_TRY(check_stack(sh, &d));
    if (!params_ok(params, d.NL) || !ssm_state || !conv_state) return SSD_ERR_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    if (d.b.L == 0) {
        if (fresh) {
            BLK_HIP(launch_fill_zero(ssm_state, (size_t)d.NL * d.b.HPN, st));
            BLK_HIP(launch_fill_zero((float*)conv_state, (size_t)d.NL * d.conv_state / 4, st));
        }
        return SSD_OK;
    }
    if (!x0 || !out) return SSD_ERR_NULL;
    const StackWs w = stack_layout(sh, d, false);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return SSD_ERR_WORKSPACE;
    char* ws = (char*)workspace;
    const size_t row = (size_t)d.b.dm * 2;
    for (int64_t k = 0; k < d.b.nseg; ++k) {
        const int64_t t0 = k * d.b.s, rows = d.b.L - t0 < d.b.s ? d.b.L - t0 : d.b.s;
        const magc_block_shape_t c = cell_shape(sh, rows);
        BlockDims dc;
        BLK_TRY(check(&c, &dc));
        const BlockWs bw = layout(dc, false);  // for the few-token path, which lays a block workspace out itself
        if (bw.total > w.inner_bytes) return SSD_ERR_WORKSPACE;
        char* bws = ws + w.inner;
        const bool zero = fresh && k == 0;
        // a few tokens: the recurrence runs on the layer's SSM state itself; a segment: through a spare state
        const bool in_place = rows <= DECODE_ROWS;
        const char* cur = (const char*)x0 + (size_t)t0 * row;
        for (int j = 0; j < d.NL; ++j) {
            float* sj = ssm_state + (size_t)j * d.b.HPN;
            char* cj = (char*)conv_state + (size_t)j * d.conv_state;
            float* ssm_out = in_place ? sj : (float*)(ws + w.fin_ssm);
            char* y = ws + w.act[j & 1];
            char* nxt = j + 1 == d.NL ? (char*)out + (size_t)t0 * row : y;  // x_{j+1} = x_j + Block_j(x_j)
            bool conv_moved = false;
            if (few_path(dc, &params[j], rows, ssm_out, cur, nxt)) {
                // generation: the residual and the move of the convolution state ride on the output product
                FewSeqs sq;
                sq.conv_final = cj;
                conv_moved = true;
                BLK_TRY(forward_few(dc, &c, &params[j], bws, bw, cur, rows, zero ? nullptr : sj, zero ? nullptr : cj, ssm_out,
                                    ws + w.fin_conv, nxt, cur, sq, st));
            } else {
                BLK_TRY(magc_block_fwd(&c, &params[j], cur, zero ? nullptr : sj, zero ? nullptr : cj, y, nullptr, nullptr, ssm_out,
                                       ws + w.fin_conv, ws + w.inner, w.inner_bytes, st));
                BLK_HIP(add_bf16(nxt, cur, y, rows * d.b.dm, st));
            }
            if (!in_place) BLK_HIP(launch_copy_f32(sj, ssm_out, d.b.HPN, st));
            if (!conv_moved) BLK_HIP(launch_copy_f32((float*)cj, (const float*)(ws + w.fin_conv), d.conv_state / 4, st));  // bf16 pairs as words
            cur = nxt;
        }
    }
    return SSD_OK;
}

// One generation step for several independent sequences at once: every parameter is read once for all of them.
extern "C" int magc_blockstack_decode(const magc_blockstack_shape_t* sh_in, const magc_block_params_t* params, int32_t nseq, const void* x0,
                                      void* out, float* ssm_state, void* conv_state, void* workspace, size_t workspace_bytes,
                                      void* hip_stream) {
    if (!sh_in) return SSD_ERR_NULL;
    magc_blockstack_shape_t one = *sh_in;  // a token per sequence whatever block.seqlen says: sizes the workspace
    one.block.seqlen = 1;
    const magc_blockstack_shape_t* sh = &one;
    StackDims d;
    BLK_TRY(check_stack(sh, &d));
    if (nseq < 0 || nseq > FEW_ROWS) return SSD_ERR_SHAPE;
    if (!params_ok(params, d.NL)) return SSD_ERR_NULL;
    if (nseq == 0) return SSD_OK;
    if (!x0 || !out || !ssm_state || !conv_state) return SSD_ERR_NULL;
    const StackWs w = stack_layout(sh, d, false);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return SSD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    char* ws = (char*)workspace;
    const size_t row = (size_t)d.b.dm * 2;
    const magc_block_shape_t c = cell_shape(sh, 1);  // a token per sequence
    BlockDims dc;
    BLK_TRY(check(&c, &dc));
    const BlockWs bw = layout(dc, false);
    if (bw.total > w.inner_bytes) return SSD_ERR_WORKSPACE;
    bool batched = nseq <= d.b.s;  // the rows of all sequences fit the buffers of one segment
    for (int j = 0; j < d.NL && batched; ++j) batched = few_path(dc, &params[j], nseq, ssm_state, x0, out);
    if (!batched) {  // shapes or alignments the generation kernels do not take: sequence by sequence
        for (int b = 0; b < nseq; ++b)
            BLK_TRY(magc_blockstack_infer(&one, params, (const char*)x0 + b * row, (char*)out + b * row, ssm_state + (size_t)b * d.NL * d.b.HPN,
                                          (char*)conv_state + (size_t)b * d.NL * d.conv_state, 0, workspace, workspace_bytes, hip_stream));
        return SSD_OK;
    }
    const char* cur = (const char*)x0;
    for (int j = 0; j < d.NL; ++j) {
        float* sj = ssm_state + (size_t)j * d.b.HPN;             // sequence 0; sequence b: NL states further on
        char* cj = (char*)conv_state + (size_t)j * d.conv_state;
        char* nxt = j + 1 == d.NL ? (char*)out : ws + w.act[j & 1];
        FewSeqs sq;
        sq.nb = nseq;
        sq.ssm_bs = (int64_t)d.NL * d.b.HPN;
        sq.conv_in_bs = (int64_t)d.NL * 3 * d.b.conv_dim;
        sq.conv_out_bs = (int64_t)3 * d.b.conv_dim;
        sq.conv_final = cj;
        sq.conv_final_bs = (size_t)d.NL * d.conv_state;
        BLK_TRY(forward_few(dc, &c, &params[j], ws + w.inner, bw, cur, 1, sj, cj, sj, ws + w.fin_conv, nxt, cur, sq, st));
        cur = nxt;
    }
    return SSD_OK;
}
