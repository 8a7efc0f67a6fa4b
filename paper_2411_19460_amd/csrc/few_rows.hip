// Generation: a token or a few at a time through a block (the recurrence of Sec. 3.1, Eq. 1 around which the
// block's other steps shrink to vectors).  Every kernel here is bound by reading each parameter once and the
// SSM state twice per call.  Up to four rows (a sequence on its own) the block's steps are folded into three
// launches that do exactly that, on the vector ALUs:
//   k_linear_few<1>  zxbcdt = RMSNorm(u) pre_norm_w W_in^T   (or plain u W_in^T)
//   k_decode_mid     convolution + SiLU, softplus(dt), the state update and y = C h + D x, token by token
//   k_linear_few<2>  out = RMSNorm(y silu(z)) norm_w W_out^T (+ the residual)
// With more rows (several sequences generated together) the per-row arithmetic would bound those kernels:
// the products then run as small MFMAs (k_linear_few_mfma), the normalisations as the library's own kernels,
// the convolution as a step of its own (k_conv_step) in front of the recurrence kernel of decode.hip.
#include "ssd_internal.h"

namespace ssdk {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float sigmoid_fast(float z) { return __builtin_amdgcn_rcpf(1.f + __expf(-z)); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// what storing a value in bf16 and reading it back leaves of it
__device__ __forceinline__ float through_bf16(float v) { return (float)(__bf16)v; }

struct FewParams {
    const __bf16 *x, *w, *z, *res;
    __bf16* out;
    const float* in_w;
    int64_t ldx, ldz, ldo, ldres;
    int rows, K, N;
    float eps;
};

// out[r, n] = sum_k f(x)[r, k] w[n, k] (+ res[r, n]) for r < rows <= R.  A wave owns CPW columns n and walks k
// with 16-byte loads, so every weight is read once, in full cache lines; the few input rows come from the
// caches.  MODE 0: f(x) = x.  MODE 1: f(x) = x / sqrt(mean x^2 + eps) * in_w.  MODE 2: the same of g = x z sigmoid(z).
// A wave sees whole rows, so the mean comes out of the same loop and scales the finished sums.  With few rows
// the operands of two k steps are requested before either is used (twice the bytes in flight per wave).
// The first workgroups also move `copy_chunks` pieces of `copy_n` 16-byte vectors from copy_src to copy_dst: a small
// state (one piece per sequence) that the kernel before this one still read in its old place.
struct FewOperands {
    const void* copy_src;
    void* copy_dst;
    int copy_n, copy_chunks;                   // vectors per chunk, chunks
    int64_t copy_src_stride, copy_dst_stride;  // vectors between chunks
};

template <int MODE, int R, int CPW>
struct FewStep {
    bf16x8 wv[CPW], xv[R], zv[MODE == 2 ? R : 1];
    float iw[MODE ? 8 : 1];

    __device__ __forceinline__ void load(const FewParams& fp, const __bf16* w0, int k) {
#pragma unroll
        for (int c = 0; c < CPW; ++c) wv[c] = *(const bf16x8*)(w0 + (int64_t)c * fp.K + k);
        if (MODE) {
            const f32x4 a = *(const f32x4*)(fp.in_w + k), b = *(const f32x4*)(fp.in_w + k + 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                iw[e] = a[e];
                iw[4 + e] = b[e];
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (r < fp.rows) {
                xv[r] = *(const bf16x8*)(fp.x + r * fp.ldx + k);
                if (MODE == 2) zv[r] = *(const bf16x8*)(fp.z + r * fp.ldz + k);
            }
        }
    }

    __device__ __forceinline__ void use(const FewParams& fp, float (&acc)[R][CPW], float (&ss)[R]) const {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if (r < fp.rows) {
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    float v = (float)xv[r][e];
                    if (MODE == 2) {
                        const float zz = (float)zv[r][e];
                        v *= zz * sigmoid_fast(zz);
                    }
                    if (MODE) {
                        ss[r] = fmaf(v, v, ss[r]);
                        v *= iw[e];
                    }
#pragma unroll
                    for (int c = 0; c < CPW; ++c) acc[r][c] = fmaf(v, (float)wv[c][e], acc[r][c]);
                }
            }
        }
    }
};

// KS waves of a workgroup share a wave's columns and take every KS-th k step each (a wave that walks all of a
// long row alone waits for one load after the other: more, shorter waves keep more bytes in flight); their
// partial sums meet in LDS.
template <int MODE, int R, int CPW, int KS>
__global__ __launch_bounds__(256) void k_linear_few(FewParams fp, FewOperands fo) {
    __shared__ float red[4][R * (CPW + 1)];
    if (fo.copy_n) {
        const int i = blockIdx.x * 256 + threadIdx.x;
        if (i < fo.copy_n * fo.copy_chunks) {
            const int c = i / fo.copy_n, v = i - c * fo.copy_n;
            ((f32x4*)fo.copy_dst)[c * fo.copy_dst_stride + v] = ((const f32x4*)fo.copy_src)[c * fo.copy_src_stride + v];
        }
    }
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int slot = wv / KS, kp = wv % KS;  // which columns of the workgroup, which share of k
    const int n0 = (blockIdx.x * (4 / KS) + slot) * CPW;
    const bool live = n0 < fp.N;
    float acc[R][CPW], ss[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        ss[r] = 0.f;
#pragma unroll
        for (int c = 0; c < CPW; ++c) acc[r][c] = 0.f;
    }
    const __bf16* w0 = fp.w + (int64_t)n0 * fp.K;
    constexpr bool TWO = R <= 4;
    constexpr int STEP = 512 * KS;  // k between a wave's consecutive steps
    if (live) {
        for (int k = lane * 8 + 512 * kp; k < fp.K; k += TWO ? 2 * STEP : STEP) {
            FewStep<MODE, R, CPW> a, b;
            const bool two = TWO && k + STEP < fp.K;
            a.load(fp, w0, k);
            if (two) b.load(fp, w0, k + STEP);
            a.use(fp, acc, ss);
            if (two) b.use(fp, acc, ss);
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (MODE) ss[r] = wave_sum(ss[r]);
#pragma unroll
        for (int c = 0; c < CPW; ++c) acc[r][c] = wave_sum(acc[r][c]);
    }
    if (KS > 1) {
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < R; ++r) {
                red[wv][r * (CPW + 1) + CPW] = ss[r];
#pragma unroll
                for (int c = 0; c < CPW; ++c) red[wv][r * (CPW + 1) + c] = acc[r][c];
            }
        }
        __syncthreads();
        if (kp != 0) return;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            ss[r] = 0.f;
#pragma unroll
            for (int c = 0; c < CPW; ++c) acc[r][c] = 0.f;
#pragma unroll
            for (int q = 0; q < KS; ++q) {  // fixed order: the result does not depend on which wave finished first
                ss[r] += red[slot * KS + q][r * (CPW + 1) + CPW];
#pragma unroll
                for (int c = 0; c < CPW; ++c) acc[r][c] += red[slot * KS + q][r * (CPW + 1) + c];
            }
        }
    }
    if (!live || lane != 0) return;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (r < fp.rows) {
            const float rstd = MODE ? rsqrtf(ss[r] / (float)fp.K + fp.eps) : 1.f;
#pragma unroll
            for (int c = 0; c < CPW; ++c) {
                float v = acc[r][c] * rstd;
                if (fp.res) v += (float)fp.res[r * fp.ldres + n0 + c];
                fp.out[r * fp.ldo + n0 + c] = (__bf16)v;
            }
        }
    }
}

template <int MODE, int CPW, int KS>
hipError_t launch_few_ck(const FewParams& fp, const FewOperands& fo, hipStream_t st) {
    const int slots = (fp.N + CPW - 1) / CPW;  // groups of CPW columns
    const dim3 grid((unsigned)((slots + 4 / KS - 1) / (4 / KS))), block(256);
    if ((int64_t)grid.x * 256 < (int64_t)fo.copy_n * fo.copy_chunks) return hipErrorInvalidValue;
    if (fp.rows <= 1) hipLaunchKernelGGL((k_linear_few<MODE, 1, CPW, KS>), grid, block, 0, st, fp, fo);
    else if (fp.rows <= 2) hipLaunchKernelGGL((k_linear_few<MODE, 2, CPW, KS>), grid, block, 0, st, fp, fo);
    else if (fp.rows <= 4) hipLaunchKernelGGL((k_linear_few<MODE, 4, CPW, KS>), grid, block, 0, st, fp, fo);
    else if (fp.rows <= 8) hipLaunchKernelGGL((k_linear_few<MODE, 8, CPW, KS>), grid, block, 0, st, fp, fo);
    else hipLaunchKernelGGL((k_linear_few<MODE, 16, CPW, KS>), grid, block, 0, st, fp, fo);
    return hipGetLastError();
}

// Long rows (the block's two products): four columns per wave share the fetched (and transformed) input rows --
// with one column per wave the input rows, re-read by every wave, are more cache traffic than the weights --
// and k is split over the four waves of the workgroup, which keeps as many waves as there are columns.  Short
// rows: no split.
template <int MODE>
hipError_t launch_few(const FewParams& fp, const FewOperands& fo, hipStream_t st) {
    if (fp.N >= 8192) return fp.K >= 2048 ? launch_few_ck<MODE, 4, 4>(fp, fo, st) : launch_few_ck<MODE, 2, 1>(fp, fo, st);
    if (fp.N >= 4096) return fp.K >= 2048 ? launch_few_ck<MODE, 1, 2>(fp, fo, st) : launch_few_ck<MODE, 1, 1>(fp, fo, st);
    return fp.K >= 2048 ? launch_few_ck<MODE, 4, 4>(fp, fo, st) : launch_few_ck<MODE, 1, 1>(fp, fo, st);
}

// More than a few rows (several sequences generated together): the same product on the matrix cores.  A
// workgroup owns 16 columns of w; its KS waves split k among themselves and each runs 16 x 16 x 32 MFMAs with the
// (at most 16) input rows as the other operand, so the arithmetic is out of the way and the kernel again only
// streams w; the partial tiles meet in LDS.  No input transform here (a normalisation in front runs as its own
// small kernel: redoing it in every wave is what would bound the kernel).
typedef float f32x4v __attribute__((ext_vector_type(4)));

template <int KS, int CG>
__global__ __launch_bounds__(KS * 64) void k_linear_few_mfma(FewParams fp, FewOperands fo) {
    __shared__ float part[KS][CG * 256];
    if (fo.copy_n) {
        const int i = blockIdx.x * (KS * 64) + threadIdx.x;
        if (i < fo.copy_n * fo.copy_chunks) {
            const int c = i / fo.copy_n, v = i - c * fo.copy_n;
            ((f32x4*)fo.copy_dst)[c * fo.copy_dst_stride + v] = ((const f32x4*)fo.copy_src)[c * fo.copy_src_stride + v];
        }
    }
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int n0 = blockIdx.x * (16 * CG);
    const int col = lane & 15, kq = lane >> 4;  // the lane's row of x and column of w; its quarter of a 32-wide k step
    const bool has_x = col < fp.rows;
    const __bf16* xr = fp.x + (int64_t)col * fp.ldx;
    const __bf16* wr = fp.w + (int64_t)(n0 + col) * fp.K;
    const int nsteps = (fp.K + 31) / 32, per = (nsteps + KS - 1) / KS;
    const int s0 = wv * per, s1 = s0 + per < nsteps ? s0 + per : nsteps;
    f32x4v acc[CG];
#pragma unroll
    for (int c = 0; c < CG; ++c) acc[c] = f32x4v{0.f, 0.f, 0.f, 0.f};
    constexpr int UN = CG > 1 ? 2 : 4;  // k steps whose operands are requested together
    for (int sb = s0; sb < s1; sb += UN) {
        bf16x8 a[UN], b[UN][CG];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = (sb + u) * 32 + 8 * kq;  // K is a multiple of 8: a lane's eight values are inside or outside as a whole
            const bool in = sb + u < s1 && k < fp.K;
#pragma unroll
            for (int e = 0; e < 8; ++e) a[u][e] = (__bf16)0.f;
            if (has_x && in) a[u] = *(const bf16x8*)(xr + k);
#pragma unroll
            for (int c = 0; c < CG; ++c) {
#pragma unroll
                for (int e = 0; e < 8; ++e) b[u][c][e] = (__bf16)0.f;
                if (in && n0 + 16 * c + col < fp.N) b[u][c] = *(const bf16x8*)(wr + (int64_t)(16 * c) * fp.K + k);
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u)
#pragma unroll
            for (int c = 0; c < CG; ++c)  // acc[c][i] = out[row 4 kq + i][column n0 + 16 c + col]
                acc[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[u], b[u][c], acc[c], 0, 0, 0);
    }
#pragma unroll
    for (int c = 0; c < CG; ++c)
#pragma unroll
        for (int i = 0; i < 4; ++i) part[wv][c * 256 + lane * 4 + i] = acc[c][i];
    __syncthreads();
    for (int t = threadIdx.x; t < CG * 256; t += KS * 64) {
        float v = 0.f;
#pragma unroll
        for (int q = 0; q < KS; ++q) v += part[q][t];
        const int c = t >> 8, l = (t & 255) >> 2, i = t & 3;
        const int r = 4 * (l >> 4) + i, n = n0 + 16 * c + (l & 15);
        if (r < fp.rows && n < fp.N) {
            if (fp.res) v += (float)fp.res[r * fp.ldres + n];
            fp.out[r * fp.ldo + n] = (__bf16)v;
        }
    }
}

hipError_t launch_few_mfma(const FewParams& fp, const FewOperands& fo, hipStream_t st) {
    // wide products: 64 columns per workgroup (the input rows are fetched once for four column groups), k split 16
    // ways; narrow ones: 16 columns, and the narrower the product, the more ways k is split -- enough waves either
    // way to keep the memory system busy
    const bool wide = fp.N >= 4096;
    const int wgs = wide ? (fp.N + 63) / 64 : (fp.N + 15) / 16;
    const int ks = wide ? 16 : wgs >= 1024 ? 4 : wgs >= 512 ? 8 : 16;
    if ((int64_t)wgs * ks * 64 < (int64_t)fo.copy_n * fo.copy_chunks) return hipErrorInvalidValue;
    if (wide) hipLaunchKernelGGL((k_linear_few_mfma<16, 4>), dim3(wgs), dim3(1024), 0, st, fp, fo);
    else if (ks == 4) hipLaunchKernelGGL((k_linear_few_mfma<4, 1>), dim3(wgs), dim3(256), 0, st, fp, fo);
    else if (ks == 8) hipLaunchKernelGGL((k_linear_few_mfma<8, 1>), dim3(wgs), dim3(512), 0, st, fp, fo);
    else hipLaunchKernelGGL((k_linear_few_mfma<16, 1>), dim3(wgs), dim3(1024), 0, st, fp, fo);
    return hipGetLastError();
}

struct MidParams {
    const __bf16* zx;   // [T, ld]: (z | xBC | dt_raw) of the tokens
    int64_t ld;
    const float *conv_w, *conv_b, *dt_bias, *A, *D;
    const __bf16* cs_in;  // [3, conv_dim] or null: the convolution's inputs of the three tokens before
    __bf16* cs_out;       // [3, conv_dim] or null; never the same buffer as cs_in
    float* state;         // [H, P, N], updated in place
    __bf16* y;            // [T, d_inner]
    int T, H, P, G, N, hpg, d_inner, conv_dim, off_xbc, off_dt;
    // several independent sequences in one launch (blockIdx.y): sequence b owns rows b T .. b T + T - 1 of zx and y
    // and the states `b` strides (elements) further on
    int64_t state_bs, cs_in_bs, cs_out_bs;
};

// input of the convolution, channel c, token `pos` of this call (negative: from the entering state)
__device__ __forceinline__ float conv_input(const MidParams& mp, int pos, int c) {
    if (pos >= 0) return (float)mp.zx[pos * mp.ld + mp.off_xbc + c];
    return mp.cs_in ? (float)mp.cs_in[(3 + pos) * mp.conv_dim + c] : 0.f;
}

// silu(bias + four taps), rounded as the block stores it between its steps
__device__ __forceinline__ float conv_output(const MidParams& mp, int t, int c) {
    const float* w = mp.conv_w + (int64_t)c * 4;
    const float pre = mp.conv_b[c] + w[0] * conv_input(mp, t - 3, c) + w[1] * conv_input(mp, t - 2, c) + w[2] * conv_input(mp, t - 1, c) +
                      w[3] * conv_input(mp, t, c);
    return through_bf16(pre * sigmoid_fast(pre));
}

// Workgroup (head h, sequence b, z): wave w owns the RPW state rows p = (4 z + w) RPW + rr, lane l their columns
// n = l, l + 64, ..., which stay in registers over the tokens of the call (requested first: nothing below waits
// for them until the first update).  Per token the workgroup convolves the B and C channels of its group into
// LDS (every workgroup of the group does: a few hundred channels against the P N elements of a head's state --
// which is why several sequences at once take more rows per wave and fewer workgroups), each wave the x channels
// of its rows.
constexpr int MID_NPL = 8;  // state columns per lane at most (N <= 512)

template <int RPW>
__global__ __launch_bounds__(256) void k_decode_mid(MidParams mp) {
    extern __shared__ float bc[];  // B[0..N), C[0..N) of the group, this token
    {  // this workgroup's sequence
        const int64_t b = blockIdx.y;
        mp.zx += b * mp.T * mp.ld;
        mp.y += b * mp.T * mp.d_inner;
        mp.state += b * mp.state_bs;
        if (mp.cs_in) mp.cs_in += b * mp.cs_in_bs;
        if (mp.cs_out) mp.cs_out += b * mp.cs_out_bs;
    }
    const int h = blockIdx.x, g = h / mp.hpg;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int p0 = (4 * blockIdx.z + w) * RPW;
    float* S = mp.state + (int64_t)h * mp.P * mp.N;
    float s[RPW][MID_NPL];
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
        for (int i = 0; i < MID_NPL; ++i) {
            const int n = lane + 64 * i;
            s[rr][i] = p0 + rr < mp.P && n < mp.N ? S[(int64_t)(p0 + rr) * mp.N + n] : 0.f;
        }
    const float Ah = mp.A[h], Dh = mp.D[h], bias_h = mp.dt_bias[h];
    const int cB = mp.d_inner + g * mp.N, cC = mp.d_inner + (mp.G + g) * mp.N;
    for (int t = 0; t < mp.T; ++t) {
        for (int i = threadIdx.x; i < 2 * mp.N; i += 256) bc[i] = conv_output(mp, t, i < mp.N ? cB + i : cC + (i - mp.N));
        const float v = (float)mp.zx[t * mp.ld + mp.off_dt + h] + bias_h;
        const float dtv = through_bf16(fmaxf(v, 0.f) + log1pf(__expf(-fabsf(v))));  // softplus
        const float a = __expf(dtv * Ah);
        float xv[RPW];
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr) xv[rr] = p0 + rr < mp.P ? conv_output(mp, t, h * mp.P + p0 + rr) : 0.f;
        __syncthreads();
#pragma unroll
        for (int rr = 0; rr < RPW; ++rr) {
            if (p0 + rr < mp.P) {
                const float dx = dtv * xv[rr];
                float acc = 0.f;
#pragma unroll
                for (int i = 0; i < MID_NPL; ++i) {
                    const int n = lane + 64 * i;
                    if (n < mp.N) {
                        s[rr][i] = a * s[rr][i] + dx * bc[n];
                        acc += bc[mp.N + n] * s[rr][i];
                    }
                }
                acc = wave_sum(acc);
                if (lane == 0) mp.y[(int64_t)t * mp.d_inner + h * mp.P + p0 + rr] = (__bf16)(acc + Dh * xv[rr]);
            }
        }
        __syncthreads();  // the next token's B and C replace these
    }
#pragma unroll
    for (int rr = 0; rr < RPW; ++rr)
#pragma unroll
        for (int i = 0; i < MID_NPL; ++i) {
            const int n = lane + 64 * i;
            if (p0 + rr < mp.P && n < mp.N) S[(int64_t)(p0 + rr) * mp.N + n] = s[rr][i];
        }
    if (mp.cs_out) {  // the last three inputs of [entering state ; this call's tokens]
        for (int i = lane; i < 3 * RPW; i += 64) {
            const int rr = i / 3, j = i - 3 * rr;
            if (p0 + rr < mp.P) mp.cs_out[j * mp.conv_dim + h * mp.P + p0 + rr] = (__bf16)conv_input(mp, mp.T - 3 + j, h * mp.P + p0 + rr);
        }
        if (h % mp.hpg == 0 && blockIdx.z == 0)  // the group's B and C channels: once
            for (int i = threadIdx.x; i < 6 * mp.N; i += 256) {
                const int j = i / (2 * mp.N), ii = i % (2 * mp.N);
                const int c = ii < mp.N ? cB + ii : cC + (ii - mp.N);
                mp.cs_out[j * mp.conv_dim + c] = (__bf16)conv_input(mp, mp.T - 3 + j, c);
            }
    }
}

// One token for each of several sequences: the convolution step by itself.  A thread owns one channel of one
// sequence -- its window of the convolution state, which it replaces in place -- and writes the activated value
// into the dense x, B or C row of its sequence; the threads behind the channels take softplus(dt) of the heads.
struct ConvStepParams {
    const __bf16* zx;  // [nb, ld]
    int64_t ld;
    const float *conv_w, *conv_b, *dt_bias;
    __bf16* cs;        // sequence b: [3, conv_dim] at cs + b cs_bs, replaced in place
    int64_t cs_bs;
    __bf16 *x, *B, *C, *dt;  // [nb, d_inner], [nb, G N], [nb, G N], [nb, H]
    int H, d_inner, gn, conv_dim, off_xbc, off_dt;
};

__global__ __launch_bounds__(256) void k_conv_step(ConvStepParams cp) {
    const int c = blockIdx.x * 256 + threadIdx.x, b = blockIdx.y;
    const __bf16* zx = cp.zx + (int64_t)b * cp.ld;
    if (c < cp.conv_dim) {
        __bf16* cs = cp.cs + (int64_t)b * cp.cs_bs;
        const float s0 = (float)cs[c], s1 = (float)cs[cp.conv_dim + c], s2 = (float)cs[2 * cp.conv_dim + c];
        const __bf16 ub = zx[cp.off_xbc + c];
        const float u = (float)ub;
        const float* w = cp.conv_w + (int64_t)c * 4;
        const float pre = cp.conv_b[c] + w[0] * s0 + w[1] * s1 + w[2] * s2 + w[3] * u;
        const __bf16 o = (__bf16)(pre * sigmoid_fast(pre));
        if (c < cp.d_inner) cp.x[(int64_t)b * cp.d_inner + c] = o;
        else if (c < cp.d_inner + cp.gn) cp.B[(int64_t)b * cp.gn + (c - cp.d_inner)] = o;
        else cp.C[(int64_t)b * cp.gn + (c - cp.d_inner - cp.gn)] = o;
        cs[c] = (__bf16)s1;
        cs[cp.conv_dim + c] = (__bf16)s2;
        cs[2 * cp.conv_dim + c] = ub;
    } else if (c < cp.conv_dim + cp.H) {
        const int h = c - cp.conv_dim;
        const float v = (float)zx[cp.off_dt + h] + cp.dt_bias[h];
        cp.dt[(int64_t)b * cp.H + h] = (__bf16)(fmaxf(v, 0.f) + log1pf(__expf(-fabsf(v))));  // softplus
    }
}

bool al16(const void* p) { return ((uintptr_t)p & 15) == 0; }

}  // namespace

bool few_rows_supported(const FewRowsJob& j) {
    if (j.rows < 1 || j.rows > FEW_ROWS || j.K <= 0 || j.N <= 0 || ((j.K | j.N) & 7)) return false;
    if (!j.x || !j.w || !j.out || !al16(j.x) || !al16(j.w) || (j.ldx & 7) || j.ldx < j.K || j.ldo < j.N) return false;
    if (j.mode < 0 || j.mode > 2) return false;
    if (j.mode && (!j.in_w || !al16(j.in_w))) return false;
    if (j.mode == 2 && (!j.z || !al16(j.z) || (j.ldz & 7) || j.ldz < j.K)) return false;
    if (j.res && j.ldres < j.N) return false;
    if (j.copy_bytes) {
        const size_t chunks = j.copy_chunks > 0 ? j.copy_chunks : 1;
        if (!j.copy_src || !j.copy_dst || !al16(j.copy_src) || !al16(j.copy_dst) || (j.copy_bytes & 15) || j.copy_chunks < 0 ||
            ((j.copy_src_stride | j.copy_dst_stride) & 15) || j.copy_bytes / 16 * chunks > (size_t)j.N * 16)  // one vector per thread of the smallest launch these products use
            return false;
    }
    return true;
}

hipError_t launch_linear_few_rows(const FewRowsJob& j, hipStream_t st) {
    if (!few_rows_supported(j)) return hipErrorInvalidValue;
    FewParams fp;
    fp.x = (const __bf16*)j.x;
    fp.w = (const __bf16*)j.w;
    fp.z = (const __bf16*)j.z;
    fp.res = (const __bf16*)j.res;
    fp.out = (__bf16*)j.out;
    fp.in_w = j.in_w;
    fp.ldx = j.ldx;
    fp.ldz = j.ldz;
    fp.ldo = j.ldo;
    fp.ldres = j.ldres;
    fp.rows = j.rows;
    fp.K = j.K;
    fp.N = j.N;
    fp.eps = j.eps;
    FewOperands fo;
    fo.copy_src = j.copy_src;
    fo.copy_dst = j.copy_dst;
    fo.copy_n = (int)(j.copy_bytes / 16);
    fo.copy_chunks = j.copy_bytes ? (j.copy_chunks > 0 ? j.copy_chunks : 1) : 0;
    fo.copy_src_stride = (int64_t)(j.copy_src_stride / 16);
    fo.copy_dst_stride = (int64_t)(j.copy_dst_stride / 16);
    if (j.mode == 0 && j.rows > FEW_ROWS_VALU) return launch_few_mfma(fp, fo, st);
    return j.mode == 0 ? launch_few<0>(fp, fo, st) : j.mode == 1 ? launch_few<1>(fp, fo, st) : launch_few<2>(fp, fo, st);
}

hipError_t launch_decode_mid(const DecodeMidJob& j, hipStream_t st) {
    const int nb = j.nb > 0 ? j.nb : 1;
    if (nb > 65535 || (int64_t)nb * j.T > FEW_ROWS) return hipErrorInvalidValue;
    if (j.T < 1 || j.T > FEW_ROWS || j.H <= 0 || j.H > 65535 || j.P <= 0 || j.G <= 0 || j.N <= 0 || j.H % j.G) return hipErrorInvalidValue;
    if (!j.zx || !j.conv_w || !j.conv_b || !j.dt_bias || !j.A || !j.D || !j.state || !j.y || (j.cs_out && j.cs_out == j.cs_in))
        return hipErrorInvalidValue;
    if (j.N > 64 * MID_NPL || j.P > 256) return hipErrorInvalidValue;  // a state row in a wave's registers, a row per wave
    MidParams mp;
    mp.zx = (const __bf16*)j.zx;
    mp.ld = j.ld;
    mp.conv_w = j.conv_w;
    mp.conv_b = j.conv_b;
    mp.dt_bias = j.dt_bias;
    mp.A = j.A;
    mp.D = j.D;
    mp.cs_in = (const __bf16*)j.cs_in;
    mp.cs_out = (__bf16*)j.cs_out;
    mp.state = j.state;
    mp.y = (__bf16*)j.y;
    mp.T = j.T;
    mp.H = j.H;
    mp.P = j.P;
    mp.G = j.G;
    mp.N = j.N;
    mp.hpg = j.H / j.G;
    mp.d_inner = j.H * j.P;
    mp.conv_dim = mp.d_inner + 2 * j.G * j.N;
    mp.off_xbc = mp.d_inner;
    mp.off_dt = mp.d_inner + mp.conv_dim;
    mp.state_bs = j.state_bs;
    mp.cs_in_bs = j.cs_in_bs;
    mp.cs_out_bs = j.cs_out_bs;
    // rows per wave: one where that gives few enough workgroups (every one of them convolves its group's B and C
    // channels), else 4 or 16
    const size_t lds = (size_t)2 * j.N * sizeof(float);
    auto wgs = [&](int rpw) { return (int64_t)j.H * nb * ((j.P + 4 * rpw - 1) / (4 * rpw)); };
    if (wgs(1) <= 8192)
        hipLaunchKernelGGL(k_decode_mid<1>, dim3(j.H, nb, (j.P + 3) / 4), dim3(256), lds, st, mp);
    else if (wgs(4) <= 2048)
        hipLaunchKernelGGL(k_decode_mid<4>, dim3(j.H, nb, (j.P + 15) / 16), dim3(256), lds, st, mp);
    else
        hipLaunchKernelGGL(k_decode_mid<16>, dim3(j.H, nb, (j.P + 63) / 64), dim3(256), lds, st, mp);
    return hipGetLastError();
}

hipError_t launch_conv_step(const ConvStepJob& j, hipStream_t st) {
    if (j.nb < 1 || j.nb > 65535 || j.H <= 0 || j.P <= 0 || j.G <= 0 || j.N <= 0) return hipErrorInvalidValue;
    if (!j.zx || !j.conv_w || !j.conv_b || !j.dt_bias || !j.cs || !j.x || !j.B || !j.C || !j.dt) return hipErrorInvalidValue;
    ConvStepParams cp;
    cp.zx = (const __bf16*)j.zx;
    cp.ld = j.ld;
    cp.conv_w = j.conv_w;
    cp.conv_b = j.conv_b;
    cp.dt_bias = j.dt_bias;
    cp.cs = (__bf16*)j.cs;
    cp.cs_bs = j.cs_bs;
    cp.x = (__bf16*)j.x;
    cp.B = (__bf16*)j.B;
    cp.C = (__bf16*)j.C;
    cp.dt = (__bf16*)j.dt;
    cp.H = j.H;
    cp.d_inner = j.H * j.P;
    cp.gn = j.G * j.N;
    cp.conv_dim = cp.d_inner + 2 * cp.gn;
    cp.off_xbc = cp.d_inner;
    cp.off_dt = cp.d_inner + cp.conv_dim;
    hipLaunchKernelGGL(k_conv_step, dim3((cp.conv_dim + cp.H + 255) / 256, j.nb), dim3(256), 0, st, cp);
    return hipGetLastError();
}

}  // namespace ssdk
