// Causal depthwise convolution (kernel 4) + bias + SiLU of the Mamba-2 block, forward and backward,
// with the three-token convolution state that MA-GC keeps next to the SSM state in every sequence
// checkpoint (App. C, Tab. 7: the per-checkpoint constant counts the SSM state plus three tokens of the
// convolution's channels).  A segment is processed from its stored state exactly as the SSD segment is:
//     pre[t,c] = bias[c] + sum_{k=0..3} w[c,k] u[t-3+k, c]      (u[-3..-1] = state_in, zeros if absent)
//     out[t,c] = pre / (1 + exp(-pre))
// HBM-bound: every thread owns V consecutive channels (16 bytes) and walks TT consecutive tokens with
// the window in registers, so every input row is read once (plus a three-row halo per TT tokens).
#include <string.h>

#include "ssd_internal.h"

namespace ssdk {
namespace {

constexpr int CONV_K = 4;
constexpr int FWD_TT = 64;    // most tokens per thread, forward
constexpr int BWD_TT = 256;   // most tokens per thread, backward (also the granularity of the dw / dbias partial sums)
constexpr int MIN_TT = 16;    // shorter runs re-read too much of the three-token halo

struct ConvParams {
    const void* u;
    const void* dout;
    const void* state_in;   // [Bt][3][C] storage dtype or null
    const float* dstate_out;  // [Bt][3][C] fp32 or null: gradient reaching the last three rows of u from the right
    void* out;
    void* du;
    void* state_out;    // [Bt][3][C] storage dtype or null
    float* dstate_in;   // [Bt][3][C] fp32 or null
    const float* w;     // [C][4]
    const float* bias;  // [C] or null
    float* part;        // [Bt][ntiles][5][C] partial sums of dw (k = 0..3) and dbias
    int64_t L, u_bs, o_bs;  // tokens; batch stride of u / du and of out / dout in elements
    int64_t u_rs;           // elements between consecutive tokens of u / du (out / dout: C)
    int C, ntiles;
    int tt;             // tokens per thread of this launch
    // out / dout as three dense tensors side by side instead of one: channels [cb[k], cb[k+1]) live in
    // part[k] with rows cb[k+1] - cb[k] apart (the block's x | B | C, each the shape the scan wants)
    int split;
    int cb[4];
    void* out3[3];
    const void* dout3[3];
};

// Where this thread's channels c0.. of out / dout live: base pointer, batch and row stride, first column.
struct OutSlot {
    void* out;
    const void* dout;
    int64_t bs, rs;
    int c;
};
__device__ __forceinline__ OutSlot out_slot(const ConvParams& cp, int c0) {
    OutSlot o;
    if (!cp.split) {
        o.out = cp.out;
        o.dout = cp.dout;
        o.bs = cp.o_bs;
        o.rs = cp.C;
        o.c = c0;
    } else {
        const int k = c0 >= cp.cb[2] ? 2 : c0 >= cp.cb[1] ? 1 : 0;
        o.out = cp.out3[k];
        o.dout = cp.dout3[k];
        o.rs = cp.cb[k + 1] - cp.cb[k];
        o.bs = cp.L * o.rs;
        o.c = c0 - cp.cb[k];
    }
    return o;
}

template <typename T, int V>
struct Vec;
template <>
struct Vec<float, 1> {
    static __device__ __forceinline__ void ld(const void* p, int64_t i, float (&v)[1]) { v[0] = ((const float*)p)[i]; }
    static __device__ __forceinline__ void st(void* p, int64_t i, const float (&v)[1]) { ((float*)p)[i] = v[0]; }
};
template <>
struct Vec<float, 4> {
    static __device__ __forceinline__ void ld(const void* p, int64_t i, float (&v)[4]) {
        const float4 t = *(const float4*)((const float*)p + i);
        v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
    }
    static __device__ __forceinline__ void st(void* p, int64_t i, const float (&v)[4]) {
        *(float4*)((float*)p + i) = make_float4(v[0], v[1], v[2], v[3]);
    }
};
template <>
struct Vec<bf16_t, 1> {
    static __device__ __forceinline__ void ld(const void* p, int64_t i, float (&v)[1]) { v[0] = bf16_to_float(((const bf16_t*)p)[i]); }
    static __device__ __forceinline__ void st(void* p, int64_t i, const float (&v)[1]) { ((bf16_t*)p)[i] = float_to_bf16(v[0]); }
};
template <>
struct Vec<bf16_t, 8> {
    typedef __bf16 b8 __attribute__((ext_vector_type(8)));
    static __device__ __forceinline__ void ld(const void* p, int64_t i, float (&v)[8]) {
        const b8 t = *(const b8*)((const __bf16*)p + i);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (float)t[e];
    }
    static __device__ __forceinline__ void st(void* p, int64_t i, const float (&v)[8]) {
        b8 t;
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = (__bf16)v[e];
        *(b8*)((__bf16*)p + i) = t;
    }
};

// sigmoid through the hardware reciprocal (1 ulp) instead of an IEEE division: the kernels here are close
// enough to the VALU limit for the ten extra instructions per element to show
__device__ __forceinline__ float sigmoid_fast(float z) { return __builtin_amdgcn_rcpf(1.f + __expf(-z)); }
__device__ __forceinline__ float silu(float z) { return z * sigmoid_fast(z); }
// d silu / dz = s (1 + z (1 - s)), s = sigmoid(z)
__device__ __forceinline__ float dsilu(float z) {
    const float s = sigmoid_fast(z);
    return s * (1.f + z * (1.f - s));
}

// Row t of u for this thread's channels: from the tensor (t >= 0), the entering state (t >= -3) or zeros.
template <typename T, int V>
__device__ __forceinline__ void load_row(const ConvParams& cp, int64_t b, int64_t t, int c0, float (&v)[V]) {
    if (t >= 0 && t < cp.L) {
        Vec<T, V>::ld(cp.u, b * cp.u_bs + t * cp.u_rs + c0, v);
    } else if (t < 0 && t >= -3 && cp.state_in) {
        Vec<T, V>::ld(cp.state_in, (b * 3 + (t + 3)) * cp.C + c0, v);
    } else {
#pragma unroll
        for (int e = 0; e < V; ++e) v[e] = 0.f;
    }
}

template <typename T, int V>
__global__ __launch_bounds__(64) void k_conv_fwd(ConvParams cp) {
    const int c0 = (blockIdx.x * 64 + threadIdx.x) * V;
    if (c0 >= cp.C) return;
    const int64_t b = blockIdx.z, t0 = (int64_t)blockIdx.y * cp.tt;
    const OutSlot os = out_slot(cp, c0);
    float w[V][CONV_K], bias[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
#pragma unroll
        for (int k = 0; k < CONV_K; ++k) w[e][k] = cp.w[(c0 + e) * CONV_K + k];
        bias[e] = cp.bias ? cp.bias[c0 + e] : 0.f;
    }
    float win[3][V];  // u[t-3], u[t-2], u[t-1]
#pragma unroll
    for (int j = 0; j < 3; ++j) load_row<T, V>(cp, b, t0 - 3 + j, c0, win[j]);
    const int64_t t1 = t0 + cp.tt < cp.L ? t0 + cp.tt : cp.L;
    constexpr int U = 4;  // four rows requested together, then consumed in order
    for (int64_t t = t0; t < t1; t += U) {
        float cur[U][V];
#pragma unroll
        for (int j = 0; j < U; ++j)
            if (t + j < t1) Vec<T, V>::ld(cp.u, b * cp.u_bs + (t + j) * cp.u_rs + c0, cur[j]);
#pragma unroll
        for (int j = 0; j < U; ++j) {
            if (t + j >= t1) break;
            float o[V];
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float pre = bias[e] + w[e][0] * win[0][e] + w[e][1] * win[1][e] + w[e][2] * win[2][e] + w[e][3] * cur[j][e];
                o[e] = silu(pre);
                win[0][e] = win[1][e];
                win[1][e] = win[2][e];
                win[2][e] = cur[j][e];
            }
            Vec<T, V>::st(os.out, b * os.bs + (t + j) * os.rs + os.c, o);
        }
    }
    // the state leaving the segment: the last three rows of [state_in ; u]
    if (cp.state_out && t1 == cp.L) {
#pragma unroll
        for (int j = 0; j < 3; ++j) Vec<T, V>::st(cp.state_out, (b * 3 + j) * cp.C + c0, win[j]);
    }
}

// Backward.  g[t] = dout[t] silu'(pre[t]);  du[t] = sum_k w[k] g[t+3-k]  (g beyond the segment is 0; what
// the segment on the right contributes to the last three rows arrives as dstate_out);
// dw[k] = sum_t g[t] u[t-3+k];  dbias = sum_t g[t];  dstate_in[j] = du[-3+j].
template <typename T, int V>
__global__ __launch_bounds__(64) void k_conv_bwd(ConvParams cp) {
    const int c0 = (blockIdx.x * 64 + threadIdx.x) * V;
    if (c0 >= cp.C) return;
    const int64_t b = blockIdx.z, t0 = (int64_t)blockIdx.y * cp.tt;
    const OutSlot os = out_slot(cp, c0);
    float w[V][CONV_K], bias[V];
#pragma unroll
    for (int e = 0; e < V; ++e) {
#pragma unroll
        for (int k = 0; k < CONV_K; ++k) w[e][k] = cp.w[(c0 + e) * CONV_K + k];
        bias[e] = cp.bias ? cp.bias[c0 + e] : 0.f;
    }
    float acc[5][V];
#pragma unroll
    for (int k = 0; k < 5; ++k)
#pragma unroll
        for (int e = 0; e < V; ++e) acc[k][e] = 0.f;
    float win[3][V];  // u[t-3], u[t-2], u[t-1]
#pragma unroll
    for (int j = 0; j < 3; ++j) load_row<T, V>(cp, b, t0 - 3 + j, c0, win[j]);
    float gw[3][V];   // g[t-3], g[t-2], g[t-1]; before the tile (or the sequence) they are not needed: zeros
#pragma unroll
    for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int e = 0; e < V; ++e) gw[j][e] = 0.f;
    const int64_t t1 = t0 + cp.tt < cp.L ? t0 + cp.tt : cp.L;  // own tokens: [t0, t1)
    // the first tile also produces the gradient of the entering state, du[-3..-1]; its g window starts at 0 anyway
    const int64_t first_out = (t0 == 0 && cp.dstate_in) ? -3 : t0;
    // one token: g[t] from its rows of u and dout (zeros beyond the sequence), then du[t-3]
    auto token = [&](int64_t t, const float (&cur)[V], const float (&dv)[V]) {
        float g[V];
        if (t < cp.L) {
#pragma unroll
            for (int e = 0; e < V; ++e) {
                const float pre = bias[e] + w[e][0] * win[0][e] + w[e][1] * win[1][e] + w[e][2] * win[2][e] + w[e][3] * cur[e];
                g[e] = dv[e] * dsilu(pre);
            }
            if (t < t1) {  // own token: its share of dw and dbias
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    acc[0][e] += g[e] * win[0][e];
                    acc[1][e] += g[e] * win[1][e];
                    acc[2][e] += g[e] * win[2][e];
                    acc[3][e] += g[e] * cur[e];
                    acc[4][e] += g[e];
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e) g[e] = 0.f;
        }
        // du[t-3] = w3 g[t-3] + w2 g[t-2] + w1 g[t-1] + w0 g[t]
        const int64_t to = t - 3;
        if (to >= first_out && to < t1) {
            float o[V];
#pragma unroll
            for (int e = 0; e < V; ++e) o[e] = w[e][3] * gw[0][e] + w[e][2] * gw[1][e] + w[e][1] * gw[2][e] + w[e][0] * g[e];
            if (to >= 0) {
                if (cp.dstate_out && to >= cp.L - 3) {  // one of the last three rows: add what arrives from the right
                    const int64_t j = to - (cp.L - 3);
#pragma unroll
                    for (int e = 0; e < V; ++e) o[e] += cp.dstate_out[(b * 3 + j) * cp.C + c0 + e];
                }
                Vec<T, V>::st(cp.du, b * cp.u_bs + to * cp.u_rs + c0, o);
            } else {
                // a row of the entering state; when the sequence is shorter than three tokens, part of the
                // state passes straight through to state_out and takes dstate_out's gradient with it
                const int64_t jr = to + 3;  // 0..2
                if (cp.dstate_out && cp.L < 3 && jr >= cp.L) {
                    const int64_t j = jr - cp.L;
#pragma unroll
                    for (int e = 0; e < V; ++e) o[e] += cp.dstate_out[(b * 3 + j) * cp.C + c0 + e];
                }
#pragma unroll
                for (int e = 0; e < V; ++e) cp.dstate_in[(b * 3 + jr) * cp.C + c0 + e] = o[e];
            }
        }
#pragma unroll
        for (int e = 0; e < V; ++e) {
            gw[0][e] = gw[1][e];
            gw[1][e] = gw[2][e];
            gw[2][e] = g[e];
            win[0][e] = win[1][e];
            win[1][e] = win[2][e];
            win[2][e] = t < cp.L ? cur[e] : 0.f;
        }
    };
    for (int64_t t = t0; t < t1 + 3; ++t) {
        float cur[V], dv[V];
        if (t < cp.L) {
            Vec<T, V>::ld(cp.u, b * cp.u_bs + t * cp.u_rs + c0, cur);
            Vec<T, V>::ld(os.dout, b * os.bs + t * os.rs + os.c, dv);
        } else {
#pragma unroll
            for (int e = 0; e < V; ++e) cur[e] = dv[e] = 0.f;
        }
        token(t, cur, dv);
    }
    float* part = cp.part + ((b * cp.ntiles + blockIdx.y) * 5) * (int64_t)cp.C;
#pragma unroll
    for (int k = 0; k < 5; ++k)
#pragma unroll
        for (int e = 0; e < V; ++e) part[(int64_t)k * cp.C + c0 + e] = acc[k][e];
}

// dw[c][k] (k < 4) and dbias[c]: sum of the partial sums of all (batch, tile) pairs, in a fixed order.
// A workgroup owns 64 consecutive entries of the [5][C] rows; its four waves sum every fourth part each
// (four loads in flight per lane), wave 0 adds the four results.
__global__ __launch_bounds__(256) void k_conv_reduce(const float* part, int64_t nparts, int C, float* dw, float* dbias, int accumulate) {
    __shared__ float red[4][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int i = blockIdx.x * 64 + lane;  // over 5 * C
    const bool live = i < 5 * C;
    float s = 0.f;
    if (live) {
        const float* src = part + i;
        const int64_t stride = 5 * (int64_t)C;
        int64_t p = wv;
        for (; p + 12 < nparts; p += 16) {
            const float a0 = src[p * stride], a1 = src[(p + 4) * stride], a2 = src[(p + 8) * stride], a3 = src[(p + 12) * stride];
            s += a0;
            s += a1;
            s += a2;
            s += a3;
        }
        for (; p < nparts; p += 4) s += src[p * stride];
    }
    red[wv][lane] = s;
    __syncthreads();
    if (wv == 0 && live) {
        s = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
        const int k = i / C, c = i - k * C;
        if (k < 4) {
            float* o = dw + (int64_t)c * 4 + k;
            *o = accumulate ? *o + s : s;
        } else if (dbias) {
            dbias[c] = accumulate ? dbias[c] + s : s;
        }
    }
}

int check(const ssd_conv_shape_t* sh) {
    if (!sh) return SSD_ERR_NULL;
    if (sh->dtype != SSD_F32 && sh->dtype != SSD_BF16) return SSD_ERR_DTYPE;
    if (sh->batch <= 0 || sh->batch > 65535 || sh->seqlen < 0 || sh->channels <= 0) return SSD_ERR_SHAPE;
    if ((sh->seqlen + FWD_TT - 1) / FWD_TT > 65535) return SSD_ERR_SHAPE;  // grid.y (long sequences run FWD_TT tokens per thread)
    if (sh->u_row_stride && sh->u_row_stride < sh->channels) return SSD_ERR_SHAPE;
    if (sh->batch_stride && sh->batch_stride < sh->seqlen * (sh->u_row_stride ? sh->u_row_stride : sh->channels)) return SSD_ERR_SHAPE;
    return SSD_OK;
}

// Tokens per thread: the most (fewest halo re-reads, fewest partial sums) that still gives the launch about
// 2048 waves -- a segment-sized call would otherwise leave most of the machine idle.
int pick_tt(const ssd_conv_shape_t* sh, int most) {
    const int64_t col_waves = ((int64_t)sh->channels / 8 + 63) / 64 * sh->batch;  // waves per token tile
    int tt = most;
    while (tt > MIN_TT && (sh->seqlen + tt - 1) / tt * col_waves < 2048) tt >>= 1;
    return tt;
}
int ntiles_bwd(const ssd_conv_shape_t* sh) {
    const int tt = pick_tt(sh, BWD_TT);
    return (int)((sh->seqlen + tt - 1) / tt);
}

}  // namespace
}  // namespace ssdk

using namespace ssdk;

extern "C" size_t ssd_conv1d_workspace_bytes(const ssd_conv_shape_t* sh) {
    if (check(sh) != SSD_OK) return 0;
    const size_t n = (size_t)sh->batch * (size_t)(ntiles_bwd(sh) > 0 ? ntiles_bwd(sh) : 1) * 5 * (size_t)sh->channels * 4;
    return (n + 255) & ~(size_t)255;
}

namespace ssdk {
namespace {

// split: the three-part form of out / dout; every boundary a multiple of the vector width or the kernels fall
// back to one channel per thread
bool bind_split(ConvParams& cp, const ConvSplit* sp, bool bwd) {
    if (!sp) return true;
    if (sp->c1 <= 0 || sp->c2 <= sp->c1 || sp->c2 >= cp.C) return false;
    cp.split = 1;
    cp.cb[0] = 0;
    cp.cb[1] = sp->c1;
    cp.cb[2] = sp->c2;
    cp.cb[3] = cp.C;
    for (int k = 0; k < 3; ++k) {
        if (cp.L > 0 && !sp->p[k]) return false;
        if (bwd) cp.dout3[k] = sp->p[k];
        else cp.out3[k] = sp->p[k];
    }
    return true;
}

int vec_width(const ConvParams& cp, bool bf) {
    int all = cp.C | (int)cp.u_rs;
    if (cp.split) all |= cp.cb[1] | cp.cb[2];
    return bf ? (all % 8 == 0 ? 8 : 1) : (all % 4 == 0 ? 4 : 1);
}

int conv_fwd_impl(const ssd_conv_shape_t* sh, const void* u, const float* w, const float* bias, const void* state_in, void* out,
                  const ConvSplit* split, void* state_out, void* hip_stream) {
    int rc = check(sh);
    if (rc != SSD_OK) return rc;
    if (!w) return SSD_ERR_NULL;
    if (sh->seqlen > 0 && (!u || (!out && !split))) return SSD_ERR_NULL;
    ConvParams cp;
    memset(&cp, 0, sizeof(cp));
    cp.u = u;
    cp.out = out;
    cp.state_in = state_in;
    cp.state_out = state_out;
    cp.w = w;
    cp.bias = bias;
    cp.L = sh->seqlen;
    cp.C = sh->channels;
    cp.u_rs = sh->u_row_stride ? sh->u_row_stride : sh->channels;
    cp.u_bs = sh->batch_stride ? sh->batch_stride : sh->seqlen * cp.u_rs;
    cp.o_bs = sh->batch_stride ? sh->batch_stride : sh->seqlen * sh->channels;
    if (!bind_split(cp, split, false)) return SSD_ERR_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    const bool bf = sh->dtype == SSD_BF16;
    const int V = vec_width(cp, bf);
    // an empty sequence still hands the state on: one tile, whose token loop is empty
    cp.tt = pick_tt(sh, FWD_TT);
    const dim3 grid((cp.C / V + 63) / 64, (unsigned)(cp.L > 0 ? (cp.L + cp.tt - 1) / cp.tt : 1), (unsigned)sh->batch);
    if (bf && V == 8) hipLaunchKernelGGL((k_conv_fwd<bf16_t, 8>), grid, dim3(64), 0, st, cp);
    else if (bf) hipLaunchKernelGGL((k_conv_fwd<bf16_t, 1>), grid, dim3(64), 0, st, cp);
    else if (V == 4) hipLaunchKernelGGL((k_conv_fwd<float, 4>), grid, dim3(64), 0, st, cp);
    else hipLaunchKernelGGL((k_conv_fwd<float, 1>), grid, dim3(64), 0, st, cp);
    return hipGetLastError() == hipSuccess ? SSD_OK : SSD_ERR_LAUNCH;
}

int conv_bwd_impl(const ssd_conv_shape_t* sh, const void* u, const float* w, const float* bias, const void* state_in, const void* dout,
                  const ConvSplit* split, const float* dstate_out, void* du, float* dw, float* dbias, float* dstate_in, void* workspace,
                  size_t workspace_bytes, uint32_t flags, void* hip_stream) {
    int rc = check(sh);
    if (rc != SSD_OK) return rc;
    if (flags & ~(uint32_t)SSD_FLAG_ACCUM_PARAM) return SSD_ERR_ARG;
    if (!w || !dw) return SSD_ERR_NULL;
    if (sh->seqlen > 0 && (!u || (!dout && !split) || !du)) return SSD_ERR_NULL;
    if (sh->seqlen > 0 && du == dout) return SSD_ERR_ARG;
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < ssd_conv1d_workspace_bytes(sh)) return SSD_ERR_WORKSPACE;
    ConvParams cp;
    memset(&cp, 0, sizeof(cp));
    cp.u = u;
    cp.dout = dout;
    cp.du = du;
    cp.state_in = state_in;
    cp.dstate_out = dstate_out;
    cp.dstate_in = dstate_in;
    cp.w = w;
    cp.bias = bias;
    cp.part = (float*)workspace;
    cp.L = sh->seqlen;
    cp.C = sh->channels;
    cp.u_rs = sh->u_row_stride ? sh->u_row_stride : sh->channels;
    cp.u_bs = sh->batch_stride ? sh->batch_stride : sh->seqlen * cp.u_rs;
    cp.o_bs = sh->batch_stride ? sh->batch_stride : sh->seqlen * sh->channels;
    cp.tt = pick_tt(sh, BWD_TT);
    cp.ntiles = ntiles_bwd(sh) > 0 ? ntiles_bwd(sh) : 1;
    if (!bind_split(cp, split, true)) return SSD_ERR_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    const bool bf = sh->dtype == SSD_BF16;
    const int V = vec_width(cp, bf);
    const dim3 grid((cp.C / V + 63) / 64, (unsigned)cp.ntiles, (unsigned)sh->batch);
    if (bf && V == 8) hipLaunchKernelGGL((k_conv_bwd<bf16_t, 8>), grid, dim3(64), 0, st, cp);
    else if (bf) hipLaunchKernelGGL((k_conv_bwd<bf16_t, 1>), grid, dim3(64), 0, st, cp);
    else if (V == 4) hipLaunchKernelGGL((k_conv_bwd<float, 4>), grid, dim3(64), 0, st, cp);
    else hipLaunchKernelGGL((k_conv_bwd<float, 1>), grid, dim3(64), 0, st, cp);
    if (hipGetLastError() != hipSuccess) return SSD_ERR_LAUNCH;
    hipLaunchKernelGGL(k_conv_reduce, dim3((5 * cp.C + 63) / 64), dim3(256), 0, st, cp.part, (int64_t)sh->batch * cp.ntiles,
                       cp.C, dw, dbias, (flags & SSD_FLAG_ACCUM_PARAM) ? 1 : 0);
    return hipGetLastError() == hipSuccess ? SSD_OK : SSD_ERR_LAUNCH;
}

}  // namespace

int conv1d_fwd_split(const ssd_conv_shape_t* sh, const void* u, const float* w, const float* bias, const void* state_in,
                     const ConvSplit& out, void* state_out, hipStream_t st) {
    return conv_fwd_impl(sh, u, w, bias, state_in, nullptr, &out, state_out, st);
}

int conv1d_bwd_split(const ssd_conv_shape_t* sh, const void* u, const float* w, const float* bias, const void* state_in,
                     const ConvSplit& dout, const float* dstate_out, void* du, float* dw, float* dbias, float* dstate_in,
                     void* workspace, size_t workspace_bytes, uint32_t flags, hipStream_t st) {
    return conv_bwd_impl(sh, u, w, bias, state_in, nullptr, &dout, dstate_out, du, dw, dbias, dstate_in, workspace, workspace_bytes,
                         flags, st);
}

}  // namespace ssdk

extern "C" int ssd_conv1d_fwd(const ssd_conv_shape_t* sh, const void* u, const float* w, const float* bias,
                              const void* state_in, void* out, void* state_out, void* hip_stream) {
    return conv_fwd_impl(sh, u, w, bias, state_in, out, nullptr, state_out, hip_stream);
}

extern "C" int ssd_conv1d_bwd(const ssd_conv_shape_t* sh, const void* u, const float* w, const float* bias,
                              const void* state_in, const void* dout, const float* dstate_out, void* du, float* dw,
                              float* dbias, float* dstate_in, void* workspace, size_t workspace_bytes, uint32_t flags,
                              void* hip_stream) {
    return conv_bwd_impl(sh, u, w, bias, state_in, dout, nullptr, dstate_out, du, dw, dbias, dstate_in, workspace, workspace_bytes,
                         flags, hip_stream);
}
