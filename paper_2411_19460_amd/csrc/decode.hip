// Recurrent form of the layer (Sec. 3.1, Eq. 1 in the Mamba-2 form), token by token:
//     state <- exp(dt_t A) state + dt_t x_t (x) B_t ;   y_t = C_t state + D x_t
// the constant-memory step that continues a sequence after a prefill (ssd_fwd's final_state).
// Any P, N, fp32 or bf16 storage; bound by reading and writing the fp32 state: once per call where a state
// row fits a wave's registers (N <= 256), else once per token.
#include "ssd_internal.h"

namespace ssdk {
namespace {

struct DecodeParams {
    const void *x, *dt, *Bm, *Cm;
    const uint8_t* reset;  // optional [Bt][T]: non-zero = the state is dropped before this token
    const float *A, *D;
    float* state;
    void* y;
    int64_t T, xs_b, dts_b, bcs_b;
    int64_t state_bs;  // floats between the states of consecutive batch entries (dense: H P N)
    int H, P, G, N, hpg;
    float skip_add;  // 1 under the residual flag: y = x + layer(x)
};

template <typename T>
__device__ __forceinline__ float ld(const void* p, int64_t i);
template <>
__device__ __forceinline__ float ld<float>(const void* p, int64_t i) { return ((const float*)p)[i]; }
template <>
__device__ __forceinline__ float ld<bf16_t>(const void* p, int64_t i) { return bf16_to_float(((const bf16_t*)p)[i]); }
template <typename T>
__device__ __forceinline__ void st(void* p, int64_t i, float v);
template <>
__device__ __forceinline__ void st<float>(void* p, int64_t i, float v) { ((float*)p)[i] = v; }
template <>
__device__ __forceinline__ void st<bf16_t>(void* p, int64_t i, float v) { ((bf16_t*)p)[i] = float_to_bf16(v); }

// Workgroup (head, batch, z) owns the state rows p = 4 z + w (wave w), and further rows in steps of
// 4 gridDim.z; lane l the columns n = l, l + 64, ...  A lane only ever touches its own state elements
// and rows are independent recurrences, so the token loop needs no synchronisation at all.
template <typename T>
__global__ __launch_bounds__(256) void k_decode(DecodeParams dp) {
    const int h = blockIdx.x, b = blockIdx.y, g = h / dp.hpg;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const float Ah = dp.A[h], Dh = dp.D[h] + dp.skip_add;
    float* S = dp.state + (int64_t)b * dp.state_bs + (int64_t)h * dp.P * dp.N;
    for (int64_t t = 0; t < dp.T; ++t) {
        const float dtv = ld<T>(dp.dt, (int64_t)b * dp.dts_b + t * dp.H + h);
        const float a = (dp.reset && dp.reset[(int64_t)b * dp.T + t]) ? 0.f : __expf(dtv * Ah);
        const int64_t bc = (int64_t)b * dp.bcs_b + (t * dp.G + g) * dp.N;
        const int64_t xo = (int64_t)b * dp.xs_b + (t * dp.H + h) * dp.P;
        for (int p = 4 * blockIdx.z + w; p < dp.P; p += 4 * gridDim.z) {
            const float xv = ld<T>(dp.x, xo + p);
            const float dx = dtv * xv;
            float acc = 0.f;
            for (int n = lane; n < dp.N; n += 64) {
                const float hn = a * S[(int64_t)p * dp.N + n] + dx * ld<T>(dp.Bm, bc + n);
                S[(int64_t)p * dp.N + n] = hn;
                acc += ld<T>(dp.Cm, bc + n) * hn;
            }
            for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
            if (lane == 0) st<T>(dp.y, xo + p, acc + Dh * xv);
        }
    }
}

// The same for N <= 64 NPL with the wave's state rows in registers over all tokens of the call: U rows per wave
// (p = 4 z + w + 4 u gridDim.z), all of them requested before the first is used, the B and C values of a token
// fetched once for all rows.  The state is read once and written once per call instead of once per token.
template <typename T, int NPL, int U>
__global__ __launch_bounds__(256) void k_decode_reg(DecodeParams dp) {
    const int h = blockIdx.x, b = blockIdx.y, g = h / dp.hpg;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const float Ah = dp.A[h], Dh = dp.D[h] + dp.skip_add;
    float* S = dp.state + (int64_t)b * dp.state_bs + (int64_t)h * dp.P * dp.N;
    const int pstep = 4 * gridDim.z, p0 = 4 * blockIdx.z + w;
    float s[U][NPL];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < NPL; ++i) {
            const int p = p0 + u * pstep, n = lane + 64 * i;
            s[u][i] = p < dp.P && n < dp.N ? S[(int64_t)p * dp.N + n] : 0.f;
        }
    for (int64_t t = 0; t < dp.T; ++t) {
        const float dtv = ld<T>(dp.dt, (int64_t)b * dp.dts_b + t * dp.H + h);
        const bool drop = dp.reset && dp.reset[(int64_t)b * dp.T + t];
        const float a = drop ? 0.f : __expf(dtv * Ah);
        const int64_t bc = (int64_t)b * dp.bcs_b + (t * dp.G + g) * dp.N;
        const int64_t xo = (int64_t)b * dp.xs_b + (t * dp.H + h) * dp.P;
        float bv[NPL], cv[NPL];
#pragma unroll
        for (int i = 0; i < NPL; ++i) {
            const int n = lane + 64 * i;
            bv[i] = n < dp.N ? ld<T>(dp.Bm, bc + n) : 0.f;
            cv[i] = n < dp.N ? ld<T>(dp.Cm, bc + n) : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int p = p0 + u * pstep;
            if (p < dp.P) {
                const float xv = ld<T>(dp.x, xo + p);
                const float dx = dtv * xv;
                float acc = 0.f;
#pragma unroll
                for (int i = 0; i < NPL; ++i) {
                    s[u][i] = a * s[u][i] + dx * bv[i];
                    acc += cv[i] * s[u][i];
                }
                for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
                if (lane == 0) st<T>(dp.y, xo + p, acc + Dh * xv);
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < NPL; ++i) {
            const int p = p0 + u * pstep, n = lane + 64 * i;
            if (p < dp.P && n < dp.N) S[(int64_t)p * dp.N + n] = s[u][i];
        }
}

// Four consecutive values of B, C (storage type) as floats; 8- or 16-byte loads.
template <typename T>
__device__ __forceinline__ void ld4(const void* p, int64_t i, float (&v)[4]);
template <>
__device__ __forceinline__ void ld4<float>(const void* p, int64_t i, float (&v)[4]) {
    const float4 t = *(const float4*)((const float*)p + i);
    v[0] = t.x; v[1] = t.y; v[2] = t.z; v[3] = t.w;
}
template <>
__device__ __forceinline__ void ld4<bf16_t>(const void* p, int64_t i, float (&v)[4]) {
    const uint2 t = *(const uint2*)((const bf16_t*)p + i);
    v[0] = __uint_as_float(t.x << 16); v[1] = __uint_as_float(t.x & 0xffff0000u);
    v[2] = __uint_as_float(t.y << 16); v[3] = __uint_as_float(t.y & 0xffff0000u);
}

// The same again with 16-byte accesses to the state (N a multiple of 4, N <= 128 NV): half a wave owns a row,
// lane l of the half the columns 4 l .. 4 l + 3 (+ 128 i); a wave walks U pairs of rows.
template <typename T, int NV, int U>
__global__ __launch_bounds__(256) void k_decode_reg4(DecodeParams dp) {
    const int h = blockIdx.x, b = blockIdx.y, g = h / dp.hpg;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, half = lane >> 5, l32 = lane & 31;
    const float Ah = dp.A[h], Dh = dp.D[h] + dp.skip_add;
    float* S = dp.state + (int64_t)b * dp.state_bs + (int64_t)h * dp.P * dp.N;
    const int p0 = (4 * blockIdx.z + w) * 2 * U + half;  // rows p0, p0 + 2, ...
    float4 s[U][NV];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int p = p0 + 2 * u, n = 4 * l32 + 128 * i;
            s[u][i] = p < dp.P && n < dp.N ? *(const float4*)(S + (int64_t)p * dp.N + n) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    for (int64_t t = 0; t < dp.T; ++t) {
        const float dtv = ld<T>(dp.dt, (int64_t)b * dp.dts_b + t * dp.H + h);
        const bool drop = dp.reset && dp.reset[(int64_t)b * dp.T + t];
        const float a = drop ? 0.f : __expf(dtv * Ah);
        const int64_t bc = (int64_t)b * dp.bcs_b + (t * dp.G + g) * dp.N;
        const int64_t xo = (int64_t)b * dp.xs_b + (t * dp.H + h) * dp.P;
        float bv[NV][4], cv[NV][4];
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int n = 4 * l32 + 128 * i;
            if (n < dp.N) {
                ld4<T>(dp.Bm, bc + n, bv[i]);
                ld4<T>(dp.Cm, bc + n, cv[i]);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) bv[i][e] = cv[i][e] = 0.f;
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int p = p0 + 2 * u;
            const bool live = p < dp.P;
            const float xv = live ? ld<T>(dp.x, xo + p) : 0.f;
            const float dx = dtv * xv;
            float acc = 0.f;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
                s[u][i].x = a * s[u][i].x + dx * bv[i][0];
                s[u][i].y = a * s[u][i].y + dx * bv[i][1];
                s[u][i].z = a * s[u][i].z + dx * bv[i][2];
                s[u][i].w = a * s[u][i].w + dx * bv[i][3];
                acc += cv[i][0] * s[u][i].x + cv[i][1] * s[u][i].y + cv[i][2] * s[u][i].z + cv[i][3] * s[u][i].w;
            }
            for (int off = 16; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);  // within the half wave
            if (live && l32 == 0) st<T>(dp.y, xo + p, acc + Dh * xv);
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int i = 0; i < NV; ++i) {
            const int p = p0 + 2 * u, n = 4 * l32 + 128 * i;
            if (p < dp.P && n < dp.N) *(float4*)(S + (int64_t)p * dp.N + n) = s[u][i];
        }
}

// Picks the kernel: state rows in registers when a row fits four values per lane, several rows per wave when
// one per wave would make more workgroups than the machine holds at a time.
template <typename T>
hipError_t launch_decode_kernel(const DecodeParams& dp, int nb, hipStream_t s) {
    const int rows4 = (dp.P + 3) / 4;
    const bool vec_ok = dp.N % 4 == 0 && ((uintptr_t)dp.state & 15) == 0 && dp.state_bs % 4 == 0 && ((uintptr_t)dp.Bm & 15) == 0 &&
                        ((uintptr_t)dp.Cm & 15) == 0 && dp.bcs_b % 4 == 0;
    if (dp.N <= 256 && vec_ok) {  // 16-byte state accesses
        const int rows8 = (dp.P + 7) / 8;
        const bool many = (int64_t)dp.H * nb * rows8 > 4096;
        const int u = many ? 4 : 1, gz = (rows8 + u - 1) / u;
        const dim3 grid(dp.H, nb, gz);
        if (dp.N <= 128) {
            if (many) hipLaunchKernelGGL((k_decode_reg4<T, 1, 4>), grid, dim3(256), 0, s, dp);
            else hipLaunchKernelGGL((k_decode_reg4<T, 1, 1>), grid, dim3(256), 0, s, dp);
        } else {
            if (many) hipLaunchKernelGGL((k_decode_reg4<T, 2, 4>), grid, dim3(256), 0, s, dp);
            else hipLaunchKernelGGL((k_decode_reg4<T, 2, 1>), grid, dim3(256), 0, s, dp);
        }
    } else if (dp.N <= 256) {
        const bool many = (int64_t)dp.H * nb * rows4 > 4096;
        const int u = many ? 4 : 1, gz = (rows4 + u - 1) / u;
        const dim3 grid(dp.H, nb, gz);
        if (dp.N <= 128) {
            if (many) hipLaunchKernelGGL((k_decode_reg<T, 2, 4>), grid, dim3(256), 0, s, dp);
            else hipLaunchKernelGGL((k_decode_reg<T, 2, 1>), grid, dim3(256), 0, s, dp);
        } else {
            if (many) hipLaunchKernelGGL((k_decode_reg<T, 4, 4>), grid, dim3(256), 0, s, dp);
            else hipLaunchKernelGGL((k_decode_reg<T, 4, 1>), grid, dim3(256), 0, s, dp);
        }
    } else {
        hipLaunchKernelGGL(k_decode<T>, dim3(dp.H, nb, rows4 < 64 ? rows4 : 64), dim3(256), 0, s, dp);
    }
    return hipGetLastError();
}

}  // namespace

// One token for each of `nb` sequences whose states lie state_bs floats apart (bf16 storage): x [nb, H, P],
// dt [nb, H], B, C [nb, G, N] dense -> y [nb, H, P].
hipError_t launch_decode_strided(int nb, int H, int P, int G, int N, const void* x, const void* dt, const float* A, const void* B,
                                 const void* C, const float* D, float* state, int64_t state_bs, void* y, hipStream_t st) {
    if (nb <= 0 || nb > 65535 || H <= 0 || H > 65535 || P <= 0 || G <= 0 || N <= 0 || H % G) return hipErrorInvalidValue;
    DecodeParams dp;
    dp.x = x;
    dp.dt = dt;
    dp.Bm = B;
    dp.Cm = C;
    dp.A = A;
    dp.D = D;
    dp.state = state;
    dp.reset = nullptr;
    dp.y = y;
    dp.T = 1;
    dp.H = H;
    dp.P = P;
    dp.G = G;
    dp.N = N;
    dp.hpg = H / G;
    dp.xs_b = (int64_t)H * P;
    dp.dts_b = H;
    dp.bcs_b = (int64_t)G * N;
    dp.state_bs = state_bs;
    dp.skip_add = 0.f;
    return launch_decode_kernel<bf16_t>(dp, nb, st);
}

}  // namespace ssdk

using namespace ssdk;

extern "C" int ssd_decode(const ssd_shape_t* sh, const void* x, const void* dt, const float* A, const void* B,
                          const void* C, const float* D, float* state, void* y, uint32_t flags, void* hip_stream) {
    if (!sh) return SSD_ERR_NULL;
    if (sh->dtype != SSD_F32 && sh->dtype != SSD_BF16) return SSD_ERR_DTYPE;
    if (sh->batch <= 0 || sh->seqlen < 0 || sh->nheads <= 0 || sh->headdim <= 0 || sh->ngroups <= 0 || sh->dstate <= 0)
        return SSD_ERR_SHAPE;
    if (sh->batch > 65535 || sh->nheads > 65535) return SSD_ERR_SHAPE;
    if (sh->nheads % sh->ngroups != 0) return SSD_ERR_DIVISIBILITY;
    if (flags & ~(uint32_t)SSD_FLAG_RESIDUAL) return SSD_ERR_ARG;
    if (sh->seqlen == 0) return SSD_OK;
    if (!x || !dt || !A || !B || !C || !D || !state || !y) return SSD_ERR_NULL;
    DecodeParams dp;
    dp.x = x;
    dp.dt = dt;
    dp.Bm = B;
    dp.Cm = C;
    dp.A = A;
    dp.D = D;
    dp.state = state;
    dp.reset = sh->seq_reset;
    dp.y = y;
    dp.T = sh->seqlen;
    dp.H = sh->nheads;
    dp.P = sh->headdim;
    dp.G = sh->ngroups;
    dp.N = sh->dstate;
    dp.hpg = dp.H / dp.G;
    dp.xs_b = sh->x_batch_stride ? sh->x_batch_stride : dp.T * dp.H * dp.P;
    dp.dts_b = sh->dt_batch_stride ? sh->dt_batch_stride : dp.T * dp.H;
    dp.bcs_b = sh->bc_batch_stride ? sh->bc_batch_stride : dp.T * dp.G * dp.N;
    if (dp.xs_b < dp.T * dp.H * dp.P || dp.dts_b < dp.T * dp.H || dp.bcs_b < dp.T * dp.G * dp.N) return SSD_ERR_SHAPE;
    dp.state_bs = (int64_t)dp.H * dp.P * dp.N;
    dp.skip_add = (flags & SSD_FLAG_RESIDUAL) ? 1.f : 0.f;
    hipStream_t s = (hipStream_t)hip_stream;
    const hipError_t e = sh->dtype == SSD_BF16 ? launch_decode_kernel<bf16_t>(dp, (int)sh->batch, s) : launch_decode_kernel<float>(dp, (int)sh->batch, s);
    return e == hipSuccess ? SSD_OK : SSD_ERR_LAUNCH;
}
