// The two projections of the Mamba-2 block (dense layers without bias, bf16 storage, fp32 accumulation):
//     out[t,o] = sum_i x[t,i] w[o,i];    dx[t,i] = sum_o dout[t,o] w[o,i];    dw[o,i] = sum_t dout[t,o] x[t,i]
// (the input projection in front of the convolution, whose output width is the larger part of the per-token
// grid-cell activations of App. C, Tab. 7, and the output projection behind the gated normalisation).
// These are dense contractions far above the machine's flop/byte ridge: matrix-core bound.
//
// One kernel, C[M,N] = op(A) op(B)^T with fp32 accumulators in v_mfma_f32_32x32x16_bf16 tiles, for the three
// operand layouts the three products need: an operand is either stored with the contraction index
// contiguous ("k-major": rows of x for the forward product) or with it as the row index (x and dout for
// dw, w for dx).  Both kinds are staged in LDS exactly as they lie in memory (16-byte vectors); k-major
// tiles are read back as plain 16-byte operands, the others through the transposing LDS read.
// Workgroup tile 256 x 128, K step 64, four waves of 128 x 64 (4 x 2 MFMA tiles, 128 accumulator
// registers): 6 operand reads per 8 MFMAs keeps the LDS below its bandwidth.  The next K step's global
// loads are in flight while the current one is multiplied.  Workgroup ids are remapped so that each XCD
// works on a compact block of the tile grid (its L2 then holds the A and B panels that block shares).
#include <string.h>

#include "mfma_common.h"

namespace ssdk {
namespace {

using namespace mf;

constexpr int BM = 256, BN = 128, BKK = 64;
constexpr int KPITCH = 144;        // bytes per LDS row of a k-major tile: 64 k (128 bytes) + 16 pad
constexpr int APITCH_T = 2 * BM + 16;  // bytes per LDS row (one k) of a tile stored [k][m]
constexpr int BPITCH_T = 2 * BN + 16;

struct GemmParams {
    const bf16_t* A;
    const bf16_t* B;
    void* C;
    int64_t lda, ldb, ldc;
    int M, N, K;
    int tiles_m, tiles_n;
    int c_f32;       // C is fp32 (else bf16)
    int accumulate;  // fp32 only: C += product
};

// Tile of this workgroup.  Hardware hands consecutive workgroup ids to the eight XCDs in turn; id -> (id % 8,
// id / 8) gives every XCD a contiguous eighth of a walk that goes down groups of eight row tiles column by
// column, so the workgroups resident on one XCD at a time share a few A row panels and B column panels.
__device__ __forceinline__ void tile_of(const GemmParams& gp, int& tm, int& tn) {
    const int nt = gp.tiles_m * gp.tiles_n;
    int id = blockIdx.x;
    if (nt % 8 == 0) id = (id & 7) * (nt >> 3) + (id >> 3);
    const int per_group = 8 * gp.tiles_n;
    const int grp = id / per_group, in = id - grp * per_group;
    const int first = grp * 8;
    const int gsz = gp.tiles_m - first < 8 ? gp.tiles_m - first : 8;
    tm = first + in % gsz;
    tn = in / gsz;
}

// Global -> registers for one K step of one operand.  ROWS = tile extent along the operand's own index (m
// or n).  k-major: ROWS rows of 8 vectors; otherwise 64 k-rows of ROWS / 8 vectors.  Out-of-range vectors
// are zeros (all extents are multiples of 8, so a vector is inside or outside as a whole).
template <int ROWS, bool KMAJOR>
__device__ __forceinline__ void load_tile(const bf16_t* base, int64_t ld, int r0, int rmax, int k0, int kmax, int tid,
                                          bf16x8 (&reg)[ROWS / 32]) {
    bf16x8 zero;
#pragma unroll
    for (int e = 0; e < 8; ++e) zero[e] = (__bf16)0.f;
#pragma unroll
    for (int i = 0; i < ROWS / 32; ++i) {
        const int v = tid + 256 * i;
        if (KMAJOR) {
            const int row = r0 + (v >> 3), k = k0 + (v & 7) * 8;
            reg[i] = (row < rmax && k < kmax) ? *(const bf16x8*)(base + (int64_t)row * ld + k) : zero;
        } else {
            constexpr int VPR = ROWS / 8;
            const int k = k0 + v / VPR, row = r0 + (v % VPR) * 8;
            reg[i] = (row < rmax && k < kmax) ? *(const bf16x8*)(base + (int64_t)k * ld + row) : zero;
        }
    }
}

template <int ROWS, bool KMAJOR>
__device__ __forceinline__ void store_tile(char* lds, int tid, const bf16x8 (&reg)[ROWS / 32]) {
#pragma unroll
    for (int i = 0; i < ROWS / 32; ++i) {
        const int v = tid + 256 * i;
        if (KMAJOR) {
            *(bf16x8*)(lds + (v >> 3) * KPITCH + (v & 7) * 16) = reg[i];
        } else {
            constexpr int VPR = ROWS / 8;
            *(bf16x8*)(lds + (v / VPR) * (2 * ROWS + 16) + (v % VPR) * 16) = reg[i];
        }
    }
}

// MFMA operand for rows r0 .. r0+31 of the tile, k = kk .. kk+15
template <int ROWS, bool KMAJOR>
__device__ __forceinline__ bf16x8 operand(const char* lds, int r0, int kk, int lane) {
    if (KMAJOR) return *(const bf16x8*)(lds + (r0 + (lane & 31)) * KPITCH + (kk + 8 * (lane >> 5)) * 2);
    return frag_tr(lds, 2 * ROWS + 16, kk, r0, lane);
}

template <bool AK, bool BK>
__global__ __launch_bounds__(256, 2) void k_gemm(GemmParams gp) {
    constexpr int A_BYTES = AK ? BM * KPITCH : BKK * APITCH_T;
    constexpr int B_BYTES = BK ? BN * KPITCH : BKK * BPITCH_T;
    __shared__ __attribute__((aligned(16))) char lds[A_BYTES + B_BYTES];
    char* As = lds;
    char* Bs = lds + A_BYTES;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w >> 1, wn = w & 1;
    int tm, tn;
    tile_of(gp, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[4][2];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = zero16();

    bf16x8 ra[BM / 32], rb[BN / 32];
    load_tile<BM, AK>(gp.A, gp.lda, m0, gp.M, 0, gp.K, tid, ra);
    load_tile<BN, BK>(gp.B, gp.ldb, n0, gp.N, 0, gp.K, tid, rb);
    for (int k0 = 0; k0 < gp.K; k0 += BKK) {
        store_tile<BM, AK>(As, tid, ra);
        store_tile<BN, BK>(Bs, tid, rb);
        __syncthreads();
        if (k0 + BKK < gp.K) {  // next step's loads fly during the products
            load_tile<BM, AK>(gp.A, gp.lda, m0, gp.M, k0 + BKK, gp.K, tid, ra);
            load_tile<BN, BK>(gp.B, gp.ldb, n0, gp.N, k0 + BKK, gp.K, tid, rb);
        }
#pragma unroll
        for (int kk = 0; kk < BKK; kk += 16) {
            bf16x8 a[4], b[2];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = operand<BM, AK>(As, wm * 128 + i * 32, kk, lane);
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = operand<BN, BK>(Bs, wn * 64 + j * 32, kk, lane);
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = mfma(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }

    // accumulator register r of a lane: row acc_row(r, lane), column lane % 32 of its 32 x 32 tile
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn * 64 + j * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = m0 + wm * 128 + i * 32 + acc_row(r, lane);
                if (row < gp.M && col < gp.N) {
                    const int64_t o = (int64_t)row * gp.ldc + col;
                    if (gp.c_f32) {
                        float* c = (float*)gp.C + o;
                        *c = gp.accumulate ? *c + acc[i][j][r] : acc[i][j][r];
                    } else {
                        ((__bf16*)gp.C)[o] = (__bf16)acc[i][j][r];
                    }
                }
            }
        }
    }
}

bool ok_ptr(const void* p) { return p && ((uintptr_t)p & 15) == 0; }

template <bool AK, bool BK>
hipError_t launch_gemm(GemmParams gp, hipStream_t st) {
    gp.tiles_m = (gp.M + BM - 1) / BM;
    gp.tiles_n = (gp.N + BN - 1) / BN;
    hipLaunchKernelGGL((k_gemm<AK, BK>), dim3(gp.tiles_m * gp.tiles_n), dim3(256), 0, st, gp);
    return hipGetLastError();
}

int check(int64_t rows, int32_t in_dim, int32_t out_dim, int64_t ldx, int64_t ldo) {
    if (rows < 0 || rows > 0x7fffffff || in_dim <= 0 || out_dim <= 0) return SSD_ERR_SHAPE;
    if ((in_dim | out_dim) & 7) return SSD_ERR_DIVISIBILITY;  // 16-byte vectors of bf16
    if ((ldx && (ldx < in_dim || (ldx & 7))) || (ldo && (ldo < out_dim || (ldo & 7)))) return SSD_ERR_SHAPE;
    const int64_t tiles = ((rows + BM - 1) / BM) * (((int64_t)out_dim + BN - 1) / BN);
    const int64_t tiles_w = (((int64_t)out_dim + BM - 1) / BM) * (((int64_t)in_dim + BN - 1) / BN);
    if (tiles > 0x7fffffff || tiles_w > 0x7fffffff) return SSD_ERR_SHAPE;
    return SSD_OK;
}

}  // namespace
}  // namespace ssdk

using namespace ssdk;

extern "C" int ssd_linear_fwd(int64_t rows, int32_t in_dim, int32_t out_dim, const void* x, int64_t x_row_stride,
                              const void* w, void* out, int64_t out_row_stride, void* hip_stream) {
    const int rc = check(rows, in_dim, out_dim, x_row_stride, out_row_stride);
    if (rc != SSD_OK) return rc;
    if (rows == 0) return SSD_OK;
    if (!x || !w || !out) return SSD_ERR_NULL;
    if (!ok_ptr(x) || !ok_ptr(w) || !ok_ptr(out)) return SSD_ERR_ARG;
    GemmParams gp;
    memset(&gp, 0, sizeof(gp));
    gp.A = (const bf16_t*)x;   // [rows, in]   k-major
    gp.B = (const bf16_t*)w;   // [out, in]    k-major
    gp.C = out;
    gp.lda = x_row_stride ? x_row_stride : in_dim;
    gp.ldb = in_dim;
    gp.ldc = out_row_stride ? out_row_stride : out_dim;
    gp.M = (int)rows;
    gp.N = out_dim;
    gp.K = in_dim;
    return launch_gemm<true, true>(gp, (hipStream_t)hip_stream) == hipSuccess ? SSD_OK : SSD_ERR_LAUNCH;
}

extern "C" int ssd_linear_bwd(int64_t rows, int32_t in_dim, int32_t out_dim, const void* x, int64_t x_row_stride,
                              const void* w, const void* dout, int64_t dout_row_stride, void* dx, int64_t dx_row_stride,
                              float* dw, uint32_t flags, void* hip_stream) {
    int rc = check(rows, in_dim, out_dim, x_row_stride, dout_row_stride);
    if (rc != SSD_OK) return rc;
    if (dx_row_stride && (dx_row_stride < in_dim || (dx_row_stride & 7))) return SSD_ERR_SHAPE;
    if (flags & ~(uint32_t)SSD_FLAG_ACCUM_PARAM) return SSD_ERR_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    const int accumulate = (flags & SSD_FLAG_ACCUM_PARAM) ? 1 : 0;
    if (rows == 0) {
        if (dw && !accumulate && launch_fill_zero(dw, (size_t)out_dim * in_dim, st) != hipSuccess) return SSD_ERR_LAUNCH;
        return SSD_OK;
    }
    if (!dout || (dx && !w) || (dw && !x)) return SSD_ERR_NULL;
    if (!ok_ptr(dout) || (dx && (!ok_ptr(dx) || !ok_ptr(w))) || (dw && (!ok_ptr(x) || !ok_ptr(dw)))) return SSD_ERR_ARG;
    GemmParams gp;
    const int64_t ldd = dout_row_stride ? dout_row_stride : out_dim;
    if (dx) {  // dx[rows, in] = dout[rows, out] w[out, in]: contraction over out; w holds it as the row index
        memset(&gp, 0, sizeof(gp));
        gp.A = (const bf16_t*)dout;
        gp.B = (const bf16_t*)w;
        gp.C = dx;
        gp.lda = ldd;
        gp.ldb = in_dim;
        gp.ldc = dx_row_stride ? dx_row_stride : in_dim;
        gp.M = (int)rows;
        gp.N = in_dim;
        gp.K = out_dim;
        if (launch_gemm<true, false>(gp, st) != hipSuccess) return SSD_ERR_LAUNCH;
    }
    if (dw) {  // dw[out, in] = dout^T x: contraction over the rows, the row index of both operands
        memset(&gp, 0, sizeof(gp));
        gp.A = (const bf16_t*)dout;
        gp.B = (const bf16_t*)x;
        gp.C = dw;
        gp.lda = ldd;
        gp.ldb = x_row_stride ? x_row_stride : in_dim;
        gp.ldc = in_dim;
        gp.M = out_dim;
        gp.N = in_dim;
        gp.K = (int)rows;
        gp.c_f32 = 1;
        gp.accumulate = accumulate;
        if (launch_gemm<false, false>(gp, st) != hipSuccess) return SSD_ERR_LAUNCH;
    }
    return SSD_OK;
}
