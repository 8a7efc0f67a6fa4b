// The two projections of the Mamba-2 block (dense layers without bias, bf16 storage, fp32 accumulation):
//     out[t,o] = sum_i x[t,i] w[o,i];    dx[t,i] = sum_o dout[t,o] w[o,i];    dw[o,i] = sum_t dout[t,o] x[t,i]
// (the input projection in front of the convolution, whose output width is the larger part of the per-token
// grid-cell activations of App. C, Tab. 7, and the output projection behind the gated normalisation).
// These are dense contractions far above the machine's flop/byte ridge: matrix-core bound.
//
// One scheme, C[M,N] = op(A) op(B)^T with fp32 accumulators in v_mfma_f32_32x32x16_bf16 tiles, for the three
// operand layouts the three products need: an operand is either stored with the contraction index
// contiguous ("k-major": rows of x for the forward product) or with it as the row index (x and dout for
// dw, w for dx).  Both kinds are staged in LDS exactly as they lie in memory (16-byte vectors); k-major
// tiles are read back as plain 16-byte operands, the others through the transposing LDS read.
// Two tilings: 256 x 256 per workgroup (four waves of 128 x 128: the whole accumulator file, one workgroup per
// compute unit, hand-laid-out K step; k_gemm_big) wherever that yields enough tiles, else 256 x 128 (two
// workgroups per compute unit; k_gemm).  Workgroup ids are remapped so that each XCD works on a compact
// block of the tile grid (its L2 then holds the A and B panels that block shares).
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "mfma_common.h"

namespace ssdk {
namespace {

using namespace mf;

constexpr int BKK = 64;            // K step
constexpr int KPITCH = 144;        // bytes per LDS row of a k-major tile: 64 k (128 bytes) + 16 pad

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

// bytes of one operand tile in LDS: k-major [ROWS][64 k] (rows padded by 16 bytes) or [64 k][ROWS] (by 64)
template <int ROWS, bool KMAJOR>
constexpr int tile_bytes() { return KMAJOR ? ROWS * KPITCH : BKK * (2 * ROWS + 64); }
// Row pitch of a tile stored [k][ROWS]: 64 bytes of padding put consecutive k rows 16 banks apart, so the four
// k rows (32 bytes each per half-wave) that one transposing read touches fall into distinct banks.
template <int ROWS>
constexpr int tpitch() { return 2 * ROWS + 64; }

// Global -> registers for one K step of one operand.  ROWS = tile extent along the operand's own index (m
// or n).  k-major: ROWS rows of 8 vectors; otherwise 64 k-rows of ROWS / 8 vectors.  `origin` points at the
// tile's first element of this K step (wave-uniform: scalar registers); a thread's vectors lie a fixed
// number of rows apart, so one 32-bit byte offset per thread addresses them all.  MASK: vectors outside
// rows_left x k_left are zeros (all extents are multiples of 8: a vector is inside or outside as a whole).
template <int ROWS, bool KMAJOR>
__device__ __forceinline__ uint32_t tile_voff(int64_t ld, int tid) {
    constexpr int VPR = KMAJOR ? 8 : ROWS / 8;  // vectors per memory row of the tile
    return (uint32_t)(tid / VPR) * (uint32_t)(ld * 2) + (uint32_t)(tid % VPR) * 16;
}

template <int ROWS, bool KMAJOR, bool MASK, int I0 = 0, int I1 = ROWS / 32>
__device__ __forceinline__ void load_tile(const bf16_t* origin, int64_t ld, uint32_t voff, int rows_left, int k_left, int tid,
                                          bf16x8 (&reg)[ROWS / 32]) {
    constexpr int VPR = KMAJOR ? 8 : ROWS / 8;
    constexpr int RSTEP = 256 / VPR;  // memory rows between a thread's consecutive vectors
#pragma unroll
    for (int i = I0; i < I1; ++i) {
        bool in = true;
        if (MASK) {
            const int mrow = tid / VPR + RSTEP * i, mcol = (tid % VPR) * 8;  // memory row / first column of the vector
            in = KMAJOR ? (mrow < rows_left && mcol < k_left) : (mrow < k_left && mcol < rows_left);
        }
        if (in) {
            reg[i] = *(const bf16x8*)((const char*)origin + (size_t)i * RSTEP * (size_t)(ld * 2) + (size_t)voff);
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) reg[i][e] = (__bf16)0.f;
        }
    }
}

template <int ROWS, bool KMAJOR, int I0 = 0, int I1 = ROWS / 32>
__device__ __forceinline__ void store_tile(char* lds, int tid, const bf16x8 (&reg)[ROWS / 32]) {
#pragma unroll
    for (int i = I0; i < I1; ++i) {
        const int v = tid + 256 * i;
        if (KMAJOR) {
            *(bf16x8*)(lds + (v >> 3) * KPITCH + (v & 7) * 16) = reg[i];
        } else {
            constexpr int VPR = ROWS / 8;
            *(bf16x8*)(lds + (v / VPR) * tpitch<ROWS>() + (v % VPR) * 16) = reg[i];
        }
    }
}

// MFMA operand for rows r0 .. r0+31 of the tile, k = kk .. kk+15
template <int ROWS, bool KMAJOR>
__device__ __forceinline__ bf16x8 operand(const char* lds, int r0, int kk, int lane) {
    if (KMAJOR) return *(const bf16x8*)(lds + (r0 + (lane & 31)) * KPITCH + (kk + 8 * (lane >> 5)) * 2);
    return frag_tr(lds, tpitch<ROWS>(), kk, r0, lane);
}

// The MFMAs are issued with the B operand first, so an accumulator tile holds the transposed product: lane
// -> row m = lane % 32 of C, registers 4q .. 4q+3 -> the four consecutive columns 8q + 4 (lane / 32) + 0..3.
// Every lane thus stores 8 bytes (bf16) or 16 bytes (fp32) at a time.  `whole`: the workgroup's tile lies
// inside C (no bounds checks; N is a multiple of 8, so a group of four columns is inside or outside as one).
template <int WI, int WJ>
__device__ __forceinline__ void store_acc(const GemmParams& gp, const f32x16 (&acc)[WI][WJ], int row0, int col0, int lane, bool whole) {
    const int row_l = row0 + (lane & 31), col_l = col0 + (lane >> 5) * 4;
#pragma unroll
    for (int i = 0; i < WI; ++i) {
        const int row = row_l + i * 32;
#pragma unroll
        for (int j = 0; j < WJ; ++j) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int col = col_l + j * 32 + q * 8;
                if (whole || (row < gp.M && col < gp.N)) {
                    const int64_t o = (int64_t)row * gp.ldc + col;
                    const f32x16& t = acc[i][j];
                    if (gp.c_f32) {
                        float4* c = (float4*)((float*)gp.C + o);
                        float4 v = make_float4(t[4 * q], t[4 * q + 1], t[4 * q + 2], t[4 * q + 3]);
                        if (gp.accumulate) {
                            const float4 old = *c;
                            v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w;
                        }
                        *c = v;
                    } else {
                        bf16x4 v;
                        v[0] = (__bf16)t[4 * q]; v[1] = (__bf16)t[4 * q + 1]; v[2] = (__bf16)t[4 * q + 2]; v[3] = (__bf16)t[4 * q + 3];
                        *(bf16x4*)((__bf16*)gp.C + o) = v;
                    }
                }
            }
        }
    }
}

// WI x WJ MFMA tiles per wave, 2 x 2 waves: workgroup tile (64 WI) x (64 WJ), one LDS buffer, two barriers per
// K step; registers and LDS leave room for two workgroups per compute unit, which cover each other's waits.
// Used where the large tiles below would be too few to fill the machine.
template <bool AK, bool BK, int WI, int WJ>
__global__ __launch_bounds__(256, 2) void k_gemm(GemmParams gp) {
    constexpr int BM = 64 * WI, BN = 64 * WJ;
    constexpr int A_BYTES = tile_bytes<BM, AK>();
    extern __shared__ __attribute__((aligned(16))) char lds[];  // A tile, B tile
    char* As = lds;
    char* Bs = lds + A_BYTES;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int wm = w >> 1, wn = w & 1;
    int tm, tn;
    tile_of(gp, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[WI][WJ];
#pragma unroll
    for (int i = 0; i < WI; ++i)
#pragma unroll
        for (int j = 0; j < WJ; ++j) acc[i][j] = zero16();

    // tiles that lie wholly inside the matrices take the unmasked loads for every whole K step
    const bool interior = m0 + BM <= gp.M && n0 + BN <= gp.N;
    const uint32_t va = tile_voff<BM, AK>(gp.lda, tid), vb = tile_voff<BN, BK>(gp.ldb, tid);
    bf16x8 ra[BM / 32], rb[BN / 32];
    auto fetch = [&](int k0) {
        const bf16_t* ao = AK ? gp.A + (int64_t)m0 * gp.lda + k0 : gp.A + (int64_t)k0 * gp.lda + m0;
        const bf16_t* bo = BK ? gp.B + (int64_t)n0 * gp.ldb + k0 : gp.B + (int64_t)k0 * gp.ldb + n0;
        if (interior && k0 + BKK <= gp.K) {
            load_tile<BM, AK, false>(ao, gp.lda, va, 0, 0, tid, ra);
            load_tile<BN, BK, false>(bo, gp.ldb, vb, 0, 0, tid, rb);
        } else {
            load_tile<BM, AK, true>(ao, gp.lda, va, gp.M - m0, gp.K - k0, tid, ra);
            load_tile<BN, BK, true>(bo, gp.ldb, vb, gp.N - n0, gp.K - k0, tid, rb);
        }
    };
    fetch(0);
    for (int k0 = 0; k0 < gp.K; k0 += BKK) {
        store_tile<BM, AK>(As, tid, ra);
        store_tile<BN, BK>(Bs, tid, rb);
        __syncthreads();
        if (k0 + BKK < gp.K) fetch(k0 + BKK);  // next step's loads fly during the products
#pragma unroll
        for (int kk = 0; kk < BKK; kk += 16) {
            bf16x8 a[WI], b[WJ];
#pragma unroll
            for (int i = 0; i < WI; ++i) a[i] = operand<BM, AK>(As, wm * 32 * WI + i * 32, kk, lane);
#pragma unroll
            for (int j = 0; j < WJ; ++j) b[j] = operand<BN, BK>(Bs, wn * 32 * WJ + j * 32, kk, lane);
#pragma unroll
            for (int i = 0; i < WI; ++i)
#pragma unroll
                for (int j = 0; j < WJ; ++j) acc[i][j] = mfma(b[j], a[i], acc[i][j]);
        }
        __syncthreads();
    }

    store_acc<WI, WJ>(gp, acc, m0 + wm * 32 * WI, n0 + wn * 32 * WJ, lane, interior);
}

// 256 x 256 tile, four waves of 128 x 128 (4 x 4 MFMA tiles: the whole accumulator register file), one
// workgroup per compute unit, two LDS buffers.  With a single wave per SIMD nothing else hides latency, so
// the K step is laid out by hand as 16 units of four MFMAs (one A operand against the four B operands of
// its k slice); behind each MFMA sit the LDS reads of later operands and (last eight units) one vector of
// the next tile's LDS writes with the global load that refills its register for the tile after that.
// Registers thus hold the tile two K steps ahead of the one being multiplied: a vector is written to LDS
// in the second half of a step and its register is refilled at once, so that a load has a whole step of
// MFMA time to arrive.
struct BigCtx {
    const bf16_t* a_org;  // tile origin at k = 0
    const bf16_t* b_org;
    int64_t lda, ldb, a_kstep, b_kstep;
    uint32_t va, vb;
    int rows_a, rows_b, K;  // extents left from the tile origin (masks)
    int tid, lane, wm, wn;
};

// One K step.  STEADY: the registers hold a next tile, there is one after it, and neither needs masks --
// straight-line code (no branches: the compiler then counts outstanding loads exactly instead of draining
// them at every join).  Otherwise the same step with run-time conditions, for the last steps and edge tiles.
template <bool AK, bool BK, bool STEADY>
__device__ __forceinline__ void big_step(const BigCtx& cx, f32x16 (&acc)[4][4], bf16x8 (&ra)[8], bf16x8 (&rb)[8], const char* As,
                                         char* An, int k0) {
    constexpr int BM = 256, BN = 256;
    constexpr int A_BYTES = tile_bytes<BM, AK>();
    const char* Bs = As + A_BYTES;
    char* Bn = An + A_BYTES;
    const int k2 = k0 + 2 * BKK;
    const bool more = STEADY || k0 + BKK < cx.K;
    const bool more2 = STEADY || k2 < cx.K;
    const bf16_t* ao = cx.a_org + (int64_t)k2 * cx.a_kstep;
    const bf16_t* bo = cx.b_org + (int64_t)k2 * cx.b_kstep;
    const int lane = cx.lane, tid = cx.tid;
    bf16x8 aq[2], bq[2][4];
    aq[0] = operand<BM, AK>(As, cx.wm * 128, 0, lane);
#pragma unroll
    for (int j = 0; j < 4; ++j) bq[0][j] = operand<BN, BK>(Bs, cx.wn * 128 + j * 32, 0, lane);
    // An MFMA keeps the matrix pipe busy for 32 cycles but takes only a few to issue: every memory
    // instruction is placed right behind an MFMA, so that it issues in that MFMA's shadow.
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int kk = u >> 2, i = u & 3;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[i][j] = mfma(bq[kk & 1][j], aq[u & 1], acc[i][j]);
            // operand reads: the next unit's A operand, and over unit 1 of a k slice the next slice's B operands
            if (j == 0 && u + 1 < 16) aq[(u + 1) & 1] = operand<BM, AK>(As, cx.wm * 128 + ((u + 1) & 3) * 32, ((u + 1) >> 2) * 16, lane);
            if (i == 1 && kk < 3) bq[(kk + 1) & 1][j] = operand<BN, BK>(Bs, cx.wn * 128 + j * 32, (kk + 1) * 16, lane);
            if (STEADY) {
                // units 8..15: behind MFMA 0 a vector of A, behind MFMA 2 a vector of B goes to LDS and its register is refilled
#define GEMM_PART(U, J, OP_A, V)                                                                  \
    if (u == U && j == J) {                                                                       \
        if (OP_A) {                                                                               \
            store_tile<BM, AK, V, V + 1>(An, tid, ra);                                            \
            load_tile<BM, AK, false, V, V + 1>(ao, cx.lda, cx.va, 0, 0, tid, ra);                 \
        } else {                                                                                  \
            store_tile<BN, BK, V, V + 1>(Bn, tid, rb);                                            \
            load_tile<BN, BK, false, V, V + 1>(bo, cx.ldb, cx.vb, 0, 0, tid, rb);                 \
        }                                                                                         \
    }
                GEMM_PART(8, 0, true, 0) GEMM_PART(8, 2, false, 0) GEMM_PART(9, 0, true, 1) GEMM_PART(9, 2, false, 1)
                GEMM_PART(10, 0, true, 2) GEMM_PART(10, 2, false, 2) GEMM_PART(11, 0, true, 3) GEMM_PART(11, 2, false, 3)
                GEMM_PART(12, 0, true, 4) GEMM_PART(12, 2, false, 4) GEMM_PART(13, 0, true, 5) GEMM_PART(13, 2, false, 5)
                GEMM_PART(14, 0, true, 6) GEMM_PART(14, 2, false, 6) GEMM_PART(15, 0, true, 7) GEMM_PART(15, 2, false, 7)
#undef GEMM_PART
            } else if (u == 8 && j == 0 && more) {
                store_tile<BM, AK>(An, tid, ra);
                store_tile<BN, BK>(Bn, tid, rb);
                if (more2) {
                    load_tile<BM, AK, true>(ao, cx.lda, cx.va, cx.rows_a, cx.K - k2, tid, ra);
                    load_tile<BN, BK, true>(bo, cx.ldb, cx.vb, cx.rows_b, cx.K - k2, tid, rb);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

template <bool AK, bool BK>
__global__ __launch_bounds__(256, 1) void k_gemm_big(GemmParams gp) {
    constexpr int BM = 256, BN = 256;
    constexpr int A_BYTES = tile_bytes<BM, AK>(), B_BYTES = tile_bytes<BN, BK>();
    extern __shared__ __attribute__((aligned(16))) char lds[];  // 2 x (A tile, B tile)
    const int tid = threadIdx.x, w = tid >> 6;
    int tm, tn;
    tile_of(gp, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = zero16();

    const bool interior = m0 + BM <= gp.M && n0 + BN <= gp.N;
    BigCtx cx;
    cx.a_org = AK ? gp.A + (int64_t)m0 * gp.lda : gp.A + m0;
    cx.b_org = BK ? gp.B + (int64_t)n0 * gp.ldb : gp.B + n0;
    cx.lda = gp.lda;
    cx.ldb = gp.ldb;
    cx.a_kstep = AK ? 1 : gp.lda;  // elements per unit of k
    cx.b_kstep = BK ? 1 : gp.ldb;
    cx.va = tile_voff<BM, AK>(gp.lda, tid);
    cx.vb = tile_voff<BN, BK>(gp.ldb, tid);
    cx.rows_a = gp.M - m0;
    cx.rows_b = gp.N - n0;
    cx.K = gp.K;
    cx.tid = tid;
    cx.lane = tid & 63;
    cx.wm = w >> 1;
    cx.wn = w & 1;
    const int lane = cx.lane, wm = cx.wm, wn = cx.wn;

    bf16x8 ra[8], rb[8];
    const bool steady = interior && 3 * BKK <= gp.K;  // at least one step of the straight-line loop
    if (steady) {
        // the same order of loads (A and B vector by vector) as inside the loop, so that the count of
        // loads still outstanding at the loop's first LDS write is the same on entry and on every repeat
#define GEMM_PRO(P, KOFF)                                                                                          \
    load_tile<BM, AK, false, P, P + 1>(cx.a_org + (int64_t)(KOFF) * cx.a_kstep, gp.lda, cx.va, 0, 0, tid, ra);      \
    load_tile<BN, BK, false, P, P + 1>(cx.b_org + (int64_t)(KOFF) * cx.b_kstep, gp.ldb, cx.vb, 0, 0, tid, rb);
        GEMM_PRO(0, 0) GEMM_PRO(1, 0) GEMM_PRO(2, 0) GEMM_PRO(3, 0) GEMM_PRO(4, 0) GEMM_PRO(5, 0) GEMM_PRO(6, 0) GEMM_PRO(7, 0)
        store_tile<BM, AK>(lds, tid, ra);
        store_tile<BN, BK>(lds + A_BYTES, tid, rb);
        GEMM_PRO(0, BKK) GEMM_PRO(1, BKK) GEMM_PRO(2, BKK) GEMM_PRO(3, BKK) GEMM_PRO(4, BKK) GEMM_PRO(5, BKK) GEMM_PRO(6, BKK) GEMM_PRO(7, BKK)
#undef GEMM_PRO
    } else {
        load_tile<BM, AK, true>(cx.a_org, gp.lda, cx.va, cx.rows_a, gp.K, tid, ra);
        load_tile<BN, BK, true>(cx.b_org, gp.ldb, cx.vb, cx.rows_b, gp.K, tid, rb);
        store_tile<BM, AK>(lds, tid, ra);
        store_tile<BN, BK>(lds + A_BYTES, tid, rb);
        if (BKK < gp.K) {
            load_tile<BM, AK, true>(cx.a_org + (int64_t)BKK * cx.a_kstep, gp.lda, cx.va, cx.rows_a, gp.K - BKK, tid, ra);
            load_tile<BN, BK, true>(cx.b_org + (int64_t)BKK * cx.b_kstep, gp.ldb, cx.vb, cx.rows_b, gp.K - BKK, tid, rb);
        }
    }
    __syncthreads();
    int cur = 0, k0 = 0;
    if (steady) {  // steps whose next two tiles are whole
        for (; k0 + 3 * BKK <= gp.K; k0 += BKK) {
            big_step<AK, BK, true>(cx, acc, ra, rb, lds + cur * (A_BYTES + B_BYTES), lds + (cur ^ 1) * (A_BYTES + B_BYTES), k0);
            cur ^= 1;
            __syncthreads();
        }
    }
    for (; k0 < gp.K; k0 += BKK) {
        big_step<AK, BK, false>(cx, acc, ra, rb, lds + cur * (A_BYTES + B_BYTES), lds + (cur ^ 1) * (A_BYTES + B_BYTES), k0);
        cur ^= 1;
        __syncthreads();
    }

    if (gp.c_f32) {  // weight gradients: K is the token count, the epilogue does not matter
        store_acc<4, 4>(gp, acc, m0 + wm * 128, n0 + wn * 128, lane, interior);
        return;
    }
    // bf16 result: through LDS (free now; every wave has left the K loop behind the last barrier), so that
    // a store instruction writes whole 256-byte row pieces instead of 32 scattered 16-byte ones.  Each wave
    // transposes its own 128 x 128 tile in a private patch: lane -> row lane % 32, four consecutive columns
    // per register group (see store_acc) on the way in, 16-byte vectors of a row on the way out.
    constexpr int EPITCH = 256 + 16;
    char* patch = lds + w * (128 * EPITCH);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x16& t = acc[i][j];
                bf16x4 v;
                v[0] = (__bf16)t[4 * q]; v[1] = (__bf16)t[4 * q + 1]; v[2] = (__bf16)t[4 * q + 2]; v[3] = (__bf16)t[4 * q + 3];
                *(bf16x4*)(patch + (i * 32 + (lane & 31)) * EPITCH + (j * 32 + q * 8 + (lane >> 5) * 4) * 2) = v;
            }
    const int col = n0 + wn * 128 + (lane & 15) * 8;
#pragma unroll 8
    for (int it = 0; it < 32; ++it) {
        const int r = it * 4 + (lane >> 4), row = m0 + wm * 128 + r;
        const bf16x8 v = *(const bf16x8*)(patch + r * EPITCH + (lane & 15) * 16);
        if (interior || (row < gp.M && col < gp.N)) *(bf16x8*)((__bf16*)gp.C + (int64_t)row * gp.ldc + col) = v;
    }
}

bool ok_ptr(const void* p) { return p && ((uintptr_t)p & 15) == 0; }

template <bool AK, bool BK, int WI, int WJ>
hipError_t launch_cfg(GemmParams gp, hipStream_t st) {
    constexpr int BM = 64 * WI, BN = 64 * WJ;
    constexpr int LDS = tile_bytes<BM, AK>() + tile_bytes<BN, BK>();
    static_assert(LDS <= 65536, "beyond the default dynamic LDS limit");
    gp.tiles_m = (gp.M + BM - 1) / BM;
    gp.tiles_n = (gp.N + BN - 1) / BN;
    hipLaunchKernelGGL((k_gemm<AK, BK, WI, WJ>), dim3(gp.tiles_m * gp.tiles_n), dim3(256), LDS, st, gp);
    return hipGetLastError();
}

template <bool AK, bool BK>
hipError_t launch_big(GemmParams gp, hipStream_t st) {
    constexpr int LDS = 2 * (tile_bytes<256, AK>() + tile_bytes<256, BK>());
    static bool raised[64];  // per device: the kernel uses more dynamic LDS than the default limit
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    if (!raised[dev]) {
        hipError_t e = hipFuncSetAttribute((const void*)k_gemm_big<AK, BK>, hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        if (e != hipSuccess) return e;
        raised[dev] = true;
    }
    gp.tiles_m = (gp.M + 255) / 256;
    gp.tiles_n = (gp.N + 255) / 256;
    hipLaunchKernelGGL((k_gemm_big<AK, BK>), dim3(gp.tiles_m * gp.tiles_n), dim3(256), LDS, st, gp);
    return hipGetLastError();
}

// 256 x 256 tiles (one workgroup per compute unit) unless there are too few of them to occupy half the
// machine; then 256 x 128 tiles, two workgroups per compute unit.  SSD_MAGC_GEMM_TILE=128 / 256 in the
// environment forces one of the two (a diagnostic).
template <bool AK, bool BK>
hipError_t launch_gemm(const GemmParams& gp, hipStream_t st) {
    static const int forced = [] {
        const char* e = getenv("SSD_MAGC_GEMM_TILE");
        return e ? atoi(e) : 0;
    }();
    bool big = true;
    if (forced == 128) big = false;
    if (forced != 128 && forced != 256) {
        big = (int64_t)((gp.M + 255) / 256) * ((gp.N + 255) / 256) >= 128;
    }
    return big ? launch_big<AK, BK>(gp, st) : launch_cfg<AK, BK, 4, 2>(gp, st);
}

// The two gradient products of a call are independent (both read dout; they write dx and dw).  One of them
// alone often leaves compute units idle -- a segment of 4096 rows gives the input gradient of the 2.7B block's
// input projection 160 tiles for 256 units -- so the weight gradient runs on a library stream of default
// priority, forked from and joined into the caller's stream with events, and the two fill the machine together.
struct Side {
    hipStream_t st = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    SideStream outer;  // the same stream with a pair of events of its own, for callers inside the library
    bool ok = false;
};
std::mutex g_side_mu;

// Created on first use on a device (or by ssd_init), under a lock; a partial failure releases what was created.
Side* side_for_current_device() {
    static Side sides[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(g_side_mu);
    Side& s = sides[dev];
    if (s.ok) return &s;
    Side q;
    bool good = hipStreamCreateWithFlags(&q.st, hipStreamNonBlocking) == hipSuccess;
    hipEvent_t* evs[] = {&q.fork, &q.join, &q.outer.fork, &q.outer.join};
    for (hipEvent_t* e : evs) good = good && hipEventCreateWithFlags(e, hipEventDisableTiming) == hipSuccess;
    if (!good) {
        for (hipEvent_t* e : evs)
            if (*e) (void)hipEventDestroy(*e);
        if (q.st) (void)hipStreamDestroy(q.st);
        return nullptr;
    }
    q.outer.st = q.st;
    q.ok = true;
    s = q;
    return &s;
}

}  // namespace

SideStream* side_stream() {
    if (serial_mode()) return nullptr;
    Side* s = side_for_current_device();
    return s ? &s->outer : nullptr;
}

namespace {

int check(int64_t rows, int32_t in_dim, int32_t out_dim, int64_t ldx, int64_t ldo) {
    if (rows < 0 || rows > 0x7fffffff || in_dim <= 0 || out_dim <= 0) return SSD_ERR_SHAPE;
    if ((in_dim | out_dim) & 7) return SSD_ERR_DIVISIBILITY;  // 16-byte vectors of bf16
    if ((ldx && (ldx < in_dim || (ldx & 7))) || (ldo && (ldo < out_dim || (ldo & 7)))) return SSD_ERR_SHAPE;
    const int64_t tiles = ((rows + 255) / 256) * (((int64_t)out_dim + 127) / 128);
    const int64_t tiles_w = (((int64_t)out_dim + 255) / 256) * (((int64_t)in_dim + 127) / 128);
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
    if (rows <= FEW_ROWS) {  // a token or a few: bound by reading w once, not by the matrix cores
        FewRowsJob j;
        memset(&j, 0, sizeof(j));
        j.rows = (int)rows;
        j.K = in_dim;
        j.N = out_dim;
        j.x = x;
        j.ldx = x_row_stride ? x_row_stride : in_dim;
        j.w = w;
        j.out = out;
        j.ldo = out_row_stride ? out_row_stride : out_dim;
        if (few_rows_supported(j)) return launch_linear_few_rows(j, (hipStream_t)hip_stream) == hipSuccess ? SSD_OK : SSD_ERR_LAUNCH;
    }
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
    // both products wanted: the weight gradient goes to the side stream (see Side)
    Side* side = dx && dw && !serial_mode() ? side_for_current_device() : nullptr;
    hipStream_t st_w = st;
    if (side) {
        if (hipEventRecord(side->fork, st) != hipSuccess || hipStreamWaitEvent(side->st, side->fork, 0) != hipSuccess) return SSD_ERR_LAUNCH;
        st_w = side->st;
    }
    int status = SSD_OK;
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
        if (launch_gemm<true, false>(gp, st) != hipSuccess) status = SSD_ERR_LAUNCH;
    }
    if (dw && status == SSD_OK) {  // dw[out, in] = dout^T x: contraction over the rows, the row index of both operands
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
        if (launch_gemm<false, false>(gp, st_w) != hipSuccess) status = SSD_ERR_LAUNCH;
    }
    // whatever reached the side stream ends before the caller's next work, also after a failed launch
    if (side && (hipEventRecord(side->join, side->st) != hipSuccess || hipStreamWaitEvent(st, side->join, 0) != hipSuccess)) return SSD_ERR_LAUNCH;
    return status;
}

// Calibration: what the matrix cores deliver when nothing else is in the way -- every wave issues
// `iters` rounds of sixteen independent 32 x 32 x 16 bf16 MFMAs on registers (no memory traffic), four
// waves per compute unit over the whole chip.  bench.py times it (--calibrate-mfma) to put the sustained
// clock of the matrix pipes next to the nominal peak.
namespace ssdk {
namespace {
__global__ __launch_bounds__(256, 1) void k_mfma_peak(int iters, float* sink) {
    f32x16 acc[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = zero16();
    bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        a[e] = (__bf16)(float)(threadIdx.x & 3);
        b[e] = (__bf16)(float)(e & 1);
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[i] = mfma(a, b, acc[i]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += acc[i][0];
    if (s == -1.f) sink[0] = s;  // never true: keeps the products alive
}
}  // namespace
}  // namespace ssdk

extern "C" int ssd_prof_mfma_peak(int32_t iters, int32_t workgroups, float* sink, void* hip_stream) {
    if (iters <= 0 || workgroups <= 0 || !sink) return SSD_ERR_ARG;
    hipLaunchKernelGGL(k_mfma_peak, dim3(workgroups), dim3(256), 0, (hipStream_t)hip_stream, iters, sink);
    return hipGetLastError() == hipSuccess ? SSD_OK : SSD_ERR_LAUNCH;
}

// Clock probe: one wave that sleeps until the constant 100 MHz counter has advanced by `ticks` and reports how
// many shader-clock cycles went by meanwhile.  Launched on a second stream next to a kernel under test it
// shows the clock that kernel really runs at (the power management lowers it under heavy load), which is what
// a cycle count or a fraction of the nominal peak has to be read against.
namespace ssdk {
namespace {
__global__ __launch_bounds__(64) void k_clock_probe(unsigned long long* out, unsigned long long ticks) {
    const unsigned long long w0 = wall_clock64(), c0 = clock64();
    unsigned long long w = w0;
    // an iteration takes about a microsecond (100 ticks): the time limit ends the loop long before the count does
    for (unsigned long long i = 0; i < ticks && w - w0 < ticks; ++i) {
        __builtin_amdgcn_s_sleep(32);
        w = wall_clock64();
    }
    if (threadIdx.x == 0) {
        out[0] = w - w0;
        out[1] = clock64() - c0;
    }
}
}  // namespace
}  // namespace ssdk

extern "C" int ssd_prof_clock_probe(uint64_t ticks, uint64_t* out, void* hip_stream) {
    if (!out || ticks == 0 || ticks > 100000000ull) return SSD_ERR_ARG;  // at most a second
    hipLaunchKernelGGL(k_clock_probe, dim3(1), dim3(64), 0, (hipStream_t)hip_stream, (unsigned long long*)out, (unsigned long long)ticks);
    return hipGetLastError() == hipSuccess ? SSD_OK : SSD_ERR_LAUNCH;
}
