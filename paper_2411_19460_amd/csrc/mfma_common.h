// Helpers shared by the matrix-core translation units (gfx950, wave64): vector types, the
// v_mfma_f32_32x32x16_bf16 wrapper, its accumulator layout, and operand-fragment loads from
// row-major global memory and from token-major LDS tiles (transpose load).
#pragma once
#include "ssd_internal.h"

namespace ssdk {
namespace mf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

constexpr int P_ = 64, N_ = 128, BLK = 64;
constexpr int XPITCH = 144;  // bytes per LDS row of a [token][64] bf16 tile (128 + 16 pad)
constexpr int BPITCH = 272;  // bytes per LDS row of a [token][128] bf16 tile (256 + 16 pad)
constexpr int NTH = 256;
constexpr float LOG2E = 1.4426950408889634f;

static __device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row (of the 32 x 32 result tile) held in accumulator register r of this lane; the column is lane % 32.
static __device__ __forceinline__ int acc_row(int r, int lane) { return (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3); }

// MFMA operand out of a row-major matrix (global memory): row = row0 + lane % 32, eight consecutive k
// starting at k0 + 8 * (lane / 32).
static __device__ __forceinline__ bf16x8 frag_rows(const bf16_t* base, int64_t row_stride, int row0, int k0, int lane) {
    return *(const bf16x8*)(base + (int64_t)(row0 + (lane & 31)) * row_stride + k0 + 8 * (lane >> 5));
}

// MFMA operand out of an LDS tile stored [k][m] (pitch in bytes): rows m0 .. m0+31 of the transpose,
// k0 .. k0+15.  Within a group of 16 lanes the transpose load returns to lane r the four k-rows
// addressed by lanes {r/4, r/4+4, r/4+8, r/4+12}... arranged so that, with the addresses below, lane r
// ends up with T[kb .. kb+3][mb + r].
static __device__ __forceinline__ bf16x8 frag_tr(const char* tile, int pitch, int k0, int m0, int lane) {
    const int g = lane >> 4, r = lane & 15;
    const char* p = tile + (k0 + 8 * (g >> 1) + (r >> 2)) * pitch + (m0 + 16 * (g & 1) + 4 * (r & 3)) * 2;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * pitch));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}

static __device__ __forceinline__ bf16x8 scale8(bf16x8 v, float s) {
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (__bf16)((float)v[e] * s);
    return o;
}

static __device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int r = 0; r < 16; ++r) z[r] = 0.f;
    return z;
}

}  // namespace mf
}  // namespace ssdk
