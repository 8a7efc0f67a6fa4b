// Gradients of B and C for one segment on the matrix cores (gfx950, bf16 in / fp32 accumulate).
// With M = the masked, decayed score matrix of a chunk (Sec. 3.1, Eq. 1 unrolled over the chunk),
//   dG[i][j] = sum over the heads of the group of  dt_j decay(i,j) (dY_i . x_j),   j <= i
//   dC_i     = sum_j dG[i][j] B_j  +  sum_heads exp(cum_i) dY_i^T Hprev
//   dB_j     = sum_i dG[i][j] C_i  +  sum_heads exp(T - cum_j) dt_j x_j^T dHnext
// Three kernels:
//   mk_dG       : one workgroup per (batch, chunk, group, head slice); the whole lower triangle of dG
//                 (36 tiles of 32 x 32 when Q = 256, four or five per wave) stays in accumulators while the workgroup walks
//                 the heads of its slice; dY and x tiles are staged in LDS once per head (next head
//                 prefetched in registers).  Writes one bf16 partial sum per slice and, per head, the
//                 chunk-local part of the gradient of cum: row sums minus column sums of
//                 E = (dY x^T) (.) M, each element entering both with the same value, so that their
//                 cancellation in the reverse cumulative sum is exact.
//   mk_dBC_part : the two head sums on the right, same organisation, accumulators [Q x 128] per
//                 (chunk, role, slice); the per-token weight is folded into the staged operand.
//   mk_dBC_final: sums the slices, contracts dG with B / dG^T with C, adds the head sums, rounds once.
// The decay of an off-diagonal tile is the product of a per-row factor, a per-column factor and a
// per-tile scalar, all <= 1 (32-token granularity); diagonal tiles evaluate exp() per element.
#include "ddt_finalize.h"
#include "dual_body.h"
#include "mfma_common.h"

namespace ssdk {
namespace {

using namespace mf;

constexpr int TP = 80;  // bytes per LDS row of a [32][32] bf16 tile (64 + 16 pad)

__device__ __forceinline__ bf16x8 lds_rows(const char* tile, int pitch, int row0, int k0, int lane) {
    return *(const bf16x8*)(tile + (row0 + (lane & 31)) * pitch + (k0 + 8 * (lane >> 5)) * 2);
}

// ---------------------------------------------------------------------------------------------
// Which 32 x 32 tiles (ti, tj <= ti) of the lower triangle each wave of mk_dG owns, as runs of tiles
// of one tile row (at most two runs per wave).  Q = 256: eight waves; waves v and v + 4 run on the same
// SIMD and together hold tile rows 7 - v and v (nine tiles per SIMD, at most five per wave).  Smaller
// chunks: wave v owns tile row v.  slot0(v) is the index of the wave's first tile in a flat numbering.
template <int Q>
struct DgMap {
    static constexpr int NT = Q / 32, NWV = NT, MAXT = NT, NSLOT = NT * (NT + 1) / 2;
    static __device__ __forceinline__ int count(int v) { return v + 1; }
    static __device__ __forceinline__ int ti(int v, int) { return v; }
    static __device__ __forceinline__ int tj(int, int k) { return k; }
    static __device__ __forceinline__ int slot0(int v) { return v * (v + 1) / 2; }
    // flat index of tile (ti, tj); the (wave, run) pairs that hold the row sums of tile row r (second: -1 = none)
    static __device__ __forceinline__ int slot_of(int ti, int tj) { return ti * (ti + 1) / 2 + tj; }
    static __device__ __forceinline__ int row_wave(int r, int) { return r; }
    static __device__ __forceinline__ int row_run(int, int which) { return which == 0 ? 0 : -1; }
};
template <>
struct DgMap<256> {
    static constexpr int NT = 8, NWV = 8, MAXT = 5, NSLOT = 36;
    static constexpr int CNT[8] = {5, 4, 4, 5, 4, 5, 5, 4};
    static constexpr int SLOT0[8] = {0, 5, 9, 13, 18, 22, 27, 32};
    static constexpr int TI[8][5] = {{7, 7, 7, 7, 0}, {6, 6, 6, 6, 0}, {5, 5, 5, 5, 0}, {4, 4, 4, 4, 4},
                                     {7, 7, 7, 7, 0}, {6, 6, 6, 1, 1}, {5, 5, 2, 2, 2}, {3, 3, 3, 3, 0}};
    static constexpr int TJ[8][5] = {{0, 1, 2, 3, 0}, {0, 1, 2, 3, 0}, {0, 1, 2, 3, 0}, {0, 1, 2, 3, 4},
                                     {4, 5, 6, 7, 0}, {4, 5, 6, 0, 1}, {4, 5, 0, 1, 2}, {0, 1, 2, 3, 0}};
    static __device__ __forceinline__ int count(int v) { return CNT[v]; }
    static __device__ __forceinline__ int ti(int v, int k) { return TI[v][k]; }
    static __device__ __forceinline__ int tj(int v, int k) { return TJ[v][k]; }
    static __device__ __forceinline__ int slot0(int v) { return SLOT0[v]; }
    // Tile row r: rows 5..7 are split over waves 7 - r (columns 0..3) and 11 - r (the rest), both as their
    // first run; row 4 is wave 3's only run, row 3 wave 7's; rows 0, 1, 2 are the second run of waves 0, 5, 6.
    static __device__ __forceinline__ int low_wave(int r) { return r == 0 ? 0 : 4 + r; }
    static __device__ __forceinline__ int row_wave(int r, int which) {
        return r >= 5 ? (which == 0 ? 7 - r : 11 - r) : (r == 4 ? 3 : (r == 3 ? 7 : low_wave(r)));
    }
    static __device__ __forceinline__ int row_run(int r, int which) {
        return r >= 5 ? 0 : (which == 1 ? -1 : (r >= 3 ? 0 : 1));
    }
    // flat index of tile (ti, tj): the position of the tile in its wave's list
    static __device__ __forceinline__ int slot_of(int ti, int tj) {
        const int v = ti >= 5 ? (tj < 4 ? 7 - ti : 11 - ti) : (ti == 4 ? 3 : (ti == 3 ? 7 : low_wave(ti)));
        const int k = ti >= 5 ? (tj < 4 ? tj : tj - 4) : (ti >= 3 ? tj : CNT[v] - (ti + 1) + tj);
        return SLOT0[v] + k;
    }
};

template <int Q>
struct DgLds {
    char dy[Q * XPITCH];
    char x[Q * XPITCH];
    float c2[Q];    // cum * log2(e)
    float dtl[Q];   // dt
    float rowf[Q];  // exp(cum_i - cum[start of i's 32-token tile - 1])
    float colf[Q];  // exp(cum[end of j's tile] - cum_j) * dt_j
    uint32_t gq[DgMap<Q>::NSLOT][8][64];         // scores G of every owned tile in accumulator layout, two bf16 per word
    float rsum[DgMap<Q>::NWV][2][32];            // per wave and tile-row run: row sums of E over the run's tiles
    float csum[DgMap<Q>::NSLOT][32];             // per tile: column sums of E
};

template <int Q>
struct DgPre {
    static constexpr int NV = Q * 8 / (64 * DgMap<Q>::NWV);  // 16-byte vectors of each tile per thread
    bf16x8 dy[NV], x[NV];
    float cum, dtf, cstart, cend;
};

template <int Q>
__device__ __forceinline__ void dg_load(DgPre<Q>& pr, const SegParams& sp, int b, int c, int h, int tid) {
    constexpr int NTHR = 64 * DgMap<Q>::NWV;
    const int64_t xt = (int64_t)sp.H * P_;
    const int64_t xrow = ((int64_t)c * Q * sp.H + h) * P_;
    const bf16_t* xg = (const bf16_t*)sp.x + (int64_t)b * sp.xs_b + xrow;
    const bf16_t* dyg = (const bf16_t*)sp.dy + (int64_t)b * sp.dys_b + xrow;
    // addresses = a wave-uniform base (scalar registers) + one 32-bit byte offset per lane
    const uint32_t rowbytes = (uint32_t)xt * 2, off = (uint32_t)(tid >> 3) * rowbytes + (uint32_t)(tid & 7) * 16;
#pragma unroll
    for (int k = 0; k < DgPre<Q>::NV; ++k) {
        const size_t step = (size_t)k * (NTHR / 8) * rowbytes;
        pr.dy[k] = *(const bf16x8*)((const char*)dyg + step + (size_t)off);
        pr.x[k] = *(const bf16x8*)((const char*)xg + step + (size_t)off);
    }
    if (tid < Q) {
        const int64_t cbase = (((int64_t)b * sp.H + h) * sp.nc + c) * Q;
        const float* cum = sp.cum + cbase;
        const int t0 = tid & ~31;
        pr.cum = cum[tid];
        pr.dtf = sp.dtf[cbase + tid];
        pr.cstart = cum[t0 > 0 ? t0 - 1 : 0];
        pr.cend = cum[t0 + 31];
    }
}

template <int Q>
__device__ __forceinline__ void dg_store(const DgPre<Q>& pr, DgLds<Q>& L, int tid) {
    constexpr int NTHR = 64 * DgMap<Q>::NWV;
#pragma unroll
    for (int k = 0; k < DgPre<Q>::NV; ++k) {
        const int v = tid + NTHR * k, row = v >> 3, seg = v & 7;
        *(bf16x8*)(L.dy + row * XPITCH + seg * 16) = pr.dy[k];
        *(bf16x8*)(L.x + row * XPITCH + seg * 16) = pr.x[k];
    }
    if (tid < Q) {
        L.c2[tid] = pr.cum * LOG2E;
        L.dtl[tid] = pr.dtf;
        L.rowf[tid] = __builtin_amdgcn_exp2f((pr.cum - (tid >= 32 ? pr.cstart : 0.f)) * LOG2E);
        L.colf[tid] = __builtin_amdgcn_exp2f((pr.cend - pr.cum) * LOG2E) * pr.dtf;
    }
}

// One tile (ti, tj) of one head: t = dY[ti] x[tj]^T; w = t (.) decay (.) dt is added to the dG
// accumulator; E = w (.) G are the element-wise products whose row sums minus column sums give the
// chunk-local part of the gradient of cum -- every E[i][j] enters both sums with the same rounded
// value.  Row sums go into rowacc (still per lane), column sums into csum[slot].
// ti and tj are wave-uniform run-time values (one code path for every wave).
template <int Q>
__device__ __forceinline__ void dg_tile(f32x16& acc, f32x16& rowacc, int ti, int tj, int slot, DgLds<Q>& L, int lane) {
    const char* pa = L.dy + (32 * ti + (lane & 31)) * XPITCH + 16 * (lane >> 5);
    const char* pb = L.x + (32 * tj + (lane & 31)) * XPITCH + 16 * (lane >> 5);
    f32x16 t = zero16();
    {   // all eight operand reads in flight before the first MFMA (one LDS latency per tile instead of four)
        bf16x8 fa[4], fb[4];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            fa[ks] = *(const bf16x8*)(pa + 32 * ks);
            fb[ks] = *(const bf16x8*)(pb + 32 * ks);
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) t = mfma(fa[ks], fb[ks], t);
    }
    const int j = 32 * tj + (lane & 31);
    const float* rowp = (ti != tj ? L.rowf : L.c2) + 32 * ti + 4 * (lane >> 5);
    if (ti != tj) {
        const float m = __builtin_amdgcn_exp2f(L.c2[32 * ti - 1] - L.c2[32 * tj + 31]);
        const float f = L.colf[j] * m;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 rf = *(const float4*)(rowp + 8 * q);
            t[4 * q + 0] *= rf.x * f;
            t[4 * q + 1] *= rf.y * f;
            t[4 * q + 2] *= rf.z * f;
            t[4 * q + 3] *= rf.w * f;
        }
    } else {
        const float cj = L.c2[j], dj = L.dtl[j];
        const int il = (lane & 31) - 4 * (lane >> 5);  // j - (first row of register group 0), tile-local
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 ci = *(const float4*)(rowp + 8 * q);
            const float cv[4] = {ci.x, ci.y, ci.z, ci.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float f = __builtin_amdgcn_exp2f(fminf(cv[e] - cj, 0.f)) * dj;
                t[4 * q + e] = (il <= 8 * q + e) ? t[4 * q + e] * f : 0.f;
            }
        }
    }
    float cs = 0.f;
#pragma unroll
    for (int r2 = 0; r2 < 8; ++r2) {
        const uint32_t g2 = L.gq[slot][r2][lane];
        const float g0 = __builtin_bit_cast(float, g2 << 16), g1 = __builtin_bit_cast(float, g2 & 0xffff0000u);
        acc[2 * r2] += t[2 * r2];
        acc[2 * r2 + 1] += t[2 * r2 + 1];
        const float e0 = t[2 * r2] * g0, e1 = t[2 * r2 + 1] * g1;
        rowacc[2 * r2] += e0;
        rowacc[2 * r2 + 1] += e1;
        cs += e0 + e1;
    }
    cs += __shfl_xor(cs, 32, 64);
    if (lane < 32) L.csum[slot][lane] = cs;
}

// Lane exchanges without LDS addressing: DPP within a row of 16 lanes, ds_swizzle across rows.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float xor16_f(float v) {  // lane ^ 16 (bit-mask swizzle: and 0x1F, or 0, xor 0x10)
    return __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));
}

// Sum of each of the 16 registers over the 32 lanes of a half wave.  First step across the two rows of 16 lanes
// (lane ^ 16, ds_swizzle): afterwards the lanes of the even row keep the sums of registers 0..7, those of the odd
// row the sums of registers 8..15.  Then a butterfly inside the row of 16 lanes with DPP adds (lane ^ 1, lane ^ 2,
// mirror of 8, mirror of 16): every lane of a row ends with the eight totals of its row's registers, and the first
// lane of each row writes them, dst[row] being the tile-local row of the register for the lane's half.
// (The two candidates of the first step are pinned in registers for a moment: a select between sums of two
// elements of one register vector would otherwise be rewritten as a dynamically indexed element, i.e. a chain of
// sixteen compare-and-select instructions.)
__device__ __forceinline__ void row_reduce_store(const f32x16& v, float* dst, int lane) {
    float a[8];
    const bool odd_row = lane & 16;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        float lo = v[r] + xor16_f(v[r]), hi = v[r + 8] + xor16_f(v[r + 8]);
        asm volatile("" : "+v"(lo), "+v"(hi));
        a[r] = odd_row ? hi : lo;
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        a[r] += dpp_f<0xB1>(a[r]);   // lane ^ 1
        a[r] += dpp_f<0x4E>(a[r]);   // lane ^ 2
        a[r] += dpp_f<0x141>(a[r]);  // the other quad of the same 8 lanes (row_half_mirror)
        a[r] += dpp_f<0x140>(a[r]);  // the other 8 lanes of the row (row_mirror)
    }
    if ((lane & 15) == 0) {  // registers R = 8 (odd row) + r: tile-local row 8 (R / 4) + 4 (lane / 32) + R % 4
        float* o = dst + (odd_row ? 16 : 0) + 4 * (lane >> 5);
        *(float4*)o = make_float4(a[0], a[1], a[2], a[3]);
        *(float4*)(o + 8) = make_float4(a[4], a[5], a[6], a[7]);
    }
}

// Where the partial sums of one tile row lie in LDS (wave-uniform; worked out once per workgroup).
template <int Q>
struct DgRowSrc {
    int cs[DgMap<Q>::NT];  // float offsets of the column sums of tiles (ti, row), ti = row .. NT-1, into csum; -1: none
    int rs0, rs1;          // float offsets of the (at most two) row-sum runs into rsum; rs1 = -1: none
};

template <int Q>
__device__ __forceinline__ DgRowSrc<Q> dg_row_src(int tt) {
    typedef DgMap<Q> M;
    DgRowSrc<Q> r;
#pragma unroll
    for (int ti = 0; ti < M::NT; ++ti) r.cs[ti] = ti >= tt ? M::slot_of(ti, tt) * 32 : -1;
    r.rs0 = (M::row_wave(tt, 0) * 2 + M::row_run(tt, 0)) * 32;
    r.rs1 = M::row_run(tt, 1) >= 0 ? (M::row_wave(tt, 1) * 2 + M::row_run(tt, 1)) * 32 : -1;
    return r;
}

// Chunk-local part of the gradient of cum for head h, from the E sums of the head just finished:
// gintra_i = sum_{j<=i} E[i][j] - sum_{i'>=i} E[i'][i], summed in a fixed order.  Wave w combines tile
// row w (32 tokens, one per lane of its first half); the reads are independent of each other.
template <int Q>
__device__ __forceinline__ void dg_emit_sums(const SegParams& sp, const DgLds<Q>& L, const DgRowSrc<Q>& src, int b, int c, int h,
                                             int w, int lane) {
    typedef DgMap<Q> M;
    static_assert(M::NWV == M::NT, "one wave per tile row");
    if (lane < 32) {
        const float* rsum = &L.rsum[0][0][0];
        const float* csum = &L.csum[0][0];
        float rs = rsum[src.rs0 + lane];
        if (src.rs1 >= 0) rs += rsum[src.rs1 + lane];
        float cs = 0.f;
#pragma unroll
        for (int ti = 0; ti < M::NT; ++ti)
            if (src.cs[ti] >= 0) cs += csum[src.cs[ti] + lane];
        sp.gintra[(((int64_t)b * sp.H + h) * sp.nc + c) * Q + 32 * w + lane] = rs - cs;
    }
}

template <int Q>
__device__ __forceinline__ void dg_body(const SegParams& sp, DgLds<Q>& L, int z, int nblk) {
    typedef DgMap<Q> M;
    constexpr int MAXT = M::MAXT;
    [[maybe_unused]] const int zlog = z;
    if ((nblk & 7) == 0) z = (z & 7) * (nblk >> 3) + (z >> 3);
    const int ns = sp.dg_split, slice = z % ns;
    z /= ns;
    const int g = z % sp.G, c = (z / sp.G) % sp.nc, b = z / (sp.G * sp.nc);
    const int hps = sp.hpg / ns, h0 = g * sp.hpg + slice * hps;
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int cnt = M::count(w), slot0 = M::slot0(w);
    // prologue: the scores of the owned tiles in accumulator layout
    {
        const bf16_t* Gd = (const bf16_t*)sp.Gm + (((int64_t)b * sp.nc + c) * sp.G + g) * (2 * Q * Q);
#pragma unroll
        for (int k = 0; k < MAXT; ++k)
            if (k < cnt) {
                const int ti = M::ti(w, k), tj = M::tj(w, k);
                const bf16_t* gp = Gd + (int64_t)(32 * ti + 4 * (lane >> 5)) * Q + 32 * tj + (lane & 31);
#pragma unroll
                for (int r2 = 0; r2 < 8; ++r2) {
                    const int r = 2 * r2, row = 8 * (r >> 2) + (r & 3);
                    const uint32_t lo = gp[(int64_t)row * Q].v, hi = gp[(int64_t)(row + 1) * Q].v;
                    L.gq[slot0 + k][r2][lane] = lo | (hi << 16);
                }
            }
    }
    const DgRowSrc<Q> rsrc = dg_row_src<Q>(w);
    f32x16 acc[MAXT];
#pragma unroll
    for (int k = 0; k < MAXT; ++k) acc[k] = zero16();
    DgPre<Q> pr;
    dg_load<Q>(pr, sp, b, c, h0, tid);
    for (int hh = 0; hh < hps; ++hh) {
        SSDK_STAMP(1, 0);
        __syncthreads();
        SSDK_STAMP(1, 1);
        if (hh > 0) dg_emit_sums<Q>(sp, L, rsrc, b, c, h0 + hh - 1, w, lane);
        dg_store<Q>(pr, L, tid);
        SSDK_STAMP(1, 2);
        __syncthreads();
        SSDK_STAMP(1, 3);
        if (hh + 1 < hps) dg_load<Q>(pr, sp, b, c, h0 + hh + 1, tid);
        SSDK_STAMP(1, 4);
        f32x16 rowacc = zero16();
        int prev = M::ti(w, 0), run = 0;
#pragma unroll
        for (int k = 0; k < MAXT; ++k)
            if (k < cnt) {
                int ti = M::ti(w, k), tj = M::tj(w, k);
                // keep the per-tile address arithmetic inside the head loop (hoisted out, it costs more
                // registers than it saves instructions)
                asm volatile("" : "+s"(ti), "+s"(tj));
                if (ti != prev) {  // a new tile row starts: flush the row sums of the finished run
                    row_reduce_store(rowacc, L.rsum[w][run], lane);
                    rowacc = zero16();
                    prev = ti;
                    ++run;
                }
                dg_tile<Q>(acc[k], rowacc, ti, tj, slot0 + k, L, lane);
            }
        row_reduce_store(rowacc, L.rsum[w][run], lane);
        SSDK_STAMP(1, 5);
    }
    __syncthreads();
    dg_emit_sums<Q>(sp, L, rsrc, b, c, h0 + hps - 1, w, lane);
    // partial sum of this slice, bf16, tile by tile: tile (ti, tj) is the 32 x 32 row-major block number ti NT + tj,
    // so that the pass that sums the slices reads whole cache lines (tiles above the diagonal are never touched)
    __bf16* out = (__bf16*)sp.dG + ((((int64_t)b * sp.nc + c) * sp.G + g) * ns + slice) * ((int64_t)Q * Q);
#pragma unroll
    for (int k = 0; k < MAXT; ++k)
        if (k < cnt) {
            __bf16* o = out + ((M::ti(w, k) * M::NT + M::tj(w, k)) * 32 + 4 * (lane >> 5)) * 32 + (lane & 31);
#pragma unroll
            for (int r = 0; r < 16; ++r) o[(8 * (r >> 2) + (r & 3)) * 32] = (__bf16)acc[k][r];
        }
}

template <int Q>
__global__ __launch_bounds__(64 * DgMap<Q>::NWV) void mk_dG(SegParams sp) {
    __shared__ __attribute__((aligned(16))) DgLds<Q> L;
    dg_body<Q>(sp, L, blockIdx.x, gridDim.x);
}

// ---------------------------------------------------------------------------------------------
// Head sums of dC (role 0) and dB (role 1):
//   role 0:  part[i][n] = sum_h exp(cum_h,i) (dY_h,i . Hprev_h[:, n])
//   role 1:  part[j][n] = sum_h exp(T_h - cum_h,j) dt_h,j (x_h,j . dHnext_h[:, n])
// and, per head, the two per-token dot products through the chunk-boundary states that enter the
// gradient of cum (same staged operands, contracted the other way round):
//   role 0:  gterm_i = exp(cum_i)          dY_i . (Hprev  C_i)
//   role 1:  sterm_j = exp(T - cum_j) dt_j x_j  . (dHnext B_j)
// Wave w owns RT row tiles (row group w / 2) and one half of the state columns (w % 2).
template <int Q>
struct PartCfg {
    static constexpr int RT = Q >= 256 ? 2 : 1;       // 32-row tiles per wave
    static constexpr int NWV = 2 * (Q / 32) / RT;     // waves
    static constexpr int NTHR = 64 * NWV;
    static constexpr int TV = Q * 8 / NTHR;           // 16-byte vectors of the token tile per thread
    static constexpr int SV = P_ * 16 / NTHR;         // of the state
};

template <int Q>
struct PartBuf {
    char tile[Q * XPITCH];  // weight * dY or weight * x, token-major
    char st[P_ * BPITCH];   // Hprev or dHnext, [p][n] bf16
};
// Two buffers: a head is contracted out of one while the next head is staged into the other (one barrier per head).
template <int Q>
struct PartLds {
    PartBuf<Q> b[2];
};

template <int Q>
struct PartPre {
    bf16x8 t[PartCfg<Q>::TV];
    float cv[PartCfg<Q>::TV], dv[PartCfg<Q>::TV];  // cum and dt of the vector's token
    float T;                                       // cum at the end of the chunk
    bf16x8 sv[PartCfg<Q>::SV];
};

template <int Q>
__device__ __forceinline__ void part_load(PartPre<Q>& pr, const SegParams& sp, int role, int b, int c, int h, int tid) {
    typedef PartCfg<Q> CF;
    const int64_t xt = (int64_t)sp.H * P_;
    const int64_t xrow = ((int64_t)c * Q * sp.H + h) * P_;
    const bf16_t* src = role == 0 ? (const bf16_t*)sp.dy + (int64_t)b * sp.dys_b + xrow
                                  : (const bf16_t*)sp.x + (int64_t)b * sp.xs_b + xrow;
    const int64_t cbase = (((int64_t)b * sp.H + h) * sp.nc + c) * Q;
    // loads only: no arithmetic on the loaded values here, so that nothing waits for them early
    pr.T = sp.cum[cbase + Q - 1];
    // addresses = a wave-uniform base (scalar registers) + one 32-bit byte offset per lane
    const uint32_t rowbytes = (uint32_t)xt * 2, off = (uint32_t)(tid >> 3) * rowbytes + (uint32_t)(tid & 7) * 16;
    const uint32_t roff = (uint32_t)(tid >> 3) * 4;
#pragma unroll
    for (int k = 0; k < CF::TV; ++k) {
        pr.t[k] = *(const bf16x8*)((const char*)src + (size_t)k * (CF::NTHR / 8) * rowbytes + (size_t)off);
        pr.cv[k] = *(const float*)((const char*)(sp.cum + cbase + k * (CF::NTHR / 8)) + (size_t)roff);
        pr.dv[k] = *(const float*)((const char*)(sp.dtf + cbase + k * (CF::NTHR / 8)) + (size_t)roff);
    }
    const bf16_t* S = (role == 0 ? sp.states_bf : sp.dstates_bf) + (((int64_t)b * sp.nc + c) * sp.H + h) * (P_ * N_);
    const uint32_t soff = (uint32_t)tid * 16;
    // the state tile has this one reader: streaming load (the token tile above is shared with the other passes)
#pragma unroll
    for (int k = 0; k < CF::SV; ++k) pr.sv[k] = __builtin_nontemporal_load((const bf16x8*)((const char*)S + (size_t)k * CF::NTHR * 16 + (size_t)soff));
}

template <int Q>
__device__ __forceinline__ void part_store(const PartPre<Q>& pr, PartBuf<Q>& L, int role, int tid) {
    typedef PartCfg<Q> CF;
#pragma unroll
    for (int k = 0; k < CF::TV; ++k) {
        const int v = tid + CF::NTHR * k, row = v >> 3, seg = v & 7;
        const float wgt = role == 0 ? __expf(pr.cv[k]) : __expf(pr.T - pr.cv[k]) * pr.dv[k];
        *(bf16x8*)(L.tile + row * XPITCH + seg * 16) = scale8(pr.t[k], wgt);
    }
#pragma unroll
    for (int k = 0; k < CF::SV; ++k) {
        const int v = tid + CF::NTHR * k, row = v >> 4, seg = v & 15;
        *(bf16x8*)(L.st + row * BPITCH + seg * 16) = pr.sv[k];
    }
}

template <int Q>
__device__ __forceinline__ void part_body(const SegParams& sp, PartLds<Q>& LL, int z, int nblk) {
    typedef PartCfg<Q> CF;
    constexpr int RT = CF::RT;
    [[maybe_unused]] const int zlog = z;
    if ((nblk & 7) == 0) z = (z & 7) * (nblk >> 3) + (z >> 3);
    const int ns = sp.part_split, slice = z % ns;
    z /= ns;
    const int role = z & 1;
    z >>= 1;
    const int g = z % sp.G, c = (z / sp.G) % sp.nc, b = z / (sp.G * sp.nc);
    const int hps = sp.hpg / ns, h0 = g * sp.hpg + slice * hps;
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), rg = w >> 1, nh = w & 1;
    f32x16 acc[RT][2];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) acc[rt][0] = acc[rt][1] = zero16();
    // wave w < Q/32 also owns token tile w of the per-token dot product through the state:
    // its rows of C (role 0) or B (role 1) stay in registers
    const bool has_dots = w < Q / 32;
    bf16x8 rf[N_ / 16];
    if (has_dots) {
        const int64_t bt = (int64_t)sp.G * N_;
        const bf16_t* rowop = (role ? (const bf16_t*)sp.Bm : (const bf16_t*)sp.Cm) + (int64_t)b * sp.bcs_b + ((int64_t)c * Q * sp.G + g) * N_;
#pragma unroll
        for (int ks = 0; ks < N_ / 16; ++ks) rf[ks] = frag_rows(rowop, bt, 32 * w, 16 * ks, lane);
    }
    // Order of the heads.  When this pass runs beside the other two head-walking passes with half as many slices
    // (twice the heads per workgroup, at about twice their pace per head), it alternates between the two half
    // slices -- heads 0, n/2, 1, n/2 + 1, ... -- so that it reads a head's x / dY tile while the two workgroups of
    // the other passes that walk those halves are on it too and the tile is still in the L2 slice they share.
    const bool alt = sp.part_alternate && (hps & 1) == 0;
    auto head_at = [&](int i) { return h0 + (alt ? (i >> 1) + (i & 1) * (hps >> 1) : i); };
    PartPre<Q> pr;
    part_load<Q>(pr, sp, role, b, c, head_at(0), tid);
    part_store<Q>(pr, LL.b[0], role, tid);
    if (hps > 1) part_load<Q>(pr, sp, role, b, c, head_at(1), tid);
    __syncthreads();
    // The two waves of a SIMD (w and w + NWV / 2) take the phases of a head in different orders -- the later one stages the
    // next head (vector ALU work) first, the other last -- so that one is on the vector ALUs while the other feeds the
    // matrix core.  The next head goes into the other LDS buffer, which nobody reads during this iteration.
    const bool stage_first = w >= CF::NWV / 2;
    for (int hh = 0; hh < hps; ++hh) {
        SSDK_STAMP(2, 0);
        const PartBuf<Q>& L = LL.b[hh & 1];
        if (stage_first) {
            if (hh + 1 < hps) part_store<Q>(pr, LL.b[(hh + 1) & 1], role, tid);
            if (hh + 2 < hps) part_load<Q>(pr, sp, role, b, c, head_at(hh + 2), tid);
        }
        {   // operand reads run one contraction step ahead of their MFMAs
            bf16x8 fb0 = frag_tr(L.st, BPITCH, 0, 64 * nh, lane), fb1 = frag_tr(L.st, BPITCH, 0, 64 * nh + 32, lane);
            bf16x8 fa[RT];
#pragma unroll
            for (int rt = 0; rt < RT; ++rt) fa[rt] = lds_rows(L.tile, XPITCH, 32 * (rg * RT + rt), 0, lane);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                bf16x8 nb0 = fb0, nb1 = fb1, na[RT];
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) na[rt] = fa[rt];
                if (ks + 1 < 4) {
                    nb0 = frag_tr(L.st, BPITCH, 16 * (ks + 1), 64 * nh, lane);
                    nb1 = frag_tr(L.st, BPITCH, 16 * (ks + 1), 64 * nh + 32, lane);
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) na[rt] = lds_rows(L.tile, XPITCH, 32 * (rg * RT + rt), 16 * (ks + 1), lane);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    acc[rt][0] = mfma(fa[rt], fb0, acc[rt][0]);
                    acc[rt][1] = mfma(fa[rt], fb1, acc[rt][1]);
                }
                fb0 = nb0;
                fb1 = nb1;
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) fa[rt] = na[rt];
            }
        }
        SSDK_STAMP(2, 1);
        if (has_dots) {
            // z^T[p][i] = (state C_i)[p] (role 1: (state B_j)[p]); the staged tile already carries the token's weight
            f32x16 z0 = zero16(), z1 = zero16();
            bf16x8 a0 = lds_rows(L.st, BPITCH, 0, 0, lane), a1 = lds_rows(L.st, BPITCH, 32, 0, lane);
#pragma unroll
            for (int ks = 0; ks < N_ / 16; ++ks) {
                bf16x8 n0 = a0, n1 = a1;
                if (ks + 1 < N_ / 16) {
                    n0 = lds_rows(L.st, BPITCH, 0, 16 * (ks + 1), lane);
                    n1 = lds_rows(L.st, BPITCH, 32, 16 * (ks + 1), lane);
                }
                __builtin_amdgcn_sched_barrier(0);
                z0 = mfma(a0, rf[ks], z0);
                z1 = mfma(a1, rf[ks], z1);
                a0 = n0;
                a1 = n1;
            }
            const int tok = 32 * w + (lane & 31);
            float sdot = 0.f;
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bf16x4 o = *(const bf16x4*)(L.tile + tok * XPITCH + (32 * pt + 8 * q + 4 * (lane >> 5)) * 2);
#pragma unroll
                    for (int e = 0; e < 4; ++e) sdot += (float)o[e] * (pt ? z1 : z0)[4 * q + e];
                }
            sdot += __shfl_xor(sdot, 32, 64);
            if (lane < 32) (role ? sp.sterm : sp.gterm)[(((int64_t)b * sp.H + head_at(hh)) * sp.nc + c) * Q + tok] = sdot;
        }
        SSDK_STAMP(2, 2);
        // the next head: its loads were issued a whole head ago; stage it into the other buffer, then ask for the one after
        if (!stage_first && hh + 1 < hps) part_store<Q>(pr, LL.b[(hh + 1) & 1], role, tid);
        SSDK_STAMP(2, 3);
        if (!stage_first && hh + 2 < hps) part_load<Q>(pr, sp, role, b, c, head_at(hh + 2), tid);
        SSDK_STAMP(2, 4);
        __syncthreads();
        SSDK_STAMP(2, 5);
    }
    float* part = sp.dbc_part + (((((int64_t)b * sp.nc + c) * sp.G + g) * ns + slice) * 2 + role) * ((int64_t)Q * N_);
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                part[(int64_t)(32 * (rg * RT + rt) + acc_row(r, lane)) * N_ + 64 * nh + 32 * nt + (lane & 31)] = acc[rt][nt][r];
}

template <int Q>
__global__ __launch_bounds__(PartCfg<Q>::NTHR) void mk_dBC_part(SegParams sp) {
    __shared__ __attribute__((aligned(16))) PartLds<Q> L;
    part_body<Q>(sp, L, blockIdx.x, gridDim.x);
}

// ---------------------------------------------------------------------------------------------
// The three head-walking passes of the backward sweep that follow the state scans -- dx (reverse dual
// form), dG and the dB / dC head sums -- as one launch: they read the same dY and x tiles, and
// workgroups that run side by side find in cache what their neighbours fetched.  Needs the three
// passes to use the same workgroup size (Q = 256).  With equal workgroup counts, a multiple of 8, the
// passes alternate in groups of 8 consecutive workgroup ids, so that the workgroups of the three
// passes that work on one chunk land on the same XCD (ids are dealt round-robin over the 8 XCDs) and are
// dispatched together.
template <int Q>
union TrioLds {
    dualk::DualLds<Q> dual;
    DgLds<Q> dg;
    PartLds<Q> part;
};

template <int Q>
__global__ __launch_bounds__(512) void mk_bwd_trio(SegParams sp, int n_dual, int n_dg, int n_part) {
    static_assert(dualk::DualCfg<Q>::NTHR == 512 && 64 * DgMap<Q>::NWV == 512 && PartCfg<Q>::NTHR == 512, "one workgroup size");
    __shared__ __attribute__((aligned(16))) TrioLds<Q> L;
    int z = blockIdx.x, pass;
    if (n_dual == n_dg && n_dg == n_part && (n_dual & 7) == 0) {
        pass = (z >> 3) % 3;
        z = ((z >> 3) / 3) * 8 + (z & 7);
    } else {
        pass = z < n_dual ? 0 : (z < n_dual + n_dg ? 1 : 2);
        z -= pass == 0 ? 0 : (pass == 1 ? n_dual : n_dual + n_dg);
    }
    if (pass == 0)
        dualk::dual_body<Q, 2>(sp, L.dual, z, n_dual);
    else if (pass == 1)
        dg_body<Q>(sp, L.dg, z, n_dg);
    else
        part_body<Q>(sp, L.part, z, n_part);
}

// ---------------------------------------------------------------------------------------------
// dC rows (role 0) / dB rows (role 1) of one 32-token tile R of one (chunk, group):
//   role 0: out[i][n] = sum_{tj <= R} dG[R-tile rows][tj-tile cols] B[tj-tile rows][n] + head sums
//   role 1: out[j][n] = sum_{ti >= R} dG[ti-tile rows][R-tile cols]^T C[ti-tile rows][n] + head sums
// The waves share out the halves of the needed dG tiles and sum their slices into LDS (bf16); then every wave
// owns 32 state columns of the contraction.
template <int Q>
struct FinLds {
    char tiles[Q / 32][32 * TP];
    char slab[64 * BPITCH];  // rows of B / C along the contraction, 64 at a time
};

// Small footprint on purpose (37 KB of LDS): the kernel only streams partial sums.
template <int Q>
__device__ __forceinline__ void final_body(const SegParams& sp, FinLds<Q>& L, int z) {
    constexpr int NT = Q / 32;
    const int R = z % NT;
    z /= NT;
    const int role = z & 1;
    z >>= 1;
    const int g = z % sp.G, c = (z / sp.G) % sp.nc, b = z / (sp.G * sp.nc);
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int64_t bcg = ((int64_t)b * sp.nc + c) * sp.G + g;
    const int64_t bt = (int64_t)sp.G * N_;
    const int64_t bbase = (int64_t)b * sp.bcs_b + ((int64_t)c * Q * sp.G + g) * N_;
    const bf16_t* rhs = (role == 0 ? (const bf16_t*)sp.Bm : (const bf16_t*)sp.Cm) + bbase;
    const int k_lo = role == 0 ? 0 : R, k_hi = role == 0 ? R : NT - 1;  // tiles along the contraction
    const int ns = sp.dg_split;
    const bf16_t* dg = (const bf16_t*)sp.dG + bcg * ns * ((int64_t)Q * Q);
    const int ps = sp.part_split;
    const float* part = sp.dbc_part + (bcg * ps * 2 + role) * ((int64_t)Q * N_);
    f32x16 acc = zero16();
    // Everything below is a chain of memory round trips on a workgroup that has the compute unit almost to itself,
    // so each step asks for what the next one needs before it works: the first rows of B / C before the tile sums,
    // the head sums before the contraction.
    const int p_lo = k_lo >> 1, p_hi = k_hi >> 1;  // pairs of tiles along the contraction
    constexpr int SV = 64 * 16 / NTH;              // 16-byte pieces of a 64-row slab per thread
    bf16x8 sv[SV];
#pragma unroll
    for (int k = 0; k < SV; ++k) {
        const int v = tid + NTH * k, row = v >> 4, seg = v & 15;
        sv[k] = *(const bf16x8*)(rhs + (int64_t)(64 * p_lo + row) * bt + seg * 8);
    }
    // sum the slices of the needed dG tiles: items (tile, half of its rows), two items and eight slices of each in
    // flight per wave; one 16-byte piece per lane and item
    const int nitems = 2 * (k_hi - k_lo + 1);
    for (int it = w; it < nitems; it += 2 * (NTH / 64)) {
        const bf16_t* src[2];
        char* dst[2];
        const bool two = it + NTH / 64 < nitems;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int item = q == 0 || two ? it + q * (NTH / 64) : it;
            const int tk = k_lo + (item >> 1), half = item & 1;
            const int ti = role == 0 ? R : tk, tj = role == 0 ? tk : R;
            const int v = lane + 64 * half, row = v >> 2, seg = v & 3;
            src[q] = dg + ((ti * NT + tj) * 32 + row) * 32 + seg * 8;  // tile-major, see dg_body
            dst[q] = L.tiles[tk] + row * TP + seg * 16;
        }
        float sm[2][8];
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int e = 0; e < 8; ++e) sm[q][e] = 0.f;
        int sl = 0;
        for (; sl + 8 <= ns; sl += 8) {  // summation order stays slice 0, 1, 2, ...
            bf16x8 vv[2][8];
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int u = 0; u < 8; ++u) vv[q][u] = *(const bf16x8*)(src[q] + (int64_t)(sl + u) * Q * Q);
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int u = 0; u < 8; ++u)
#pragma unroll
                    for (int e = 0; e < 8; ++e) sm[q][e] += (float)vv[q][u][e];
        }
        for (; sl < ns; ++sl) {
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const bf16x8 vv = *(const bf16x8*)(src[q] + (int64_t)sl * Q * Q);
#pragma unroll
                for (int e = 0; e < 8; ++e) sm[q][e] += (float)vv[e];
            }
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (__bf16)sm[q][e];
            if (q == 0 || two) *(bf16x8*)dst[q] = o;
        }
    }
    // the head sums of this workgroup's rows, up to four slices asked for now and added after the contraction
    constexpr int PSR = 4;
    float pv[PSR][16];
#pragma unroll
    for (int s4 = 0; s4 < PSR; ++s4)
#pragma unroll
        for (int r = 0; r < 16; ++r)
            pv[s4][r] = s4 < ps ? part[(int64_t)s4 * 2 * Q * N_ + (int64_t)(32 * R + acc_row(r, lane)) * N_ + 32 * w + (lane & 31)] : 0.f;
    // contraction with the rows of B (role 0) / C (role 1), 64 rows (two tiles) per step
    for (int pr = p_lo; pr <= p_hi; ++pr) {
        if (pr > p_lo) __syncthreads();  // every wave is done with the previous rows
#pragma unroll
        for (int k = 0; k < SV; ++k) {
            const int v = tid + NTH * k, row = v >> 4, seg = v & 15;
            *(bf16x8*)(L.slab + row * BPITCH + seg * 16) = sv[k];
        }
        if (pr < p_hi) {
#pragma unroll
            for (int k = 0; k < SV; ++k) {
                const int v = tid + NTH * k, row = v >> 4, seg = v & 15;
                sv[k] = *(const bf16x8*)(rhs + (int64_t)(64 * (pr + 1) + row) * bt + seg * 8);
            }
        }
        __syncthreads();  // the rows (and, the first time, the summed tiles) are in place
        const char* slab = L.slab;
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
            const int tk = 2 * pr + t2;
            if (tk < k_lo || tk > k_hi) continue;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                // role 0: tile is [i][j], operand rows i, contraction j: plain rows.
                // role 1: tile is [i][j], operand rows j, contraction i: transpose load.
                const bf16x8 fa = role == 0 ? lds_rows(L.tiles[tk], TP, 0, 16 * ks, lane) : frag_tr(L.tiles[tk], TP, 16 * ks, 0, lane);
                const bf16x8 fb = frag_tr(slab, BPITCH, 32 * t2 + 16 * ks, 32 * w, lane);
                acc = mfma(fa, fb, acc);
            }
        }
    }
    bf16_t* out = (role == 0 ? (bf16_t*)sp.dC : (bf16_t*)sp.dB) + bbase;
#pragma unroll
    for (int s4 = 0; s4 < PSR; ++s4)  // slice order 0, 1, 2, ...
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] += pv[s4][r];
    for (int s = PSR; s < ps; ++s) {
        float pw[16];
#pragma unroll
        for (int r = 0; r < 16; ++r)
            pw[r] = part[(int64_t)s * 2 * Q * N_ + (int64_t)(32 * R + acc_row(r, lane)) * N_ + 32 * w + (lane & 31)];
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] += pw[r];
    }
#pragma unroll
    for (int r = 0; r < 16; ++r)
        out[(int64_t)(32 * R + acc_row(r, lane)) * bt + 32 * w + (lane & 31)] = float_to_bf16(acc[r]);
}

template <int Q>
__global__ __launch_bounds__(NTH) void mk_dBC_final(SegParams sp) {
    __shared__ __attribute__((aligned(16))) FinLds<Q> L;
    final_body<Q>(sp, L, blockIdx.x);
}

// The two steps behind the head-walking passes -- dB / dC from the partial sums, and ddt with the chunk's dA / dD
// partial sums from the per-token scalars -- as one launch (chunk 256: both run 256 threads per workgroup): the
// first n_final workgroups do the former, the rest one (chunk, head) of the latter each.
union FinDdtLds {
    FinLds<256> fin;
    float s[2][256];
};

__global__ __launch_bounds__(NTH) void mk_final_ddt(SegParams sp, int n_final) {
    __shared__ __attribute__((aligned(16))) FinDdtLds L;
    int z = blockIdx.x;
    if (z < n_final) {
        final_body<256>(sp, L.fin, z);
    } else {
        z -= n_final;
        const int c = z % sp.nc;
        z /= sp.nc;
        ddt_finalize_body(sp, L.s[0], L.s[1], c, z % sp.H, z / sp.H,
                          [&](int64_t idx, float v) { ((bf16_t*)sp.ddt)[idx] = float_to_bf16(v); });
    }
}

template <int Q>
hipError_t grad_bc_q(const SegParams& sp0, bool with_dual, hipStream_t st) {
    SegParams sp = sp0;
    const int n_dg = sp.Bt * sp.nc * sp.G * sp.dg_split, n_part = sp.Bt * sp.nc * sp.G * 2 * sp.part_split;
    if (with_dual) {
        if (Q != 256) return hipErrorInvalidValue;
        sp.dual_split = pick_split(sp.hpg, (int64_t)sp.Bt * sp.nc * sp.G, sp.wg_target);
        const int n_dual = sp.Bt * sp.nc * sp.G * sp.dual_split;
        sp.part_alternate = sp.dual_split == 2 * sp.part_split && sp.dg_split == sp.dual_split;
        SSDK_LAUNCH(K_MFMA_BWD_TRIO, st, mk_bwd_trio<256>, dim3(n_dual + n_dg + n_part), dim3(512), sp, n_dual, n_dg, n_part);
    } else {
        SSDK_LAUNCH(K_MFMA_DG, st, mk_dG<Q>, dim3(n_dg), dim3(64 * DgMap<Q>::NWV), sp);
        SSDK_LAUNCH(K_MFMA_DBC, st, mk_dBC_part<Q>, dim3(n_part), dim3(PartCfg<Q>::NTHR), sp);
    }
    const int n_final = sp.Bt * sp.nc * sp.G * 2 * (Q / 32);
    if (Q == 256 && (sp.flags & SSD_INTERNAL_SPLIT_GTERM))  // the caller has asked for the scalar step in the same launch
        SSDK_LAUNCH(K_MFMA_FINAL_DDT, st, mk_final_ddt, dim3(n_final + sp.nc * sp.H * sp.Bt), dim3(NTH), sp, n_final);
    else
        SSDK_LAUNCH(K_MFMA_DBC_FINAL, st, mk_dBC_final<Q>, dim3(n_final), dim3(NTH), sp);
    return hipSuccess;
}

}  // namespace

hipError_t mfma_launch_grad_bc(const SegParams& sp, bool with_dual, hipStream_t st) {
    switch (sp.Q) {
        case 64: return grad_bc_q<64>(sp, with_dual, st);
        case 128: return grad_bc_q<128>(sp, with_dual, st);
        case 256: return grad_bc_q<256>(sp, with_dual, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ssdk
