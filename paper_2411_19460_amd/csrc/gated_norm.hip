// Gated RMS normalisation of the Mamba-2 block (between the SSD output y and the output projection),
// forward and backward:
//     g = y * silu(z);    out[t,c] = g[t,c] / sqrt(mean_{group(c)} g[t,.]^2 + eps) * w[c]
// y and z are the two activations a grid cell of MA-GC keeps per token (App. C, Tab. 7: C_grid counts the
// input projection's output, which holds z, plus the d_inner values of y), so the backward pass recomputes
// everything else from them.
// HBM-bound.  A workgroup (long segments) or a wave (short ones) owns one (token, group) segment at a
// time: its values stay in registers in storage precision as 16-byte vectors, the two sums over the
// segment are wave reductions (plus one LDS exchange per row between waves), the results leave as 16-byte
// vectors: every input is read once, every output written once.  A thread sees the same channels in
// every row, so the weight and the running weight-gradient sums are registers; the partial sums of all
// workgroups are finished by a fixed-order reduction kernel.
#include <string.h>

#include <initializer_list>

#include "ssd_internal.h"

namespace ssdk {
namespace {

constexpr int ROWS_PER_WG = 64;  // rows per tile in the backward kernels: granularity of the dw partial sums
constexpr int ROWS_PER_WG_FWD = 16;
constexpr int MAX_VPL = 8;       // most 16-byte vectors per thread the register-resident kernels are built for

struct NormParams {
    const void* y;
    const void* z;
    const void* dout;
    const float* w;
    void* out;
    void* dy;
    void* dz;
    float* part;  // [ntiles * slots][C] partial sums of dw
    int64_t T, y_rs, z_rs;  // rows; elements between rows of y / dy and of z / dz (out, dout are dense)
    int C, G, gs, ntiles, tile_rows;
    float eps;
};

typedef __bf16 b8 __attribute__((ext_vector_type(8)));

template <typename T>
struct Pk;
template <>
struct Pk<bf16_t> {
    static constexpr int V = 8;
    typedef b8 pack;
    static __device__ __forceinline__ pack ld(const void* p, int64_t i) { return *(const pack*)((const __bf16*)p + i); }
    static __device__ __forceinline__ void st(void* p, int64_t i, pack v) { *(pack*)((__bf16*)p + i) = v; }
    static __device__ __forceinline__ float get(const pack& v, int e) { return (float)v[e]; }
    static __device__ __forceinline__ void set(pack& v, int e, float f) { v[e] = (__bf16)f; }
    static __device__ __forceinline__ float ld1(const void* p, int64_t i) { return bf16_to_float(((const bf16_t*)p)[i]); }
    static __device__ __forceinline__ void st1(void* p, int64_t i, float f) { ((bf16_t*)p)[i] = float_to_bf16(f); }
};
template <>
struct Pk<float> {
    static constexpr int V = 4;
    typedef float4 pack;
    static __device__ __forceinline__ pack ld(const void* p, int64_t i) { return *(const pack*)((const float*)p + i); }
    static __device__ __forceinline__ void st(void* p, int64_t i, pack v) { *(pack*)((float*)p + i) = v; }
    static __device__ __forceinline__ float get(const pack& v, int e) { return e == 0 ? v.x : e == 1 ? v.y : e == 2 ? v.z : v.w; }
    static __device__ __forceinline__ void set(pack& v, int e, float f) {
        if (e == 0) v.x = f;
        else if (e == 1) v.y = f;
        else if (e == 2) v.z = f;
        else v.w = f;
    }
    static __device__ __forceinline__ float ld1(const void* p, int64_t i) { return ((const float*)p)[i]; }
    static __device__ __forceinline__ void st1(void* p, int64_t i, float f) { ((float*)p)[i] = f; }
};

// through the hardware reciprocal (1 ulp): an IEEE division costs ten instructions more per element, which
// shows in kernels this close to the VALU limit
__device__ __forceinline__ float sigmoidf(float z) { return __builtin_amdgcn_rcpf(1.f + __expf(-z)); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Register-resident kernel: grid (workgroups, G), 256 threads.  A (row, group) segment is shared by WPS waves
// (4: the whole workgroup, for long segments; 1: one wave each, for short ones); the workgroup's 4 / WPS
// slots walk the 64 rows of each of its tiles.  A thread owns the same channels in every row (vector
// i * 64 * WPS + its index within the slot), so the weight and the weight-gradient sums stay in its registers.
template <typename T, int VPL, int WPS, bool BWD, bool GATED>
__global__ __launch_bounds__(256) void k_gated_norm(NormParams np) {
    constexpr int V = Pk<T>::V;
    constexpr int NSLOT = 4 / WPS;
    typedef typename Pk<T>::pack pack;
    __shared__ float red[2][4][2];  // [row parity][wave][sum]: partial sums of the waves that share a segment
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int slot = wv / WPS, lid = (wv % WPS) * 64 + lane;
    const int c_base = blockIdx.y * np.gs;
    const int nvec = np.gs / V;
    float wr[VPL][V], acc[BWD ? VPL : 1][V];
#pragma unroll
    for (int i = 0; i < VPL; ++i) {
        const int v = i * 64 * WPS + lid;
#pragma unroll
        for (int e = 0; e < V; ++e) {
            wr[i][e] = v < nvec ? np.w[c_base + v * V + e] : 0.f;
            if (BWD) acc[i][e] = 0.f;
        }
    }
    const float inv_n = 1.f / (float)np.gs;
    int parity = 0;
    // a workgroup walks tiles blockIdx.x, blockIdx.x + gridDim.x, ... of np.tile_rows rows; slot `slot` takes
    // every NSLOT-th row of each
    const int tr = np.tile_rows;
    const int64_t nrows_wg = ((int64_t)np.ntiles - blockIdx.x + gridDim.x - 1) / gridDim.x * tr;
    auto row_of = [&](int64_t q) { return ((int64_t)blockIdx.x + (q / tr) * gridDim.x) * tr + q % tr; };
    auto load_row = [&](int64_t r, pack (&yv)[VPL], pack (&zv)[VPL], pack (&dv)[BWD ? VPL : 1]) {
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int v = i * 64 * WPS + lid;
            if (v < nvec) {
                yv[i] = Pk<T>::ld(np.y, r * np.y_rs + c_base + v * V);
                if (GATED) zv[i] = Pk<T>::ld(np.z, r * np.z_rs + c_base + v * V);
                if (BWD) dv[i] = Pk<T>::ld(np.dout, r * (int64_t)np.C + c_base + v * V);
            }
        }
    };
    // forward: the next row is fetched while this one is worked on (the backward kernel has no registers to
    // spare for that and more bytes in flight per row anyway)
    constexpr bool PREFETCH = !BWD;
    pack ny[VPL], nz[VPL], nd[BWD ? VPL : 1];
    if (PREFETCH && slot < nrows_wg && row_of(slot) < np.T) load_row(row_of(slot), ny, nz, nd);
    for (int64_t q = slot; q < nrows_wg; q += NSLOT, parity ^= 1) {
        const int64_t r = row_of(q);
        if (r >= np.T) break;  // only the last tile is short; uniform over the waves that share a segment
        pack yv[VPL], zv[VPL], dv[BWD ? VPL : 1];
        if (PREFETCH) {
#pragma unroll
            for (int i = 0; i < VPL; ++i) {
                yv[i] = ny[i];
                if (GATED) zv[i] = nz[i];
            }
            if (q + NSLOT < nrows_wg && row_of(q + NSLOT) < np.T) load_row(row_of(q + NSLOT), ny, nz, nd);
        } else {
            load_row(r, yv, zv, dv);
        }
        // first pass: the gated values (kept for the second pass: the sigmoid is the expensive part), the
        // sum of g^2 and (backward) of dout * w * g over the segment
        float gv[VPL][V], sv[BWD ? VPL : 1][V];
        float s1 = 0.f, s2 = 0.f;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            if (i * 64 * WPS + lid < nvec) {
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const float zz = GATED ? Pk<T>::get(zv[i], e) : 0.f;
                    const float sg = GATED ? sigmoidf(zz) : 1.f;
                    const float g = GATED ? Pk<T>::get(yv[i], e) * zz * sg : Pk<T>::get(yv[i], e);  // no gate: plain RMS norm
                    gv[i][e] = g;
                    if (BWD) sv[i][e] = sg;
                    s1 = fmaf(g, g, s1);
                    if (BWD) s2 = fmaf(Pk<T>::get(dv[i], e) * wr[i][e], g, s2);
                }
            }
        }
        s1 = wave_sum(s1);
        if (BWD) s2 = wave_sum(s2);
        if (WPS > 1) {  // one barrier per row: the two parities keep a fast wave out of the slots still being read
            if (lane == 0) {
                red[parity][wv][0] = s1;
                red[parity][wv][1] = s2;
            }
            __syncthreads();
            s1 = (red[parity][0][0] + red[parity][1][0]) + (red[parity][2][0] + red[parity][3][0]);
            s2 = (red[parity][0][1] + red[parity][1][1]) + (red[parity][2][1] + red[parity][3][1]);
        }
        const float rstd = rsqrtf(s1 * inv_n + np.eps);
        const float m = BWD ? s2 * inv_n * rstd : 0.f;  // mean of dghat * ghat
        // second pass: the outputs
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int v = i * 64 * WPS + lid;
            if (v < nvec) {
                pack o1, o2;
#pragma unroll
                for (int e = 0; e < V; ++e) {
                    const float ghat = gv[i][e] * rstd;
                    if (!BWD) {
                        Pk<T>::set(o1, e, ghat * wr[i][e]);
                    } else {
                        const float d = Pk<T>::get(dv[i], e);
                        const float dg = rstd * (d * wr[i][e] - ghat * m);
                        if (GATED) {
                            const float zz = Pk<T>::get(zv[i], e), yy = Pk<T>::get(yv[i], e), sg = sv[i][e];
                            Pk<T>::set(o1, e, dg * zz * sg);                              // dy
                            Pk<T>::set(o2, e, dg * yy * sg * (1.f + zz * (1.f - sg)));    // dz
                        } else {
                            Pk<T>::set(o1, e, dg);
                        }
                        acc[i][e] = fmaf(d, ghat, acc[i][e]);
                    }
                }
                if (!BWD) {
                    Pk<T>::st(np.out, r * (int64_t)np.C + c_base + v * V, o1);
                } else {
                    Pk<T>::st(np.dy, r * np.y_rs + c_base + v * V, o1);
                    if (GATED) Pk<T>::st(np.dz, r * np.z_rs + c_base + v * V, o2);
                }
            }
        }
    }
    if (BWD) {  // dw of this slot's rows (zeros if it had none): partial row (workgroup, slot)
        float* part = np.part + ((int64_t)blockIdx.x * NSLOT + slot) * np.C + c_base;
#pragma unroll
        for (int i = 0; i < VPL; ++i) {
            const int v = i * 64 * WPS + lid;
            if (v < nvec) {
#pragma unroll
                for (int e = 0; e < V; ++e) part[v * V + e] = acc[i][e];
            }
        }
    }
}

// Any group size, any alignment: one wave per (row, group), three passes over the segment through the
// caches, element by element.  Same arithmetic in the same order per element; the sums over the segment
// are taken in a different order than in the kernel above.
template <typename T, bool BWD, bool GATED>
__global__ __launch_bounds__(256) void k_gated_norm_any(NormParams np) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int grp = blockIdx.y;
    const int c_base = grp * np.gs;
    const float inv_n = 1.f / (float)np.gs;
    const int64_t r0 = (int64_t)blockIdx.x * ROWS_PER_WG;
    // partial sums of dw: slot (tile * 4 + wave) is this wave's alone, written on its first row, added to after
    float* part = BWD ? np.part + ((int64_t)blockIdx.x * 4 + wv) * np.C + c_base : nullptr;
    bool first = true;
    for (int rr = wv; rr < ROWS_PER_WG; rr += 4) {
        const int64_t r = r0 + rr;
        if (r >= np.T) break;
        float s1 = 0.f, s2 = 0.f;
        for (int c = lane; c < np.gs; c += 64) {
            const float zz = GATED ? Pk<T>::ld1(np.z, r * np.z_rs + c_base + c) : 0.f;
            const float g = Pk<T>::ld1(np.y, r * np.y_rs + c_base + c) * (GATED ? zz * sigmoidf(zz) : 1.f);
            s1 = fmaf(g, g, s1);
            if (BWD) s2 = fmaf(Pk<T>::ld1(np.dout, r * (int64_t)np.C + c_base + c) * np.w[c_base + c], g, s2);
        }
        s1 = wave_sum(s1);
        const float rstd = rsqrtf(s1 * inv_n + np.eps);
        float m = 0.f;
        if (BWD) m = wave_sum(s2) * inv_n * rstd;
        for (int c = lane; c < np.gs; c += 64) {
            const float zz = GATED ? Pk<T>::ld1(np.z, r * np.z_rs + c_base + c) : 0.f, yy = Pk<T>::ld1(np.y, r * np.y_rs + c_base + c);
            const float sg = GATED ? sigmoidf(zz) : 1.f;
            const float ghat = (GATED ? yy * zz * sg : yy) * rstd;
            const float wc = np.w[c_base + c];
            if (!BWD) {
                Pk<T>::st1(np.out, r * (int64_t)np.C + c_base + c, ghat * wc);
            } else {
                const float d = Pk<T>::ld1(np.dout, r * (int64_t)np.C + c_base + c);
                const float dg = rstd * (d * wc - ghat * m);
                Pk<T>::st1(np.dy, r * np.y_rs + c_base + c, GATED ? dg * zz * sg : dg);
                if (GATED) Pk<T>::st1(np.dz, r * np.z_rs + c_base + c, dg * yy * sg * (1.f + zz * (1.f - sg)));
                part[c] = first ? d * ghat : fmaf(d, ghat, part[c]);
            }
        }
        first = false;
    }
    if (BWD && first) {  // a wave without rows still owns its slot
        for (int c = lane; c < np.gs; c += 64) part[c] = 0.f;
    }
}

// dw[c] = sum over the partial sums, in a fixed order: a workgroup owns 64 channels, its four waves sum
// every fourth part each (four loads in flight per lane), wave 0 adds the four results.
__global__ __launch_bounds__(256) void k_norm_reduce(const float* part, int64_t nparts, int C, float* dw, int accumulate) {
    __shared__ float red[4][64];
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane;
    const bool live = c < C;
    float s = 0.f;
    if (live) {
        const float* src = part + c;
        int64_t p = wv;
        for (; p + 12 < nparts; p += 16) {
            const float a0 = src[p * C], a1 = src[(p + 4) * C], a2 = src[(p + 8) * C], a3 = src[(p + 12) * C];
            s += a0;
            s += a1;
            s += a2;
            s += a3;
        }
        for (; p < nparts; p += 4) s += src[p * C];
    }
    red[wv][lane] = s;
    __syncthreads();
    if (wv == 0 && live) {
        s = (red[0][lane] + red[1][lane]) + (red[2][lane] + red[3][lane]);
        dw[c] = accumulate ? dw[c] + s : s;
    }
}

struct NormDims {
    int64_t T, y_rs, z_rs;
    int C, G, gs, ntiles;
    bool bf16;
};

int check(const ssd_norm_shape_t* sh, NormDims* d) {
    if (!sh) return SSD_ERR_NULL;
    if (sh->dtype != SSD_F32 && sh->dtype != SSD_BF16) return SSD_ERR_DTYPE;
    if (sh->rows < 0 || sh->dim <= 0 || sh->ngroups <= 0 || sh->ngroups > 65535) return SSD_ERR_SHAPE;
    if (sh->dim % sh->ngroups) return SSD_ERR_DIVISIBILITY;
    if (!(sh->eps >= 0.f)) return SSD_ERR_ARG;
    if ((sh->y_row_stride && sh->y_row_stride < sh->dim) || (sh->z_row_stride && sh->z_row_stride < sh->dim)) return SSD_ERR_SHAPE;
    d->T = sh->rows;
    d->C = sh->dim;
    d->G = sh->ngroups;
    d->gs = sh->dim / sh->ngroups;
    d->y_rs = sh->y_row_stride ? sh->y_row_stride : sh->dim;
    d->z_rs = sh->z_row_stride ? sh->z_row_stride : sh->dim;
    d->ntiles = (int)((sh->rows + ROWS_PER_WG - 1) / ROWS_PER_WG);
    if ((sh->rows + ROWS_PER_WG - 1) / ROWS_PER_WG > 0x7fffffff) return SSD_ERR_SHAPE;
    d->bf16 = sh->dtype == SSD_BF16;
    return SSD_OK;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// How the register-resident kernel is instantiated for a shape: vectors per lane and waves per segment;
// vpl = 0 if the shape needs the element-wise kernel.
struct FastCfg {
    int vpl, wps;
};
FastCfg pick_fast(const NormDims& d, std::initializer_list<const void*> ptrs) {
    const int V = d.bf16 ? 8 : 4;
    if (d.gs % V || d.C % V || d.y_rs % V || d.z_rs % V) return {0, 0};
    for (const void* p : ptrs)
        if (!aligned16(p)) return {0, 0};
    const int nvec = d.gs / V;
    if (nvec <= 64) return {1, 1};
    if (nvec <= 128) return {2, 1};
    const int need = (nvec + 255) / 256;
    for (int v : {1, 2, 3, 4, 6, MAX_VPL})
        if (need <= v) return {v, 4};
    return {0, 0};
}

// Tiling of the rows for the register-resident kernels.  Backward: 64-row tiles, every tile its own
// workgroup up to about three workgroups per compute unit, beyond that equal shares of tiles (fewer partial
// sums of dw, the weight loaded once per workgroup).  Forward: no partial sums, registers for five
// workgroups per compute unit: 16-row tiles.  Short calls take smaller tiles.
struct FastGrid {
    int tile_rows, ntiles, nwg;
};
FastGrid fast_grid(const NormDims& d, bool bwd) {
    FastGrid g;
    const int per_cu = bwd ? 3 : 5;
    const int target = 256 * per_cu / d.G > 0 ? 256 * per_cu / d.G : 1;
    // fewer rows per tile when the call is short (a segment at a time), so that it still fills the machine
    g.tile_rows = bwd ? ROWS_PER_WG : ROWS_PER_WG_FWD;
    // (down to single rows forward -- a handful of tokens in generation; the backward pass keeps four, its
    // partial sums of dw are per workgroup)
    while (g.tile_rows > (bwd ? 4 : 1) && (d.T + g.tile_rows - 1) / g.tile_rows < target) g.tile_rows >>= 1;
    g.ntiles = (int)((d.T + g.tile_rows - 1) / g.tile_rows);
    if (g.ntiles <= target) {
        g.nwg = g.ntiles;
    } else {
        const int per = (g.ntiles + target - 1) / target;
        g.nwg = (g.ntiles + per - 1) / per;
    }
    return g;
}

template <typename T, bool BWD, bool GATED>
hipError_t launch_fast(const NormDims& d, const NormParams& np0, FastCfg f, hipStream_t st) {
    const FastGrid fg = fast_grid(d, BWD);
    NormParams np = np0;
    np.ntiles = fg.ntiles;
    np.tile_rows = fg.tile_rows;
    const dim3 grid(fg.nwg, np.G), block(256);
#define NORM_CASE(N, W)                                                                    \
    if (f.vpl == N && f.wps == W) {                                                        \
        hipLaunchKernelGGL((k_gated_norm<T, N, W, BWD, GATED>), grid, block, 0, st, np);   \
        return hipGetLastError();                                                          \
    }
    NORM_CASE(1, 1)
    NORM_CASE(2, 1)
    NORM_CASE(1, 4)
    NORM_CASE(2, 4)
    NORM_CASE(3, 4)
    NORM_CASE(4, 4)
    NORM_CASE(6, 4)
    NORM_CASE(8, 4)
#undef NORM_CASE
    return hipErrorInvalidValue;
}

template <bool BWD, bool GATED>
hipError_t launch_g(const NormDims& d, const NormParams& np, FastCfg f, hipStream_t st) {
    if (f.vpl) return d.bf16 ? launch_fast<bf16_t, BWD, GATED>(d, np, f, st) : launch_fast<float, BWD, GATED>(d, np, f, st);
    const dim3 grid(np.ntiles, np.G), block(256);
    if (d.bf16)
        hipLaunchKernelGGL((k_gated_norm_any<bf16_t, BWD, GATED>), grid, block, 0, st, np);
    else
        hipLaunchKernelGGL((k_gated_norm_any<float, BWD, GATED>), grid, block, 0, st, np);
    return hipGetLastError();
}

// np.z == NULL: no gate (plain RMS normalisation of y); the kernels then never touch z or dz
template <bool BWD>
hipError_t launch(const NormDims& d, const NormParams& np, FastCfg f, hipStream_t st) {
    return np.z ? launch_g<BWD, true>(d, np, f, st) : launch_g<BWD, false>(d, np, f, st);
}

NormParams params(const NormDims& d, const ssd_norm_shape_t* sh) {
    NormParams np;
    memset(&np, 0, sizeof(np));
    np.T = d.T;
    np.y_rs = d.y_rs;
    np.z_rs = d.z_rs;
    np.C = d.C;
    np.G = d.G;
    np.gs = d.gs;
    np.ntiles = d.ntiles;
    np.tile_rows = ROWS_PER_WG;
    np.eps = sh->eps;
    return np;
}

}  // namespace
}  // namespace ssdk

using namespace ssdk;

// up to four partial rows of dw per tile (one per slot of the workgroup)
extern "C" size_t ssd_gated_norm_workspace_bytes(const ssd_norm_shape_t* sh) {
    NormDims d;
    if (check(sh, &d) != SSD_OK) return 0;
    // partial rows of dw: four per 64-row tile (element-wise kernel) or up to four per workgroup (register-resident one)
    size_t rows = (size_t)(d.ntiles > 0 ? d.ntiles : 1);
    const size_t fast = d.T > 0 ? (size_t)fast_grid(d, true).nwg : 0;
    rows = fast > rows ? fast : rows;
    const size_t n = rows * 4 * (size_t)d.C * 4;
    return (n + 255) & ~(size_t)255;
}

extern "C" int ssd_gated_norm_fwd(const ssd_norm_shape_t* sh, const void* y, const void* z, const float* w, void* out,
                                  void* hip_stream) {
    NormDims d;
    const int rc = check(sh, &d);
    if (rc != SSD_OK) return rc;
    if (d.T == 0) return SSD_OK;
    if (!y || !w || !out) return SSD_ERR_NULL;  // z == NULL: no gate
    NormParams np = params(d, sh);
    np.y = y;
    np.z = z;
    np.w = w;
    np.out = out;
    return launch<false>(d, np, pick_fast(d, {y, z, out}), (hipStream_t)hip_stream) == hipSuccess ? SSD_OK : SSD_ERR_LAUNCH;
}

extern "C" int ssd_gated_norm_bwd(const ssd_norm_shape_t* sh, const void* y, const void* z, const float* w, const void* dout,
                                  void* dy, void* dz, float* dw, void* workspace, size_t workspace_bytes, uint32_t flags,
                                  void* hip_stream) {
    NormDims d;
    const int rc = check(sh, &d);
    if (rc != SSD_OK) return rc;
    if (flags & ~(uint32_t)SSD_FLAG_ACCUM_PARAM) return SSD_ERR_ARG;
    if (!dw) return SSD_ERR_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    const int accumulate = (flags & SSD_FLAG_ACCUM_PARAM) ? 1 : 0;
    if (d.T == 0) {
        if (accumulate) return SSD_OK;
        return launch_fill_zero(dw, (size_t)d.C, st) == hipSuccess ? SSD_OK : SSD_ERR_LAUNCH;
    }
    if (!y || !w || !dout || !dy || (z && !dz)) return SSD_ERR_NULL;  // z == NULL: no gate, dz is not written
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < ssd_gated_norm_workspace_bytes(sh)) return SSD_ERR_WORKSPACE;
    NormParams np = params(d, sh);
    np.y = y;
    np.z = z;
    np.w = w;
    np.dout = dout;
    np.dy = dy;
    np.dz = z ? dz : nullptr;
    np.part = (float*)workspace;
    const FastCfg f = pick_fast(d, {y, z, dout, dy, z ? dz : nullptr});
    const int64_t nparts = f.vpl ? (int64_t)fast_grid(d, true).nwg * (4 / f.wps) : (int64_t)d.ntiles * 4;
    if ((size_t)nparts * d.C * 4 > workspace_bytes) return SSD_ERR_WORKSPACE;  // cannot happen with the documented size
    if (launch<true>(d, np, f, st) != hipSuccess) return SSD_ERR_LAUNCH;
    hipLaunchKernelGGL(k_norm_reduce, dim3((d.C + 63) / 64), dim3(256), 0, st, np.part, nparts, d.C, dw, accumulate);
    return hipGetLastError() == hipSuccess ? SSD_OK : SSD_ERR_LAUNCH;
}
