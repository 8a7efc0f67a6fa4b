// The last step of the backward pass of one chunk and head, shared by the shape-generic kernels and the
// matrix-core path: da = reverse cumulative sum of the gradient of cum (+ the chunk-end term), ddt = A da + f,
// and the chunk's partial sums of dA and dD.
#pragma once
#include "ssd_internal.h"

namespace ssdk {

// One workgroup (blockDim.x threads, a power of two >= Q) per (chunk c, head h, batch b); s and s2 are two arrays
// of blockDim.x floats in LDS; store(index into ddt, value) writes one element of ddt in its storage type.
template <class Store>
__device__ __forceinline__ void ddt_finalize_body(const SegParams& sp, float* s, float* s2, int c, int h, int b, Store store) {
    const int i = threadIdx.x;
    const int Q = sp.Q;
    const int64_t cbase = (((int64_t)b * sp.H + h) * sp.nc + c) * Q;
    // reverse order so that an inclusive forward scan yields the suffix sums
    const int ri = Q - 1 - i;
    // Matrix-core path: the gradient of cum_i arrives as gterm_i + gintra_i - sterm_i, and the gradient of
    // cum at the chunk end carries + sum_j sterm_j (the chunk state depends on T - cum_j): the very same
    // sterm values enter with both signs, so their cancellation in the suffix sums is exact.
    float gt = 0.f, st_sum = 0.f;
    const bool split = sp.flags & SSD_INTERNAL_SPLIT_GTERM;
    if (i < Q) {
        gt = sp.gterm[cbase + ri];
        if (split) {
            const float sv = sp.sterm[cbase + ri];
            gt += sp.gintra[cbase + ri] - sv;
            st_sum = sv;
        }
    }
    if (split) {
        s2[i] = st_sum;
        __syncthreads();
        for (int off = blockDim.x >> 1; off > 0; off >>= 1) {
            if (i < off) s2[i] += s2[i + off];
            __syncthreads();
        }
        st_sum = s2[0];
        __syncthreads();
    }
    s[i] = gt;
    __syncthreads();
    for (int off = 1; off < (int)blockDim.x; off <<= 1) {
        const float v = (i >= off) ? s[i - off] : 0.f;
        __syncthreads();
        s[i] += v;
        __syncthreads();
    }
    float tail = 0.f;
    const float* tp = sp.tail_part + ((((int64_t)b * sp.H + h) * sp.nc + c)) * sp.nslice;
    for (int k = 0; k < sp.nslice; ++k) tail += tp[k];
    tail += st_sum;
    float pa = 0.f, pd = 0.f;
    if (i < Q) {
        const float da = s[i] + tail;  // belongs to token ri
        const float d = sp.dtf[cbase + ri];
        store((int64_t)b * sp.dts_b + ((int64_t)c * Q + ri) * sp.H + h, sp.A[h] * da + sp.fterm[cbase + ri]);
        pa = d * da;
        pd = sp.dDrow[cbase + ri];
    }
    __syncthreads();
    s[i] = pa;
    s2[i] = pd;
    __syncthreads();
    for (int off = blockDim.x >> 1; off > 0; off >>= 1) {
        if (i < off) {
            s[i] += s[i + off];
            s2[i] += s2[i + off];
        }
        __syncthreads();
    }
    if (i == 0) {
        sp.dA_part[((int64_t)b * sp.nc_total + sp.chunk0 + c) * sp.H + h] = s[0];
        sp.dD_part[((int64_t)b * sp.nc_total + sp.chunk0 + c) * sp.H + h] = s2[0];
    }
}

}  // namespace ssdk
