// The "dual form" passes of the chunked selective scan on the matrix cores (gfx950, bf16 in / fp32
// accumulate): for one chunk of Q tokens, the quadratic form of Eq. 1 unrolled over the chunk plus
// the term through the chunk's entering state (forward) or leaving state adjoint (reverse).
// Computed transposed, so that a lane owns a token:
//   EPI 0 (forward output):   yhat^T[p][i] = sum_{j<=i} G[i][j] decay(i,j) dt_j x_j[p] + exp(cum_i) (Hprev C_i)[p];
//                             y = yhat + D x  (+ x under the residual flag)
//   EPI 2 (backward):         u^T[p][j] = sum_{i>=j} G[i][j] decay(i,j) dY_i[p] + exp(T - cum_j) (dHnext B_j)[p];
//                             dx = dt u + D dY (+ dY), f_j = x_j . u_j (the direct part of ddt) and dY_j . x_j (for dD)
// (The gradient of cum is not formed here: it is assembled from the E sums of the dG kernel and the
// state dot products of the head-sum kernel.)
//
// Organisation.  One workgroup owns one (batch, chunk, group) and a slice of that group's heads and
// walks the heads one after the other.  It has one wave per 32-token tile of the chunk; the tile
// index is a wave-uniform run-time value (one code path for every wave).  Everything
// that does not depend on the head -- the wave's rows of the score matrix G = C B^T (or of its
// transpose) and of C (or B) -- is fetched once and stays in registers as MFMA operands for all
// heads of the slice.  Per head, the token-major operand (x or dY, Q x 64) and the state (64 x 128)
// are prefetched into registers while the previous head is being computed, then staged in LDS
// (plain and pre-scaled copy of the tile, see the decay factorisation in mfma_kernels.hip); outputs
// go through a per-wave LDS patch so that global stores are whole 128-byte rows.
// With Q = 256 the eight waves are paired on the four SIMDs so that each SIMD sees the same amount
// of causal work (tiles t and 7 - t).
#pragma once
#include "mfma_common.h"

namespace ssdk {
namespace dualk {

using namespace mf;

constexpr int GO_MAX = 12;  // score-matrix fragments of the off-diagonal blocks a wave keeps (three blocks of four steps)
constexpr int RF_N = N_ / 16;

template <int Q>
struct DualCfg {
    static constexpr int NT = Q / 32;           // token tiles = waves
    static constexpr int NTHR = 64 * NT;
    static constexpr int NB = Q / BLK;
    static constexpr int XV = Q * 8 / NTHR;     // 16-byte vectors of the token-major tile per thread (= 4)
    static constexpr int SV = P_ * 16 / NTHR;   // 16-byte vectors of the state per thread
};

template <int Q>
struct DualLds {
    char raw[Q * XPITCH];    // x (forward) or dY (reverse), token-major
    char scl[Q * XPITCH];    // eout*dt*x      or ein*dY
    char st[P_ * BPITCH];    // entering state / leaving adjoint, [p][n] bf16
    float cum2[Q];           // cum * log2(e)
    float fac[Q];            // ein (forward) or eout (reverse): applied per output token
    float dtl[Q];            // dt
    char priv[Q / 32][32 * XPITCH];  // per-wave patch for the row-major epilogue
};

// Registers holding the next head's operands while the current head is computed.
template <int Q>
struct Pre {
    bf16x8 xt[DualCfg<Q>::XV];
    float sc[DualCfg<Q>::XV], sc2[DualCfg<Q>::XV];  // per-token scale factors, multiplied at staging time
    bf16x8 sv[DualCfg<Q>::SV];
    float cum, dtf, fac;
    float Dh;       // D of the head
    bf16x8 own[4];  // reverse: the wave's own 32 rows of x as whole rows (for the epilogue's dot products)
};

struct HeadCtx {
    const bf16_t* xg;   // x rows of this chunk and head
    const bf16_t* dyg;  // dY rows (EPI 2)
    bf16_t* outp;       // y (EPI 0) or dx (EPI 2)
    float* fterm;
    float* dDrow;
    int64_t xt;
    float Dh;
};

__device__ __forceinline__ void lds_wave_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

__device__ __forceinline__ bf16x8 frag_lds_rows(const char* tile, int pitch, int row0, int k0, int lane) {
    return *(const bf16x8*)(tile + (row0 + (lane & 31)) * pitch + (k0 + 8 * (lane >> 5)) * 2);
}

template <int Q, bool REV>
__device__ __forceinline__ void load_pre(Pre<Q>& pr, const SegParams& sp, int b, int c, int h, int tid, int tok0) {
    typedef DualCfg<Q> CF;
    const int64_t xt = (int64_t)sp.H * P_;
    const int64_t cbase = (((int64_t)b * sp.H + h) * sp.nc + c) * Q;
    const bf16_t* src = (REV ? (const bf16_t*)sp.dy + (int64_t)b * sp.dys_b : (const bf16_t*)sp.x + (int64_t)b * sp.xs_b) +
                        ((int64_t)c * Q * sp.H + h) * P_;
    // addresses = a wave-uniform base (scalar registers) + one 32-bit byte offset per lane
    const uint32_t rowbytes = (uint32_t)xt * 2;
    const uint32_t xoff = (uint32_t)(tid >> 3) * rowbytes + (uint32_t)(tid & 7) * 16, roff = (uint32_t)(tid >> 3) * 4;
    constexpr int RSTEP = CF::NTHR / 8;  // rows between a thread's consecutive vectors
#pragma unroll
    for (int k = 0; k < CF::XV; ++k) {
        pr.xt[k] = *(const bf16x8*)((const char*)src + (size_t)k * RSTEP * rowbytes + (size_t)xoff);
        const float* f1 = (REV ? sp.ein : sp.dtf) + cbase + k * RSTEP;
        pr.sc[k] = *(const float*)((const char*)f1 + (size_t)roff);
        if (!REV) pr.sc2[k] = *(const float*)((const char*)(sp.eout + cbase + k * RSTEP) + (size_t)roff);
    }
    const bf16_t* S = (REV ? sp.dstates_bf : sp.states_bf) + (((int64_t)b * sp.nc + c) * sp.H + h) * (P_ * N_);
    const uint32_t soff = (uint32_t)tid * 16;
    // the state tile has this one reader: streaming load
#pragma unroll
    for (int k = 0; k < CF::SV; ++k) pr.sv[k] = __builtin_nontemporal_load((const bf16x8*)((const char*)S + (size_t)k * CF::NTHR * 16 + (size_t)soff));
    if (tid < Q) {
        pr.cum = sp.cum[cbase + tid];
        pr.dtf = sp.dtf[cbase + tid];
        pr.fac = REV ? sp.eout[cbase + tid] : sp.ein[cbase + tid];
    }
    pr.Dh = sp.D[h];
    if (REV) {  // lane -> (row lane / 8, 16-byte piece lane % 8) of each 8-row group of the wave's tile
        const bf16_t* xg = (const bf16_t*)sp.x + (int64_t)b * sp.xs_b + ((int64_t)c * Q * sp.H + h) * P_;
        const uint32_t ooff = (uint32_t)((tid >> 3) & 7) * rowbytes + (uint32_t)(tid & 7) * 16;
#pragma unroll
        for (int it = 0; it < 4; ++it)
            pr.own[it] = *(const bf16x8*)((const char*)(xg + (int64_t)(tok0 + 8 * it) * xt) + (size_t)ooff);
    }
}

template <int Q, bool REV>
__device__ __forceinline__ void store_pre(const Pre<Q>& pr, DualLds<Q>& L, int tid, int w) {
    typedef DualCfg<Q> CF;
    if (REV) {  // the wave's own x rows wait in its patch for the epilogue (the patch is idle until then)
        const int lane = tid & 63;
#pragma unroll
        for (int it = 0; it < 4; ++it) *(bf16x8*)(L.priv[w] + ((lane >> 3) + 8 * it) * XPITCH + (lane & 7) * 16) = pr.own[it];
    }
#pragma unroll
    for (int k = 0; k < CF::XV; ++k) {
        const int v = tid + CF::NTHR * k, row = v >> 3, seg = v & 7;
        *(bf16x8*)(L.raw + row * XPITCH + seg * 16) = pr.xt[k];
        *(bf16x8*)(L.scl + row * XPITCH + seg * 16) = scale8(pr.xt[k], REV ? pr.sc[k] : pr.sc[k] * pr.sc2[k]);
    }
#pragma unroll
    for (int k = 0; k < CF::SV; ++k) {
        const int v = tid + CF::NTHR * k, row = v >> 4, seg = v & 15;
        *(bf16x8*)(L.st + row * BPITCH + seg * 16) = pr.sv[k];
    }
    if (tid < Q) {
        // one address, three immediate offsets: cum2, fac and dtl lie one after the other
        static_assert(offsetof(DualLds<Q>, fac) == offsetof(DualLds<Q>, cum2) + Q * sizeof(float) &&
                      offsetof(DualLds<Q>, dtl) == offsetof(DualLds<Q>, cum2) + 2 * Q * sizeof(float), "contiguous per-token rows");
        float* row = L.cum2 + tid;
        row[0] = pr.cum * LOG2E;
        row[Q] = pr.fac;
        row[2 * Q] = pr.dtf;
    }
}

// Persistent operands of tile T (wave-uniform run-time value): the rows TOK0 .. TOK0+31 of the score
// matrix (forward: G, columns = earlier tokens; reverse: G^T, columns = later tokens) for the diagonal
// 64-token block (gd) and for the off-diagonal blocks (go, block K at go[4K + ks] forward and at
// go[4(K-1) + ks] reverse), and the same rows of C (forward) or B (reverse).
template <int Q, bool REV>
__device__ __forceinline__ void tile_load(bf16x8 (&go)[GO_MAX], bf16x8 (&gd)[4], bf16x8 (&rf)[RF_N], const bf16_t* Mat,
                                          const bf16_t* rowop, int64_t bt, int T, int lane) {
    constexpr int NB = Q / BLK;
    const int I = T >> 1, tok0 = 32 * T;
#pragma unroll
    for (int n = 0; n < NB - 1; ++n) {
        const int K = REV ? n + 1 : n;
        if (REV ? K > I : K < I) {
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) go[4 * n + ks] = frag_rows(Mat, Q, tok0, 16 * (4 * K + ks), lane);
        }
    }
    // the diagonal block carries the causal mask already (it does not depend on the head): scores of the
    // contraction tokens beyond the lane's own token (forward) / before it (reverse) are zero
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const bf16x8 v = frag_rows(Mat, Q, tok0, 16 * (4 * I + ks), lane);
        const int kk0 = 16 * (4 * I + ks) + 8 * (lane >> 5), tok = tok0 + (lane & 31);
#pragma unroll
        for (int e = 0; e < 8; ++e) gd[ks][e] = (REV ? kk0 + e >= tok : kk0 + e <= tok) ? v[e] : (__bf16)0.f;
    }
#pragma unroll
    for (int ks = 0; ks < RF_N; ++ks) rf[ks] = frag_rows(rowop, bt, tok0, 16 * ks, lane);
}

template <int Q, int EPI>
__device__ __forceinline__ void tile_compute(const bf16x8 (&go)[GO_MAX], const bf16x8 (&gd)[4], const bf16x8 (&rf)[RF_N],
                                             DualLds<Q>& L, const HeadCtx& cx, int T, int lane, int w) {
    constexpr bool REV = EPI == 2;
    constexpr int NB = Q / BLK;
    const int I = T >> 1, odd = T & 1, tok0 = 32 * T;
    const int tl = lane & 31, tok = tok0 + tl;
    char* priv = L.priv[w];
    const float lane_c2 = L.cum2[tok], lane_fac = L.fac[tok];
    f32x16 acc0 = zero16(), acc1 = zero16();
    // Operand reads from LDS run one contraction step ahead of the MFMAs that use them (the scheduling
    // barriers keep the compiler from sinking a read next to its use, where every MFMA would wait a full
    // LDS latency).
    // term through the chunk's entering state (forward) / leaving adjoint (reverse)
    {
        bf16x8 a0 = frag_lds_rows(L.st, BPITCH, 0, 0, lane), a1 = frag_lds_rows(L.st, BPITCH, 32, 0, lane);
#pragma unroll
        for (int ks = 0; ks < RF_N; ++ks) {
            bf16x8 n0 = a0, n1 = a1;
            if (ks + 1 < RF_N) {
                n0 = frag_lds_rows(L.st, BPITCH, 0, 16 * (ks + 1), lane);
                n1 = frag_lds_rows(L.st, BPITCH, 32, 16 * (ks + 1), lane);
            }
            __builtin_amdgcn_sched_barrier(0);
            acc0 = mfma(a0, rf[ks], acc0);
            acc1 = mfma(a1, rf[ks], acc1);
            a0 = n0;
            a1 = n1;
        }
    }
    // off-diagonal 64-token blocks, Horner in the block decays (forward: K = 0 .. I-1; reverse: K = NB-1 .. I+1)
#pragma unroll
    for (int n = 0; n < NB - 1; ++n) {
        const int K = REV ? NB - 1 - n : n;
        if (REV ? K > I : K < I) {
            bf16x8 a0 = frag_tr(L.scl, XPITCH, K * BLK, 0, lane), a1 = frag_tr(L.scl, XPITCH, K * BLK, 32, lane);
            const float sK = __builtin_amdgcn_exp2f(L.cum2[K * BLK + BLK - 1] - (K > 0 ? L.cum2[K * BLK - 1] : 0.f));
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                acc0[r] *= sK;
                acc1[r] *= sK;
            }
#pragma unroll
            for (int ks = 0; ks < BLK / 16; ++ks) {
                bf16x8 n0 = a0, n1 = a1;
                if (ks + 1 < BLK / 16) {
                    n0 = frag_tr(L.scl, XPITCH, K * BLK + 16 * (ks + 1), 0, lane);
                    n1 = frag_tr(L.scl, XPITCH, K * BLK + 16 * (ks + 1), 32, lane);
                }
                __builtin_amdgcn_sched_barrier(0);
                const bf16x8 fb = go[4 * (REV ? K - 1 : K) + ks];
                acc0 = mfma(a0, fb, acc0);
                acc1 = mfma(a1, fb, acc1);
                a0 = n0;
                a1 = n1;
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        acc0[r] *= lane_fac;
        acc1[r] *= lane_fac;
    }
    // diagonal block: the mask and the decay (and, forward, dt_j) are evaluated per element.  Forward,
    // an even tile stops after its own 32 tokens; reverse, an odd tile starts at its own.  The operand
    // reads of a step are issued before the arithmetic that builds its masked scores.
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        if (REV ? (odd && ks < 2) : (!odd && ks >= 2)) continue;
        const int k0 = I * BLK + 16 * ks;
        const bf16x8 a0 = frag_tr(L.raw, XPITCH, k0, 0, lane), a1 = frag_tr(L.raw, XPITCH, k0, 32, lane);
        const bf16x8 gv = gd[ks];
        const int kk0 = k0 + 8 * (lane >> 5);
        const float4 ca = *(const float4*)(L.cum2 + kk0), cb = *(const float4*)(L.cum2 + kk0 + 4);
        float4 da = make_float4(0.f, 0.f, 0.f, 0.f), db = da;
        if (!REV) {
            da = *(const float4*)(L.dtl + kk0);
            db = *(const float4*)(L.dtl + kk0 + 4);
        }
        __builtin_amdgcn_sched_barrier(0);
        const float cv[8] = {ca.x, ca.y, ca.z, ca.w, cb.x, cb.y, cb.z, cb.w};
        const float dv[8] = {da.x, da.y, da.z, da.w, db.x, db.y, db.z, db.w};
        bf16x8 fb;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            // masked scores are zero; the clamp keeps their factor finite (it is <= 0 wherever the score is not masked)
            const float diff = REV ? cv[e] - lane_c2 : lane_c2 - cv[e];
            float f = (float)gv[e] * __builtin_amdgcn_exp2f(fminf(diff, 0.f));
            if (!REV) f *= dv[e];
            fb[e] = (__bf16)f;
        }
        acc0 = mfma(a0, fb, acc0);
        acc1 = mfma(a1, fb, acc1);
    }
    // whole-row global accesses of the epilogue: lane -> (row lane / 8, 16-byte piece lane % 8) of an 8-row group
    const uint32_t rowoff = ((uint32_t)(lane >> 3) * (uint32_t)cx.xt + (uint32_t)(lane & 7) * 8) * 2;
    // epilogue: in the accumulators this lane owns token `tok` and, per register group q, four
    // consecutive channels; rows travel through the wave's LDS patch to and from whole-row accesses.
    // Reverse, the wave's own 32 rows of x have been waiting in its patch since the staging phase.
    float s_a = 0.f, s_b = 0.f;
    const float dtok = REV ? L.dtl[tok] : 0.f;
    // one half of the channels at a time: the results of a half replace, in the patch, the x values of
    // that half, which nothing reads any more (fewer values held in registers at once)
#pragma unroll
    for (int pt = 0; pt < 2; ++pt) {
        bf16x4 outv[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int p4 = 32 * pt + 8 * q + 4 * (lane >> 5);
            const bf16x4 mine = *(const bf16x4*)(L.raw + tok * XPITCH + p4 * 2);  // x (EPI 0) or dY (EPI 2)
            if (EPI == 0) {
#pragma unroll
                for (int e = 0; e < 4; ++e) outv[q][e] = (__bf16)((pt ? acc1 : acc0)[4 * q + e] + cx.Dh * (float)mine[e]);
            } else {
                const bf16x4 other = *(const bf16x4*)(priv + tl * XPITCH + p4 * 2);  // x
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float u = (pt ? acc1 : acc0)[4 * q + e];
                    outv[q][e] = (__bf16)(dtok * u + cx.Dh * (float)mine[e]);
                    s_a += (float)other[e] * u;
                    s_b += (float)mine[e] * (float)other[e];
                }
            }
        }
        if (EPI == 2) lds_wave_fence();  // every read of this half's x from the patch is done
#pragma unroll
        for (int q = 0; q < 4; ++q) *(bf16x4*)(priv + tl * XPITCH + (32 * pt + 8 * q + 4 * (lane >> 5)) * 2) = outv[q];
    }
    lds_wave_fence();
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int row = (lane >> 3) + 8 * it;
        const bf16x8 v = *(const bf16x8*)(priv + row * XPITCH + (lane & 7) * 16);
        // written once and not read again by this step: a streaming store leaves the L2 to the tiles the passes share
        __builtin_nontemporal_store(v, (bf16x8*)((char*)(cx.outp + (int64_t)(tok0 + 8 * it) * cx.xt) + (size_t)rowoff));
    }
    if (EPI != 0) {
        s_a += __shfl_xor(s_a, 32, 64);
        s_b += __shfl_xor(s_b, 32, 64);
        if (lane < 32) {
            cx.fterm[tok] = s_a;
            cx.dDrow[tok] = s_b;
        }
    }
}

// The body of one workgroup: z = its index among the nblk workgroups of this pass.
template <int Q, int EPI>
__device__ __forceinline__ void dual_body(const SegParams& sp, DualLds<Q>& L, int z, int nblk) {
    constexpr bool REV = EPI == 2;
    // workgroups that share a (chunk, group) -- hence G, C, B -- get consecutive logical ids and, when the
    // grid divides evenly, land on the same XCD (hardware deals workgroup ids round-robin over 8 XCDs)
    [[maybe_unused]] const int zlog = z;
    if ((nblk & 7) == 0) z = (z & 7) * (nblk >> 3) + (z >> 3);
    const int ns = sp.dual_split, slice = z % ns;
    z /= ns;
    const int g = z % sp.G, c = (z / sp.G) % sp.nc, b = z / (sp.G * sp.nc);
    const int hps = sp.hpg / ns, h0 = g * sp.hpg + slice * hps;
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Q = 256: waves w and w + 4 share a SIMD and take tiles t and 7 - t (equal causal work per SIMD)
    const int T = (Q == 256 && w >= 4) ? 11 - w : w;
    const int64_t xt = (int64_t)sp.H * P_, bt = (int64_t)sp.G * N_;

    const bf16_t* Gd = (const bf16_t*)sp.Gm + (((int64_t)b * sp.nc + c) * sp.G + g) * (2 * Q * Q);
    const bf16_t* Mat = REV ? Gd + Q * Q : Gd;  // rows = output token, columns = contraction token
    const bf16_t* rowop = (REV ? (const bf16_t*)sp.Bm : (const bf16_t*)sp.Cm) + (int64_t)b * sp.bcs_b +
                          ((int64_t)c * Q * sp.G + g) * N_;
    bf16x8 go[GO_MAX], gd[4], rf[RF_N];
    HeadCtx cx;
    tile_load<Q, REV>(go, gd, rf, Mat, rowop, bt, T, lane);
    Pre<Q> pr;
    load_pre<Q, REV>(pr, sp, b, c, h0, tid, 32 * T);
    for (int hh = 0; hh < hps; ++hh) {
        const int h = h0 + hh;
        // the thread index as the optimiser cannot see through: addresses derived from it are formed anew
        // for every head instead of being kept in registers across the whole loop
        int tv = tid;
        asm volatile("" : "+v"(tv));
        SSDK_STAMP(EPI == 2 ? 0 : 3, 0);
        __syncthreads();  // every wave is done with the previous head's tiles
        SSDK_STAMP(EPI == 2 ? 0 : 3, 1);
        cx.Dh = pr.Dh + ((sp.flags & SSD_FLAG_RESIDUAL) ? 1.f : 0.f);
        store_pre<Q, REV>(pr, L, tv, w);
        SSDK_STAMP(EPI == 2 ? 0 : 3, 2);
        __syncthreads();
        SSDK_STAMP(EPI == 2 ? 0 : 3, 3);
        if (hh + 1 < hps) load_pre<Q, REV>(pr, sp, b, c, h + 1, tv, 32 * T);
        SSDK_STAMP(EPI == 2 ? 0 : 3, 4);
        const int64_t cbase = (((int64_t)b * sp.H + h) * sp.nc + c) * Q;
        const int64_t xrow = ((int64_t)c * Q * sp.H + h) * P_;
        cx.xg = (const bf16_t*)sp.x + (int64_t)b * sp.xs_b + xrow;
        cx.dyg = EPI == 0 ? nullptr : (const bf16_t*)sp.dy + (int64_t)b * sp.dys_b + xrow;
        cx.outp = EPI == 0 ? (bf16_t*)sp.y + (int64_t)b * sp.ys_b + xrow : (bf16_t*)sp.dx + (int64_t)b * sp.dxs_b + xrow;
        cx.fterm = sp.fterm + cbase;
        cx.dDrow = sp.dDrow + cbase;
        cx.xt = xt;
        tile_compute<Q, EPI>(go, gd, rf, L, cx, T, lane, w);
        SSDK_STAMP(EPI == 2 ? 0 : 3, 5);
    }
}

}  // namespace dualk
}  // namespace ssdk
