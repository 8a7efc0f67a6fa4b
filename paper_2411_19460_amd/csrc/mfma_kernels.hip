// Matrix-core (MFMA, bf16 in / fp32 accumulate) kernels of the chunked selective scan for gfx950.
// Shape: P = 64 channels per head, N = 128 states, chunk Q in {64, 128, 256}; wave64; every contraction
// runs on v_mfma_f32_32x32x16_bf16.
//
// Numerical scheme for the decay mask exp(cum_i - cum_j) of the dual form (Sec. 3.1, Eq. 1 unrolled
// over a chunk).  The chunk is cut into blocks of 64 tokens.  With
//     ein_i  = exp(cum_i - cum[start of i's block - 1])      (<= 1)
//     eout_j = exp(cum[end of j's block] - cum_j)            (<= 1)
//     s_K    = exp(cum[end of block K] - cum[start of K - 1]) (<= 1, the block's total decay)
// one has, for i in block I and j in block J < I,
//     exp(cum_i - cum_j) = ein_i * (prod_{J<K<I} s_K) * eout_j,
// so the off-diagonal blocks are pure MFMA work on the raw scores G = C B^T and on operands that were
// scaled once per token while being staged into LDS; the product over K is applied Horner-style by
// scaling the accumulator with the scalar s_K between blocks (this is the state recurrence at
// 64-token granularity), and ein / eout is applied once per output row.  Only the four diagonal
// 64 x 64 blocks evaluate exp() per element.  Every exponent is <= 0: nothing can overflow, and an
// underflow only happens where the exact value underflows too.
//
// Operands whose contraction index is the token index live token-major in memory; they are staged
// in LDS as [token][channel] and read with the LDS transpose load (ds_read_b64_tr_b16), which hands
// each lane four consecutive tokens of one channel -- the layout an MFMA operand needs.
#include "mfma_common.h"

namespace ssdk {
namespace {

using namespace mf;

// ---------------------------------------------------------------------------------------------
// Decay preparation: cum (chunk-local inclusive cumsum of dt*A), dt in fp32, ein, eout.
template <int Q>
__device__ __forceinline__ void prep_body(const SegParams& sp, float* s, int c, int h, int b) {
    const int i = threadIdx.x;
    const float d = bf16_to_float(((const bf16_t*)sp.dt)[(int64_t)b * sp.dts_b + ((int64_t)c * Q + i) * sp.H + h]);
    s[i] = d * sp.A[h] + ((sp.reset && sp.reset[(int64_t)b * sp.reset_bs + (int64_t)c * Q + i]) ? RESET_LOG_DECAY : 0.f);
    __syncthreads();
    for (int off = 1; off < Q; off <<= 1) {
        const float v = (i >= off) ? s[i - off] : 0.f;
        __syncthreads();
        s[i] += v;
        __syncthreads();
    }
    const int bs = (i / BLK) * BLK;
    const float before = bs > 0 ? s[bs - 1] : 0.f;
    const int64_t o = (((int64_t)b * sp.H + h) * sp.nc + c) * Q + i;
    sp.cum[o] = s[i];
    sp.dtf[o] = d;
    sp.ein[o] = __expf(s[i] - before);
    sp.eout[o] = __expf(s[bs + BLK - 1] - s[i]);
}

template <int Q>
__global__ __launch_bounds__(Q) void mk_prep(SegParams sp) {
    __shared__ float s[Q];
    prep_body<Q>(sp, s, blockIdx.x, blockIdx.y, blockIdx.z);
}

// ---------------------------------------------------------------------------------------------
// Scores of one chunk and group: G[i][j] = C_i . B_j and its transpose, bf16, for the 64 x 64 blocks
// on and below the diagonal.  Layout in the scratch area: G [Q][Q] then GT [Q][Q].
template <int Q>
__device__ __forceinline__ void cb_body(const SegParams& sp, int z, int pair) {
    constexpr int NB = Q / BLK;
    const int g = z % sp.G, c = (z / sp.G) % sp.nc, b = z / (sp.G * sp.nc);
    int I = 0, rem = pair;  // pair enumerates the block pairs (I, J <= I)
    while (rem > I) {
        rem -= I + 1;
        ++I;
    }
    const int J = rem;
    if (I >= NB) return;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int i0 = I * BLK + (w >> 1) * 32, j0 = J * BLK + (w & 1) * 32;
    const int64_t ts = (int64_t)sp.G * N_;
    const bf16_t* Cm = (const bf16_t*)sp.Cm + (int64_t)b * sp.bcs_b + ((int64_t)c * Q * sp.G + g) * N_;
    const bf16_t* Bm = (const bf16_t*)sp.Bm + (int64_t)b * sp.bcs_b + ((int64_t)c * Q * sp.G + g) * N_;
    f32x16 a1 = zero16(), a2 = zero16();
#pragma unroll
    for (int ks = 0; ks < N_ / 16; ++ks) {
        const bf16x8 fc = frag_rows(Cm, ts, i0, 16 * ks, lane);
        const bf16x8 fb = frag_rows(Bm, ts, j0, 16 * ks, lane);
        a1 = mfma(fc, fb, a1);  // a1[r] = G[i0 + acc_row(r)][j0 + lane%32]
        a2 = mfma(fb, fc, a2);  // a2[r] = G[i0 + lane%32][j0 + acc_row(r)]
    }
    bf16_t* Gd = (bf16_t*)sp.Gm + (((int64_t)b * sp.nc + c) * sp.G + g) * (2 * Q * Q);
    bf16_t* GTd = Gd + Q * Q;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        bf16x4 v1, v2;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            v1[e] = (__bf16)a1[4 * q + e];
            v2[e] = (__bf16)a2[4 * q + e];
        }
        const int rr = 8 * q + 4 * (lane >> 5);
        *(bf16x4*)(GTd + (int64_t)(j0 + (lane & 31)) * Q + i0 + rr) = v1;
        *(bf16x4*)(Gd + (int64_t)(i0 + (lane & 31)) * Q + j0 + rr) = v2;
    }
}

template <int Q>
__global__ __launch_bounds__(NTH) void mk_cb(SegParams sp) {
    cb_body<Q>(sp, blockIdx.x, blockIdx.y);
}

// The two steps that need nothing but the inputs -- decay preparation and scores -- as one launch (chunk 256: both
// run 256 threads per workgroup): the first n_prep workgroups do one (chunk, head) of the former each, the rest one
// 64 x 64 block pair of the latter.
__global__ __launch_bounds__(NTH) void mk_prep_cb(SegParams sp, int n_prep) {
    constexpr int Q = 256, NPAIR = (Q / BLK) * (Q / BLK + 1) / 2;
    __shared__ float s[Q];
    int z = blockIdx.x;
    if (z < n_prep) {
        const int c = z % sp.nc;
        z /= sp.nc;
        prep_body<Q>(sp, s, c, z % sp.H, z / sp.H);
    } else {
        z -= n_prep;
        cb_body<Q>(sp, z / NPAIR, z % NPAIR);
    }
}

// ---------------------------------------------------------------------------------------------
// role 0: states_bf[b,c,h]  = sum_j exp(T - cum_j) dt_j x_j (x) B_j      (chunk state, bf16 [P][N])
// role 1: dstates_bf[b,c,h] = sum_i exp(cum_i) dY_i (x) C_i              (local state adjoint)
// (fp32 accumulation, one rounding to bf16: the consumers take these as bf16 MFMA operands anyway,
// and the scans carry the running state in fp32 registers.)
// One workgroup per (batch, chunk, group, role, head slice); eight waves, wave w owning the 32 x 32
// output tile (p half w / 4, state columns 32 (w % 4)).  The B (or C) rows of the chunk do not depend on
// the head: they go through LDS once and each wave keeps its Q/16 operand fragments in registers
// for every head of the slice.  Per head the token-major tile (x or dY, weighted per token) is
// prefetched in registers during the previous head, staged in LDS and read with transpose loads.
template <int Q>
union OuterLds {
    char bc[Q * BPITCH];  // B or C rows of the chunk (prologue only: each wave takes its fragments, then the space is xt)
    char xt[Q * XPITCH];  // weight * x or weight * dY
};

constexpr int OUTER_THR = 512;

template <int Q>
struct OuterPre {
    static constexpr int NV = Q * 8 / OUTER_THR > 0 ? Q * 8 / OUTER_THR : 1;
    bf16x8 t[NV];
    float cv[NV], dv[NV];  // cum and dt of the vector's token
    float T;               // cum at the end of the chunk
};

// Loads only: no arithmetic on the loaded values here, so that nothing waits for them before the
// next head's staging (the weights are formed in outer_weight at that point).
template <int Q>
__device__ __forceinline__ void outer_load(OuterPre<Q>& pr, const SegParams& sp, int role, int b, int c, int h, int tid) {
    const int64_t xt = (int64_t)sp.H * P_;
    const int64_t xrow = ((int64_t)c * Q * sp.H + h) * P_;
    const bf16_t* src = role == 0 ? (const bf16_t*)sp.x + (int64_t)b * sp.xs_b + xrow
                                  : (const bf16_t*)sp.dy + (int64_t)b * sp.dys_b + xrow;
    const int64_t cbase = (((int64_t)b * sp.H + h) * sp.nc + c) * Q;
    pr.T = sp.cum[cbase + Q - 1];
    // addresses = a wave-uniform base (scalar registers) + one 32-bit byte offset per lane
    const int t8 = tid % (Q * 8);  // Q = 64: one vector per thread
    const uint32_t rowbytes = (uint32_t)xt * 2, off = (uint32_t)(t8 >> 3) * rowbytes + (uint32_t)(t8 & 7) * 16;
    const uint32_t roff = (uint32_t)(t8 >> 3) * 4;
#pragma unroll
    for (int k = 0; k < OuterPre<Q>::NV; ++k) {
        // one reader per launch: streaming load (keeps the L2 for the kernels of other segments that do share tiles)
        pr.t[k] = __builtin_nontemporal_load((const bf16x8*)((const char*)src + (size_t)k * (OUTER_THR / 8) * rowbytes + (size_t)off));
        pr.cv[k] = *(const float*)((const char*)(sp.cum + cbase + k * (OUTER_THR / 8)) + (size_t)roff);
        pr.dv[k] = *(const float*)((const char*)(sp.dtf + cbase + k * (OUTER_THR / 8)) + (size_t)roff);
    }
}

template <int Q>
__device__ __forceinline__ float outer_weight(const OuterPre<Q>& pr, int role, int k) {
    return role == 0 ? __expf(pr.T - pr.cv[k]) * pr.dv[k] : __expf(pr.cv[k]);
}

// Two workgroups per compute unit (70 KB of LDS, at most 128 registers): one stages its next head while the
// other contracts.
template <int Q, bool F32OUT>
__global__ __launch_bounds__(OUTER_THR, 2) void mk_chunk_outer(SegParams sp, int nroles) {
    constexpr int KS = Q / 16;
    __shared__ __attribute__((aligned(16))) OuterLds<Q> L;
    int z = blockIdx.x;
    [[maybe_unused]] const int zlog = z;
    if ((gridDim.x & 7) == 0) z = (z & 7) * (gridDim.x >> 3) + (z >> 3);
    const int ns = sp.outer_split, slice = z % ns;
    z /= ns;
    const int role = z % nroles;
    z /= nroles;
    const int g = z % sp.G, c = (z / sp.G) % sp.nc, b = z / (sp.G * sp.nc);
    const int hps = sp.hpg / ns, h0 = g * sp.hpg + slice * hps;
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), ph = w >> 2, nt = w & 3;
    const int64_t bt = (int64_t)sp.G * N_;
    OuterPre<Q> pr;
    outer_load<Q>(pr, sp, role, b, c, h0, tid);
    // prologue: B (role 0) or C (role 1) rows -> LDS -> this wave's fragments
    const bf16_t* rhs = (role == 0 ? (const bf16_t*)sp.Bm : (const bf16_t*)sp.Cm) + (int64_t)b * sp.bcs_b + ((int64_t)c * Q * sp.G + g) * N_;
    for (int v = tid; v < Q * 16; v += OUTER_THR) {
        const int row = v >> 4, seg = v & 15;
        *(bf16x8*)(L.bc + row * BPITCH + seg * 16) = *(const bf16x8*)(rhs + (int64_t)row * bt + seg * 8);
    }
    __syncthreads();
    bf16x8 fb[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) fb[ks] = frag_tr(L.bc, BPITCH, 16 * ks, 32 * nt, lane);
    for (int hh = 0; hh < hps; ++hh) {
        const int h = h0 + hh;
        SSDK_STAMP(4, 0);
        __syncthreads();
        SSDK_STAMP(4, 1);
#pragma unroll
        for (int k = 0; k < OuterPre<Q>::NV; ++k) {
            const int v = tid + OUTER_THR * k, row = v >> 3, seg = v & 7;
            if (v < Q * 8) *(bf16x8*)(L.xt + row * XPITCH + seg * 16) = scale8(pr.t[k], outer_weight<Q>(pr, role, k));
        }
        SSDK_STAMP(4, 2);
        __syncthreads();
        SSDK_STAMP(4, 3);
        if (hh + 1 < hps) outer_load<Q>(pr, sp, role, b, c, h + 1, tid);
        SSDK_STAMP(4, 4);
        f32x16 acc = zero16();
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) acc = mfma(frag_tr(L.xt, XPITCH, 16 * ks, 32 * ph, lane), fb[ks], acc);
        const int64_t so = (((int64_t)b * sp.nc + c) * sp.H + h) * (P_ * N_);
        if (F32OUT) {  // fp32 scan input, in an array of its own
            float* out = (role == 0 ? sp.states : sp.dstates) + so;
#pragma unroll
            for (int r = 0; r < 16; ++r) out[(32 * ph + acc_row(r, lane)) * N_ + 32 * nt + (lane & 31)] = acc[r];
        } else {
            // bf16, into the slot where the scan will put the state entering the chunk (total adjoint leaving it)
            __bf16* out = (__bf16*)(role == 0 ? sp.states_bf : sp.dstates_bf) + so;
#pragma unroll
            for (int r = 0; r < 16; ++r) out[(32 * ph + acc_row(r, lane)) * N_ + 32 * nt + (lane & 31)] = (__bf16)acc[r];
        }
        SSDK_STAMP(4, 5);
    }
}

// ---------------------------------------------------------------------------------------------
// Inter-chunk state passing over a segment (four state elements per thread).  The running state is
// carried in fp32 registers (checkpoints and the final state are stored from them); the state
// entering each chunk is emitted as the bf16 copy the contraction kernels read, nothing else.
__device__ __forceinline__ bf16x4 to_bf16x4(const float4 v) {
    bf16x4 r;
    r[0] = (__bf16)v.x; r[1] = (__bf16)v.y; r[2] = (__bf16)v.z; r[3] = (__bf16)v.w;
    return r;
}

template <bool F32IN>  // F32IN: the chunk states arrive in fp32 (SSD_FLAG_FP32_CHUNK_STATES), else as bf16 in place
__global__ __launch_bounds__(NTH) void mk_scan_fwd(SegParams sp) {
    constexpr int PN = P_ * N_;
    const int e = (blockIdx.x * NTH + threadIdx.x) * 4, h = blockIdx.y, b = blockIdx.z;
    const int64_t bh = (int64_t)h * PN + e;
    float4 hc = sp.state_in ? *(const float4*)(sp.state_in + (int64_t)b * sp.state_in_bs + bh) : make_float4(0.f, 0.f, 0.f, 0.f);
    if (!sp.state_in && sp.state_in16) {  // bf16 checkpoint
        const bf16x4 v = *(const bf16x4*)(sp.state_in16 + (int64_t)b * sp.state_in_bs + bh);
        hc = make_float4((float)v[0], (float)v[1], (float)v[2], (float)v[3]);
    }
    if (sp.bnd_write) *(float4*)(sp.bnd_write + (int64_t)b * sp.bnd_write_bs + bh) = hc;
    if (sp.bnd_write16) *(bf16x4*)(sp.bnd_write16 + (int64_t)b * sp.bnd_write_bs + bh) = to_bf16x4(hc);
    const float* cum = sp.cum + ((int64_t)b * sp.H + h) * sp.nc * sp.Q;
    constexpr bool f32in = F32IN;
    constexpr int U = 8;  // chunks whose loads are in flight together (the recurrence itself is serial)
    for (int c0 = 0; c0 < sp.nc; c0 += U) {
        float4 sv[U];
        float av[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u < sp.nc ? c0 + u : sp.nc - 1;
            if (f32in) {  // chunk state kept in fp32 (an array of its own)
                sv[u] = *(const float4*)(sp.states + (((int64_t)b * sp.nc + c) * sp.H + h) * PN + e);
            } else {      // chunk state (bf16), about to be replaced in place by the state entering the chunk
                const bf16x4 sb = *(const bf16x4*)(sp.states_bf + (((int64_t)b * sp.nc + c) * sp.H + h) * PN + e);
                sv[u] = make_float4((float)sb[0], (float)sb[1], (float)sb[2], (float)sb[3]);
            }
            av[u] = cum[(int64_t)c * sp.Q + sp.Q - 1];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 + u;
            if (c < sp.nc) {
                const bf16x4 hb = to_bf16x4(hc);  // the entering state is kept in bf16 only
                *(bf16x4*)(sp.states_bf + (((int64_t)b * sp.nc + c) * sp.H + h) * PN + e) = hb;
                const float a = __expf(av[u]);
                const float4 s = sv[u];
                hc.x = a * hc.x + s.x; hc.y = a * hc.y + s.y; hc.z = a * hc.z + s.z; hc.w = a * hc.w + s.w;
            }
        }
    }
    if (sp.state_out) *(float4*)(sp.state_out + (int64_t)b * sp.state_out_bs + bh) = hc;
    if (sp.state_out2) *(float4*)(sp.state_out2 + (int64_t)b * sp.state_out2_bs + bh) = hc;
    if (sp.state_out16) *(bf16x4*)(sp.state_out16 + (int64_t)b * sp.state_out16_bs + bh) = to_bf16x4(hc);
}

// Reverse pass over the chunk-state adjoints; emits the bf16 copies and the per-wave partial sums
// of exp(T_c) <dHnext_c, Hprev_c>, the gradient of the chunk's total decay through the carried state
// (fixed summation order).
template <bool F32IN>
__global__ __launch_bounds__(NTH) void mk_scan_bwd(SegParams sp) {
    constexpr int PN = P_ * N_;
    const int e = (blockIdx.x * NTH + threadIdx.x) * 4, h = blockIdx.y, b = blockIdx.z;
    const int64_t ce = ((int64_t)b * sp.H + h) * PN + e;
    float4 g = *(const float4*)(sp.dcarry + ce);
    const float* cum = sp.cum + ((int64_t)b * sp.H + h) * sp.nc * sp.Q;
    constexpr bool f32in = F32IN;
    constexpr int U = 4;  // chunks whose loads are in flight together
    for (int c0 = sp.nc - 1; c0 >= 0; c0 -= U) {
        float4 lv[U], hv[U];
        float av[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 - u >= 0 ? c0 - u : 0;
            if (f32in) {  // local adjoint kept in fp32 (an array of its own)
                lv[u] = *(const float4*)(sp.dstates + (((int64_t)b * sp.nc + c) * sp.H + h) * PN + e);
            } else {      // local adjoint (bf16), about to be replaced in place by the total adjoint leaving the chunk
                const bf16x4 lb = *(const bf16x4*)(sp.dstates_bf + (((int64_t)b * sp.nc + c) * sp.H + h) * PN + e);
                lv[u] = make_float4((float)lb[0], (float)lb[1], (float)lb[2], (float)lb[3]);
            }
            av[u] = cum[(int64_t)c * sp.Q + sp.Q - 1];
            // state entering chunk c (bf16 copy)
            {
                const bf16x4 hb = *(const bf16x4*)(sp.states_bf + (((int64_t)b * sp.nc + c) * sp.H + h) * PN + e);
                hv[u] = make_float4((float)hb[0], (float)hb[1], (float)hb[2], (float)hb[3]);
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int c = c0 - u;
            if (c < 0) break;  // uniform
            bf16x4 gb;  // the total adjoint is kept in bf16 only
            gb[0] = (__bf16)g.x; gb[1] = (__bf16)g.y; gb[2] = (__bf16)g.z; gb[3] = (__bf16)g.w;
            *(bf16x4*)(sp.dstates_bf + (((int64_t)b * sp.nc + c) * sp.H + h) * PN + e) = gb;
            const float a = __expf(av[u]);
            const float4 hp = hv[u];
            float part = a * (g.x * hp.x + g.y * hp.y + g.z * hp.z + g.w * hp.w);
            for (int off = 32; off > 0; off >>= 1) part += __shfl_down(part, off, 64);
            if ((threadIdx.x & 63) == 0)  // one partial sum per wave; summed later in a fixed order
                sp.tail_part[(((int64_t)b * sp.H + h) * sp.nc + c) * sp.nslice + blockIdx.x * (NTH / 64) + (threadIdx.x >> 6)] = part;
            const float4 loc = lv[u];
            g.x = a * g.x + loc.x; g.y = a * g.y + loc.y; g.z = a * g.z + loc.z; g.w = a * g.w + loc.w;
        }
    }
    *(float4*)(sp.dcarry + ce) = g;
    if (sp.dinit_out) *(float4*)(sp.dinit_out + ce) = g;
}

template <int Q>
hipError_t fwd_q(const SegParams& sp, bool need_y, hipStream_t st) {
    constexpr int NB = Q / BLK;
    const int n_prep = sp.nc * sp.H * sp.Bt, n_cb = sp.Bt * sp.nc * sp.G * (NB * (NB + 1) / 2);
    if (Q == 256)
        SSDK_LAUNCH(K_MFMA_PREP_CB, st, mk_prep_cb, dim3(n_prep + n_cb), dim3(NTH), sp, n_prep);
    else
        SSDK_LAUNCH(K_CUMSUM, st, mk_prep<Q>, dim3(sp.nc, sp.H, sp.Bt), dim3(Q), sp);
    {   // chunk states; on the backward path (need_y false) the local state adjoints ride in the same launch
        SegParams so = sp;
        const int nroles = need_y ? 1 : 2;
        so.outer_split = pick_split(sp.hpg, (int64_t)sp.Bt * sp.nc * sp.G * nroles, sp.wg_target);
        if (sp.flags & SSD_FLAG_FP32_CHUNK_STATES)
            SSDK_LAUNCH(need_y ? K_MFMA_CHUNK_STATE : K_MFMA_DSTATE, st, (mk_chunk_outer<Q, true>), dim3(sp.Bt * sp.nc * sp.G * nroles * so.outer_split), dim3(OUTER_THR), so, nroles);
        else
            SSDK_LAUNCH(need_y ? K_MFMA_CHUNK_STATE : K_MFMA_DSTATE, st, (mk_chunk_outer<Q, false>), dim3(sp.Bt * sp.nc * sp.G * nroles * so.outer_split), dim3(OUTER_THR), so, nroles);
    }
    if (Q != 256) SSDK_LAUNCH(K_MFMA_CB, st, mk_cb<Q>, dim3(sp.Bt * sp.nc * sp.G, NB * (NB + 1) / 2), dim3(NTH), sp);
    // the scan is the only step that needs the previous segment (its leaving state)
    if (need_y && sp.ev_wait && hipStreamWaitEvent(st, sp.ev_wait, 0) != hipSuccess) return hipErrorUnknown;
    if (sp.flags & SSD_FLAG_FP32_CHUNK_STATES)
        SSDK_LAUNCH(K_SCAN_FWD, st, mk_scan_fwd<true>, dim3(P_ * N_ / 4 / NTH, sp.H, sp.Bt), dim3(NTH), sp);
    else
        SSDK_LAUNCH(K_SCAN_FWD, st, mk_scan_fwd<false>, dim3(P_ * N_ / 4 / NTH, sp.H, sp.Bt), dim3(NTH), sp);
    if (need_y && sp.ev_record && hipEventRecord(sp.ev_record, st) != hipSuccess) return hipErrorUnknown;
    if (need_y) {
        hipError_t e = mfma_launch_dual(sp, 0, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <int Q>
hipError_t bwd_q(const SegParams& sp0, hipStream_t st) {
    SegParams sp = sp0;
    sp.nslice = P_ * N_ / 4 / 64;  // partial sums written by mk_scan_bwd: one per wave
    // the reverse scan is the only step that needs the segment to the right (its entering-state adjoint)
    if (sp.ev_wait && hipStreamWaitEvent(st, sp.ev_wait, 0) != hipSuccess) return hipErrorUnknown;
    if (sp.flags & SSD_FLAG_FP32_CHUNK_STATES)
        SSDK_LAUNCH(K_SCAN_BWD, st, mk_scan_bwd<true>, dim3(P_ * N_ / 4 / NTH, sp.H, sp.Bt), dim3(NTH), sp);
    else
        SSDK_LAUNCH(K_SCAN_BWD, st, mk_scan_bwd<false>, dim3(P_ * N_ / 4 / NTH, sp.H, sp.Bt), dim3(NTH), sp);
    if (sp.ev_record && hipEventRecord(sp.ev_record, st) != hipSuccess) return hipErrorUnknown;
    // dx, dG and the dB / dC head sums (which also write the chunk-local part of the gradient of cum
    // and the state dot products): one launch when the three share a workgroup size
    const bool trio = Q == 256;
    hipError_t e = trio ? hipSuccess : mfma_launch_dual(sp, 2, st);
    if (e != hipSuccess) return e;
    sp.flags |= SSD_INTERNAL_SPLIT_GTERM;  // the gradient of cum arrives in three pieces
    e = mfma_launch_grad_bc(sp, trio, st);   // chunk 256: ddt and the dA / dD partial sums ride in its last launch
    if (e != hipSuccess) return e;
    if (Q != 256) {
        e = generic_backward_scalars(sp, st);
        if (e != hipSuccess) return e;
    } else if (!sp.defer_param) {
        e = launch_param_reduce(sp, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

bool mfma_path_supported(const ssd_shape_t& s) {
    return s.dtype == SSD_BF16 && s.headdim == P_ && s.dstate == N_ && (s.chunk == 64 || s.chunk == 128 || s.chunk == 256);
}

hipError_t mfma_forward_segment(const SegParams& sp, bool need_y, hipStream_t st) {
    switch (sp.Q) {
        case 64: return fwd_q<64>(sp, need_y, st);
        case 128: return fwd_q<128>(sp, need_y, st);
        case 256: return fwd_q<256>(sp, need_y, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t mfma_backward_segment(const SegParams& sp, hipStream_t st) {
    switch (sp.Q) {
        case 64: return bwd_q<64>(sp, st);
        case 128: return bwd_q<128>(sp, st);
        case 256: return bwd_q<256>(sp, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ssdk
