// C-ABI entry points for one SSD layer: argument validation, workspace partitioning and the
// segment loops of the MA-GC sequence axis (paper Sec. 3.2/3.3, Alg. 1 and Alg. 2).
#include <stdlib.h>
#include <string.h>

#include <mutex>

#include "ssd_internal.h"

namespace ssdk {

inline size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }

int pick_split(int heads_per_group, int64_t base, int target) {
    for (int ns = 1; ns <= heads_per_group; ++ns)
        if (heads_per_group % ns == 0 && base * ns >= target) return ns;
    return heads_per_group;
}

// Returns SSD_OK and fills d, or the validation error.
int check_shape(const ssd_shape_t* sh, Dims* d) {
    if (!sh) return SSD_ERR_NULL;
    if (sh->dtype != SSD_F32 && sh->dtype != SSD_BF16) return SSD_ERR_DTYPE;
    if (sh->batch <= 0 || sh->seqlen < 0 || sh->nheads <= 0 || sh->headdim <= 0 || sh->ngroups <= 0 ||
        sh->dstate <= 0 || sh->chunk <= 0)
        return SSD_ERR_SHAPE;
    if (sh->chunk > 1024 || sh->headdim > 256 || sh->dstate > 256) return SSD_ERR_SHAPE;
    if (sh->batch > 65535 || sh->nheads > 65535) return SSD_ERR_SHAPE;
    if (sh->nheads % sh->ngroups != 0) return SSD_ERR_DIVISIBILITY;
    if (sh->seqlen > 0) {
        if (sh->segment <= 0) return SSD_ERR_SHAPE;
        if (sh->segment % sh->chunk != 0) return SSD_ERR_DIVISIBILITY;
    }
    d->Bt = sh->batch;
    d->L = sh->seqlen;
    d->s = sh->seqlen > 0 ? sh->segment : 0;
    d->H = sh->nheads;
    d->P = sh->headdim;
    d->G = sh->ngroups;
    d->N = sh->dstate;
    d->Q = sh->chunk;
    d->hpg = d->H / d->G;
    d->nc = sh->seqlen > 0 ? (int)(sh->segment / sh->chunk) : 0;
    d->nseg = sh->seqlen > 0 ? (sh->seqlen + sh->segment - 1) / sh->segment : 0;
    d->tail = sh->seqlen > 0 ? sh->seqlen % sh->segment : 0;
    d->nc_tail = (int)((d->tail + sh->chunk - 1) / sh->chunk);
    d->bf16 = sh->dtype == SSD_BF16;
    d->esz = d->bf16 ? 2 : 4;
    d->xs_b = sh->x_batch_stride ? sh->x_batch_stride : d->L * d->H * d->P;
    d->dts_b = sh->dt_batch_stride ? sh->dt_batch_stride : d->L * d->H;
    d->bcs_b = sh->bc_batch_stride ? sh->bc_batch_stride : d->L * d->G * d->N;
    d->reset = sh->seq_reset;
    if (d->xs_b < d->L * d->H * d->P || d->dts_b < d->L * d->H || d->bcs_b < d->L * d->G * d->N) return SSD_ERR_SHAPE;
    // every launch keeps its largest grid dimension below 2^31
    const int64_t blocks = d->Bt * (int64_t)d->nc * d->H * 2;
    if (blocks >= ((int64_t)1 << 31) || (int64_t)sh->segment / sh->chunk >= ((int64_t)1 << 24)) return SSD_ERR_SHAPE;
    return SSD_OK;
}

WsLayout ws_layout(const Dims& d, bool bwd, bool mfma, int wg_target, bool fp32cs) {
    WsLayout w;
    memset(&w, 0, sizeof(w));
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off += align_up(bytes);
        return o;
    };
    const size_t tok = (size_t)d.Bt * d.H * d.nc * d.Q * 4;
    const size_t PN = (size_t)d.P * d.N;
    w.nslice = (int)((PN + 255) / 256);
    w.cum = take(tok);
    w.dtf = take(tok);
    w.states = w.states_bf = w.dstates = w.dstates_bf = w.dbc_part = WS_NONE;  // present on one path only
    if (!mfma) w.states = take((size_t)d.Bt * (d.nc + 1) * d.H * PN * 4);
    if (mfma && fp32cs) w.states = take((size_t)d.Bt * d.nc * d.H * PN * 4);  // slot c: chunk state c (scan input)
    w.Gm = take((size_t)d.Bt * d.nc * d.G * d.Q * d.Q * 4);
    w.ein = take(tok);
    w.eout = take(tok);
    if (mfma) w.states_bf = take((size_t)d.Bt * d.nc * d.H * PN * 2);
    const int64_t groups = d.Bt * (int64_t)d.nc * d.G;
    w.dg_split = pick_split(d.hpg, groups, wg_target);
    w.part_split = pick_split(d.hpg, groups * 2, wg_target);
    if (bwd) {
        if (!mfma || fp32cs) w.dstates = take((size_t)d.Bt * d.nc * d.H * PN * 4);
        if (mfma) w.dstates_bf = take((size_t)d.Bt * d.nc * d.H * PN * 2);
        {   // fp32 head sum (generic kernels) or one bf16 partial sum per head slice (MFMA kernels)
            const size_t per = mfma ? (size_t)d.Q * d.Q * 2 * w.dg_split : (size_t)d.Q * d.Q * 4;
            w.dG = take((size_t)d.Bt * d.nc * d.G * per);
        }
        if (mfma) w.dbc_part = take((size_t)d.Bt * d.nc * d.G * w.part_split * 2 * d.Q * d.N * 4);
        w.gterm = take(tok);
        w.sterm = take(tok);
        w.gintra = take(tok);
        w.fterm = take(tok);
        w.dDrow = take(tok);
        w.tail_part = take((size_t)d.Bt * d.H * d.nc * w.nslice * 4);
        w.dA_part = take((size_t)d.Bt * d.nc * d.H * 4);
        w.dD_part = take((size_t)d.Bt * d.nc * d.H * 4);
        w.dcarry = take((size_t)d.Bt * d.H * PN * 4);
    }
    w.total = off;
    return w;
}

void bind_workspace(SegParams& sp, const WsLayout& w, void* workspace, bool bwd) {
    char* base = (char*)workspace;
    auto at = [&](size_t off) { return off == WS_NONE ? nullptr : base + off; };
    sp.cum = (float*)(base + w.cum);
    sp.dtf = (float*)(base + w.dtf);
    sp.states = (float*)at(w.states);
    sp.Gm = (float*)(base + w.Gm);
    sp.nslice = w.nslice;
    sp.ein = (float*)(base + w.ein);
    sp.eout = (float*)(base + w.eout);
    sp.states_bf = (bf16_t*)at(w.states_bf);
    sp.dg_split = w.dg_split;
    sp.part_split = w.part_split;
    if (bwd) {
        sp.dstates_bf = (bf16_t*)at(w.dstates_bf);
        sp.dbc_part = (float*)at(w.dbc_part);
        sp.dstates = (float*)at(w.dstates);
        sp.dG = (float*)(base + w.dG);
        sp.gterm = (float*)(base + w.gterm);
        sp.sterm = (float*)(base + w.sterm);
        sp.gintra = (float*)(base + w.gintra);
        sp.fterm = (float*)(base + w.fterm);
        sp.dDrow = (float*)(base + w.dDrow);
        sp.tail_part = (float*)(base + w.tail_part);
        sp.dA_part = (float*)(base + w.dA_part);
        sp.dD_part = (float*)(base + w.dD_part);
        sp.dcarry = (float*)(base + w.dcarry);
    }
}

void base_params(SegParams& sp, const Dims& d, uint32_t flags) {
    memset(&sp, 0, sizeof(sp));
    sp.Bt = (int)d.Bt;
    sp.H = d.H;
    sp.P = d.P;
    sp.G = d.G;
    sp.N = d.N;
    sp.Q = d.Q;
    sp.nc = d.nc;
    sp.hpg = d.hpg;
    sp.xs_b = sp.ys_b = sp.dys_b = sp.dxs_b = d.xs_b;
    sp.dts_b = d.dts_b;
    sp.bcs_b = d.bcs_b;
    sp.flags = flags;
    sp.nc_total = d.nc;
    sp.wg_target = 256;
#ifdef SSDK_STAMPS
    sp.stamps = g_stamps;
#endif
}

static inline const void* off(const void* p, int64_t elems, size_t esz) { return p ? (const char*)p + elems * (int64_t)esz : nullptr; }
static inline void* off(void* p, int64_t elems, size_t esz) { return p ? (char*)p + elems * (int64_t)esz : nullptr; }

bool use_mfma(const ssd_shape_t& sh, uint32_t flags) {
    return !(flags & SSD_FLAG_GENERIC_KERNELS) && mfma_path_supported(sh);
}

// Points the scan of segment k at its entering state and at the places its leaving state goes.
static void wire_states(SegParams& sp, const Dims& d, int64_t k, const float* init_state, const float* bnd_ro,
                        float* bnd_rw, float* final_state) {
    const int64_t HPN = (int64_t)d.H * d.P * d.N;
    if (k == 0 || !bnd_ro) {
        sp.state_in = init_state;
        sp.state_in_bs = HPN;
    } else {
        sp.state_in = bnd_ro + k * HPN;
        sp.state_in_bs = d.nseg * HPN;
    }
    sp.bnd_write = nullptr;
    sp.state_out = nullptr;
    sp.state_out2 = nullptr;
    sp.state_in16 = nullptr;
    sp.bnd_write16 = nullptr;
    sp.state_out16 = nullptr;
    if (bnd_rw) {
        if (k == 0) {
            sp.bnd_write = bnd_rw;
            sp.bnd_write_bs = d.nseg * HPN;
        }
        if (k + 1 < d.nseg) {
            sp.state_out = bnd_rw + (k + 1) * HPN;
            sp.state_out_bs = d.nseg * HPN;
        }
    }
    if (k + 1 == d.nseg && final_state) {
        sp.state_out2 = final_state;
        sp.state_out2_bs = HPN;
    }
}

// ---- several segments in flight ---------------------------------------------------------------
// Consecutive segments depend on each other only through the state scan.  With more than one
// segment, segment k runs on lane k % NPIPE -- lane 0 is the caller's stream, the others are internal
// streams (default priority) -- each lane with its own per-segment scratch; events order the scans.
// This overlaps one segment's launch gaps, tails and bandwidth-bound kernels with another's matrix work.
constexpr int NPIPE = 4;  // segments in flight (the caller's stream + NPIPE - 1 internal ones)
struct Pipe {
    hipStream_t aux[NPIPE] = {};       // aux[0] is unused: lane 0 is the caller's stream
    hipEvent_t fork = nullptr, join[NPIPE] = {}, scan[NPIPE] = {};
    bool ok = false;
};

// Created on the first call that needs them on a device (or by ssd_init), under a lock; a partial failure
// releases what was created and leaves the entry unset, so that a later call tries again.
static std::mutex g_pipe_mu;

static Pipe* pipe_for_current_device() {
    static Pipe pipes[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(g_pipe_mu);
    Pipe& p = pipes[dev];
    if (p.ok) return &p;
    Pipe q;
    bool good = hipEventCreateWithFlags(&q.fork, hipEventDisableTiming) == hipSuccess;
    for (int i = 0; good && i < NPIPE; ++i) {
        if (i > 0) good = hipStreamCreateWithFlags(&q.aux[i], hipStreamNonBlocking) == hipSuccess;
        good = good && hipEventCreateWithFlags(&q.join[i], hipEventDisableTiming) == hipSuccess;
        good = good && hipEventCreateWithFlags(&q.scan[i], hipEventDisableTiming) == hipSuccess;
    }
    if (!good) {
        if (q.fork) (void)hipEventDestroy(q.fork);
        for (int i = 0; i < NPIPE; ++i) {
            if (q.aux[i]) (void)hipStreamDestroy(q.aux[i]);
            if (q.join[i]) (void)hipEventDestroy(q.join[i]);
            if (q.scan[i]) (void)hipEventDestroy(q.scan[i]);
        }
        return nullptr;
    }
    q.ok = true;
    p = q;
    return &p;
}

// Forward without checkpoints (boundary_states == NULL, several segments): the state leaving one
// segment reaches the next through two buffers used alternately (the scans are ordered by events, so
// a buffer is rewritten only after its reader has finished).
static size_t carry_bytes(const Dims& d) { return d.nseg > 1 ? 2 * align_up((size_t)d.Bt * d.H * d.P * d.N * 4) : 0; }

// A short last segment (seqlen not a multiple of segment, or of chunk) is run on padded copies of its
// tokens: the padding tokens have dt = 0 and x = B = C = dy = 0, i.e. they are identity steps of the
// recurrence that add nothing to any gradient.  Offsets (bytes) of the copies behind the scratch blocks.
struct TailStage {
    size_t x, dt, B, C, y, dy, dx, ddt, dB, dC, reset, total;
    int64_t T;  // tokens of the padded segment
};
static TailStage tail_stage(const Dims& d, bool bwd) {
    TailStage t;
    memset(&t, 0, sizeof(t));
    if (!d.tail) return t;
    t.T = (int64_t)d.nc_tail * d.Q;
    size_t off = 0;
    auto take = [&](size_t row_elems) {
        size_t o = off;
        off += align_up((size_t)d.Bt * t.T * row_elems * d.esz);
        return o;
    };
    const size_t hp = (size_t)d.H * d.P, gn = (size_t)d.G * d.N;
    t.x = take(hp);
    t.dt = take(d.H);
    t.B = take(gn);
    t.C = take(gn);
    if (!bwd) {
        t.y = take(hp);
    } else {
        t.dy = take(hp);
        t.dx = take(hp);
        t.ddt = take(d.H);
        t.dB = take(gn);
        t.dC = take(gn);
    }
    if (d.reset) {
        t.reset = off;
        off += align_up((size_t)d.Bt * t.T);
    }
    t.total = off;
    return t;
}

// Bytes of the arrays shared by all scratch blocks: the dA / dD partial sums of every chunk.
static size_t shared_bytes(const Dims& d) { return 2 * align_up((size_t)d.Bt * d.nseg * d.nc * d.H * 4); }

// SSD_MAGC_SERIAL=1 in the environment keeps every segment on the caller's stream (diagnostics: per-kernel
// timings are only meaningful when kernels do not overlap).
static bool g_serial = false;  // ssd_prof_serialize

bool serial_mode() {
    static const bool serial = [] {
        const char* v = getenv("SSD_MAGC_SERIAL");
        return v && v[0] == '1';
    }();
    return serial || g_serial;
}

// SSD_MAGC_LANES=n (1 .. NPIPE) in the environment caps the segments in flight (measurements; the default is NPIPE).
static int lanes(const Dims& d, bool mfma, bool one_stream = false) {
    static const int cap = [] {
        const char* v = getenv("SSD_MAGC_LANES");
        const int n = v ? atoi(v) : NPIPE;
        return n < 1 ? 1 : (n > NPIPE ? NPIPE : n);
    }();
    if (!mfma || one_stream || serial_mode() || d.nseg <= 1) return 1;
    return d.nseg < cap ? (int)d.nseg : cap;
}

// Workgroups a launch should have at least.  One segment at a time: one per compute unit.  Several
// segments in flight: half as many, twice as long -- launches of the other lanes fill the machine, and
// the per-workgroup prologue (fetching the operands shared by all heads) is paid half as often.
static int wg_target(int nlanes) { return nlanes > 1 ? 128 : 256; }

static bool fork_lanes(Pipe* pp, int n, hipStream_t st) {
    if (n <= 1) return true;
    if (hipEventRecord(pp->fork, st) != hipSuccess) return false;
    for (int i = 1; i < n; ++i)
        if (hipStreamWaitEvent(pp->aux[i], pp->fork, 0) != hipSuccess) return false;
    return true;
}

static bool join_lanes(Pipe* pp, int n, hipStream_t st) {
    for (int i = 1; i < n; ++i)
        if (hipEventRecord(pp->join[i], pp->aux[i]) != hipSuccess || hipStreamWaitEvent(st, pp->join[i], 0) != hipSuccess) return false;
    return true;
}

}  // namespace ssdk

using namespace ssdk;

#ifdef SSDK_STAMPS
namespace ssdk {
unsigned long long* g_stamps = nullptr;
}
extern "C" void ssd_debug_stamps(void* p) { ssdk::g_stamps = (unsigned long long*)p; }
#endif

extern "C" size_t ssd_workspace_bytes_flags(const ssd_shape_t* shape, int32_t is_backward, uint32_t flags) {
    Dims d;
    if (check_shape(shape, &d) != SSD_OK) return 0;
    // never 0 for a valid shape, so that 0 unambiguously means "invalid"
    const bool mfma = use_mfma(*shape, flags);
    const int nl = lanes(d, mfma);
    const size_t block = align_up(ws_layout(d, is_backward != 0, mfma, wg_target(nl), (flags & SSD_FLAG_FP32_CHUNK_STATES) != 0).total);
    const size_t t = nl * block + (is_backward ? shared_bytes(d) : carry_bytes(d)) + tail_stage(d, is_backward != 0).total;
    return t ? t : 256;
}

extern "C" size_t ssd_workspace_bytes(const ssd_shape_t* shape, int32_t is_backward) {
    return ssd_workspace_bytes_flags(shape, is_backward, 0);
}

// one_stream: everything stays on the caller's stream (no library stream or event is touched).
static int fwd_impl(const ssd_shape_t* shape, const void* x, const void* dt, const float* A, const void* B,
                    const void* C, const float* D, const float* init_state, void* y, float* final_state,
                    void* boundary_states, void* workspace, size_t workspace_bytes, uint32_t flags,
                    void* hip_stream, bool one_stream) {
    Dims d;
    int rc = check_shape(shape, &d);
    if (rc != SSD_OK) return rc;
    if (flags & ~(uint32_t)(SSD_FLAG_RESIDUAL | SSD_FLAG_GENERIC_KERNELS | SSD_FLAG_ACCUM_PARAM | SSD_FLAG_BF16_CHECKPOINTS | SSD_FLAG_FP32_CHUNK_STATES))
        return SSD_ERR_ARG;
    const bool ck16 = (flags & SSD_FLAG_BF16_CHECKPOINTS) && boundary_states;
    float* bnd32 = ck16 ? nullptr : (float*)boundary_states;
    bf16_t* bnd16 = ck16 ? (bf16_t*)boundary_states : nullptr;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t HPN = (size_t)d.H * d.P * d.N;
    if (d.L == 0) {  // empty sequence: the state passes through untouched
        if (final_state) {
            hipError_t e = init_state ? launch_copy_f32(final_state, init_state, (size_t)d.Bt * HPN, st)
                                      : launch_fill_zero(final_state, (size_t)d.Bt * HPN, st);
            if (e != hipSuccess) return SSD_ERR_LAUNCH;
        }
        return SSD_OK;
    }
    if (!x || !dt || !A || !B || !C || !D || !y) return SSD_ERR_NULL;
    const bool mfma = use_mfma(*shape, flags);
    const int nl = lanes(d, mfma, one_stream);
    const WsLayout w = ws_layout(d, false, mfma, wg_target(nl), (flags & SSD_FLAG_FP32_CHUNK_STATES) != 0);
    const size_t block = align_up(w.total);
    const TailStage ts = tail_stage(d, false);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < nl * block + carry_bytes(d) + ts.total) return SSD_ERR_WORKSPACE;
    char* stage = (char*)workspace + nl * block + carry_bytes(d);
    float* carry[2] = {(float*)((char*)workspace + nl * block), (float*)((char*)workspace + nl * block + carry_bytes(d) / 2)};
    Pipe* pp = nl > 1 ? pipe_for_current_device() : nullptr;
    if (nl > 1 && !pp) return SSD_ERR_LAUNCH;

    SegParams sps[NPIPE];
    for (int i = 0; i < nl; ++i) {
        base_params(sps[i], d, flags);
        sps[i].wg_target = wg_target(nl);
        bind_workspace(sps[i], w, (char*)workspace + i * block, false);
        sps[i].A = A;
        sps[i].D = D;
    }
    if (!fork_lanes(pp, nl, st)) return SSD_ERR_LAUNCH;
    for (int64_t k = 0; k < d.nseg; ++k) {
        const int ln = (int)(k % nl);
        SegParams& sp = sps[ln];
        hipStream_t sk = ln ? pp->aux[ln] : st;
        const int64_t t0 = k * d.s;
        const bool short_seg = d.tail && k + 1 == d.nseg;
        const int HP = d.H * d.P, GN = d.G * d.N;
        if (!short_seg) {
            sp.x = off(x, t0 * HP, d.esz);
            sp.y = off(y, t0 * HP, d.esz);
            sp.dt = off(dt, t0 * d.H, d.esz);
            sp.Bm = off(B, t0 * GN, d.esz);
            sp.Cm = off(C, t0 * GN, d.esz);
            sp.xs_b = sp.ys_b = d.xs_b;
            sp.dts_b = d.dts_b;
            sp.bcs_b = d.bcs_b;
            sp.nc = d.nc;
            sp.reset = d.reset ? d.reset + t0 : nullptr;
            sp.reset_bs = d.L;
        } else {  // padded copies of the last tokens (see TailStage)
            const int tv = (int)d.tail, T = (int)ts.T;
            hipError_t es = launch_stage_rows(stage + ts.x, (int64_t)T * HP, off(x, t0 * HP, d.esz), d.xs_b, tv, T, HP, sp.Bt, d.esz, sk);
            if (es == hipSuccess) es = launch_stage_rows(stage + ts.dt, (int64_t)T * d.H, off(dt, t0 * d.H, d.esz), d.dts_b, tv, T, d.H, sp.Bt, d.esz, sk);
            if (es == hipSuccess) es = launch_stage_rows(stage + ts.B, (int64_t)T * GN, off(B, t0 * GN, d.esz), d.bcs_b, tv, T, GN, sp.Bt, d.esz, sk);
            if (es == hipSuccess) es = launch_stage_rows(stage + ts.C, (int64_t)T * GN, off(C, t0 * GN, d.esz), d.bcs_b, tv, T, GN, sp.Bt, d.esz, sk);
            if (es == hipSuccess && d.reset) es = launch_stage_rows(stage + ts.reset, T, d.reset + t0, d.L, tv, T, 1, sp.Bt, 1, sk);
            if (es != hipSuccess) {
                (void)join_lanes(pp, nl, st);
                return SSD_ERR_LAUNCH;
            }
            sp.x = stage + ts.x;
            sp.y = stage + ts.y;
            sp.dt = stage + ts.dt;
            sp.Bm = stage + ts.B;
            sp.Cm = stage + ts.C;
            sp.xs_b = sp.ys_b = (int64_t)T * HP;
            sp.dts_b = (int64_t)T * d.H;
            sp.bcs_b = (int64_t)T * GN;
            sp.nc = d.nc_tail;
            sp.reset = d.reset ? (const uint8_t*)(stage + ts.reset) : nullptr;
            sp.reset_bs = T;
        }
        wire_states(sp, d, k, init_state, bnd32, bnd32, final_state);
        if (bnd16) {  // bf16 checkpoints: rounded copies; the fp32 state itself travels through the carry buffers
            if (k == 0) {
                sp.bnd_write16 = bnd16;
                sp.bnd_write_bs = d.nseg * (int64_t)HPN;
            }
            if (k + 1 < d.nseg) {
                sp.state_out16 = bnd16 + (k + 1) * (int64_t)HPN;
                sp.state_out16_bs = d.nseg * (int64_t)HPN;
            }
        }
        if (!bnd32 && d.nseg > 1) {  // no fp32 checkpoints: hand the state on through the carry buffers
            if (k > 0) {
                sp.state_in = carry[k & 1];
                sp.state_in_bs = (int64_t)HPN;
            }
            if (k + 1 < d.nseg) {
                sp.state_out = carry[(k + 1) & 1];
                sp.state_out_bs = (int64_t)HPN;
            }
        }
        sp.ev_wait = (nl > 1 && k > 0) ? pp->scan[(k - 1) % nl] : nullptr;
        sp.ev_record = (nl > 1 && k + 1 < d.nseg) ? pp->scan[ln] : nullptr;
        hipError_t e = mfma ? mfma_forward_segment(sp, true, sk) : generic_forward_segment(sp, d.bf16, true, sk);
        if (e == hipSuccess && short_seg)  // the valid rows of y go back to the caller's tensor
            e = launch_stage_rows(off(y, t0 * HP, d.esz), d.xs_b, stage + ts.y, (int64_t)ts.T * HP, (int)d.tail, (int)d.tail, HP, sp.Bt, d.esz, sk);
        if (e != hipSuccess) {
            (void)join_lanes(pp, nl, st);  // whatever was enqueued on the library's streams still ends before the caller's next work
            return SSD_ERR_LAUNCH;
        }
    }
    if (!join_lanes(pp, nl, st)) return SSD_ERR_LAUNCH;
    return SSD_OK;
}

extern "C" int ssd_fwd(const ssd_shape_t* shape, const void* x, const void* dt, const float* A, const void* B,
                       const void* C, const float* D, const float* init_state, void* y, float* final_state,
                       void* boundary_states, void* workspace, size_t workspace_bytes, uint32_t flags,
                       void* hip_stream) {
    return fwd_impl(shape, x, dt, A, B, C, D, init_state, y, final_state, boundary_states, workspace, workspace_bytes,
                    flags, hip_stream, false);
}

// ---- forward pass for callers that cannot allocate -------------------------------------------------
// The per-segment scratch lives in a file-scope device array instead of a caller's workspace.  Every
// device the library runs on holds its own copy of the array, at its own address, until the process ends;
// the address is looked up once per device (hipGetSymbolAddress with that device current) and only that
// pointer -- never the array's name, which in host code is a stand-in and not a device address -- is
// handed to the kernels.
namespace ssdk {
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)SSD_STATIC_SCRATCH_MIB << 20;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];

static std::mutex g_scratch_mu;
static void* g_scratch_ptr[64] = {};

// The array's address on the current device (looked up on first use there), or NULL on failure.
static void* static_scratch() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
        g_scratch_ptr[dev] = p;
    }
    return g_scratch_ptr[dev];
}

// Scratch bytes of a forward call that stays on one stream.
static size_t fwd_bytes_one_stream(const ssd_shape_t* shape, uint32_t flags) {
    Dims d;
    if (check_shape(shape, &d) != SSD_OK) return 0;
    const bool mfma = use_mfma(*shape, flags);
    const size_t t = align_up(ws_layout(d, false, mfma, wg_target(1), (flags & SSD_FLAG_FP32_CHUNK_STATES) != 0).total) + carry_bytes(d) + tail_stage(d, false).total;
    return t ? t : 256;
}
}  // namespace ssdk

extern "C" int ssd_init(void) {
    // everything the library creates lazily on a device: the scratch array's address, the streams and events of
    // the segments in flight, the side stream of the projections
    const bool a = static_scratch() != nullptr, b = pipe_for_current_device() != nullptr;
    const bool c = serial_mode() || side_stream() != nullptr;
    return a && b && c ? SSD_OK : SSD_ERR_LAUNCH;
}

extern "C" size_t ssd_fwd_static_bytes(const ssd_shape_t* shape, uint32_t flags) { return fwd_bytes_one_stream(shape, flags); }

extern "C" int ssd_fwd_static(const ssd_shape_t* shape, const void* x, const void* dt, const float* A, const void* B,
                              const void* C, const float* D, const float* init_state, void* y, float* final_state,
                              void* boundary_states, uint32_t flags, void* hip_stream) {
    Dims d;
    const int rc = check_shape(shape, &d);
    if (rc != SSD_OK) return rc;
    const size_t need = fwd_bytes_one_stream(shape, flags);
    if (need > STATIC_SCRATCH_BYTES) return SSD_ERR_WORKSPACE;  // beyond the array: use ssd_fwd with a workspace
    void* ws = static_scratch();
    if (!ws) return SSD_ERR_LAUNCH;
    // Nothing in the scratch has to start at zero: every array in it is written by the kernel that
    // precedes its first reader within the same call.
    return fwd_impl(shape, x, dt, A, B, C, D, init_state, y, final_state, boundary_states, ws, need, flags, hip_stream, true);
}

extern "C" int ssd_bwd(const ssd_shape_t* shape, const void* x, const void* dt, const float* A, const void* B,
                       const void* C, const float* D, const float* init_state, const void* dy,
                       const float* dfinal_state, const void* boundary_states, void* dx, void* ddt, float* dA,
                       void* dB, void* dC, float* dD, float* dinit_state, void* workspace, size_t workspace_bytes,
                       uint32_t flags, void* hip_stream) {
    Dims d;
    int rc = check_shape(shape, &d);
    if (rc != SSD_OK) return rc;
    if (flags & ~(uint32_t)(SSD_FLAG_RESIDUAL | SSD_FLAG_GENERIC_KERNELS | SSD_FLAG_ACCUM_PARAM | SSD_FLAG_BF16_CHECKPOINTS | SSD_FLAG_FP32_CHUNK_STATES))
        return SSD_ERR_ARG;
    const bool ck16 = (flags & SSD_FLAG_BF16_CHECKPOINTS) && boundary_states;
    if (!dA || !dD) return SSD_ERR_NULL;
    hipStream_t st = (hipStream_t)hip_stream;
    const size_t HPN = (size_t)d.H * d.P * d.N;
    if (d.L == 0) {  // empty sequence: the state adjoint passes through, parameter gradients are zero
        hipError_t e = hipSuccess;
        if (dinit_state)
            e = dfinal_state ? launch_copy_f32(dinit_state, dfinal_state, (size_t)d.Bt * HPN, st)
                             : launch_fill_zero(dinit_state, (size_t)d.Bt * HPN, st);
        if (e == hipSuccess && !(flags & SSD_FLAG_ACCUM_PARAM)) {
            e = launch_fill_zero(dA, d.H, st);
            if (e == hipSuccess) e = launch_fill_zero(dD, d.H, st);
        }
        return e == hipSuccess ? SSD_OK : SSD_ERR_LAUNCH;
    }
    if (!x || !dt || !A || !B || !C || !D || !dy || !dx || !ddt || !dB || !dC) return SSD_ERR_NULL;
    if (dx == dy) return SSD_ERR_ARG;
    if (!boundary_states && d.nseg > 1) return SSD_ERR_NULL;
    const bool mfma = use_mfma(*shape, flags);
    const int nl = lanes(d, mfma);
    const WsLayout w = ws_layout(d, true, mfma, wg_target(nl), (flags & SSD_FLAG_FP32_CHUNK_STATES) != 0);
    const size_t block = align_up(w.total);
    const TailStage ts = tail_stage(d, true);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < nl * block + shared_bytes(d) + ts.total) return SSD_ERR_WORKSPACE;
    char* stage = (char*)workspace + nl * block + shared_bytes(d);
    Pipe* pp = nl > 1 ? pipe_for_current_device() : nullptr;
    if (nl > 1 && !pp) return SSD_ERR_LAUNCH;

    // shared by all scratch blocks: the carried state adjoint and the dA / dD partial sums of every chunk
    float* part_all = (float*)((char*)workspace + nl * block);
    SegParams sps[NPIPE];
    for (int i = 0; i < nl; ++i) {
        SegParams& sp = sps[i];
        base_params(sp, d, flags);
        sp.wg_target = wg_target(nl);
        bind_workspace(sp, w, (char*)workspace + i * block, true);
        sp.A = A;
        sp.D = D;
        sp.dA = dA;
        sp.dD = dD;
        sp.dcarry = sps[0].dcarry;
        sp.dA_part = part_all;
        sp.dD_part = (float*)((char*)part_all + shared_bytes(d) / 2);
        sp.nc_total = (int)(d.tail ? (d.nseg - 1) * d.nc + d.nc_tail : d.nseg * d.nc);  // chunks that write dA / dD partial sums
        sp.defer_param = 1;
    }
    hipError_t e = dfinal_state ? launch_copy_f32(sps[0].dcarry, dfinal_state, (size_t)d.Bt * HPN, st)
                                : launch_fill_zero(sps[0].dcarry, (size_t)d.Bt * HPN, st);
    if (e != hipSuccess) return SSD_ERR_LAUNCH;
    if (!fork_lanes(pp, nl, st)) return SSD_ERR_LAUNCH;
    for (int64_t k = d.nseg - 1, it = 0; k >= 0; --k, ++it) {
        const int ln = (int)(it % nl);
        SegParams& sp = sps[ln];
        hipStream_t sk = ln ? pp->aux[ln] : st;
        const int64_t t0 = k * d.s;
        const bool short_seg = d.tail && k + 1 == d.nseg;
        const int HP = d.H * d.P, GN = d.G * d.N;
        if (!short_seg) {
            sp.x = off(x, t0 * HP, d.esz);
            sp.dy = off(dy, t0 * HP, d.esz);
            sp.dx = off(dx, t0 * HP, d.esz);
            sp.dt = off(dt, t0 * d.H, d.esz);
            sp.ddt = off(ddt, t0 * d.H, d.esz);
            sp.Bm = off(B, t0 * GN, d.esz);
            sp.Cm = off(C, t0 * GN, d.esz);
            sp.dB = off(dB, t0 * GN, d.esz);
            sp.dC = off(dC, t0 * GN, d.esz);
            sp.xs_b = sp.ys_b = sp.dys_b = sp.dxs_b = d.xs_b;
            sp.dts_b = d.dts_b;
            sp.bcs_b = d.bcs_b;
            sp.nc = d.nc;
            sp.reset = d.reset ? d.reset + t0 : nullptr;
            sp.reset_bs = d.L;
        } else {  // padded copies of the last tokens (see TailStage); results come back after the segment
            const int tv = (int)d.tail, T = (int)ts.T;
            e = launch_stage_rows(stage + ts.x, (int64_t)T * HP, off(x, t0 * HP, d.esz), d.xs_b, tv, T, HP, sp.Bt, d.esz, sk);
            if (e == hipSuccess) e = launch_stage_rows(stage + ts.dy, (int64_t)T * HP, off(dy, t0 * HP, d.esz), d.xs_b, tv, T, HP, sp.Bt, d.esz, sk);
            if (e == hipSuccess) e = launch_stage_rows(stage + ts.dt, (int64_t)T * d.H, off(dt, t0 * d.H, d.esz), d.dts_b, tv, T, d.H, sp.Bt, d.esz, sk);
            if (e == hipSuccess) e = launch_stage_rows(stage + ts.B, (int64_t)T * GN, off(B, t0 * GN, d.esz), d.bcs_b, tv, T, GN, sp.Bt, d.esz, sk);
            if (e == hipSuccess) e = launch_stage_rows(stage + ts.C, (int64_t)T * GN, off(C, t0 * GN, d.esz), d.bcs_b, tv, T, GN, sp.Bt, d.esz, sk);
            if (e == hipSuccess && d.reset) e = launch_stage_rows(stage + ts.reset, T, d.reset + t0, d.L, tv, T, 1, sp.Bt, 1, sk);
            if (e != hipSuccess) {
                (void)join_lanes(pp, nl, st);
                return SSD_ERR_LAUNCH;
            }
            sp.x = stage + ts.x;
            sp.dy = stage + ts.dy;
            sp.dx = stage + ts.dx;
            sp.dt = stage + ts.dt;
            sp.ddt = stage + ts.ddt;
            sp.Bm = stage + ts.B;
            sp.Cm = stage + ts.C;
            sp.dB = stage + ts.dB;
            sp.dC = stage + ts.dC;
            sp.xs_b = sp.ys_b = sp.dys_b = sp.dxs_b = (int64_t)T * HP;
            sp.dts_b = (int64_t)T * d.H;
            sp.bcs_b = (int64_t)T * GN;
            sp.nc = d.nc_tail;
            sp.reset = d.reset ? (const uint8_t*)(stage + ts.reset) : nullptr;
            sp.reset_bs = T;
        }
        sp.chunk0 = (int)(k * d.nc);
        // restore: per-chunk entering states of this segment from its checkpoint
        wire_states(sp, d, k, init_state, ck16 ? nullptr : (const float*)boundary_states, nullptr, nullptr);
        if (ck16 && k > 0) {  // restart from the rounded checkpoint
            sp.state_in = nullptr;
            sp.state_in16 = (const bf16_t*)boundary_states + k * (int64_t)HPN;
            sp.state_in_bs = d.nseg * (int64_t)HPN;
        }
        sp.ev_wait = sp.ev_record = nullptr;
        e = mfma ? mfma_forward_segment(sp, false, sk) : generic_forward_segment(sp, d.bf16, false, sk);
        if (e == hipSuccess) {
            sp.dinit_out = (k == 0) ? dinit_state : nullptr;
            sp.ev_wait = (nl > 1 && it > 0) ? pp->scan[(it - 1) % nl] : nullptr;
            sp.ev_record = (nl > 1 && k > 0) ? pp->scan[ln] : nullptr;
            e = mfma ? mfma_backward_segment(sp, sk) : generic_backward_segment(sp, d.bf16, sk);
        }
        if (e == hipSuccess && short_seg) {  // the valid rows of the results go back to the caller's tensors
            const int tv = (int)d.tail;
            e = launch_stage_rows(off(dx, t0 * HP, d.esz), d.xs_b, stage + ts.dx, (int64_t)ts.T * HP, tv, tv, HP, sp.Bt, d.esz, sk);
            if (e == hipSuccess) e = launch_stage_rows(off(ddt, t0 * d.H, d.esz), d.dts_b, stage + ts.ddt, (int64_t)ts.T * d.H, tv, tv, d.H, sp.Bt, d.esz, sk);
            if (e == hipSuccess) e = launch_stage_rows(off(dB, t0 * GN, d.esz), d.bcs_b, stage + ts.dB, (int64_t)ts.T * GN, tv, tv, GN, sp.Bt, d.esz, sk);
            if (e == hipSuccess) e = launch_stage_rows(off(dC, t0 * GN, d.esz), d.bcs_b, stage + ts.dC, (int64_t)ts.T * GN, tv, tv, GN, sp.Bt, d.esz, sk);
        }
        if (e != hipSuccess) {
            (void)join_lanes(pp, nl, st);  // whatever was enqueued on the library's streams still ends before the caller's next work
            return SSD_ERR_LAUNCH;
        }
    }
    if (!join_lanes(pp, nl, st)) return SSD_ERR_LAUNCH;
    sps[0].accumulate = (flags & SSD_FLAG_ACCUM_PARAM) ? 1 : 0;
    if (launch_param_reduce(sps[0], st) != hipSuccess) return SSD_ERR_LAUNCH;
    return SSD_OK;
}

extern "C" int ssd_prof_serialize(int32_t on) {
    g_serial = on != 0;
    return SSD_OK;
}

extern "C" const char* ssd_strerror(int status) {
    switch (status) {
        case SSD_OK: return "ok";
        case SSD_ERR_NULL: return "a required pointer is NULL";
        case SSD_ERR_SHAPE: return "a dimension is non-positive or exceeds a kernel limit";
        case SSD_ERR_DIVISIBILITY: return "nheads % ngroups or segment % chunk is not zero (stack: seqlen % segment)";
        case SSD_ERR_DTYPE: return "unknown dtype";
        case SSD_ERR_WORKSPACE: return "workspace is NULL, not 256-byte aligned, or too small";
        case SSD_ERR_LAUNCH: return "a HIP launch failed";
        case SSD_ERR_BUDGET: return "no admissible checkpoint plan fits the budget";
        case SSD_ERR_ARG: return "invalid argument";
        default: return "unknown status";
    }
}
