// Residual stack of SSD layers on the MA-GC grid (paper Sec. 3.2/3.3): forward places the layer-
// and sequence-axis checkpoints (Alg. 1), backward restores one grid cell at a time and
// back-propagates through it (Alg. 2).  Layer j: x_{j+1} = x_j + SSD_j(x_j).
#include <string.h>

#include "ssd_internal.h"

namespace ssdk {
namespace {

inline size_t align_up(size_t v) { return (v + 255) & ~(size_t)255; }
inline const void* offc(const void* p, int64_t elems, size_t esz) { return (const char*)p + elems * (int64_t)esz; }
inline void* offm(void* p, int64_t elems, size_t esz) { return (char*)p + elems * (int64_t)esz; }

struct StackDims {
    Dims full;  // whole sequence
    Dims cell;  // one segment as its own call (seqlen = segment)
    int nl, l, nlg;
    bool mfma;         // the cell runs on the matrix-core kernels
    size_t act_bytes;  // one [Bt, s, H, P] activation buffer
    size_t HPN;
};

int check_stack(const ssd_shape_t* shape, int32_t nlayers, int32_t layer_interval, StackDims* sd) {
    int rc = check_shape(shape, &sd->full);
    if (rc != SSD_OK) return rc;
    if (nlayers <= 0 || layer_interval <= 0) return SSD_ERR_SHAPE;
    if (nlayers > 4096) return SSD_ERR_SHAPE;
    if (shape->seqlen <= 0) return SSD_ERR_SHAPE;
    if (shape->x_batch_stride || shape->dt_batch_stride || shape->bc_batch_stride) return SSD_ERR_ARG;
    if (shape->segment > 0 && shape->seqlen % shape->segment != 0) return SSD_ERR_DIVISIBILITY;  // the grid has whole cells only
    if (shape->seq_reset) return SSD_ERR_ARG;  // packed sequences are not wired through the stack
    ssd_shape_t cs = *shape;
    cs.seqlen = shape->segment;
    rc = check_shape(&cs, &sd->cell);
    if (rc != SSD_OK) return rc;
    // the cell views the full tensors: keep their batch strides
    sd->cell.xs_b = sd->full.xs_b;
    sd->cell.dts_b = sd->full.dts_b;
    sd->cell.bcs_b = sd->full.bcs_b;
    sd->mfma = use_mfma(*shape, 0);
    sd->nl = nlayers;
    sd->l = layer_interval < nlayers ? layer_interval : nlayers;
    sd->nlg = (nlayers + sd->l - 1) / sd->l;
    sd->act_bytes = align_up((size_t)sd->full.Bt * sd->full.s * sd->full.H * sd->full.P * sd->full.esz);
    sd->HPN = (size_t)sd->full.H * sd->full.P * sd->full.N;
    return SSD_OK;
}

struct StackWs {
    size_t ssd, act0, nact, dh, total;
};

StackWs stack_ws(const StackDims& sd, bool bwd) {
    StackWs w;
    size_t o = 0;
    w.ssd = o;
    o += align_up(ws_layout(sd.cell, bwd, sd.mfma).total);
    w.act0 = o;
    // fwd: two ping-pong activation buffers; bwd: the cell's (l - 1) restored layer inputs plus two gradient buffers
    w.nact = bwd ? (size_t)(sd.l - 1) + 2 : 2;
    o += w.nact * sd.act_bytes;
    w.dh = o;
    if (bwd) o += align_up((size_t)sd.nl * sd.full.Bt * sd.HPN * 4);
    w.total = o;
    return w;
}

}  // namespace
}  // namespace ssdk

using namespace ssdk;

extern "C" size_t magc_stack_workspace_bytes(const ssd_shape_t* shape, int32_t nlayers, int32_t layer_interval,
                                             int32_t is_backward) {
    StackDims sd;
    if (check_stack(shape, nlayers, layer_interval, &sd) != SSD_OK) return 0;
    return stack_ws(sd, is_backward != 0).total;
}

extern "C" int magc_stack_fwd(const ssd_shape_t* shape, int32_t nlayers, int32_t layer_interval, const void* x0,
                              const void* dt, const float* A, const void* B, const void* C, const float* D, void* out,
                              float* final_states, float* s_ckpt, void* l_ckpt, void* workspace,
                              size_t workspace_bytes, void* hip_stream) {
    StackDims sd;
    int rc = check_stack(shape, nlayers, layer_interval, &sd);
    if (rc != SSD_OK) return rc;
    if (!x0 || !dt || !A || !B || !C || !D || !out || !s_ckpt) return SSD_ERR_NULL;
    if (sd.nlg > 1 && !l_ckpt) return SSD_ERR_NULL;
    const StackWs w = stack_ws(sd, false);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return SSD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    const Dims& f = sd.full;
    const Dims& c = sd.cell;
    const bool mfma = use_mfma(*shape, 0);
    const WsLayout wl = ws_layout(c, false, mfma);
    char* wsb = (char*)workspace;
    void* act[2] = {wsb + w.act0, wsb + w.act0 + sd.act_bytes};
    const int64_t cell_bs = f.s * f.H * f.P;  // batch stride of a workspace activation buffer
    const int64_t HPN = (int64_t)sd.HPN;

    SegParams sp;
    base_params(sp, c, SSD_FLAG_RESIDUAL);
    bind_workspace(sp, wl, wsb + w.ssd, false);
    for (int64_t k = 0; k < f.nseg; ++k) {
        const int64_t t0 = k * f.s;
        const void* cur = offc(x0, t0 * f.H * f.P, f.esz);
        int64_t cur_bs = f.xs_b;
        for (int j = 0; j < sd.nl; ++j) {
            // where this layer's output lives: the stack output, a layer checkpoint, or a scratch buffer
            void* dst;
            int64_t dst_bs;
            if (j == sd.nl - 1) {
                dst = offm(out, t0 * f.H * f.P, f.esz);
                dst_bs = f.xs_b;
            } else if ((j + 1) % sd.l == 0) {
                const int64_t slot = (j + 1) / sd.l - 1;
                dst = offm(l_ckpt, slot * f.Bt * f.L * f.H * f.P + t0 * f.H * f.P, f.esz);
                dst_bs = f.xs_b;
            } else {
                dst = act[j & 1];
                dst_bs = cell_bs;
            }
            sp.x = cur;
            sp.xs_b = cur_bs;
            sp.y = dst;
            sp.ys_b = dst_bs;
            sp.dt = offc(dt, (int64_t)j * f.Bt * f.L * f.H + t0 * f.H, f.esz);
            sp.Bm = offc(B, (int64_t)j * f.Bt * f.L * f.G * f.N + t0 * f.G * f.N, f.esz);
            sp.Cm = offc(C, (int64_t)j * f.Bt * f.L * f.G * f.N + t0 * f.G * f.N, f.esz);
            sp.A = A + (int64_t)j * f.H;
            sp.D = D + (int64_t)j * f.H;
            float* sj = s_ckpt + (int64_t)j * f.Bt * f.nseg * HPN;  // [Bt, nseg, H, P, N] of layer j
            sp.state_in = (k == 0) ? nullptr : sj + k * HPN;
            sp.state_in_bs = f.nseg * HPN;
            sp.bnd_write = (k == 0) ? sj : nullptr;
            sp.bnd_write_bs = f.nseg * HPN;
            sp.state_out = (k + 1 < f.nseg) ? sj + (k + 1) * HPN : nullptr;
            sp.state_out_bs = f.nseg * HPN;
            sp.state_out2 = (k + 1 == f.nseg && final_states) ? final_states + (int64_t)j * f.Bt * HPN : nullptr;
            sp.state_out2_bs = HPN;
            hipError_t e = mfma ? mfma_forward_segment(sp, true, st) : generic_forward_segment(sp, c.bf16, true, st);
            if (e != hipSuccess) return SSD_ERR_LAUNCH;
            cur = dst;
            cur_bs = dst_bs;
        }
    }
    return SSD_OK;
}

extern "C" int magc_stack_bwd(const ssd_shape_t* shape, int32_t nlayers, int32_t layer_interval, const void* x0,
                              const void* dt, const float* A, const void* B, const void* C, const float* D,
                              const void* dout, const float* s_ckpt, const void* l_ckpt, void* dx0, void* ddt,
                              float* dA, void* dB, void* dC, float* dD, void* workspace, size_t workspace_bytes,
                              void* hip_stream) {
    StackDims sd;
    int rc = check_stack(shape, nlayers, layer_interval, &sd);
    if (rc != SSD_OK) return rc;
    if (!x0 || !dt || !A || !B || !C || !D || !dout || !s_ckpt || !dx0 || !ddt || !dA || !dB || !dC || !dD)
        return SSD_ERR_NULL;
    if (sd.nlg > 1 && !l_ckpt) return SSD_ERR_NULL;
    if (dx0 == dout) return SSD_ERR_ARG;
    const StackWs w = stack_ws(sd, true);
    if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < w.total) return SSD_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    const Dims& f = sd.full;
    const Dims& c = sd.cell;
    const bool mfma = use_mfma(*shape, 0);
    const WsLayout wl = ws_layout(c, true, mfma);
    char* wsb = (char*)workspace;
    const int64_t cell_bs = f.s * f.H * f.P;
    const int64_t HPN = (int64_t)sd.HPN;
    // activation buffers: [0, l-1) restored layer inputs of the cell, then two gradient buffers
    auto actbuf = [&](size_t i) { return (void*)(wsb + w.act0 + i * sd.act_bytes); };
    void* gbuf[2] = {actbuf((size_t)(sd.l - 1)), actbuf((size_t)(sd.l - 1) + 1)};
    float* dh = (float*)(wsb + w.dh);  // [nl, Bt, H, P, N] state adjoints carried right to left
    hipError_t e = launch_fill_zero(dh, (size_t)sd.nl * f.Bt * HPN, st);
    if (e != hipSuccess) return SSD_ERR_LAUNCH;

    SegParams sp;
    base_params(sp, c, SSD_FLAG_RESIDUAL);
    bind_workspace(sp, wl, wsb + w.ssd, true);

    auto set_layer = [&](int j, int64_t k) {
        const int64_t t0 = k * f.s;
        sp.dt = offc(dt, (int64_t)j * f.Bt * f.L * f.H + t0 * f.H, f.esz);
        sp.Bm = offc(B, (int64_t)j * f.Bt * f.L * f.G * f.N + t0 * f.G * f.N, f.esz);
        sp.Cm = offc(C, (int64_t)j * f.Bt * f.L * f.G * f.N + t0 * f.G * f.N, f.esz);
        sp.ddt = offm(ddt, (int64_t)j * f.Bt * f.L * f.H + t0 * f.H, f.esz);
        sp.dB = offm(dB, (int64_t)j * f.Bt * f.L * f.G * f.N + t0 * f.G * f.N, f.esz);
        sp.dC = offm(dC, (int64_t)j * f.Bt * f.L * f.G * f.N + t0 * f.G * f.N, f.esz);
        sp.A = A + (int64_t)j * f.H;
        sp.D = D + (int64_t)j * f.H;
        sp.dA = dA + (int64_t)j * f.H;
        sp.dD = dD + (int64_t)j * f.H;
        const float* sj = s_ckpt + (int64_t)j * f.Bt * f.nseg * HPN;
        sp.state_in = sj + k * HPN;  // slot 0 holds the (zero) initial state written by the forward pass
        sp.state_in_bs = f.nseg * HPN;
        sp.bnd_write = nullptr;
        sp.state_out = nullptr;
        sp.state_out2 = nullptr;
    };

    for (int64_t k = f.nseg - 1; k >= 0; --k) {
        const int64_t t0 = k * f.s;
        const void* g_in = offc(dout, t0 * f.H * f.P, f.esz);
        int64_t g_in_bs = f.xs_b;
        int gflip = 0;
        for (int jb = sd.nlg - 1; jb >= 0; --jb) {
            const int j_lo = jb * sd.l;
            const int j_hi = (j_lo + sd.l < sd.nl) ? j_lo + sd.l : sd.nl;  // exclusive
            // input of the block's first layer: the layer checkpoint (or the stack input)
            auto layer_input = [&](int j, const void** p, int64_t* bs) {
                if (j == j_lo) {
                    if (jb == 0) *p = offc(x0, t0 * f.H * f.P, f.esz);
                    else *p = offc(l_ckpt, (int64_t)(jb - 1) * f.Bt * f.L * f.H * f.P + t0 * f.H * f.P, f.esz);
                    *bs = f.xs_b;
                } else {
                    *p = actbuf((size_t)(j - j_lo - 1));
                    *bs = cell_bs;
                }
            };
            // restore: inputs of layers j_lo+1 .. j_hi-1 of this cell
            for (int j = j_lo; j + 1 < j_hi; ++j) {
                set_layer(j, k);
                const void* xi;
                int64_t xbs;
                layer_input(j, &xi, &xbs);
                sp.x = xi;
                sp.xs_b = xbs;
                sp.y = actbuf((size_t)(j - j_lo));
                sp.ys_b = cell_bs;
                e = mfma ? mfma_forward_segment(sp, true, st) : generic_forward_segment(sp, c.bf16, true, st);
                if (e != hipSuccess) return SSD_ERR_LAUNCH;
            }
            // back-propagate through the cell, top layer first
            for (int j = j_hi - 1; j >= j_lo; --j) {
                set_layer(j, k);
                const void* xi;
                int64_t xbs;
                layer_input(j, &xi, &xbs);
                sp.x = xi;
                sp.xs_b = xbs;
                sp.dy = g_in;
                sp.dys_b = g_in_bs;
                void* g_out;
                int64_t g_out_bs;
                if (j == 0) {
                    g_out = offm(dx0, t0 * f.H * f.P, f.esz);
                    g_out_bs = f.xs_b;
                } else {
                    g_out = gbuf[gflip];
                    g_out_bs = cell_bs;
                    gflip ^= 1;
                }
                sp.dx = g_out;
                sp.dxs_b = g_out_bs;
                // chunk states of this layer over the segment, then the backward proper
                e = mfma ? mfma_forward_segment(sp, false, st) : generic_forward_segment(sp, c.bf16, false, st);
                if (e != hipSuccess) return SSD_ERR_LAUNCH;
                float* dhj = dh + (int64_t)j * f.Bt * HPN;
                e = launch_copy_f32(sp.dcarry, dhj, (size_t)f.Bt * HPN, st);
                if (e != hipSuccess) return SSD_ERR_LAUNCH;
                sp.dinit_out = dhj;
                sp.accumulate = (k == f.nseg - 1) ? 0 : 1;
                e = mfma ? mfma_backward_segment(sp, st) : generic_backward_segment(sp, c.bf16, st);
                if (e != hipSuccess) return SSD_ERR_LAUNCH;
                g_in = g_out;
                g_in_bs = g_out_bs;
            }
        }
    }
    return SSD_OK;
}
