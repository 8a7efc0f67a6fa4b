// Checkpoint-interval planner for the MA-GC grid (host only).
// Memory model of the paper's App. C:  M(l,s) = (L S / l) C_Lckpt + (L S / s) C_Sckpt + l s C_grid + s C_state;
// with unit constants and C_state = 0 it is the model analysed in Sec. 3.3.
#include <math.h>

#include "ssd_magc.h"

namespace {

struct Terms {
    double ml, ms, mg, mt, total;
};

Terms eval(const magc_model_t& m, int64_t l, int64_t s) {
    const double L = (double)m.n_layers, S = (double)m.seqlen;
    double nl = L / (double)l, ns = S / (double)s;
    if (m.integer_counts) {
        nl = (double)((m.n_layers + l - 1) / l);
        ns = (double)((m.seqlen + s - 1) / s);
    }
    Terms t;
    t.ml = nl * S * m.c_lckpt;
    t.ms = L * ns * m.c_sckpt;
    t.mg = (double)l * (double)s * m.c_grid;
    t.mt = (double)s * m.c_state;
    t.total = t.ml + t.ms + t.mg + t.mt;
    return t;
}

}  // namespace

extern "C" int magc_plan(const magc_model_t* model, magc_plan_t* out) {
    if (!model || !out) return SSD_ERR_NULL;
    const magc_model_t& m = *model;
    if (m.n_layers <= 0 || m.seqlen <= 0) return SSD_ERR_SHAPE;
    if (m.c_lckpt < 0 || m.c_sckpt < 0 || m.c_grid < 0 || m.c_state < 0) return SSD_ERR_ARG;
    if (!(m.c_lckpt == m.c_lckpt) || !(m.c_sckpt == m.c_sckpt) || !(m.c_grid == m.c_grid) || !(m.c_state == m.c_state))
        return SSD_ERR_ARG;
    if (m.n_layers > (1 << 20) || m.seqlen > ((int64_t)1 << 40)) return SSD_ERR_SHAPE;
    const bool rule = m.s_multiple > 1 && m.seqlen >= m.s_multiple;
    const int64_t s_step = rule ? m.s_multiple : 1;
    if ((m.seqlen / s_step) * m.n_layers > ((int64_t)1 << 32)) return SSD_ERR_SHAPE;  // keeps the search bounded

    bool have = false, have_fit = false;
    int64_t bl = 0, bs = 0, fl = 0, fs = 0;
    Terms bt = {}, ft = {};
    for (int64_t l = 1; l <= m.n_layers; ++l) {
        for (int64_t s = s_step; s <= m.seqlen; s += s_step) {
            const Terms t = eval(m, l, s);
            if (!have || t.total < bt.total || (t.total == bt.total && (s > bs || (s == bs && l < bl)))) {
                have = true;
                bl = l;
                bs = s;
                bt = t;
            }
            if (m.budget > 0 && t.total <= m.budget) {
                if (!have_fit || s > fs || (s == fs && l > fl)) {
                    have_fit = true;
                    fl = l;
                    fs = s;
                    ft = t;
                }
            }
        }
    }
    const bool fit = m.budget > 0 ? have_fit : true;
    const Terms& t = (m.budget > 0 && have_fit) ? ft : bt;
    out->l = (m.budget > 0 && have_fit) ? fl : bl;
    out->s = (m.budget > 0 && have_fit) ? fs : bs;
    out->m_lckpt = t.ml;
    out->m_sckpt = t.ms;
    out->m_grid = t.mg;
    out->m_state = t.mt;
    out->m_total = t.total;
    const double L = (double)m.n_layers, S = (double)m.seqlen;
    out->regime = (L * L <= S) ? 1 : ((S * S <= L) ? 2 : 0);
    out->fits = fit ? 1 : 0;
    return fit ? SSD_OK : SSD_ERR_BUDGET;
}
