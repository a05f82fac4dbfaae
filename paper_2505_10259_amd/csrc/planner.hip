// ParaSpec planner (Section 4.3; Appendix A.1 "ParaSpec Planner"): host-side search for the batch
// sizes and the number of candidates per round that maximise the modelled throughput under the two
// GPU-memory constraints.  No device code.
//
// The throughput separates: T_prefill depends on bs_prefill only and V_prefill constrains bs_prefill
// only; T_draft depends on bs_draft only (given bs, n_cand) and enters through max(T_target, T_draft).
// So for each (bs, n_cand) the two inner parameters are chosen independently — the largest bs_prefill
// with the smallest T_prefill, the largest bs_draft with the smallest round time — which replaces the
// four-deep search by bs_max * n_cand_max * 2 bs_max evaluations.
#include <cmath>
#include <cstdint>

#include "../../include/specverify.h"

namespace {

struct Model {
    const spec_planner_profile& p;

    // E[n_generated] = sum_{k=1}^{n_cand+1} k P[n = k], P = p^(k-1) (1-p) for k <= n_cand and
    // p^n_cand for k = n_cand + 1 (Appendix A.1, "Generated Tokens")
    double expected(int n_cand) const {
        double e = 0.0;
        for (int k = 1; k <= n_cand; ++k) e += k * std::pow(p.p_accept, k - 1) * (1.0 - p.p_accept);
        e += (n_cand + 1) * std::pow(p.p_accept, n_cand);
        return e;
    }
    // T_prefill = ceil(bs / bs_prefill) * (T_c2g_para + T_gpu_comp)
    double t_prefill(int bs, int bp) const {
        double per_batch = p.t_c2g_para + p.t_gpu_prefill_comp + p.t_prefill_comp_per_seq * bp;
        return std::ceil((double)bs / bp) * per_batch;
    }
    // T_draft = ceil(bs / bs_draft) * (T_draft_prefill + (n_cand - 1) T_draft_decoding)
    double t_draft(int bs, int bd, int n_cand) const {
        double first = p.t_draft_prefill + p.t_draft_per_seq * bd;
        double later = p.t_draft_decoding + p.t_draft_per_seq * bd;
        return std::ceil((double)bs / bd) * (first + (n_cand - 1) * later);
    }
    // T_target_decoding = sum over layers of max(T_attention, T_ffn_c2g) + T_ffn_gpu,
    // T_attention = n_cand * bs * t_attention_unit; resident layers have no transfer
    double t_target(int bs, int n_cand) const {
        double t_att = n_cand * bs * p.t_attention_unit;
        double t_gpu = p.t_ffn_gpu + p.t_ffn_gpu_per_token * bs * (n_cand + 1);
        double total = 0.0;
        for (int l = 0; l < p.n_layer; ++l) {
            double c2g = l < p.n_layer_streamed ? p.t_ffn_c2g : 0.0;
            total += std::fmax(t_att, c2g) + t_gpu;
        }
        return total;
    }
    double v_prefill(int bp) const { return p.v_target_prefill + (double)bp * p.l_input * p.v_target_kv; }
    double v_decoding(int bs, int bd) const {
        double ctx = (double)p.l_input + p.n_generate;
        return p.v_target_ffn + p.v_draft + bd * ctx * p.v_draft_kv + bs * ctx * p.v_target_kv_decoding;
    }
    void fill(int bs, int bp, int bd, int n_cand, spec_plan* o) const {
        o->bs = bs; o->bs_prefill = bp; o->bs_draft = bd; o->n_cand = n_cand;
        o->v_prefill = v_prefill(bp);
        o->v_decoding = v_decoding(bs, bd);
        o->feasible = o->v_prefill <= p.gpu_mem_capacity && o->v_decoding <= p.gpu_mem_capacity;
        o->expected_tokens = expected(n_cand);
        o->n_iter = (int32_t)std::ceil(p.n_generate / o->expected_tokens);
        o->t_target_decoding = t_target(bs, n_cand);
        o->t_draft = t_draft(bs, bd, n_cand);
        o->t_round = std::fmax(o->t_target_decoding, o->t_draft);
        o->t_prefill = t_prefill(bs, bp);
        double n_gen = (double)bs * o->n_iter * o->expected_tokens;
        o->throughput = n_gen / (o->t_prefill + o->n_iter * o->t_round);
    }
};

bool valid(const spec_planner_profile* p) {
    if (!p) return false;
    if (p->n_layer <= 0 || p->n_layer_streamed < 0 || p->n_layer_streamed > p->n_layer || p->l_input <= 0 ||
        p->n_generate <= 0 || p->bs_max <= 0 || p->n_cand_max <= 0)
        return false;
    if (!(p->p_accept >= 0.0 && p->p_accept < 1.0)) return false;
    const double nonneg[] = {p->t_c2g_para, p->t_gpu_prefill_comp, p->t_ffn_c2g, p->t_ffn_gpu, p->t_attention_unit,
                             p->t_draft_prefill, p->t_draft_decoding, p->gpu_mem_capacity, p->v_target_prefill,
                             p->v_target_kv, p->v_target_ffn, p->v_draft, p->v_draft_kv, p->t_ffn_gpu_per_token,
                             p->t_draft_per_seq, p->t_prefill_comp_per_seq, p->v_target_kv_decoding};
    for (double v : nonneg)
        if (!(v >= 0.0)) return false;     // also rejects NaN
    return true;
}

}  // namespace

extern "C" int spec_plan_evaluate(const spec_planner_profile* profile, int32_t bs, int32_t bs_prefill,
                                  int32_t bs_draft, int32_t n_cand, spec_plan* out) {
    if (!valid(profile) || !out || bs <= 0 || bs_prefill <= 0 || bs_draft <= 0 || n_cand <= 0) return SPEC_ERR_ARG;
    Model{*profile}.fill(bs, bs_prefill, bs_draft, n_cand, out);
    return SPEC_OK;
}

extern "C" int spec_plan_paraspec(const spec_planner_profile* profile, spec_plan* out) {
    if (!valid(profile) || !out) return SPEC_ERR_ARG;
    const Model m{*profile};
    spec_plan best{};
    best.feasible = 0;
    for (int bs = 1; bs <= profile->bs_max; ++bs) {
        // prefill batch: smallest T_prefill among the feasible ones, largest bs_prefill on ties
        int bp_best = 0;
        double tp_best = 0.0;
        for (int bp = bs; bp >= 1; --bp) {
            if (m.v_prefill(bp) > profile->gpu_mem_capacity) continue;
            double tp = m.t_prefill(bs, bp);
            if (bp_best == 0 || tp < tp_best) { bp_best = bp; tp_best = tp; }
        }
        if (bp_best == 0) continue;
        for (int n_cand = 1; n_cand <= profile->n_cand_max; ++n_cand) {
            // draft batch: smallest round time max(T_target, T_draft), largest bs_draft on ties
            const double tt = m.t_target(bs, n_cand);
            int bd_best = 0;
            double round_best = 0.0;
            for (int bd = bs; bd >= 1; --bd) {
                if (m.v_decoding(bs, bd) > profile->gpu_mem_capacity) continue;
                double tr = std::fmax(tt, m.t_draft(bs, bd, n_cand));
                if (bd_best == 0 || tr < round_best) { bd_best = bd; round_best = tr; }
            }
            if (bd_best == 0) continue;
            spec_plan cand;
            m.fill(bs, bp_best, bd_best, n_cand, &cand);
            if (!best.feasible || cand.throughput > best.throughput) best = cand;
        }
    }
    *out = best;
    return SPEC_OK;
}
