// C ABI entry points of the operators: argument checks, plan lookup, dispatch to the kernels.
#include "internal.h"

namespace dol {

bool is_dtkp(const dol_prov *prov) { return prov && prov->kind == DOL_DTKP; }

dol_status check_prov(const dol_prov *prov, int32_t batch)
{
    if (!prov) return DOL_OK;
    if (prov->kind != DOL_DAMP && prov->kind != DOL_DTKP) return fail(DOL_EINVAL, "unknown provenance kind %d", prov->kind);
    if (prov->kind == DOL_DTKP) {
        if (prov->k < 1 || prov->k > DOL_MAX_K) return fail(DOL_EINVAL, "k = %d outside 1..%d", prov->k, DOL_MAX_K);
        if (prov->n_facts < 0 || prov->n_facts > DOL_MAX_FACTS)
            return fail(DOL_EINVAL, "n_facts = %d outside 0..%d", prov->n_facts, DOL_MAX_FACTS);
        if (!prov->fact_prob && prov->n_facts > 0 && batch > 0) return fail(DOL_EINVAL, "fact_prob is NULL");
    }
    return DOL_OK;
}

// Shape and pointer checks of one Distribution.  need_ids: the call reads sym_ids.
dol_status check_dist(const dol_dist *d, const char *name, bool dtkp, bool need_ids, bool need_prob)
{
    if (!d) return fail(DOL_EINVAL, "%s is NULL", name);
    if (d->batch < 0) return fail(DOL_ESHAPE, "%s.batch is negative", name);
    if (d->n_sym < 0 || d->n_sym > DOL_MAX_SYMBOLS) return fail(DOL_ESHAPE, "%s.n_sym = %d outside 0..%d", name, d->n_sym, DOL_MAX_SYMBOLS);
    if (d->ld < d->n_sym) return fail(DOL_ESHAPE, "%s.ld = %lld smaller than n_sym = %d", name, static_cast<long long>(d->ld), d->n_sym);
    const bool has_data = d->batch > 0 && d->n_sym > 0;
    if (has_data && need_prob && !d->prob) return fail(DOL_EINVAL, "%s.prob is NULL", name);
    if (has_data && dtkp && !d->proof_mask) return fail(DOL_EINVAL, "%s.proof_mask is NULL", name);
    if (need_ids && d->n_sym > 0) {
        if (!d->sym_ids) return fail(DOL_EINVAL, "%s.sym_ids is NULL", name);
        for (int32_t i = 1; i < d->n_sym; ++i)
            if (d->sym_ids[i - 1] >= d->sym_ids[i]) return fail(DOL_EINVAL, "%s.sym_ids not strictly ascending at %d", name, i);
    }
    return DOL_OK;
}

dol_status check_work(int64_t batch, int64_t per_sample)
{
    // one thread per element, at most 2^31-1 workgroups of >= 128 threads
    if (batch * per_sample > (int64_t(1) << 37)) return fail(DOL_EUNSUPPORTED, "batch * symbols = %lld exceeds 2^37", static_cast<long long>(batch * per_sample));
    return DOL_OK;
}

}  // namespace dol

using namespace dol;

extern "C" {

dol_status dol_apply2(const dol_dist *a, const dol_dist *b, const dol_fn_table *f, const dol_prov *prov,
                      dol_dist *out, void *hip_stream)
{
    if (!f) return fail(DOL_EINVAL, "function table is NULL");
    const bool dtkp = is_dtkp(prov);
    if (dol_status st = check_dist(a, "a", dtkp, false, !dtkp)) return st;
    if (dol_status st = check_dist(b, "b", dtkp, false, !dtkp)) return st;
    if (dol_status st = check_dist(out, "out", dtkp, false, true)) return st;
    if (dol_status st = check_prov(prov, a->batch)) return st;
    if (a->batch != b->batch || a->batch != out->batch) return fail(DOL_ESHAPE, "batch sizes differ: %d, %d, %d", a->batch, b->batch, out->batch);
    if (a->n_sym != f->na || b->n_sym != f->nb || out->n_sym != f->n_out)
        return fail(DOL_ESHAPE, "operands have %d x %d -> %d symbols, the table is %d x %d -> %d", a->n_sym, b->n_sym, out->n_sym, f->na, f->nb, f->n_out);
    if (out->sym_ids)
        for (int32_t c = 0; c < f->n_out; ++c)
            if (out->sym_ids[c] != f->out_syms[c]) return fail(DOL_EINVAL, "out.sym_ids[%d] = %d, the table produces %d there", c, out->sym_ids[c], f->out_syms[c]);
    if (dol_status st = check_work(a->batch, f->n_out)) return st;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (!dtkp)
        return launch_damp_apply2_fwd(f, a->batch, a->prob, a->ld, b->prob, b->ld, out->prob, out->ld, st);
    if (out->batch > 0 && out->n_sym > 0 && !out->proof_prob) return fail(DOL_EINVAL, "out.proof_prob is NULL");
    GroupMasks gm;
    if (dol_status s2 = make_group_masks(prov, &gm)) return s2;
    return launch_dtkp_apply2(f, a->batch, prov->k, prov->n_facts, gm, prov->fact_prob, a->proof_mask, a->proof_prob,
                              b->proof_mask, b->proof_prob, nullptr, out->proof_mask, out->proof_prob, out->prob, out->ld,
                              st);
}

dol_status dol_dtkp_apply2_input(const dol_dist *a, const int32_t *fact_of_sym_b, const dol_fn_table *f,
                                 const dol_prov *prov, dol_dist *out, void *hip_stream)
{
    if (!f) return fail(DOL_EINVAL, "function table is NULL");
    if (!is_dtkp(prov)) return fail(DOL_EINVAL, "dol_dtkp_apply2_input needs a DTKP provenance");
    if (dol_status st = check_dist(a, "a", true, false, false)) return st;
    if (dol_status st = check_dist(out, "out", true, false, true)) return st;
    if (dol_status st = check_prov(prov, a->batch)) return st;
    if (a->batch != out->batch) return fail(DOL_ESHAPE, "batch sizes differ: %d, %d", a->batch, out->batch);
    if (a->n_sym != f->na || out->n_sym != f->n_out)
        return fail(DOL_ESHAPE, "a has %d symbols and out %d, the table is %d x %d -> %d", a->n_sym, out->n_sym, f->na, f->nb, f->n_out);
    if (f->nb > 0 && !fact_of_sym_b) return fail(DOL_EINVAL, "fact_of_sym_b is NULL");
    for (int32_t j = 0; j < f->nb; ++j)
        if (fact_of_sym_b[j] < 0 || fact_of_sym_b[j] >= prov->n_facts)
            return fail(DOL_EINVAL, "fact_of_sym_b[%d] = %d outside 0..%d", j, fact_of_sym_b[j], prov->n_facts - 1);
    if (out->sym_ids)
        for (int32_t c = 0; c < f->n_out; ++c)
            if (out->sym_ids[c] != f->out_syms[c]) return fail(DOL_EINVAL, "out.sym_ids[%d] = %d, the table produces %d there", c, out->sym_ids[c], f->out_syms[c]);
    if (dol_status st = check_work(a->batch, f->n_out)) return st;
    if (a->batch == 0 || f->n_out == 0) return DOL_OK;
    if (!out->proof_prob) return fail(DOL_EINVAL, "out.proof_prob is NULL");
    GroupMasks gm;
    if (dol_status s2 = make_group_masks(prov, &gm)) return s2;
    // four words per symbol of b: its fact, the other facts of that fact's exclusion group (low, high word), 0
    std::vector<int32_t> words(4 * static_cast<size_t>(f->nb), 0);
    for (int32_t j = 0; j < f->nb; ++j) {
        const int32_t fb = fact_of_sym_b[j];
        uint64_t rival = 0;
        for (int32_t g = 0; g < gm.n; ++g)
            if ((gm.m[g] >> fb) & 1) rival |= gm.m[g];
        rival &= ~(uint64_t(1) << fb);
        words[4 * j] = fb;
        words[4 * j + 1] = static_cast<int32_t>(static_cast<uint32_t>(rival));
        words[4 * j + 2] = static_cast<int32_t>(static_cast<uint32_t>(rival >> 32));
    }
    const int32_t *d_fact_b = nullptr;
    if (dol_status s2 = get_i32_array(static_cast<int32_t>(words.size()), words.data(), &d_fact_b)) return s2;
    return launch_dtkp_apply2(f, a->batch, prov->k, prov->n_facts, gm, prov->fact_prob, a->proof_mask, a->proof_prob,
                              nullptr, nullptr, d_fact_b, out->proof_mask, out->proof_prob, out->prob, out->ld,
                              static_cast<hipStream_t>(hip_stream));
}

dol_status dol_filter(const dol_dist *d, const uint8_t *pred_mask, const dol_prov *prov, dol_dist *out,
                      void *hip_stream)
{
    const bool dtkp = is_dtkp(prov);
    if (dol_status st = check_dist(d, "d", dtkp, false, true)) return st;
    if (dol_status st = check_dist(out, "out", dtkp, false, true)) return st;
    if (dol_status st = check_prov(prov, 0)) return st;
    if (d->n_sym > 0 && !pred_mask) return fail(DOL_EINVAL, "pred_mask is NULL");
    if (d->batch != out->batch) return fail(DOL_ESHAPE, "batch sizes differ: %d, %d", d->batch, out->batch);
    const FilterPlan *plan = nullptr;
    if (dol_status st = get_filter_plan(d->n_sym, pred_mask, &plan)) return st;
    if (out->n_sym != plan->n_out) return fail(DOL_ESHAPE, "out.n_sym = %d, the predicate keeps %d symbols", out->n_sym, plan->n_out);
    if (out->sym_ids && d->sym_ids)
        for (int32_t c = 0; c < plan->n_out; ++c)
            if (out->sym_ids[c] != d->sym_ids[plan->keep_idx[c]]) return fail(DOL_EINVAL, "out.sym_ids[%d] is not the kept symbol", c);
    if (dol_status st = check_work(d->batch, d->n_sym)) return st;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (!dtkp) return launch_damp_filter_fwd(plan, d->batch, d->prob, d->ld, out->prob, out->ld, st);
    if (d->batch > 0 && d->n_sym > 0 && !d->proof_prob) return fail(DOL_EINVAL, "d.proof_prob is NULL");
    if (out->batch > 0 && out->n_sym > 0 && !out->proof_prob) return fail(DOL_EINVAL, "out.proof_prob is NULL");
    return launch_dtkp_filter(plan, d->batch, prov->k, d->proof_mask, d->proof_prob, d->prob, d->ld, out->proof_mask,
                              out->proof_prob, out->prob, out->ld, st);
}

dol_status dol_union(const dol_dist *a, const dol_dist *b, const dol_prov *prov, dol_dist *out, void *hip_stream)
{
    const bool dtkp = is_dtkp(prov);
    if (dol_status st = check_dist(a, "a", dtkp, true, !dtkp)) return st;
    if (dol_status st = check_dist(b, "b", dtkp, true, !dtkp)) return st;
    if (dol_status st = check_dist(out, "out", dtkp, false, true)) return st;
    if (dol_status st = check_prov(prov, 0)) return st;
    if (a->batch != b->batch || a->batch != out->batch) return fail(DOL_ESHAPE, "batch sizes differ: %d, %d, %d", a->batch, b->batch, out->batch);
    const UnionPlan *plan = nullptr;
    if (dol_status st = get_union_plan(a->n_sym, a->sym_ids, b->n_sym, b->sym_ids, &plan)) return st;
    if (plan->n_out > DOL_MAX_SYMBOLS) return fail(DOL_EUNSUPPORTED, "the union has %d symbols, more than %d", plan->n_out, DOL_MAX_SYMBOLS);
    if (out->n_sym != plan->n_out) return fail(DOL_ESHAPE, "out.n_sym = %d, the union has %d symbols", out->n_sym, plan->n_out);
    if (out->sym_ids)
        for (int32_t c = 0; c < plan->n_out; ++c)
            if (out->sym_ids[c] != plan->out_syms[c]) return fail(DOL_EINVAL, "out.sym_ids[%d] = %d, the union has %d there", c, out->sym_ids[c], plan->out_syms[c]);
    if (dol_status st = check_work(a->batch, plan->n_out)) return st;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (!dtkp) return launch_damp_union_fwd(plan, a->batch, a->prob, a->ld, b->prob, b->ld, out->prob, out->ld, st);
    if ((a->batch > 0 && a->n_sym > 0 && !a->proof_prob) || (b->batch > 0 && b->n_sym > 0 && !b->proof_prob) ||
        (out->batch > 0 && out->n_sym > 0 && !out->proof_prob))
        return fail(DOL_EINVAL, "proof_prob is NULL");
    return launch_dtkp_union(plan, a->batch, prov->k, a->proof_mask, a->proof_prob, b->proof_mask, b->proof_prob,
                             out->proof_mask, out->proof_prob, out->prob, out->ld, st);
}

dol_status dol_filter_union(const dol_dist *d, const uint8_t *pred_mask, const dol_dist *c, const dol_prov *prov,
                            dol_dist *out, void *hip_stream)
{
    if (is_dtkp(prov)) return fail(DOL_EUNSUPPORTED, "dol_filter_union is DAMP only: call dol_filter and dol_union");
    if (!pred_mask) return fail(DOL_EINVAL, "pred_mask is NULL");
    if (dol_status st = check_dist(d, "d", false, true, true)) return st;
    if (dol_status st = check_dist(c, "c", false, true, true)) return st;
    if (dol_status st = check_dist(out, "out", false, false, true)) return st;
    if (d->batch != c->batch || d->batch != out->batch) return fail(DOL_ESHAPE, "batch sizes differ: %d, %d, %d", d->batch, c->batch, out->batch);
    const UnionPlan *plan = nullptr;
    if (dol_status st = get_filter_union_plan(d->n_sym, d->sym_ids, pred_mask, c->n_sym, c->sym_ids, &plan)) return st;
    if (plan->n_out > DOL_MAX_SYMBOLS) return fail(DOL_EUNSUPPORTED, "the union has %d symbols, more than %d", plan->n_out, DOL_MAX_SYMBOLS);
    if (out->n_sym != plan->n_out) return fail(DOL_ESHAPE, "out.n_sym = %d, the result has %d symbols", out->n_sym, plan->n_out);
    if (out->sym_ids)
        for (int32_t u = 0; u < plan->n_out; ++u)
            if (out->sym_ids[u] != plan->out_syms[u]) return fail(DOL_EINVAL, "out.sym_ids[%d] = %d, the result has %d there", u, out->sym_ids[u], plan->out_syms[u]);
    if (dol_status st = check_work(d->batch, plan->n_out)) return st;
    return launch_damp_union_fwd(plan, d->batch, d->prob, d->ld, c->prob, c->ld, out->prob, out->ld,
                                 static_cast<hipStream_t>(hip_stream));
}

// Checks of dol_apply2_filter_union and its reverse; leaves the merge plan in *plan.
static dol_status check_apply_merge(const dol_apply_merge *m, const UnionPlan **plan)
{
    if (!m) return fail(DOL_EINVAL, "the description is NULL");
    if (!m->f || !m->pred_mask) return fail(DOL_EINVAL, "f or pred_mask is NULL");
    if (dol_status st = check_dist(m->a, "a", false, false, true)) return st;
    if (dol_status st = check_dist(m->b, "b", false, false, true)) return st;
    if (dol_status st = check_dist(m->c, "c", false, true, true)) return st;
    if (dol_status st = check_dist(m->out, "out", false, false, true)) return st;
    const dol_fn_table *f = m->f;
    if (m->a->n_sym != f->na || m->b->n_sym != f->nb)
        return fail(DOL_ESHAPE, "the table is %d x %d, its operands have %d and %d symbols", f->na, f->nb, m->a->n_sym, m->b->n_sym);
    const int32_t batch = m->a->batch;
    if (m->b->batch != batch || m->c->batch != batch || m->out->batch != batch) return fail(DOL_ESHAPE, "batch sizes differ");
    if (dol_status st = get_filter_union_plan(f->n_out, f->out_syms.data(), m->pred_mask, m->c->n_sym, m->c->sym_ids, plan)) return st;
    const UnionPlan *p = *plan;
    if (p->n_out > DOL_MAX_SYMBOLS) return fail(DOL_EUNSUPPORTED, "the union has %d symbols, more than %d", p->n_out, DOL_MAX_SYMBOLS);
    if (m->out->n_sym != p->n_out) return fail(DOL_ESHAPE, "out.n_sym = %d, the result has %d symbols", m->out->n_sym, p->n_out);
    if (m->out->sym_ids)
        for (int32_t u = 0; u < p->n_out; ++u)
            if (m->out->sym_ids[u] != p->out_syms[u])
                return fail(DOL_EINVAL, "out.sym_ids[%d] = %d, the result has %d there", u, m->out->sym_ids[u], p->out_syms[u]);
    if (!table_merge_ok(f))
        return fail(DOL_EUNSUPPORTED, "the one-launch form needs a table of at most 64 x 64 symbols producing at most 512, all counts multiples of 4");
    auto flat = [](const dol_dist *d) { return d->ld == d->n_sym && !(d->n_sym & 3) && !(reinterpret_cast<uintptr_t>(d->prob) & 15u); };
    if (!flat(m->a) || !flat(m->b) || !flat(m->c) || !flat(m->out) || m->c->n_sym < 4)
        return fail(DOL_EUNSUPPORTED, "the one-launch form needs contiguous 16-byte aligned tensors with symbol counts that are multiples of 4");
    return DOL_OK;
}

dol_status dol_apply2_filter_union(const dol_apply_merge *m, void *hip_stream)
{
    const UnionPlan *plan = nullptr;
    if (dol_status st = check_apply_merge(m, &plan)) return st;
    if (m->a->batch == 0) return DOL_OK;
    return launch_damp_table_merge_fwd(m->f, plan, m->a->batch, m->a->prob, m->b->prob, m->c->prob, m->out->prob, m->saved,
                                       static_cast<hipStream_t>(hip_stream));
}

dol_status dol_apply2_filter_union_backward(const dol_apply_merge *m, const float *grad_out, int64_t grad_out_ld, float *grad_a,
                                            float *grad_b, float *grad_c, int32_t accumulate, void *hip_stream)
{
    const UnionPlan *plan = nullptr;
    if (dol_status st = check_apply_merge(m, &plan)) return st;
    if (m->a->batch == 0 || (!grad_a && !grad_b && !grad_c)) return DOL_OK;
    if (!grad_out) return fail(DOL_EINVAL, "grad_out is NULL");
    auto off16 = [](const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) != 0; };
    if (grad_out_ld != plan->n_out || off16(grad_out) || off16(grad_a) || off16(grad_b) || off16(grad_c))
        return fail(DOL_EUNSUPPORTED, "the one-launch form needs contiguous 16-byte aligned gradient tensors");
    if (grad_a && grad_a == grad_b) return fail(DOL_EINVAL, "grad_a and grad_b are the same tensor");
    return launch_damp_table_merge_bwd(m->f, plan, m->a->batch, m->a->prob, m->b->prob, m->c->prob, grad_out, grad_a, grad_b, grad_c,
                                       m->saved, accumulate, static_cast<hipStream_t>(hip_stream));
}

dol_status dol_apply2_filter_union_forward_backward(const dol_apply_merge *m, const float *grad_out, int64_t grad_out_ld,
                                                    float *grad_a, float *grad_b, float *grad_c, int32_t accumulate,
                                                    void *hip_stream)
{
    const UnionPlan *plan = nullptr;
    if (dol_status st = check_apply_merge(m, &plan)) return st;
    if (!grad_out) return fail(DOL_EINVAL, "grad_out is NULL");
    if (!grad_a && !grad_b && !grad_c) return fail(DOL_EINVAL, "grad_a, grad_b and grad_c are all NULL");
    if (!m->saved) return fail(DOL_EINVAL, "saved is NULL: the backward pass of this call reads the forward pass's clamp words");
    auto off16 = [](const void *ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15u) != 0; };
    if (grad_out_ld != plan->n_out || off16(grad_out) || off16(grad_a) || off16(grad_b) || off16(grad_c))
        return fail(DOL_EUNSUPPORTED, "the one-launch form needs contiguous 16-byte aligned gradient tensors");
    if (grad_a && grad_a == grad_b) return fail(DOL_EINVAL, "grad_a and grad_b are the same tensor");
    if (m->a->batch == 0) return DOL_OK;
    return launch_damp_table_merge_both(m->f, plan, m->a->batch, m->a->prob, m->b->prob, m->c->prob, m->out->prob, m->saved, grad_out,
                                        grad_a, grad_b, grad_c, accumulate, static_cast<hipStream_t>(hip_stream));
}

dol_status dol_dtkp_init(dol_dist *d, const int32_t *fact_of_sym, const dol_prov *prov, void *hip_stream)
{
    if (!is_dtkp(prov)) return fail(DOL_EINVAL, "dol_dtkp_init needs a DTKP provenance");
    if (dol_status st = check_dist(d, "d", true, false, true)) return st;
    if (dol_status st = check_prov(prov, d->batch)) return st;
    if (d->n_sym == 0 || d->batch == 0) return DOL_OK;
    if (!d->proof_prob) return fail(DOL_EINVAL, "d.proof_prob is NULL");
    if (!fact_of_sym) return fail(DOL_EINVAL, "fact_of_sym is NULL");
    for (int32_t i = 0; i < d->n_sym; ++i)
        if (fact_of_sym[i] < 0 || fact_of_sym[i] >= prov->n_facts)
            return fail(DOL_EINVAL, "fact_of_sym[%d] = %d outside 0..%d", i, fact_of_sym[i], prov->n_facts - 1);
    const int32_t *d_fos = nullptr;
    if (dol_status st = get_i32_array(d->n_sym, fact_of_sym, &d_fos)) return st;
    return launch_dtkp_init(d->batch, d->n_sym, prov->k, prov->n_facts, d_fos, prov->fact_prob, d->proof_mask,
                            d->proof_prob, d->prob, d->ld, static_cast<hipStream_t>(hip_stream));
}

dol_status dol_dtkp_backward(const dol_dist *d, const dol_prov *prov, const float *grad_prob, int64_t grad_prob_ld,
                             float *grad_fact_prob, void *hip_stream)
{
    if (!is_dtkp(prov)) return fail(DOL_EINVAL, "dol_dtkp_backward needs a DTKP provenance");
    if (dol_status st = check_dist(d, "d", true, false, false)) return st;
    if (dol_status st = check_prov(prov, d->batch)) return st;
    if (d->batch == 0 || prov->n_facts == 0) return DOL_OK;
    if (!grad_fact_prob) return fail(DOL_EINVAL, "grad_fact_prob is NULL");
    if (d->n_sym > 0) {
        if (!d->proof_prob) return fail(DOL_EINVAL, "d.proof_prob is NULL");
        if (!grad_prob) return fail(DOL_EINVAL, "grad_prob is NULL");
        if (grad_prob_ld < d->n_sym) return fail(DOL_ESHAPE, "grad_prob_ld = %lld is smaller than n_sym = %d", static_cast<long long>(grad_prob_ld), d->n_sym);
    }
    return launch_dtkp_prob_bwd(d->batch, d->n_sym, prov->k, prov->n_facts, d->proof_mask, d->proof_prob, prov->fact_prob,
                                grad_prob, grad_prob_ld, grad_fact_prob, static_cast<hipStream_t>(hip_stream));
}

dol_status dol_backward(const dol_op_record *rec, const float *grad_out, float *grad_a, float *grad_b,
                        void *hip_stream)
{
    if (!rec) return fail(DOL_EINVAL, "record is NULL");
    if (is_dtkp(rec->prov)) return fail(DOL_EUNSUPPORTED, "DTKP tags carry their input facts: differentiate the final Distribution with dol_dtkp_backward");
    if (dol_status st = check_prov(rec->prov, 0)) return st;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const dol_dist *a = rec->a, *b = rec->b, *out = rec->out;
    if (dol_status s2 = check_dist(a, "rec.a", false, rec->op == DOL_OP_UNION || rec->op == DOL_OP_FILTER_UNION, true)) return s2;
    if (dol_status s2 = check_dist(out, "rec.out", false, false, rec->op == DOL_OP_APPLY2)) return s2;
    if (a->batch != out->batch) return fail(DOL_ESHAPE, "batch sizes differ: %d, %d", a->batch, out->batch);
    if (!grad_out && out->batch > 0 && out->n_sym > 0) return fail(DOL_EINVAL, "grad_out is NULL");
    switch (rec->op) {
    case DOL_OP_APPLY2: {
        const dol_fn_table *f = rec->f;
        if (!f) return fail(DOL_EINVAL, "rec.f is NULL");
        if (dol_status s2 = check_dist(b, "rec.b", false, false, true)) return s2;
        if (a->batch != b->batch) return fail(DOL_ESHAPE, "batch sizes differ: %d, %d", a->batch, b->batch);
        if (a->n_sym != f->na || b->n_sym != f->nb || out->n_sym != f->n_out)
            return fail(DOL_ESHAPE, "operands have %d x %d -> %d symbols, the table is %d x %d -> %d", a->n_sym, b->n_sym, out->n_sym, f->na, f->nb, f->n_out);
        if (dol_status s2 = check_work(a->batch, f->na + f->nb)) return s2;
        if (f->n_out == 0) {   // nothing was produced: all gradients are zero
            if (grad_a && !(rec->accumulate & 1))
                if (dol_status s2 = launch_zero_rows(a->batch, a->n_sym, grad_a, a->ld, st)) return s2;
            if (grad_b && !(rec->accumulate & 2))
                if (dol_status s2 = launch_zero_rows(b->batch, b->n_sym, grad_b, b->ld, st)) return s2;
            return DOL_OK;
        }
        return launch_damp_apply2_bwd(f, a->batch, a->prob, a->ld, b->prob, b->ld, out->prob, out->ld, grad_out,
                                      out->ld, grad_a, grad_b, rec->accumulate, st);
    }
    case DOL_OP_FILTER: {
        if (a->n_sym > 0 && !rec->pred_mask) return fail(DOL_EINVAL, "rec.pred_mask is NULL");
        const FilterPlan *plan = nullptr;
        if (dol_status s2 = get_filter_plan(a->n_sym, rec->pred_mask, &plan)) return s2;
        if (out->n_sym != plan->n_out) return fail(DOL_ESHAPE, "rec.out.n_sym = %d, the predicate keeps %d symbols", out->n_sym, plan->n_out);
        if (dol_status s2 = check_work(a->batch, a->n_sym)) return s2;
        if (!grad_a) return DOL_OK;
        return launch_damp_filter_bwd(plan, a->batch, grad_out, out->ld, grad_a, a->ld, rec->accumulate, st);
    }
    case DOL_OP_UNION: {
        if (dol_status s2 = check_dist(b, "rec.b", false, true, true)) return s2;
        if (a->batch != b->batch) return fail(DOL_ESHAPE, "batch sizes differ: %d, %d", a->batch, b->batch);
        const UnionPlan *plan = nullptr;
        if (dol_status s2 = get_union_plan(a->n_sym, a->sym_ids, b->n_sym, b->sym_ids, &plan)) return s2;
        if (out->n_sym != plan->n_out) return fail(DOL_ESHAPE, "rec.out.n_sym = %d, the union has %d symbols", out->n_sym, plan->n_out);
        if (dol_status s2 = check_work(a->batch, a->n_sym + b->n_sym)) return s2;
        return launch_damp_union_bwd(plan, a->batch, a->prob, a->ld, b->prob, b->ld, grad_out, out->ld, grad_a, grad_b,
                                     rec->accumulate, st);
    }
    case DOL_OP_FILTER_UNION: {
        if (!rec->pred_mask) return fail(DOL_EINVAL, "rec.pred_mask is NULL");
        if (dol_status s2 = check_dist(b, "rec.b", false, true, true)) return s2;
        if (a->batch != b->batch) return fail(DOL_ESHAPE, "batch sizes differ: %d, %d", a->batch, b->batch);
        const UnionPlan *plan = nullptr;
        if (dol_status s2 = get_filter_union_plan(a->n_sym, a->sym_ids, rec->pred_mask, b->n_sym, b->sym_ids, &plan)) return s2;
        if (out->n_sym != plan->n_out) return fail(DOL_ESHAPE, "rec.out.n_sym = %d, the result has %d symbols", out->n_sym, plan->n_out);
        if (dol_status s2 = check_work(a->batch, a->n_sym + b->n_sym)) return s2;
        return launch_damp_union_bwd(plan, a->batch, a->prob, a->ld, b->prob, b->ld, grad_out, out->ld, grad_a, grad_b,
                                     rec->accumulate, st);
    }
    default:
        return fail(DOL_EINVAL, "unknown operator kind %d", rec->op);
    }
}

dol_status dol_nll_grad(const dol_dist *d, const int32_t *target_col, float *grad, void *hip_stream)
{
    if (dol_status st = check_dist(d, "d", false, false, true)) return st;
    if (d->batch == 0 || d->n_sym == 0) return DOL_OK;
    if (!target_col || !grad) return fail(DOL_EINVAL, "target_col or grad is NULL");
    if (dol_status st = check_work(d->batch, d->n_sym)) return st;
    return launch_nll_grad(d->batch, d->n_sym, d->prob, d->ld, target_col, grad, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
