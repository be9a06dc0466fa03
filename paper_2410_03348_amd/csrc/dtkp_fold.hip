// Fused left fold of Apply under DTKP-AM (the loop of Fig. 2 with the top-k proofs provenance of Sec. 3.2 /
// App. A) over naturally initialised inputs: symbol i of input t carries the single proof {fact_of_sym[t][i]}.
// One wavefront owns a sample: the fact probabilities and the running Distribution's proofs (two buffers of
// S x k masks and probabilities) live in LDS, a lane owns an output symbol, streams the candidates of its tuples
// through a k-entry sorted list in registers and writes the list back to LDS for the next stage.  HBM sees the
// fact probabilities once and the final Distribution once.  Optionally the gradient of the final tag
// probabilities w.r.t. the fact probabilities follows in the same launch (lane f owns fact f).
// Candidate order, proof probabilities, exclusion test and list order are those of dol_apply2, so the result is the
// same bit for bit.  The sorted list of a column carries probabilities and the origin of each proof; masks are built
// for the k winners only, and a stage whose input brings only new, higher facts (fresh_t below) never reads one.
#include "dtkp_util.h"
#include "wave_util.h"

#include <cfloat>
#include <vector>

namespace dol {

constexpr int kDfMax = 32;              // most inputs of one fold

// The symbol side of the whole fold as one array of words, copied into LDS at the start of the kernel:
//   [0] number of inputs n, then for t = 0 .. n-1 four words: S_t, p_t, r_t, fresh_t
//   t = 0:  S_0 words at p_0: the facts of the first input's symbols
//   t >= 1: S_t + 1 words at p_t: where each output column's tuples start and end inside the stage's records;
//           the records at r_t, one per tuple in column order: first operand's symbol | second operand's FACT << 16
//           (one spare record at the end so that the read-ahead stays inside)
//   fresh_t = 1: every fact of input t lies above every fact of the inputs before it and shares no exclusion group
//           with any of them.  A proof of the running Distribution then never holds the new fact or a rival of it, and
//           the product over ascending facts is the proof's stored probability times the new fact's: the stage needs
//           no mask at all until its k winners are known.
struct DtkpFoldArgs {
    int32_t n, batch, n_facts, max_s, n_words;
    const int32_t *words;
    const uint64_t *rival;              // device [n_facts]: the other facts of each fact's exclusion group
    const float *fact_prob;
    uint64_t *om;
    float *op, *oprob;
    int64_t ldo;
    const int32_t *target;
    const float *gout;
    int64_t ldg;
    float *gfact;
};

// One stage of the fold for this wavefront's sample: the columns of the stage's table, a lane each.  KA: slots of the
// first operand's lists that can hold a proof (1 right after the natural initialisation); FRESH: see fresh_t above.
// Absent slots carry the probability -1 in LDS (0 in the result tensors).
// The list keeps, per rank, the probability and where the proof came from (record, slot of the first operand's list);
// the masks are put together for the k winners only.  A candidate whose probability differs from every kept one
// finds its rank by comparing probabilities alone; one that ties (duplicates of a kept proof always do) takes the
// full comparison of the list's contract.
template <int K, int KA, bool FRESH>
__device__ __forceinline__ void dtkp_fold_stage(const DtkpFoldArgs &A, int64_t s, int S, bool last, const uint32_t *l_ptr,
                                                const uint32_t *l_rec, const uint64_t *cm, const float *cp, uint64_t *nm,
                                                float *np, const uint64_t *rival, const float *fp, float *gh)
{
    const int lane = threadIdx.x;
    for (int c = lane; c < S; c += kWave) {
        float tp[K];
        int tid_[K];
#pragma unroll
        for (int x = 0; x < K; ++x) { tp[x] = -1.0f; tid_[x] = -1; }
        auto mask_of = [&](int id) -> uint64_t {
            const int q = id / K, x = id - q * K;
            const uint32_t r = l_rec[q];
            return cm[static_cast<int>(r & 0xffffu) * K + x] | (uint64_t(1) << (r >> 16));
        };
        // the full comparison: equal masks are one proof, order by probability, then by mask
        auto insert_tied = [&](uint64_t mask, float pr, int id) {
            uint64_t tm[K];
            bool dup = false;
#pragma unroll
            for (int y = 0; y < K; ++y) {
                tm[y] = tid_[y] >= 0 ? mask_of(tid_[y]) : kAbsent;
                dup |= tm[y] == mask;
            }
            if (dup || !TopK<K>::before(mask, pr, tm[K - 1], tp[K - 1])) return;
#pragma unroll
            for (int y = K - 1; y >= 0; --y) {
                const bool here = TopK<K>::before(mask, pr, tm[y], tp[y]);
                const bool above = y > 0 ? TopK<K>::before(mask, pr, tm[y - 1], tp[y - 1]) : false;
                if (above) { tp[y] = tp[y - 1]; tid_[y] = tid_[y - 1]; }
                else if (here) { tp[y] = pr; tid_[y] = id; }
            }
        };
        // offer < 0: nothing to offer (below every slot, absent ones included)
        // (the kept probabilities are in descending order and the offer equals none of them: the new list is the larger
        // of the first and the offer, then the median of each neighbouring pair and the offer)
        auto insert_untied = [&](float offer, int id) {
            bool gt[K];
#pragma unroll
            for (int y = 0; y < K; ++y) gt[y] = offer > tp[y];
#pragma unroll
            for (int y = K - 1; y >= 0; --y) {
                const bool above = y > 0 ? gt[y - 1] : false;
                tp[y] = y > 0 ? __builtin_amdgcn_fmed3f(tp[y - 1], tp[y], offer) : fmaxf(tp[0], offer);
                tid_[y] = above ? tid_[y - 1] : gt[y] ? id : tid_[y];
            }
        };
        const uint32_t q0 = l_ptr[c], q1 = l_ptr[c + 1];
        uint32_t rec = l_rec[q0];
        for (uint32_t q = q0; q < q1; ++q) {
            const int i = static_cast<int>(rec & 0xffffu), fb = static_cast<int>(rec >> 16);
            rec = l_rec[q + 1];                 // the next tuple's record is on its way while this one is worked on
            const float pb = 1.0f * fp[fb];
            if constexpr (FRESH) {
                float pa[KA];
#pragma unroll
                for (int x = 0; x < KA; ++x) pa[x] = cp[i * K + x];
#pragma unroll
                for (int x = 0; x < KA; ++x) {
                    const float offer = pa[x] >= 0.0f ? pa[x] * pb : -2.0f;
                    const int id = static_cast<int>(q) * K + x;
                    bool tie = false;
#pragma unroll
                    for (int y = 0; y < K; ++y) tie |= offer == tp[y];
                    if (tie) insert_tied(cm[i * K + x] | (uint64_t(1) << fb), offer, id);
                    else insert_untied(offer, id);
                }
            } else {
                uint64_t ma[KA];
                float pa[KA];
#pragma unroll
                for (int x = 0; x < KA; ++x) { ma[x] = cm[i * K + x]; pa[x] = cp[i * K + x]; }
                const uint64_t mb = uint64_t(1) << fb, bad = rival[fb];
                // kept proofs hold at most one fact per exclusion group, so the union is inconsistent exactly when
                // the first operand's proof holds a rival of the one fact the second brings.  The product over
                // ascending facts is unchanged when the fact is already there, takes one more factor when it lies
                // above every fact of the proof (ma < mb as integers), and is redone from scratch otherwise.
#pragma unroll
                for (int x = 0; x < KA; ++x) {
                    const bool ok = ma[x] != kAbsent && !(ma[x] & bad);
                    const bool plain = (ma[x] & mb) || ma[x] < mb;
                    float pr = (ma[x] & mb) ? pa[x] : pa[x] * pb;
                    if (ok && !plain) pr = proof_prob(ma[x] | mb, fp);
                    const int id = static_cast<int>(q) * K + x;
                    bool tie = false;
#pragma unroll
                    for (int y = 0; y < K; ++y) tie |= pr == tp[y];
                    if (ok && tie) insert_tied(ma[x] | mb, pr, id);
                    else insert_untied(ok ? pr : -2.0f, id);
                }
            }
        }
        float sum = 0.0f;
        uint64_t wm[K];
        float wp[K];
#pragma unroll
        for (int x = 0; x < K; ++x) {
            const bool present = tid_[x] >= 0;
            wm[x] = present ? mask_of(tid_[x]) : kAbsent;
            wp[x] = present ? tp[x] : 0.0f;
            nm[c * K + x] = wm[x];
            np[c * K + x] = present ? tp[x] : -1.0f;
            if (present) sum = sum + tp[x];
        }
        if (last) {
            const int64_t o = (s * S + c) * K;
#pragma unroll
            for (int x = 0; x < K; ++x) { A.om[o + x] = wm[x]; A.op[o + x] = wp[x]; }
            const float pr = fminf(sum, 1.0f);
            A.oprob[s * A.ldo + c] = pr;
            if (A.gfact) {                      // upstream gradient, gated by the clamp (passes on sum <= 1)
                float g;
                if (A.target) g = c == A.target[s] ? -1.0f / fmaxf(pr, FLT_MIN) : 0.0f;
                else g = A.gout[s * A.ldg + c];
                gh[c] = sum <= 1.0f ? g : 0.0f;
            }
        }
    }
}

template <int K>
__global__ void __launch_bounds__(kWave)
dtkp_fold_kernel(const DtkpFoldArgs A)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    // masks of both buffers, rivals, probabilities of both buffers, fact probabilities, gated gradients, symbol side
    uint64_t *bufm = reinterpret_cast<uint64_t *>(lds_raw);
    uint64_t *rival = bufm + 2 * A.max_s * K;
    float *bufp = reinterpret_cast<float *>(rival + 64);
    float *fp = bufp + 2 * A.max_s * K;
    float *gh = fp + 64;
    // the symbol side starts at the next multiple of 16 bytes
    const uint32_t w_off = (static_cast<uint32_t>(reinterpret_cast<unsigned char *>(gh + A.max_s) - lds_raw) + 15u) & ~15u;
    const uint32_t *w = reinterpret_cast<const uint32_t *>(lds_raw + w_off);
    const int lane = threadIdx.x;
    const int64_t s = blockIdx.x;
    const float my_fp = lane < A.n_facts ? A.fact_prob[s * A.n_facts + lane] : 1.0f;
    const uint64_t my_rival = lane < A.n_facts ? A.rival[lane] : 0;
    {   // 16 bytes per lane and four loads in flight: the words are the same for every sample and sit in L2, so what
        // this costs is round trips
        uint4 *wl = reinterpret_cast<uint4 *>(lds_raw + w_off);
        const uint4 *src = reinterpret_cast<const uint4 *>(A.words);
        const int n4 = A.n_words / 4;           // the host pads the array to whole 16-byte pieces
        for (int base = 0; base < n4; base += 4 * kWave) {
            uint4 v[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) v[k] = src[min(base + k * kWave + lane, n4 - 1)];
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (base + k * kWave + lane < n4) wl[base + k * kWave + lane] = v[k];
        }
    }
    fp[lane] = my_fp;
    rival[lane] = my_rival;
    wave_lds_fence();
    {   // natural initialisation (App. A.1)
        const int S0 = static_cast<int>(w[1]);
        const uint32_t *fact0 = w + w[2];
        for (int i = lane; i < S0; i += kWave) {
            const int f = static_cast<int>(fact0[i]);
            bufm[i * K] = uint64_t(1) << f;
            bufp[i * K] = 1.0f * fp[f];
#pragma unroll
            for (int x = 1; x < K; ++x) { bufm[i * K + x] = kAbsent; bufp[i * K + x] = -1.0f; }
        }
    }
    wave_lds_fence();
    int S = 0;
    for (int t = 1; t < A.n; ++t) {
        const uint64_t *cm = bufm + ((t - 1) & 1) * A.max_s * K;
        const float *cp = bufp + ((t - 1) & 1) * A.max_s * K;
        uint64_t *nm = bufm + (t & 1) * A.max_s * K;
        float *np = bufp + (t & 1) * A.max_s * K;
        S = static_cast<int>(w[1 + 4 * t]);
        const uint32_t *l_ptr = w + w[2 + 4 * t], *l_rec = w + w[3 + 4 * t];
        const bool last = t == A.n - 1, fresh = w[4 + 4 * t] != 0;
        if (t == 1) {                       // the first operand is naturally initialised: one proof per symbol
            if (fresh) dtkp_fold_stage<K, 1, true>(A, s, S, last, l_ptr, l_rec, cm, cp, nm, np, rival, fp, gh);
            else dtkp_fold_stage<K, 1, false>(A, s, S, last, l_ptr, l_rec, cm, cp, nm, np, rival, fp, gh);
        } else {
            if (fresh) dtkp_fold_stage<K, K, true>(A, s, S, last, l_ptr, l_rec, cm, cp, nm, np, rival, fp, gh);
            else dtkp_fold_stage<K, K, false>(A, s, S, last, l_ptr, l_rec, cm, cp, nm, np, rival, fp, gh);
        }
        wave_lds_fence();
    }
    if (!A.gfact) return;
    // d Pr / d p_f = sum over the kept proofs holding f of the product of their other facts (ascending symbol, rank)
    const int n1 = A.n - 1;
    const uint64_t *fm = bufm + (n1 & 1) * A.max_s * K;
    const uint64_t mine = uint64_t(1) << lane;
    float acc = 0.0f;
    for (int c = 0; c < S; ++c) {
        const float g = gh[c];
#pragma unroll
        for (int x = 0; x < K; ++x) {
            const uint64_t mm = fm[c * K + x];
            if (mm == kAbsent) continue;
            float others = 1.0f;
            for (uint64_t r = mm; r; r &= r - 1) {
                const int j = __builtin_ctzll(r);
                others = others * (j == lane ? 1.0f : fp[j]);
            }
            if (mm & mine) acc = __builtin_fmaf(g, others, acc);
        }
    }
    if (lane < A.n_facts) A.gfact[s * A.n_facts + lane] = acc;
}

}  // namespace dol

using namespace dol;

extern "C" dol_status dol_dtkp_fold_apply2(const dol_dtkp_fold *fold, const dol_prov *prov, void *hip_stream)
{
    if (!fold || !prov) return fail(DOL_EINVAL, "NULL argument");
    if (prov->kind != DOL_DTKP) return fail(DOL_EINVAL, "dol_dtkp_fold_apply2 needs a DTKP provenance");
    const int n = fold->n_inputs, K = prov->k;
    if (n < 2 || n > kDfMax) return fail(n < 2 ? DOL_EINVAL : DOL_EUNSUPPORTED, "n_inputs = %d outside 2..%d", n, kDfMax);
    if (K < 1 || K > DOL_MAX_K) return fail(DOL_EINVAL, "k = %d outside 1..%d", K, DOL_MAX_K);
    if (prov->n_facts < 1 || prov->n_facts > 63) return fail(DOL_EINVAL, "n_facts = %d outside 1..63", prov->n_facts);
    if (!fold->inputs || !fold->tables || !fold->fact_of_sym || !fold->out) return fail(DOL_EINVAL, "inputs, tables, fact_of_sym or out is NULL");
    DtkpFoldArgs A{};
    A.n = n;
    A.n_facts = prov->n_facts;
    std::vector<int32_t> words(1 + 4 * static_cast<size_t>(n), 0);
    words[0] = n;
    int32_t s_prev = 0, s_last = 0;
    int32_t fact_hi = -1;                   // highest fact of the inputs so far
    uint64_t facts_seen = 0;
    for (int t = 0; t < n; ++t) {
        const dol_dist *d = fold->inputs[t];
        if (!d) return fail(DOL_EINVAL, "inputs[%d] is NULL", t);
        if (d->batch < 0 || d->n_sym < 1) return fail(DOL_ESHAPE, "inputs[%d] has a bad shape", t);
        if (t == 0) A.batch = d->batch;
        if (d->batch != A.batch) return fail(DOL_ESHAPE, "inputs[%d].batch = %d, inputs[0].batch = %d", t, d->batch, A.batch);
        const int32_t *fos = fold->fact_of_sym[t];
        if (!fos) return fail(DOL_EINVAL, "fact_of_sym[%d] is NULL", t);
        for (int32_t i = 0; i < d->n_sym; ++i)
            if (fos[i] < 0 || fos[i] >= prov->n_facts)
                return fail(DOL_EINVAL, "fact_of_sym[%d][%d] = %d outside 0..%d", t, i, fos[i], prov->n_facts - 1);
        {   // fresh_t: this input's facts lie above every earlier fact and share no exclusion group with one
            bool fresh = true;
            uint64_t mine = 0;
            for (int32_t i = 0; i < d->n_sym; ++i) {
                fresh = fresh && fos[i] > fact_hi;
                mine |= uint64_t(1) << fos[i];
            }
            for (int f = 0; f < prov->n_facts && prov->fact_group && fresh; ++f)
                for (int h = 0; h < prov->n_facts && ((mine >> f) & 1); ++h)
                    if (((facts_seen >> h) & 1) && prov->fact_group[h] == prov->fact_group[f]) fresh = false;
            words[4 + 4 * t] = fresh ? 1 : 0;
            for (int32_t i = 0; i < d->n_sym; ++i) fact_hi = std::max(fact_hi, fos[i]);
            facts_seen |= mine;
        }
        if (t == 0) {
            words[1] = d->n_sym;
            words[2] = static_cast<int32_t>(words.size());
            words.insert(words.end(), fos, fos + d->n_sym);
            s_prev = s_last = A.max_s = d->n_sym;
            continue;
        }
        const dol_fn_table *f = fold->tables[t - 1];
        if (!f) return fail(DOL_EINVAL, "tables[%d] is NULL", t - 1);
        if (f->na != s_prev || f->nb != d->n_sym)
            return fail(DOL_ESHAPE, "tables[%d] is %d x %d, its operands have %d and %d symbols", t - 1, f->na, f->nb, s_prev, d->n_sym);
        if (f->n_out < 1) return fail(DOL_EUNSUPPORTED, "tables[%d] produces no symbol", t - 1);
        if (words.size() + static_cast<size_t>(f->n_out) + static_cast<size_t>(f->n_tuples) + 2 > 16000)
            return fail(DOL_EUNSUPPORTED, "the tables of the fold do not fit in LDS");
        words[1 + 4 * t] = f->n_out;
        words[2 + 4 * t] = static_cast<int32_t>(words.size());
        words.insert(words.end(), f->h_col_ptr.begin(), f->h_col_ptr.begin() + f->n_out + 1);
        words[3 + 4 * t] = static_cast<int32_t>(words.size());
        for (int64_t q = 0; q < f->n_tuples; ++q) {
            const uint32_t ij = f->h_col_ij[static_cast<size_t>(q)];
            words.push_back(static_cast<int32_t>((ij & 0xffffu) | (static_cast<uint32_t>(fos[ij >> 16]) << 16)));
        }
        words.push_back(0);
        s_prev = s_last = f->n_out;
        A.max_s = f->n_out > A.max_s ? f->n_out : A.max_s;
    }
    while (words.size() % 4) words.push_back(0);
    A.n_words = static_cast<int32_t>(words.size());
    const dol_dist *o = fold->out;
    if (o->batch != A.batch || o->n_sym != s_last || o->ld < o->n_sym)
        return fail(DOL_ESHAPE, "out has %d x %d, the fold produces %d x %d", o->batch, o->n_sym, A.batch, s_last);
    const size_t lds = static_cast<size_t>(2) * A.max_s * K * (sizeof(uint64_t) + sizeof(float)) + 64 * sizeof(uint64_t) +
                       sizeof(float) * (64 + A.max_s) + 16 + sizeof(uint32_t) * words.size();
    if (lds > 64 * 1024) return fail(DOL_EUNSUPPORTED, "the fold needs %zu bytes of LDS per sample, more than 65536", lds);
    if (A.batch == 0) return DOL_OK;
    if (!o->proof_mask || !o->proof_prob || !o->prob) return fail(DOL_EINVAL, "out.proof_mask, out.proof_prob or out.prob is NULL");
    if (!prov->fact_prob) return fail(DOL_EINVAL, "prov.fact_prob is NULL");
    {   // rival[f]: the other facts of f's exclusion group (a device array cached by content)
        std::vector<int32_t> words(2 * static_cast<size_t>(prov->n_facts), 0);
        for (int f = 0; f < prov->n_facts && prov->fact_group; ++f) {
            uint64_t r = 0;
            for (int h = 0; h < prov->n_facts; ++h)
                if (h != f && prov->fact_group[h] == prov->fact_group[f]) r |= uint64_t(1) << h;
            words[2 * f] = static_cast<int32_t>(static_cast<uint32_t>(r));
            words[2 * f + 1] = static_cast<int32_t>(static_cast<uint32_t>(r >> 32));
        }
        const int32_t *dptr = nullptr;
        if (dol_status st = get_i32_array(2 * prov->n_facts, words.data(), &dptr)) return st;
        A.rival = reinterpret_cast<const uint64_t *>(dptr);
    }
    if (dol_status st = get_i32_array(A.n_words, words.data(), &A.words)) return st;
    A.fact_prob = prov->fact_prob;
    A.om = o->proof_mask;
    A.op = o->proof_prob;
    A.oprob = o->prob;
    A.ldo = o->ld;
    A.gfact = fold->grad_fact_prob;
    A.target = fold->target_col;
    A.gout = fold->grad_out;
    A.ldg = fold->grad_out_ld;
    if (A.gfact && !A.target) {
        if (!A.gout) return fail(DOL_EINVAL, "grad_fact_prob needs target_col or grad_out");
        if (A.ldg < s_last) return fail(DOL_ESHAPE, "grad_out_ld = %lld is smaller than %d", static_cast<long long>(A.ldg), s_last);
    }
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const dim3 grid(static_cast<unsigned>(A.batch)), block(kWave);
#define DOL_DF(KK) hipLaunchKernelGGL(dtkp_fold_kernel<KK>, grid, block, lds, st, A)
    switch (K) {
    case 1: DOL_DF(1); break;
    case 2: DOL_DF(2); break;
    case 3: DOL_DF(3); break;
    case 4: DOL_DF(4); break;
    case 5: DOL_DF(5); break;
    case 6: DOL_DF(6); break;
    case 7: DOL_DF(7); break;
    default: DOL_DF(8); break;
    }
#undef DOL_DF
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}
