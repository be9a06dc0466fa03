/*
 * dolphin_hip.h -- C ABI of the MI355X (gfx950) hot path of the Dolphin
 * neurosymbolic framework (arXiv 2410.03348): batched Distribution operators
 * evaluated under a provenance.
 *
 * Vocabulary (Sec. 3.1): a Distribution maps a batch-invariant list of symbols
 * to batched tags.  Symbols live on the host as ascending int32 ids; tags live
 * on the device.  Under DAMP (Sec. 3.2, Table 1) a tag is one probability per
 * (sample, symbol).  Under DTKP-AM (Sec. 3.2, App. A) a tag is up to k proofs;
 * here a proof is a 64-bit set of input facts plus its probability, instead of
 * the paper's (k x |I|) tensor of +-inf-padded probabilities.
 *
 * General rules
 *   - "host" pointers are ordinary CPU memory, read during the call only
 *     (unless stated otherwise).  "device" pointers are HIP device memory on
 *     the current device, owned by the caller; the library never frees or
 *     reallocates them.
 *   - Every operator call is asynchronous on `hip_stream` (a hipStream_t cast
 *     to void*, NULL = the default stream), never synchronises the device and
 *     performs no allocation once its symbol-side plan exists (the first call
 *     with a new fn_table / predicate / symbol-list pair builds and uploads a
 *     small plan synchronously; later calls reuse it).
 *   - Errors are reported as a non-zero dol_status; dol_last_error() gives a
 *     thread-local message.  Argument and shape errors are detected before any
 *     launch and leave the outputs untouched.  Nothing throws or aborts.
 *   - batch == 0 or an empty symbol list is legal and does nothing.
 *   - Tag tensors are row-major [batch, ld] float with ld >= n_sym (elements).
 *   - DAMP tags must lie in [0, 1].
 */
#ifndef DOLPHIN_HIP_H
#define DOLPHIN_HIP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DOL_MAX_K 8            /* DTKP: most proofs kept per tag */
#define DOL_MAX_FACTS 63       /* DTKP: most input facts (bit 0..62); the all-ones mask marks an absent proof */
#define DOL_MAX_ARITY 6        /* most operands of dol_apply_k */
#define DOL_MAX_SYMBOLS 65535  /* most symbols per Distribution / operand of a function table */
#define DOL_ABSENT_PROOF UINT64_MAX

typedef enum {
    DOL_OK = 0,
    DOL_EINVAL = 1,        /* NULL where data is needed, bad enum, unsorted symbol ids, ... */
    DOL_ESHAPE = 2,        /* operand sizes do not fit each other or the table */
    DOL_ENOMEM = 3,        /* host or device allocation of a plan failed */
    DOL_EHIP = 4,          /* a HIP runtime call failed; message holds hipGetErrorString */
    DOL_EUNSUPPORTED = 5   /* valid request the library does not implement */
} dol_status;

typedef enum { DOL_DAMP = 0, DOL_DTKP = 1 } dol_prov_kind;

/* Provenance (Sec. 3.2): which (tag space, conjunction, disjunction) the operators use.
 * DAMP: conjunction t*t', disjunction min(1, t+t').  Only `kind` is read.
 * DTKP: conjunction = top-k over all pairs of proofs of the union of their fact sets,
 *       disjunction = top-k of the concatenation (Table 1); repeated proofs count once;
 *       order: higher probability first, ties by smaller mask.  A proof holding two
 *       facts of one exclusion group is dropped.  A proof's probability is the float
 *       product of fact_prob over its facts in ascending fact index, starting from 1. */
typedef struct {
    int32_t kind;                /* dol_prov_kind */
    int32_t k;                   /* DTKP: 1..DOL_MAX_K */
    int32_t n_facts;             /* DTKP: 0..DOL_MAX_FACTS */
    const int32_t *fact_group;   /* DTKP, host [n_facts]: exclusion group of each fact (>=0), or NULL = none */
    const float *fact_prob;      /* DTKP, device [batch, n_facts] row-major: probability of each input fact */
} dol_prov;

/* A Distribution (Sec. 3.1.1). */
typedef struct {
    int32_t batch;               /* samples */
    int32_t n_sym;               /* symbols, 0..DOL_MAX_SYMBOLS */
    int64_t ld;                  /* elements between consecutive rows of prob, >= n_sym */
    const int32_t *sym_ids;      /* host [n_sym], strictly ascending */
    float *prob;                 /* device [batch, ld]: DAMP tag; DTKP: the tag's probability (GetProbs) */
    uint64_t *proof_mask;        /* DTKP, device [batch, n_sym, k]: kept proofs by rank, absent = DOL_ABSENT_PROOF */
    float *proof_prob;           /* DTKP, device [batch, n_sym, k]: their probabilities, absent = 0 */
} dol_dist;

/* Symbol side of Apply / ApplyIf with K=2 (Sec. 3.1.2, Eq. 1-2): the user function evaluated
 * once for the whole batch over operand positions (i, j), 0 <= i < na, 0 <= j < nb.
 * The handle owns host and device copies of its index structures. */
typedef struct dol_fn_table dol_fn_table;

/* out_id: host [na*nb] row-major, the produced symbol id (>= 0) or -1 where the condition rejects (i, j). */
dol_status dol_fn_table_create_dense(int32_t na, int32_t nb, const int32_t *out_id, dol_fn_table **table);
/* The n admitted tuples (i[t], j[t]) -> out_id[t] >= 0, any order, each (i, j) at most once. */
dol_status dol_fn_table_create_sparse(int32_t na, int32_t nb, int64_t n, const int32_t *i, const int32_t *j,
                                      const int32_t *out_id, dol_fn_table **table);
/* Number of distinct produced symbols S, and their ids ascending (host [S], valid until destroy).
 * Column c of the result of dol_apply2 is symbol out_syms[c]. */
int32_t dol_fn_table_n_out(const dol_fn_table *table);
const int32_t *dol_fn_table_out_syms(const dol_fn_table *table);
/* Name of the HIP kernel that dol_apply2 (which = 0) or dol_backward (which = 1) launches for this table under
 * DAMP, as a profiler prints it without namespace and arguments (valid until destroy).  The library picks the
 * kernel from the table's structure (Sec. 3.1.2: the symbol side is known before any tag is touched). */
const char *dol_fn_table_kernel(const dol_fn_table *table, int32_t which);
/* The same for a batch of the given size with contiguous, 16-byte aligned tensors: some tables get another kernel
 * once the batch fills the chip (valid until the next call on this thread). */
const char *dol_fn_table_kernel_at(const dol_fn_table *table, int32_t which, int64_t batch);
/* Synchronises the device before releasing the device copies.  NULL is ignored. */
void dol_fn_table_destroy(dol_fn_table *table);

/* ApplyIf with K=2 (Sec. 3.1.2): the table of f_apply restricted to the tuples f_cond admits.
 * out_id: host [na*nb] row-major, f_apply(i, j) (>= 0; entries where cond is 0 are not read);
 * cond: host [na*nb], non-zero where f_cond(i, j) holds.  dol_apply2 with this table is ApplyIf. */
dol_status dol_fn_table_create_if(int32_t na, int32_t nb, const int32_t *out_id, const uint8_t *cond,
                                  dol_fn_table **table);

/* Apply, K=2 (Eq. 1-3): out(s) = disjunction over admitted (i, j) with f(i, j) = s of a(i) conjunction b(j).
 * a->n_sym == na, b->n_sym == nb, out->n_sym == S, equal batch.  prov NULL = DAMP.
 * DAMP: out->prob[s,c] = min(1, sum a.prob[s,i] * b.prob[s,j]); the sum runs over the tuples of column c
 *       in ascending (i, j) with one fused multiply-add each (this fixes the clamp decision of backward).
 * DTKP: reads a/b->proof_mask and, where not NULL, a/b->proof_prob (each entry must be its proof's probability as
 * this library computes it: the product of the fact probabilities in ascending fact index; with NULL the kernel
 * derives every probability from the masks); writes out->proof_mask, out->proof_prob and out->prob (all required). */
dol_status dol_apply2(const dol_dist *a, const dol_dist *b, const dol_fn_table *f, const dol_prov *prov,
                      dol_dist *out, void *hip_stream);

/* Apply, K=2, under DTKP-AM with an input Distribution as second operand (the shape of every fold over model
 * outputs: D_res = apply(D_res, D_i, f), Fig. 2): symbol j of the second operand is input fact fact_of_sym_b[j]
 * (host [nb], each in 0..n_facts-1) and carries the tag natural initialisation gives it (App. A.1: the single proof
 * {that fact}).  The result equals dol_dtkp_init on the operand followed by dol_apply2; the operand's tags are
 * never stored.  a, f, prov, out as for dol_apply2, and each proof of a must hold at most one fact per exclusion
 * group (every proof this library writes does): the conjunction is then inconsistent exactly when the proof holds
 * another fact of the group of the fact it is joined with, which is all this call tests. */
dol_status dol_dtkp_apply2_input(const dol_dist *a, const int32_t *fact_of_sym_b, const dol_fn_table *f,
                                 const dol_prov *prov, dol_dist *out, void *hip_stream);

/* Filter (Sec. 3.1.2): symbols whose pred_mask entry is 0 are removed, the rest keep tags and order.
 * pred_mask: host [d->n_sym].  dol_filter_plan returns the kept count and (if out_syms != NULL,
 * room for d->n_sym) the kept ids, so that the caller can allocate `out`. */
dol_status dol_filter_plan(const dol_dist *d, const uint8_t *pred_mask, int32_t *n_out, int32_t *out_syms);
dol_status dol_filter(const dol_dist *d, const uint8_t *pred_mask, const dol_prov *prov, dol_dist *out,
                      void *hip_stream);

/* Union (Sec. 3.1.2): symbols of either input (ascending merge of the id lists); a symbol of both gets the
 * disjunction of its two tags (DAMP min(1, a+b); DTKP top-k of both proof lists), others are copied.
 * dol_union_plan: merged count and ids (out_syms has room for a->n_sym + b->n_sym). */
dol_status dol_union_plan(const dol_dist *a, const dol_dist *b, int32_t *n_out, int32_t *out_syms);
dol_status dol_union(const dol_dist *a, const dol_dist *b, const dol_prov *prov, dol_dist *out, void *hip_stream);

/* union(filter(d, pred_mask), c) in one launch, DAMP only (the apply_if-then-union step of the recursion of App. B,
 * Fig. 9, once the Apply has run): the filtered Distribution is never materialised.  Same values as dol_filter
 * followed by dol_union.  dol_filter_union_plan: resulting count and ids (out_syms has room for d->n_sym + c->n_sym).
 * Backward: dol_backward with op = DOL_OP_FILTER_UNION, a = d, b = c, pred_mask and out as here; grad_a is
 * [batch, d->ld] (dropped symbols get 0). */
dol_status dol_filter_union_plan(const dol_dist *d, const uint8_t *pred_mask, const dol_dist *c, int32_t *n_out,
                                 int32_t *out_syms);
dol_status dol_filter_union(const dol_dist *d, const uint8_t *pred_mask, const dol_dist *c, const dol_prov *prov,
                            dol_dist *out, void *hip_stream);

/* union(filter(apply2(a, b, f), pred_mask), c) in ONE launch under DAMP (one step of the recursion of App. B, Fig. 9:
 * merged = union(paths, apply_if(...)), with a Filter in between as in Ex. 3.3): neither the Apply's result nor the
 * filtered Distribution ever leaves the chip.  Same values, same clamp decisions as dol_apply2 followed by
 * dol_filter_union (Eq. 1-3 with the fused multiply-add order of dol_apply2; the union's min(1, x + y) on one float add).
 *   a, b, f     as for dol_apply2
 *   pred_mask   host [dol_fn_table_n_out(f)], 1 = the produced symbol is kept
 *   c           the Distribution the kept symbols are merged with
 *   out         n_sym and sym_ids as dol_filter_union_plan gives for (a Distribution over f's symbols, pred_mask, c)
 *   saved       device [batch] int32 or NULL: the forward call leaves 1 for a sample in which some clamp acted (a sum
 *               of the Apply or of the union above 1) and 0 otherwise; the reverse call reads it and re-derives the
 *               clamp decisions only for tiles of 64 samples that hold such a sample (with NULL: for every tile)
 * dol_apply2_filter_union_backward: grad_out device [batch, grad_out_ld] w.r.t. out; grad_a, grad_b, grad_c device
 * [batch, n_sym] of a, b, c, each overwritten, or added to where `accumulate` has bit 0, 1, 2 set; any may be NULL.
 *   gh = grad_out gated by the union's clamp (symbols of both sides) -> grad_c, and, for the kept symbols of the
 *   Apply, further by [pre <= 1] -> grad_a, grad_b as dol_backward defines them.
 * Supported when the table has at most 64 x 64 symbols and produces at most 512, all symbol counts (a, b, f's result,
 * c, out) are multiples of 4 and every tensor is contiguous (ld == n_sym) and 16-byte aligned; otherwise
 * DOL_EUNSUPPORTED and the caller composes dol_apply2, dol_filter_union and dol_backward.  The first call with a table
 * builds its code (synchronously, about a second); later calls are pure asynchronous launches. */
typedef struct {
    const dol_dist *a, *b;
    const dol_fn_table *f;
    const uint8_t *pred_mask;
    const dol_dist *c;
    dol_dist *out;
    int32_t *saved;
} dol_apply_merge;
dol_status dol_apply2_filter_union(const dol_apply_merge *m, void *hip_stream);
dol_status dol_apply2_filter_union_backward(const dol_apply_merge *m, const float *grad_out, int64_t grad_out_ld, float *grad_a,
                                            float *grad_b, float *grad_c, int32_t accumulate, void *hip_stream);
/* Both of the above in ONE launch, for an upstream gradient that does not depend on this call's result (as
 * dol_fold_apply2 runs the loop of Fig. 2 both ways): out and saved are written as by dol_apply2_filter_union, the
 * gradients as by dol_apply2_filter_union_backward, bit for bit.  saved must be given. */
dol_status dol_apply2_filter_union_forward_backward(const dol_apply_merge *m, const float *grad_out, int64_t grad_out_ld,
                                                    float *grad_a, float *grad_b, float *grad_c, int32_t accumulate,
                                                    void *hip_stream);

/* DTKP natural initialisation (App. A.1): symbol i of `d` gets the single proof {fact_of_sym[i]}.
 * fact_of_sym: host [d->n_sym].  Writes proof_mask, proof_prob and prob. */
dol_status dol_dtkp_init(dol_dist *d, const int32_t *fact_of_sym, const dol_prov *prov, void *hip_stream);

/* One recorded forward operator, for the backward pass. */
typedef enum { DOL_OP_APPLY2 = 0, DOL_OP_FILTER = 1, DOL_OP_UNION = 2, DOL_OP_FILTER_UNION = 3 } dol_op_kind;
typedef struct {
    int32_t op;                  /* dol_op_kind */
    const dol_dist *a;           /* first (or only) input, as passed to the forward call, tags unchanged since */
    const dol_dist *b;           /* second input (apply2, union) or NULL */
    const dol_dist *out;         /* the forward result */
    const dol_fn_table *f;       /* apply2 */
    const uint8_t *pred_mask;    /* filter, host */
    const dol_prov *prov;        /* NULL = DAMP */
    int32_t accumulate;          /* bit 0: add into grad_a instead of overwriting it; bit 1: same for grad_b */
} dol_op_record;

/* Vector-Jacobian product of one DAMP operator (the paper relies on autograd, Sec. 3.1.1; the clamp passes
 * gradient 1 inside and on its bounds, App. A.2).  grad_out: device [batch, out->ld].
 * grad_a: device [batch, a->ld], grad_b: device [batch, b->ld]; the first n_sym entries of each row are
 * OVERWRITTEN, or added to where rec->accumulate says so (a Distribution used by several operators sums the
 * gradients of its uses); either may be NULL to skip it.
 *   apply2: gh = grad_out * [pre <= 1];  grad_a[i] = sum_j gh[col(i,j)] * b[j];  grad_b[j] = sum_i gh[col(i,j)] * a[i]
 *   filter: grad_a[i] = grad_out[position of i] for kept symbols, else 0
 *   union:  common symbols pass grad_out * [a + b <= 1] to both sides, one-sided symbols pass grad_out.
 *   filter-union: as union over the kept symbols of a; the dropped symbols of a get 0.
 * DTKP records return DOL_EUNSUPPORTED: see dol_dtkp_backward. */
dol_status dol_backward(const dol_op_record *rec, const float *grad_out, float *grad_a, float *grad_b,
                        void *hip_stream);

/* Gradient of a DTKP Distribution's tag probabilities w.r.t. the probabilities of the input facts (Sec. 3.2:
 * Pr(t) = min(1, sum_i prod_j norm(t_ij)); App. A.2: the clamp passes gradient inside and on its bounds).  A DTKP tag
 * names the input facts it rests on, so one call on the final Distribution of a program replaces the reverse sweep
 * over its operators; the proofs top-k kept are constants of the differentiation.
 *   d               the Distribution (proof_mask, proof_prob as the forward calls left them)
 *   prov            the provenance the forward calls used (same fact_prob contents)
 *   grad_prob       device [batch, grad_prob_ld]: d loss / d prob of each symbol of d
 *   grad_fact_prob  device [batch, n_facts], OVERWRITTEN:
 *                   sum over symbols with unclamped probability and their proofs holding fact f of
 *                   grad_prob * (product of the proof's other facts' probabilities)
 * Asynchronous on the stream; errors as for the other calls. */
dol_status dol_dtkp_backward(const dol_dist *d, const dol_prov *prov, const float *grad_prob, int64_t grad_prob_ld,
                             float *grad_fact_prob, void *hip_stream);

/* ---- Apply / ApplyIf over K Distributions, K = 1..DOL_MAX_ARITY (Sec. 3.1.2: Apply: D^K x (S^K -> S) -> D,
 * ApplyIf: D^K x (S^K -> S) x (S^K -> B) -> D; Eq. 1-3).  K = 1 is the unary Apply that maps every symbol through f
 * and disjoins the tags of symbols with one image.
 * Symbol side: the admitted tuples, once for the whole batch.  idx: host [n*K], idx[t*K + l] = position of tuple t's
 * symbol in operand l (0 <= . < n_sym[l]); out_id: host [n], f(tuple) >= 0, or < 0 where f_cond rejects the tuple
 * (such tuples are dropped).  Any order, each index tuple at most once.  The handle owns host and device copies. */
typedef struct dol_fnk_table dol_fnk_table;
dol_status dol_fnk_table_create(int32_t K, const int32_t *n_sym, int64_t n, const int32_t *idx,
                                const int32_t *out_id, dol_fnk_table **table);
/* Distinct produced symbols S and their ids ascending (host [S], valid until destroy): column c of the result. */
int32_t dol_fnk_table_n_out(const dol_fnk_table *table);
const int32_t *dol_fnk_table_out_syms(const dol_fnk_table *table);
/* Name of the HIP kernel that dol_apply_k (which = 0) or dol_apply_k_backward (which = 1) launches for this table
 * under DAMP, as a profiler prints it without namespace (valid until the next call on this thread); the library
 * picks it from the table's structure, as dol_fn_table_kernel does. */
const char *dol_fnk_table_kernel(const dol_fnk_table *table, int32_t which);
/* Synchronises the device before releasing the device copies.  NULL is ignored. */
void dol_fnk_table_destroy(dol_fnk_table *table);

/* out(s) = disjunction over admitted tuples with f(tuple) = s of in[0](i_0) conjunction ... conjunction in[K-1](i_{K-1}).
 * in: host array of K Distributions, in[l]->n_sym == n_sym[l]; out->n_sym == S; equal batch.  prov NULL = DAMP.
 * DAMP: out->prob[s,c] = min(1, pre), pre = float sum over the tuples of column c in ascending index order of one
 *       term each: K = 1 adds the tag; K >= 2 multiplies the first K-1 tags left to right and enters the product
 *       through one fused multiply-add with the last tag (K = 2 is dol_apply2's rule).  This fixes [pre <= 1].
 * DTKP: the conjunction of Table 1 is binary; a tuple's tag is that operation folded over the operands left to
 *       right, each intermediate pruned to its top k proofs; the disjunction is one top-k over the tuples' proofs.
 *       Reads in[l]->proof_mask and, where not NULL, proof_prob (canonical, see dol_apply2); writes out->proof_mask,
 *       out->proof_prob, out->prob. */
dol_status dol_apply_k(int32_t K, const dol_dist *const *in, const dol_fnk_table *f, const dol_prov *prov,
                       dol_dist *out, void *hip_stream);
/* Vector-Jacobian product of dol_apply_k under DAMP: gh = grad_out * [pre <= 1],
 *   grad_in[l][s, i] = sum over admitted tuples t with idx[t][l] = i of gh[s, col(t)] * prod_{m != l} in[m][s, idx[t][m]].
 * out: the forward result (prob read); grad_out: device [batch, grad_out_ld]; grad_in: host array of K device
 * pointers [batch, in[l]->ld], first n_sym[l] entries of each row OVERWRITTEN; a NULL entry is skipped. */
dol_status dol_apply_k_backward(int32_t K, const dol_dist *const *in, const dol_fnk_table *f, const dol_dist *out,
                                const float *grad_out, int64_t grad_out_ld, float *const *grad_in, void *hip_stream);

/* A left fold of Apply under DAMP (the loop of Fig. 2: D_res = apply(D_res, D_i, f)), forward and backward in
 * ONE launch: acc_1 = apply2(inputs[0], inputs[1], tables[0]), acc_t = apply2(acc_{t-1}, inputs[t], tables[t-1]).
 * Results are the same as n_inputs-1 dol_apply2 calls followed by the reverse sweep of dol_backward calls
 * (same summation order, same clamp decisions); the intermediate Distributions never leave the chip.
 *   inputs      host array of n_inputs Distributions (any ld), equal batch
 *   tables      host array of n_inputs-1 tables; tables[t-1] is (symbols of acc_{t-1}) x (symbols of inputs[t])
 *   out         the last acc (forward result), prob written; may be NULL to skip the store
 *   target_col  device [batch] int32 or NULL: if given, the upstream gradient is that of -log out[target_col]
 *               (as dol_nll_grad); else grad_out (device [batch, out_ld]) is used; both NULL = forward only
 *   grad_inputs host array of n_inputs device pointers, grad_inputs[t] is [batch, inputs[t]->ld], overwritten;
 *               NULL entries are skipped; the array itself may be NULL when no backward is asked for
 * Supported when every table is convolution-shaped (tuple (i, j) lands in column i + j, all tuples admitted:
 * sums of integer-valued symbols), inputs[t >= 1] have at most 16 symbols, n_inputs <= 32 and the per-sample
 * working set fits in LDS; otherwise DOL_EUNSUPPORTED and the caller composes dol_apply2 / dol_backward. */
typedef struct {
    int32_t n_inputs;
    const dol_dist *const *inputs;
    const dol_fn_table *const *tables;
    dol_dist *out;
    const int32_t *target_col;
    const float *grad_out;
    int64_t grad_out_ld;
    float *const *grad_inputs;
} dol_fold;
dol_status dol_fold_apply2(const dol_fold *fold, void *hip_stream);
/* Name of the kernel dol_fold_apply2 launches for this description, as a profiler prints it ("" if the
 * description is rejected).  Host only; the string belongs to the library and is valid until the calling
 * thread's next call of this function. */
const char *dol_fold_kernel(const dol_fold *fold);

/* A left fold of Apply under DTKP-AM over naturally initialised inputs (the loop of Fig. 2 with the top-k proofs
 * provenance of Sec. 3.2 / App. A), in ONE launch: symbol i of inputs[t] carries the single proof
 * {fact_of_sym[t][i]} (as dol_dtkp_init would write it), acc_1 = apply2(inputs[0], inputs[1], tables[0]),
 * acc_t = apply2(acc_{t-1}, inputs[t], tables[t-1]).  The result equals dol_dtkp_init on every input followed by
 * n_inputs-1 dol_apply2 calls, bit for bit; neither the inputs' tags nor the intermediate Distributions touch HBM.
 *   inputs          host array of n_inputs Distributions: only batch and n_sym are read
 *   fact_of_sym     host array of n_inputs host arrays [inputs[t]->n_sym]
 *   tables          host array of n_inputs-1 tables; tables[t-1] is (symbols of acc_{t-1}) x (symbols of inputs[t])
 *   out             the last acc: proof_mask, proof_prob and prob written (all required)
 *   grad_fact_prob  device [batch, n_facts] or NULL: if given, also the gradient of the loss w.r.t. the fact
 *                   probabilities as dol_dtkp_backward defines it, OVERWRITTEN; the upstream gradient is that of
 *                   -log out[target_col] (target_col: device [batch] int32) or grad_out (device [batch, grad_out_ld])
 * DOL_EUNSUPPORTED when n_inputs > 32 or two generations of proofs (2 * max symbols * k * 12 bytes) exceed 64 KB. */
typedef struct {
    int32_t n_inputs;
    const dol_dist *const *inputs;
    const int32_t *const *fact_of_sym;
    const dol_fn_table *const *tables;
    dol_dist *out;
    const int32_t *target_col;
    const float *grad_out;
    int64_t grad_out_ld;
    float *grad_fact_prob;
} dol_dtkp_fold;
dol_status dol_dtkp_fold_apply2(const dol_dtkp_fold *fold, const dol_prov *prov, void *hip_stream);

/* Repeated Apply with feedback under DAMP (the recursion of App. B, Fig. 9, run for a fixed number of rounds):
 *     r_0 = r0,   r_{t+1} = apply2(r_t, e, f)   for t = 0 .. rounds-1,
 * all rounds in ONE launch, one workgroup per sample with r_t in LDS.  The table must be square: it produces
 * exactly the symbols of its first operand (n_out == na and out_syms == r0->sym_ids), so that a round's result
 * can be the next round's first operand.  Results equal `rounds` dol_apply2 calls (same order, same clamps).
 * The reverse sweep needs the rounds in between; the caller chooses what it keeps of them:
 *
 * Full history (rounds + 1 tensors through HBM):
 *   hist  device [rounds+1, batch, na], contiguous: receives r_0 .. r_rounds; r_rounds is the result and the
 *         whole history is what dol_iterate_backward reads.
 *   dol_iterate_backward: grad_out device [batch, grad_out_ld] w.r.t. r_rounds;
 *     grad_r0 device [batch, na] contiguous or NULL; grad_e device [batch, e->ld] or NULL: the gradient w.r.t. e
 *     summed over the rounds.  Both overwritten.
 *
 * Checkpoints (only r_rounds and every ckpt_every-th round leave the chip; the reverse sweep replays each stretch
 * of ckpt_every rounds forward in LDS before walking it backwards, same arithmetic, same results bit for bit):
 *   dol_iterate_apply2_ckpt: out->prob receives r_rounds; ckpt, device [n_ckpt, batch, na] contiguous with
 *     n_ckpt = dol_iterate_ckpt_count(rounds, ckpt_every) = ceil(rounds / ckpt_every) - 1, receives r_{ckpt_every},
 *     r_{2 ckpt_every}, ... (those before r_rounds); may be NULL when n_ckpt == 0.
 *   dol_iterate_backward_ckpt: r0, e, f, rounds, ckpt_every, ckpt as in the forward call; gradients as above.
 *
 * The gradient w.r.t. e is summed in a fixed order (no atomics): two runs give the same bits.
 * DOL_EUNSUPPORTED when the table is not square, an operand has more than 4096 symbols, or the rows (for the
 * reverse sweep: ckpt_every + 3 rows of na tags, na rounded up to 512, 1024, 2048 or 4096, plus e; and one word per
 * tuple when a symbol of the first operand has more tuples than a thread keeps in registers) do not fit in 160 KB of
 * LDS.  dol_iterate_ckpt_every gives an interval that fits. */
dol_status dol_iterate_apply2(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds, float *hist,
                              void *hip_stream);
dol_status dol_iterate_backward(const dol_dist *e, const dol_fn_table *f, int32_t rounds, const float *hist,
                                const float *grad_out, int64_t grad_out_ld, float *grad_r0, float *grad_e,
                                void *hip_stream);
int32_t dol_iterate_ckpt_count(int32_t rounds, int32_t ckpt_every);
/* A checkpoint interval for `rounds` rounds of f over `batch` samples: the fewest segments whose rows fit the LDS a
 * workgroup of the reverse sweep gets (a whole compute unit's while the batch leaves units idle, its share of one
 * otherwise).  Host only, no device work; 1 when f is NULL or rounds <= 1.  Any interval >= 1 that fits is valid for the
 * calls below; this is the one the library's own measurements favour (App. B, Fig. 9: the recursion with a fixed round
 * count). */
int32_t dol_iterate_ckpt_every(const dol_fn_table *f, int32_t batch, int32_t rounds);
dol_status dol_iterate_apply2_ckpt(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds,
                                   int32_t ckpt_every, dol_dist *out, float *ckpt, void *hip_stream);
dol_status dol_iterate_backward_ckpt(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds,
                                     int32_t ckpt_every, const float *ckpt, const float *grad_out, int64_t grad_out_ld,
                                     float *grad_r0, float *grad_e, void *hip_stream);
/* dol_iterate_apply2_ckpt and dol_iterate_backward_ckpt in ONE call (as dol_fold_apply2 runs the loop of Fig. 2 both
 * ways): the rounds forward, r_rounds into out and the checkpoints into ckpt, then the reverse sweep from the upstream
 * gradient.  Up to 512 samples the call is one launch (the last segment of rounds stays in LDS between the sweeps);
 * above, it issues the two sweeps' kernels back to back on the stream.  Exactly one of target_col and grad_out is given: target_col, device [batch] with 0 <= . < na, makes the
 * loss -log r_rounds[target] (its gradient -1 / max(r, FLT_MIN) at the target, as dol_nll_grad); grad_out, device
 * [batch, grad_out_ld], is any gradient that does not depend on this call's result.  At least one of grad_r0 and
 * grad_e is given.  Results are those of the two separate calls, bit for bit. */
dol_status dol_iterate_apply2_backward(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds,
                                       int32_t ckpt_every, dol_dist *out, float *ckpt, const int32_t *target_col,
                                       const float *grad_out, int64_t grad_out_ld, float *grad_r0, float *grad_e,
                                       void *hip_stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid it): the reverse sweep of dol_iterate_backward_ckpt without a workspace argument.  The call first replays the
 * forward sweep from r0, keeping a checkpoint every 8 rounds in a 16 MiB device array built into the library (one copy
 * per device, held until the process ends), then walks the rounds backwards from it; same kernels and same results,
 * bit for bit, as dol_iterate_apply2_ckpt followed by dol_iterate_backward_ckpt with ckpt_every = 8.  It calls no
 * allocating routine.  DOL_EUNSUPPORTED (outputs untouched) when (ceil(rounds / 8) - 1) * batch * na exceeds
 * 4 194 304 floats.  Every call on a device uses that device's one array: calls that overlap on one device (two
 * streams, two threads) race; calls on one stream are safe, each rewrites the checkpoints it reads. */
dol_status dol_iterate_backward_noalloc(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds,
                                        const float *grad_out, int64_t grad_out_ld, float *grad_r0, float *grad_e,
                                        void *hip_stream);

/* Harness helper for loss = -log p[target] (Sec. 3.3 leaves the loss to the user): for every sample s,
 * grad[s, c] = -1 / max(d->prob[s, c], FLT_MIN) at c = target_col[s] and 0 elsewhere (all n_sym columns written).
 * target_col: device [batch] int32 column indices in 0..n_sym-1 (rows with an index outside get all zeros).
 * grad: device [batch, d->ld]. */
dol_status dol_nll_grad(const dol_dist *d, const int32_t *target_col, float *grad, void *hip_stream);

/* Message of the calling thread's most recent failing call ("" if none). */
const char *dol_last_error(void);
/* Library version, e.g. "0.1.0". */
const char *dol_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DOLPHIN_HIP_H */
