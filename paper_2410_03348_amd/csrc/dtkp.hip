// DTKP-AM provenance kernels (Sec. 3.2, Table 1, App. A) for gfx950, on the bitmask encoding of proofs:
// a proof is the 64-bit set of input facts it uses; its probability is the float product of the facts'
// probabilities in ascending fact index starting from 1 (absent symbols contribute 1, Sec. 3.2).
// The set union of two proofs (the paper's element-wise minimum, App. A.1) is a bitwise OR.
//
// One thread owns one (sample, output symbol) and streams every candidate proof through a k-entry sorted
// list held in registers.  Repeated proofs are one proof, so insertion first looks the mask up; the list
// order (higher probability first, ties by smaller mask) is total on distinct masks, which makes the
// result independent of the order candidates arrive in.
#include "dtkp_util.h"

namespace dol {

constexpr int kThreadsT = 128;

static inline unsigned grid_t(int64_t work) { return static_cast<unsigned>((work + kThreadsT - 1) / kThreadsT); }

// ---------------------------------------------------------------- init

__global__ void __launch_bounds__(kThreadsT)
dtkp_init_kernel(int64_t total, int32_t n_sym, int32_t k, int32_t n_facts, const int32_t *__restrict__ fact_of_sym,
                 const float *__restrict__ fact_prob, uint64_t *__restrict__ mask, float *__restrict__ pprob,
                 float *__restrict__ prob, int64_t ld)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreadsT + threadIdx.x;
    if (idx >= total) return;
    const int64_t s = idx / n_sym;
    const int32_t i = static_cast<int32_t>(idx - s * n_sym);
    const int32_t f = fact_of_sym[i];
    const float pr = 1.0f * fact_prob[s * n_facts + f];
    mask[idx * k] = uint64_t(1) << f;
    pprob[idx * k] = pr;
    for (int x = 1; x < k; ++x) { mask[idx * k + x] = kAbsent; pprob[idx * k + x] = 0.0f; }
    prob[s * ld + i] = fminf(pr, 1.0f);
}

dol_status launch_dtkp_init(int32_t batch, int32_t n_sym, int32_t k, int32_t n_facts, const int32_t *d_fact_of_sym,
                            const float *fact_prob, uint64_t *mask, float *pprob, float *prob, int64_t ld,
                            hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * n_sym;
    if (total == 0) return DOL_OK;
    hipLaunchKernelGGL(dtkp_init_kernel, dim3(grid_t(total)), dim3(kThreadsT), 0, st, total, n_sym, k, n_facts,
                       d_fact_of_sym, fact_prob, mask, pprob, prob, ld);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// ---------------------------------------------------------------- apply2

template <int K>
__global__ void __launch_bounds__(kThreadsT)
dtkp_apply2_kernel(int64_t total, int32_t S, int32_t na, int32_t nb, int32_t n_facts,
                   const uint32_t *__restrict__ col_ptr, const uint32_t *__restrict__ col_ij, GroupMasks gm,
                   const float *__restrict__ fact_prob, const uint64_t *__restrict__ am,
                   const float *__restrict__ ap, const uint64_t *__restrict__ bm, const float *__restrict__ bp,
                   uint64_t *__restrict__ om, float *__restrict__ op, float *__restrict__ oprob, int64_t ldo)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreadsT + threadIdx.x;
    if (idx >= total) return;
    const int64_t s = idx / S;
    const int32_t c = static_cast<int32_t>(idx - s * S);
    const float *fp = fact_prob + s * n_facts;
    const int64_t a0 = s * na * K, b0 = s * nb * K;
    TopK<K> top;
    top.clear();
    for (uint32_t q = col_ptr[c], q1 = col_ptr[c + 1]; q < q1; ++q) {
        const uint32_t ij = col_ij[q];
        const int64_t ia = a0 + static_cast<int64_t>(ij & 0xffffu) * K, ib = b0 + static_cast<int64_t>(ij >> 16) * K;
        uint64_t ma[K], mb[K];
        float pa[K], pb[K];
#pragma unroll
        for (int x = 0; x < K; ++x) {
            ma[x] = am[ia + x];
            mb[x] = bm[ib + x];
            pa[x] = ap ? ap[ia + x] : -1.0f;
            pb[x] = bp ? bp[ib + x] : -1.0f;
        }
#pragma unroll
        for (int x = 0; x < K; ++x) {
            if (ma[x] == kAbsent) continue;
#pragma unroll
            for (int y = 0; y < K; ++y) {
                if (mb[y] == kAbsent) continue;
                const uint64_t m = ma[x] | mb[y];
                if (proof_conflict(m, gm)) continue;
                top.insert(m, union_prob(ma[x], pa[x], mb[y], pb[y], fp));
            }
        }
    }
    oprob[s * ldo + c] = top.store(om + idx * K, op + idx * K);
}

template <int K>
static void launch_apply2_k(int64_t total, const dol_fn_table *f, int32_t n_facts, const GroupMasks &gm,
                            const float *fact_prob, const uint64_t *am, const float *ap, const uint64_t *bm,
                            const float *bp, uint64_t *om, float *op, float *oprob, int64_t ldo, hipStream_t st)
{
    hipLaunchKernelGGL(dtkp_apply2_kernel<K>, dim3(grid_t(total)), dim3(kThreadsT), 0, st, total, f->n_out, f->na,
                       f->nb, n_facts, f->col_ptr.ptr, f->col_ij.ptr, gm, fact_prob, am, ap, bm, bp, om, op, oprob, ldo);
}

#define DOL_DISPATCH_K(k, CALL)                                      \
    switch (k) {                                                     \
    case 1: CALL(1); break;                                          \
    case 2: CALL(2); break;                                          \
    case 3: CALL(3); break;                                          \
    case 4: CALL(4); break;                                          \
    case 5: CALL(5); break;                                          \
    case 6: CALL(6); break;                                          \
    case 7: CALL(7); break;                                          \
    case 8: CALL(8); break;                                          \
    default: return fail(DOL_EINVAL, "k = %d outside 1..%d", k, DOL_MAX_K); \
    }

dol_status launch_dtkp_apply2(const dol_fn_table *f, int32_t batch, int32_t k, int32_t n_facts, const GroupMasks &gm,
                              const float *fact_prob, const uint64_t *am, const float *ap, const uint64_t *bm,
                              const float *bp, uint64_t *om, float *op, float *oprob, int64_t ldo, hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * f->n_out;
    if (total == 0) return DOL_OK;
#define CALL(KK) launch_apply2_k<KK>(total, f, n_facts, gm, fact_prob, am, ap, bm, bp, om, op, oprob, ldo, st)
    DOL_DISPATCH_K(k, CALL)
#undef CALL
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// ---------------------------------------------------------------- union

template <int K>
__global__ void __launch_bounds__(kThreadsT)
dtkp_union_kernel(int64_t total, int32_t S, int32_t na, int32_t nb, const int32_t *__restrict__ ia,
                  const int32_t *__restrict__ ib, const uint64_t *__restrict__ am, const float *__restrict__ ap,
                  const uint64_t *__restrict__ bm, const float *__restrict__ bp, uint64_t *__restrict__ om,
                  float *__restrict__ op, float *__restrict__ oprob, int64_t ldo)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreadsT + threadIdx.x;
    if (idx >= total) return;
    const int64_t s = idx / S;
    const int32_t c = static_cast<int32_t>(idx - s * S);
    const int32_t i = ia[c], j = ib[c];
    TopK<K> top;
    top.clear();
    if (i >= 0) {
        const int64_t o = (s * na + i) * K;
#pragma unroll
        for (int x = 0; x < K; ++x)
            if (am[o + x] != kAbsent) top.insert(am[o + x], ap[o + x]);
    }
    if (j >= 0) {
        const int64_t o = (s * nb + j) * K;
#pragma unroll
        for (int x = 0; x < K; ++x)
            if (bm[o + x] != kAbsent) top.insert(bm[o + x], bp[o + x]);
    }
    oprob[s * ldo + c] = top.store(om + idx * K, op + idx * K);
}

dol_status launch_dtkp_union(const UnionPlan *p, int32_t batch, int32_t k, const uint64_t *am, const float *ap,
                             const uint64_t *bm, const float *bp, uint64_t *om, float *op, float *oprob, int64_t ldo,
                             hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * p->n_out;
    if (total == 0) return DOL_OK;
#define CALL(KK)                                                                                                  \
    hipLaunchKernelGGL(dtkp_union_kernel<KK>, dim3(grid_t(total)), dim3(kThreadsT), 0, st, total, p->n_out, p->na, \
                       p->nb, p->d_ia.ptr, p->d_ib.ptr, am, ap, bm, bp, om, op, oprob, ldo)
    DOL_DISPATCH_K(k, CALL)
#undef CALL
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// ---------------------------------------------------------------- filter

__global__ void __launch_bounds__(kThreadsT)
dtkp_filter_kernel(int64_t total, int32_t n_in, int32_t n_out, int32_t k, const int32_t *__restrict__ keep_idx,
                   const uint64_t *__restrict__ im, const float *__restrict__ ip, const float *__restrict__ iprob,
                   int64_t ldi, uint64_t *__restrict__ om, float *__restrict__ op, float *__restrict__ oprob,
                   int64_t ldo)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreadsT + threadIdx.x;
    if (idx >= total) return;
    const int64_t s = idx / n_out;
    const int32_t c = static_cast<int32_t>(idx - s * n_out);
    const int64_t src = (s * n_in + keep_idx[c]) * k;
    for (int x = 0; x < k; ++x) { om[idx * k + x] = im[src + x]; op[idx * k + x] = ip[src + x]; }
    oprob[s * ldo + c] = iprob[s * ldi + keep_idx[c]];
}

dol_status launch_dtkp_filter(const FilterPlan *p, int32_t batch, int32_t k, const uint64_t *im, const float *ip,
                              const float *iprob, int64_t ldi, uint64_t *om, float *op, float *oprob, int64_t ldo,
                              hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * p->n_out;
    if (total == 0) return DOL_OK;
    hipLaunchKernelGGL(dtkp_filter_kernel, dim3(grid_t(total)), dim3(kThreadsT), 0, st, total, p->n_in, p->n_out, k,
                       p->d_keep_idx.ptr, im, ip, iprob, ldi, om, op, oprob, ldo);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// ---------------------------------------------------------------- gradient of the tag probabilities

// Pr(symbol) = min(1, sum over its kept proofs of the product of their facts' probabilities) (Sec. 3.2); which
// proofs top-k kept is a constant of the differentiation and the clamp passes gradient inside and on its bound
// (App. A.2).  One wavefront per sample, lane f owns fact f and walks every proof of the sample: the control flow
// is the same in all lanes (the proof's own fact multiplies by 1), the sums run in ascending (symbol, rank) order.
__global__ void __launch_bounds__(64)
dtkp_prob_bwd_kernel(int32_t n_sym, int32_t k, int32_t n_facts, const uint64_t *__restrict__ mask,
                     const float *__restrict__ pprob, const float *__restrict__ fact_prob,
                     const float *__restrict__ g, int64_t ldg, float *__restrict__ gfact)
{
    const int64_t s = blockIdx.x;
    const int f = threadIdx.x;
    const uint64_t mine = uint64_t(1) << f;
    const float *fp = fact_prob + s * n_facts;
    float acc = 0.0f;
    for (int32_t i = 0; i < n_sym; ++i) {
        const uint64_t *m = mask + (s * n_sym + i) * k;
        const float *pp = pprob + (s * n_sym + i) * k;
        float sum = 0.0f;                   // the quantity the forward pass clamped: kept proofs in rank order
        for (int x = 0; x < k; ++x)
            if (m[x] != kAbsent) sum = sum + pp[x];
        if (!(sum <= 1.0f)) continue;
        const float gi = g[s * ldg + i];
        for (int x = 0; x < k; ++x) {
            const uint64_t mm = m[x];
            if (mm == kAbsent) continue;
            float others = 1.0f;
            for (uint64_t r = mm; r; r &= r - 1) {
                const int j = __builtin_ctzll(r);
                others = others * (j == f ? 1.0f : fp[j]);
            }
            if (mm & mine) acc = __builtin_fmaf(gi, others, acc);
        }
    }
    if (f < n_facts) gfact[s * n_facts + f] = acc;
}

dol_status launch_dtkp_prob_bwd(int32_t batch, int32_t n_sym, int32_t k, int32_t n_facts, const uint64_t *mask,
                                const float *pprob, const float *fact_prob, const float *g, int64_t ldg, float *gfact,
                                hipStream_t st)
{
    if (batch == 0 || n_facts == 0) return DOL_OK;
    hipLaunchKernelGGL(dtkp_prob_bwd_kernel, dim3(static_cast<unsigned>(batch)), dim3(64), 0, st, n_sym, k, n_facts, mask,
                       pprob, fact_prob, g, ldg, gfact);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

}  // namespace dol
