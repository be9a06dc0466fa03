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
#include "wave_util.h"

#include <algorithm>

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

// Offers every consistent union of a proof of a's symbol with a proof of b's symbol (tuple ij) to the list.
template <int K>
__device__ __forceinline__ void offer_tuple(TopK<K> &top, uint32_t ij, int64_t a0, int64_t b0, const GroupMasks &gm,
                                            const float *__restrict__ fp, const uint64_t *__restrict__ am,
                                            const float *__restrict__ ap, const uint64_t *__restrict__ bm,
                                            const float *__restrict__ bp, const int32_t *__restrict__ fact_b)
{
    const int64_t ia = a0 + static_cast<int64_t>(ij & 0xffffu) * K, ib = b0 + static_cast<int64_t>(ij >> 16) * K;
    uint64_t ma[K], mb[K];
    float pa[K], pb[K];
    if (fact_b) {
        // the second operand is an input Distribution under natural initialisation: its symbol is one fact, its
        // tag the single proof {that fact} (App. A.1); nothing of it is stored.  fact_b holds four words per symbol:
        // the fact and the mask of the other facts of its exclusion group (low, high word).  The first operand's
        // proofs hold at most one fact per exclusion group, so the union is inconsistent exactly when such a proof
        // holds a rival of the one fact the second operand brings.  The product over ascending facts is unchanged
        // when the fact is already there, takes one more factor when it lies above every fact of the proof
        // (ma < bit as integers), and is redone from scratch otherwise.
        const uint4 fr = reinterpret_cast<const uint4 *>(fact_b)[ij >> 16];
        const int fb = static_cast<int>(fr.x);
        const uint64_t bit = uint64_t(1) << fb, rival = (static_cast<uint64_t>(fr.z) << 32) | fr.y;
        const float pbit = 1.0f * fp[fb];
        load_masks<K>(am + ia, ma);
        if (ap) load_probs<K>(ap + ia, pa);
#pragma unroll
        for (int x = 0; x < K; ++x) {
            if (ma[x] == kAbsent || (ma[x] & rival)) continue;
            const bool held = (ma[x] & bit) != 0;
            const float pr = ap && (held || ma[x] < bit) ? (held ? pa[x] : pa[x] * pbit) : proof_prob(ma[x] | bit, fp);
            top.insert(ma[x] | bit, pr);
        }
        return;
    }
    load_masks<K>(am + ia, ma);
    load_masks<K>(bm + ib, mb);
#pragma unroll
    for (int x = 0; x < K; ++x) pa[x] = pb[x] = -1.0f;
    if (ap) load_probs<K>(ap + ia, pa);
    if (bp) load_probs<K>(bp + ib, pb);
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

template <int K>
__global__ void __launch_bounds__(kThreadsT)
dtkp_apply2_kernel(int64_t total, int32_t S, int32_t na, int32_t nb, int32_t n_facts, const uint32_t *__restrict__ order,
                   const uint32_t *__restrict__ ord_len, const uint32_t *__restrict__ ord_tuples, GroupMasks gm,
                   const float *__restrict__ fact_prob, const uint64_t *__restrict__ am,
                   const float *__restrict__ ap, const uint64_t *__restrict__ bm, const float *__restrict__ bp,
                   const int32_t *__restrict__ fact_b, uint64_t *__restrict__ om, float *__restrict__ op,
                   float *__restrict__ oprob, int64_t ldo)
{
    // (each XCD takes a contiguous range of samples: a sample's operand lists then fill one L2 and not all eight)
    const int64_t idx = static_cast<int64_t>(xcd_contiguous(blockIdx.x, gridDim.x)) * kThreadsT + threadIdx.x;
    if (idx >= total) return;
    const int64_t s = idx / S;
    const int64_t r = idx - s * S;
    const uint32_t len = ord_len[r];                                     // lanes of a wavefront: columns of like length,
    if (len == 0) return;                                                // the long ones left to the wavefront-per-column kernels
    const int32_t c = static_cast<int32_t>(order[r]);
    const float *fp = fact_prob + s * n_facts;
    const int64_t a0 = s * na * K, b0 = s * nb * K;
    TopK<K> top;
    top.clear();
    for (uint32_t k = 0; k < len; ++k)                                   // (the lists interleaved in that order: coalesced loads)
        offer_tuple<K>(top, ord_tuples[static_cast<size_t>(k) * S + r], a0, b0, gm, fp, am, ap, bm, bp, fact_b);
    const int64_t o = s * S + c;
    oprob[s * ldo + c] = top.store(om + o * K, op + o * K);
}

// One workgroup of 1, 4 or 16 wavefronts (by the table's longest column) per (sample, long column): every lane streams
// a share of the column's tuples through a list of its own; the lists of a wavefront then meet by log2(64) exchange
// rounds in which each lane offers its partner's entries to its own list, the wavefronts' lists through LDS and one
// more such merge.  The list order is total on distinct proofs and repeated proofs are one proof, so the result does not depend
// on how the candidates were split.
template <int K>
__global__ void __launch_bounds__(1024)
dtkp_apply2_long_kernel(int32_t n_long, const uint32_t *__restrict__ long_cols, int32_t S, int32_t na, int32_t nb,
                        int32_t n_facts, const uint32_t *__restrict__ col_ptr, const uint32_t *__restrict__ col_ij,
                        GroupMasks gm, const float *__restrict__ fact_prob, const uint64_t *__restrict__ am,
                        const float *__restrict__ ap, const uint64_t *__restrict__ bm, const float *__restrict__ bp,
                        const int32_t *__restrict__ fact_b, uint64_t *__restrict__ om, float *__restrict__ op,
                        float *__restrict__ oprob, int64_t ldo)
{
    const int64_t wg = xcd_contiguous(blockIdx.x, gridDim.x);       // a sample's columns on one XCD: its lists fill one L2
    const int64_t s = wg / n_long;
    const uint32_t c = long_cols[wg - s * n_long];
    const float *fp = fact_prob + s * n_facts;
    const int64_t a0 = s * na * K, b0 = s * nb * K;
    TopK<K> top;
    top.clear();
    for (uint32_t q = col_ptr[c] + threadIdx.x, q1 = col_ptr[c + 1]; q < q1; q += blockDim.x)
        offer_tuple<K>(top, col_ij[q], a0, b0, gm, fp, am, ap, bm, bp, fact_b);
    merge_lists<K>(top);
    if (blockDim.x > kWave) {                       // uniform: the wavefronts' lists meet in the first wavefront
        __shared__ uint64_t lm[16][K];
        __shared__ float lp[16][K];
        const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave, n_waves = blockDim.x / kWave;
        if (lane == 0) {
#pragma unroll
            for (int x = 0; x < K; ++x) { lm[wave][x] = top.m[x]; lp[wave][x] = top.p[x]; }
        }
        __syncthreads();
        if (wave != 0) return;
        top.clear();
        if (lane < n_waves) {
#pragma unroll
            for (int x = 0; x < K; ++x) { top.m[x] = lm[lane][x]; top.p[x] = lp[lane][x]; }
        }
        merge_lists<K>(top);
    }
    if (threadIdx.x == 0) {
        const int64_t idx = s * S + c;
        oprob[s * ldo + c] = top.store(om + idx * K, op + idx * K);
    }
}

// Columns of a few dozen tuples: four to a wavefront, 16 lanes each.
template <int K>
__global__ void __launch_bounds__(kWave)
dtkp_apply2_mid_kernel(int32_t n_mid, const uint32_t *__restrict__ cols, int32_t S, int32_t na, int32_t nb, int32_t n_facts,
                       const uint32_t *__restrict__ col_ptr, const uint32_t *__restrict__ col_ij, GroupMasks gm,
                       const float *__restrict__ fact_prob, const uint64_t *__restrict__ am, const float *__restrict__ ap,
                       const uint64_t *__restrict__ bm, const float *__restrict__ bp, const int32_t *__restrict__ fact_b,
                       uint64_t *__restrict__ om, float *__restrict__ op, float *__restrict__ oprob, int64_t ldo)
{
    const int32_t quads = (n_mid + 3) / 4;
    const int64_t wg = xcd_contiguous(blockIdx.x, gridDim.x);       // a sample's columns on one XCD: its lists fill one L2
    const int64_t s = wg / quads;
    const int32_t ci = static_cast<int32_t>(wg - s * quads) * 4 + static_cast<int32_t>(threadIdx.x / 16);
    if (ci >= n_mid) return;                        // a whole group of 16 lanes at once
    const uint32_t c = cols[ci];
    const float *fp = fact_prob + s * n_facts;
    const int64_t a0 = s * na * K, b0 = s * nb * K;
    TopK<K> top;
    top.clear();
    for (uint32_t q = col_ptr[c] + (threadIdx.x & 15), q1 = col_ptr[c + 1]; q < q1; q += 16)
        offer_tuple<K>(top, col_ij[q], a0, b0, gm, fp, am, ap, bm, bp, fact_b);
    merge_lists<K, 16>(top);
    if ((threadIdx.x & 15) == 0) {
        const int64_t idx = s * S + c;
        oprob[s * ldo + c] = top.store(om + idx * K, op + idx * K);
    }
}

template <int K>
static void launch_apply2_k(int64_t total, const dol_fn_table *f, int32_t n_facts, const GroupMasks &gm,
                            const float *fact_prob, const uint64_t *am, const float *ap, const uint64_t *bm,
                            const float *bp, const int32_t *fact_b, uint64_t *om, float *op, float *oprob, int64_t ldo,
                            hipStream_t st)
{
    hipLaunchKernelGGL(dtkp_apply2_kernel<K>, dim3(grid_t(total)), dim3(kThreadsT), 0, st, total, f->n_out, f->na,
                       f->nb, n_facts, f->col_order.ptr, f->ord_len.ptr, f->ord_tuples.ptr, gm, fact_prob, am, ap, bm, bp,
                       fact_b, om, op, oprob, ldo);
    const int64_t n_long = static_cast<int64_t>(f->dtkp_long_cols.n);
    const int64_t n_huge = f->n_huge_dtkp_cols, batch = total / f->n_out;
    if (n_huge > 0)                                  // the list's first n_huge columns: 16 wavefronts each
        hipLaunchKernelGGL(dtkp_apply2_long_kernel<K>, dim3(static_cast<unsigned>(batch * n_huge)), dim3(1024), 0, st,
                           static_cast<int32_t>(n_huge), f->dtkp_long_cols.ptr, f->n_out, f->na, f->nb, n_facts,
                           f->col_ptr.ptr, f->col_ij.ptr, gm, fact_prob, am, ap, bm, bp, fact_b, om, op, oprob, ldo);
    const int64_t n_wave = f->n_wave_dtkp_cols, n_mid = n_long - n_huge - n_wave;
    if (n_wave > 0)
        hipLaunchKernelGGL(dtkp_apply2_long_kernel<K>, dim3(static_cast<unsigned>(batch * n_wave)), dim3(kWave), 0, st,
                           static_cast<int32_t>(n_wave), f->dtkp_long_cols.ptr + n_huge, f->n_out, f->na, f->nb, n_facts,
                           f->col_ptr.ptr, f->col_ij.ptr, gm, fact_prob, am, ap, bm, bp, fact_b, om, op, oprob, ldo);
    if (n_mid > 0)
        hipLaunchKernelGGL(dtkp_apply2_mid_kernel<K>, dim3(static_cast<unsigned>(batch * ((n_mid + 3) / 4))), dim3(kWave), 0, st,
                           static_cast<int32_t>(n_mid), f->dtkp_long_cols.ptr + n_huge + n_wave, f->n_out, f->na, f->nb,
                           n_facts, f->col_ptr.ptr, f->col_ij.ptr, gm, fact_prob, am, ap, bm, bp, fact_b, om, op, oprob, ldo);
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
                              const float *bp, const int32_t *fact_b, uint64_t *om, float *op, float *oprob, int64_t ldo,
                              hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * f->n_out;
    if (total == 0) return DOL_OK;
    if (static_cast<int64_t>(batch) * static_cast<int64_t>(f->dtkp_long_cols.n) > 0x7fffffffLL)
        return fail(DOL_EUNSUPPORTED, "batch x long table columns exceeds 2^31");
#define CALL(KK) launch_apply2_k<KK>(total, f, n_facts, gm, fact_prob, am, ap, bm, bp, fact_b, om, op, oprob, ldo, st)
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
// (App. A.2).  One workgroup per sample; its wavefronts take 64 symbols at a time, a lane per symbol (coalesced loads
// of the proof lists).  A lane folds the clamp's gate and the upstream gradient into one coefficient per proof,
// gradient * proof probability, and adds it to a register accumulator of every fact the proof holds (the loop over
// the facts is unrolled, so the accumulators are plain registers and a fact's test is a bit-field extract).  The
// product of a proof's other facts is its probability divided by the fact's: that division happens once, on the
// accumulator's total (one rounding more than multiplying the facts out, far inside the 1e-5 bar).  A fact of
// probability (nearly) 0 cannot be divided by: its accumulator takes gradient * (the other facts multiplied out, in
// ascending order) instead.  No atomics; the sums run over a lane's symbols in ascending order, then over the lanes
// (exchange tree), then over the wavefronts in order.
constexpr int kGradWaves = 16;

template <int K>
__global__ void __launch_bounds__(kGradWaves * 64)
dtkp_prob_bwd_kernel(int32_t n_sym, int32_t n_facts, const uint64_t *__restrict__ mask,
                     const float *__restrict__ pprob, const float *__restrict__ fact_prob,
                     const float *__restrict__ g, int64_t ldg, float *__restrict__ gfact)
{
    __shared__ float part[kGradWaves][64];
    __shared__ float fp[64];
    const int64_t s = blockIdx.x;
    const int lane = threadIdx.x & 63, n_waves = blockDim.x >> 6;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));   // tells the compiler it is uniform
    if (wave == 0) fp[lane] = lane < n_facts ? fact_prob[s * n_facts + lane] : 1.0f;
    __syncthreads();
    const float pj = fp[lane];
    const uint64_t tiny = __ballot(!(pj > 1e-30f));
    float acc[64], mine_tiny = 0.0f;
#pragma unroll
    for (int j = 0; j < 64; ++j) acc[j] = 0.0f;
    for (int32_t i0 = wave * 64; i0 < n_sym; i0 += n_waves * 64) {
        const int32_t i = i0 + lane;
        uint64_t mm[K];                     // 0: absent, gated by the clamp, or past the last symbol
        float cf[K], gate_g = 0.0f;
#pragma unroll
        for (int x = 0; x < K; ++x) { mm[x] = 0; cf[x] = 0.0f; }
        if (i < n_sym) {
            const uint64_t *m = mask + (s * n_sym + i) * K;
            const float *pp = pprob + (s * n_sym + i) * K;
            uint64_t lm[K];
            float pv[K];
            load_masks<K>(m, lm);
            load_probs<K>(pp, pv);
            const float gi = g[s * ldg + i];
            float sum = 0.0f;               // the quantity the forward pass clamped: kept proofs in rank order
#pragma unroll
            for (int x = 0; x < K; ++x)
                if (lm[x] != kAbsent) sum = sum + pv[x];
            if (sum <= 1.0f) {
                gate_g = gi;
#pragma unroll
                for (int x = 0; x < K; ++x)
                    if (lm[x] != kAbsent) { mm[x] = lm[x]; cf[x] = gi * pv[x]; }
            }
        }
#pragma unroll
        for (int j0 = 0; j0 < 64; j0 += 8) {
            if (j0 >= n_facts) continue;    // (uniform; facts past n_facts are in no proof)
#pragma unroll
            for (int j = j0; j < j0 + 8; ++j) {
#pragma unroll
                for (int x = 0; x < K; ++x) {
                    const int word = static_cast<int>(static_cast<uint32_t>(j < 32 ? mm[x] : mm[x] >> 32));
                    const int held = __builtin_amdgcn_sbfe(word, j & 31, 1);                    // all ones: the proof holds fact j
                    acc[j] = acc[j] + __builtin_bit_cast(float, held & __builtin_bit_cast(int, cf[x]));
                }
            }
        }
        for (uint64_t tm = tiny; tm; tm &= tm - 1) {                     // (uniform) facts that cannot be divided by
            const int j = __builtin_ctzll(tm);
            float t = 0.0f;
#pragma unroll
            for (int x = 0; x < K; ++x) {
                if (!((mm[x] >> j) & 1)) continue;
                float others = 1.0f;
                for (uint64_t r = mm[x] & ~(uint64_t(1) << j); r; r &= r - 1) others = others * fp[__builtin_ctzll(r)];
                t = __builtin_fmaf(gate_g, others, t);
            }
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) t += __shfl_xor(t, d, 64);
            if (lane == j) mine_tiny = mine_tiny + t;
        }
    }
    float mine = 0.0f;                      // lane j ends with this wavefront's total of fact j
#pragma unroll
    for (int j0 = 0; j0 < 64; j0 += 8) {
        if (j0 >= n_facts) continue;
#pragma unroll
        for (int j = j0; j < j0 + 8; ++j) {
            float v = acc[j];
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
            if (lane == j) mine = v;
        }
    }
    mine = pj > 1e-30f ? mine * __builtin_amdgcn_rcpf(pj) : mine_tiny;
    part[wave][lane] = mine;
    __syncthreads();
    if (wave == 0 && lane < n_facts) {
        float tot = 0.0f;
        for (int w = 0; w < n_waves; ++w) tot = tot + part[w][lane];
        gfact[s * n_facts + lane] = tot;
    }
}

dol_status launch_dtkp_prob_bwd(int32_t batch, int32_t n_sym, int32_t k, int32_t n_facts, const uint64_t *mask,
                                const float *pprob, const float *fact_prob, const float *g, int64_t ldg, float *gfact,
                                hipStream_t st)
{
    if (batch == 0 || n_facts == 0) return DOL_OK;
    const int waves = std::max(1, std::min(kGradWaves, (n_sym + 63) / 64));
#define CALL(K)                                                                                                        \
    hipLaunchKernelGGL(dtkp_prob_bwd_kernel<K>, dim3(static_cast<unsigned>(batch)), dim3(64 * waves), 0, st, n_sym,     \
                       n_facts, mask, pprob, fact_prob, g, ldg, gfact)
    DOL_DISPATCH_K(k, CALL)
#undef CALL
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

}  // namespace dol
