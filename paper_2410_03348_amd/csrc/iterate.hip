// Repeated DAMP Apply with feedback (the fixed-round form of the recursion of App. B, Fig. 9):
//     r_{t+1}[c] = min(1, sum over the tuples (i, j) of column c of r_t[i] * e[j]),
// every round in one launch.  One workgroup of 1024 threads owns a sample: r_t, r_{t+1} and the second
// operand sit in LDS; the function table never changes between rounds, so every thread keeps the tuples of
// its own columns (rows, for the reverse sweep) in registers and a round is one burst of LDS reads, a short
// fma chain and a barrier.  Tuples beyond the first few of a column are read through the caches; rows with
// more than 64 tuples are summed by the whole workgroup.  Summation order and clamp decisions are those of
// dol_apply2 / dol_backward.
#include "internal.h"
#include "wave_util.h"

namespace dol {

constexpr int kItThreads = 1024;
constexpr int kItWaves = kItThreads / kWave;
constexpr int kItMaxK = 4;              // columns per thread: na, nb up to 2048
constexpr int kItMaxRow = kItThreads * kItMaxK;
constexpr int kItCacheA = 6;            // tuples of a column / of a row of the first operand kept in registers

// The tuples [q0, q1) of one column or row: the first N in registers, the rest behind `list`.
template <int N>
struct Cached {
    uint32_t t[N];
    uint32_t q0, q1;
};

// Register slots past the end of a short list hold `dummy`, a tuple that points at the zero entries kept
// behind both operand rows: its product is an exact +0 added after the real tuples, so no slot needs a branch.
template <int N>
__device__ __forceinline__ void load_cached(Cached<N> &c, const uint32_t *__restrict__ ptr,
                                            const uint32_t *__restrict__ list, int r, int n, uint32_t dummy)
{
    c.q0 = c.q1 = 0;
    if (r < n) { c.q0 = ptr[r]; c.q1 = ptr[r + 1]; }
#pragma unroll
    for (int x = 0; x < N; ++x) c.t[x] = c.q0 + x < c.q1 ? list[c.q0 + x] : dummy;
}

// sum over the tuples of x[lo16] * y[hi16], in list order, one fma each, starting from 0
template <int N>
__device__ __forceinline__ float dot_lo_hi(const Cached<N> &c, const uint32_t *__restrict__ list, const float *x,
                                           const float *y)
{
    float acc = 0.0f;
#pragma unroll
    for (int k = 0; k < N; ++k) acc = __builtin_fmaf(x[c.t[k] & 0xffffu], y[c.t[k] >> 16], acc);
    for (uint32_t q = c.q0 + N; q < c.q1; ++q) {
        const uint32_t t = list[q];
        acc = __builtin_fmaf(x[t & 0xffffu], y[t >> 16], acc);
    }
    return acc;
}

// ---------------------------------------------------------------- forward

template <int K>
__global__ void __launch_bounds__(kItThreads)
damp_iterate_fwd_kernel(int32_t batch, int32_t na, int32_t nb, int32_t rounds, const uint32_t *__restrict__ col_ptr,
                        const uint32_t *__restrict__ col_ij, const float *__restrict__ r0, int64_t ldr,
                        const float *__restrict__ e, int64_t lde, float *__restrict__ hist)
{
    extern __shared__ float lds[];          // r (two rows of na + 1), e (nb + 1): each row ends with a zero
    float *r_cur = lds, *r_nxt = lds + na + 1;
    float *le = lds + 2 * (na + 1);
    const int tid = threadIdx.x;
    const int64_t s = blockIdx.x;
    const int64_t plane = static_cast<int64_t>(batch) * na;
    float *hs = hist + s * na;
    for (int c = tid; c < na; c += kItThreads) { const float v = r0[s * ldr + c]; r_cur[c] = v; hs[c] = v; }
    for (int j = tid; j < nb; j += kItThreads) le[j] = e[s * lde + j];
    if (tid == 0) { r_cur[na] = 0.0f; r_nxt[na] = 0.0f; le[nb] = 0.0f; }
    Cached<kItCacheA> col[K];
#pragma unroll
    for (int k = 0; k < K; ++k) load_cached(col[k], col_ptr, col_ij, tid + kItThreads * k, na, pack16(na, nb));
    lds_barrier();
    for (int t = 0; t < rounds; ++t) {
        float *ht = hs + (t + 1) * plane;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int c = tid + kItThreads * k;
            if (c < na) {
                const float v = fminf(dot_lo_hi(col[k], col_ij, r_cur, le), 1.0f);
                r_nxt[c] = v;
                ht[c] = v;
            }
        }
        lds_barrier();
        float *sw = r_cur; r_cur = r_nxt; r_nxt = sw;
    }
}

// ---------------------------------------------------------------- backward

struct ItTable {
    const uint32_t *col_ptr, *col_ij, *rowa_ptr, *rowa_jc, *rowb_ptr, *rowb_ic, *long_rows;
    int32_t n_long;
};

constexpr int kItLongCache = 2;         // long rows whose tuples the threads keep in registers
constexpr int kItAhead = 4;             // reverse sweep: rounds between requesting a row of the history and using it

// Sum of x over the workgroup (every thread gets the total); `red` holds one float per wavefront and must not
// be in use by an earlier call that other threads may still be reading.
__device__ __forceinline__ float block_sum(float x, float *red)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = x;
    lds_barrier();
    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < kItWaves; ++w) tot += red[w];
    return tot;
}

// Reverse sweep, one barrier per round.  At the start of round t (t = rounds - 1 .. 0) LDS holds gh = the gradient
// reaching the unclamped sums of round t + 1, r_t and r_{t-1}.  A thread owns the same symbols i of the first
// operand in every round.  For each tuple (i, j, c) of its rows it reads e[j] and gh[c] once: e[j] * gh[c] goes
// into g[i] = d loss / d r_t[i], and r_t[i] * gh[c], the tuple's share of d loss / d e[j], into a register that
// belongs to the tuple and runs over all rounds; the shares meet in LDS after the last round.  g[i] is gated
// with the clamp decision of round t (re-derived from r_{t-1} only where r_t[i] sits on the clamp) and becomes
// the next round's gh.  r_{t-2} arrives from HBM through a ring of registers requested kItAhead rounds earlier.
template <int K>                        // symbols of the first operand per thread
__global__ void __launch_bounds__(kItThreads)
damp_iterate_bwd_kernel(int32_t batch, int32_t na, int32_t nb, int32_t rounds, ItTable T,
                        const float *__restrict__ e, int64_t lde, const float *__restrict__ hist,
                        const float *__restrict__ gout, int64_t ldg, float *__restrict__ grad_r0,
                        float *__restrict__ grad_e, int64_t ldge)
{
    extern __shared__ float lds[];          // gh[2], r[3]: rows of na + 1; e, ge: nb + 1; red[kItLongCache][kItWaves]
    const int na1 = na + 1;                 // operand rows end with a zero entry (see load_cached)
    float *gh_cur = lds, *gh_nxt = lds + na1, *h_cur = lds + 2 * na1, *h_pre = lds + 3 * na1, *h_in = lds + 4 * na1;
    float *le = lds + 5 * na1, *ge = le + nb + 1, *red = ge + nb + 1;
    const int tid = threadIdx.x;
    const int64_t s = blockIdx.x;
    const int64_t plane = static_cast<int64_t>(batch) * na;
    const float *hs = hist + s * na;
    if (rounds == 0) {
        if (grad_r0)
            for (int c = tid; c < na; c += kItThreads) grad_r0[s * na + c] = gout[s * ldg + c];
        if (grad_e)
            for (int j = tid; j < nb; j += kItThreads) grad_e[s * ldge + j] = 0.0f;
        return;
    }
    for (int c = tid; c < na; c += kItThreads) {
        h_cur[c] = hs[(rounds - 1) * plane + c];
        h_pre[c] = hs[max(rounds - 2, 0) * plane + c];
    }
    for (int j = tid; j <= nb; j += kItThreads) { le[j] = j < nb ? e[s * lde + j] : 0.0f; ge[j] = 0.0f; }
    if (tid == 0) { gh_cur[na] = 0.0f; gh_nxt[na] = 0.0f; h_cur[na] = 0.0f; h_pre[na] = 0.0f; h_in[na] = 0.0f; }
    Cached<kItCacheA> col[K], rowa[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        load_cached(col[k], T.col_ptr, T.col_ij, tid + kItThreads * k, na, pack16(na, nb));
        load_cached(rowa[k], T.rowa_ptr, T.rowa_jc, tid + kItThreads * k, na, pack16(nb, na));
    }
    // The first kItLongCache rows of the first operand with many tuples are summed by the whole workgroup: which
    // rows they are and this thread's share of their tuples are the same in every round.
    int lx[kItLongCache];
    bool l_on[kItLongCache];
    uint32_t ent_l[kItLongCache][kItMaxK];
    int n_long_a = 0;
    for (int l = 0; l < T.n_long; ++l) n_long_a += static_cast<int>(T.long_rows[l]) < na;   // rows of a come first
#pragma unroll
    for (int l = 0; l < kItLongCache; ++l) {
        l_on[l] = l < n_long_a;
        lx[l] = l_on[l] ? static_cast<int>(T.long_rows[l]) : -1;
        const uint32_t q0 = l_on[l] ? T.rowa_ptr[lx[l]] : 0u;
        const uint32_t len = l_on[l] ? T.rowa_ptr[lx[l] + 1] - q0 : 0u;
#pragma unroll
        for (int k = 0; k < kItMaxK; ++k)          // a row has at most nb <= kItMaxRow tuples
            ent_l[l][k] = static_cast<uint32_t>(tid + kItThreads * k) < len ? T.rowa_jc[q0 + tid + kItThreads * k] : pack16(nb, na);
    }
    int wide_a[K];                          // index of the workgroup-summed row that is this thread's, or -1
#pragma unroll
    for (int k = 0; k < K; ++k) {
        wide_a[k] = -1;
#pragma unroll
        for (int l = 0; l < kItLongCache; ++l)
            if (l_on[l] && lx[l] == tid + kItThreads * k) wide_a[k] = l;
    }
    float share[K][kItCacheA], share_l[kItLongCache][kItMaxK];
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
        for (int x = 0; x < kItCacheA; ++x) share[k][x] = 0.0f;
#pragma unroll
    for (int l = 0; l < kItLongCache; ++l)
#pragma unroll
        for (int k = 0; k < kItMaxK; ++k) share_l[l][k] = 0.0f;
    lds_barrier();
    // gradient reaching the unclamped sums of the last round: r_rounds < 1 means the clamp did not act
#pragma unroll
    for (int k = 0; k < K; ++k) {
        const int c = tid + kItThreads * k;
        if (c < na) {
            float gv = gout[s * ldg + c];
            if (hs[rounds * plane + c] >= 1.0f && !(dot_lo_hi(col[k], T.col_ij, h_cur, le) <= 1.0f)) gv = 0.0f;
            gh_cur[c] = gv;
        }
    }
    lds_barrier();
    // One round.  `slot` carries this thread's piece of r_{t-2} from memory: with `primed` it was requested
    // kItAhead rounds ago and is re-armed here for round t - kItAhead; otherwise it is requested at the start of
    // the round.  The requests are unconditional (indices clamped) so that the wait in front of their use counts
    // exactly the younger requests in flight.
    auto round_body = [&](int t, float (&slot)[K], bool primed) {
        if (!primed) {
#pragma unroll
            for (int k = 0; k < K; ++k)
                slot[k] = hs[max(t - 2, 0) * plane + min(tid + kItThreads * k, na - 1)];
        }
        float wide_tot[kItLongCache];
#pragma unroll
        for (int l = 0; l < kItLongCache; ++l) {
            wide_tot[l] = 0.0f;
            if (l_on[l]) {
                const float ri = h_cur[lx[l]];
                float acc = 0.0f;
#pragma unroll
                for (int k = 0; k < kItMaxK; ++k) {
                    const float ghc = gh_cur[ent_l[l][k] >> 16];
                    acc = __builtin_fmaf(le[ent_l[l][k] & 0xffffu], ghc, acc);
                    share_l[l][k] = __builtin_fmaf(ri, ghc, share_l[l][k]);
                }
                wide_tot[l] = block_sum(acc, red + l * kItWaves);
            }
        }
        float g[K], ri[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {           // rowa tuples are (j | column << 16)
            const int i = tid + kItThreads * k;
            ri[k] = h_cur[min(i, na)];
            float acc = 0.0f;
            if (wide_a[k] < 0) {
#pragma unroll
                for (int x = 0; x < kItCacheA; ++x) {
                    const float ghc = gh_cur[rowa[k].t[x] >> 16];
                    acc = __builtin_fmaf(le[rowa[k].t[x] & 0xffffu], ghc, acc);
                    share[k][x] = __builtin_fmaf(ri[k], ghc, share[k][x]);
                }
                for (uint32_t q = rowa[k].q0 + kItCacheA; q < rowa[k].q1; ++q) {   // tuples past the registers
                    const uint32_t tu = T.rowa_jc[q];
                    const float ghc = gh_cur[tu >> 16];
                    acc = __builtin_fmaf(le[tu & 0xffffu], ghc, acc);
                    atomicAdd(&ge[tu & 0xffffu], ri[k] * ghc);
                }
            } else {
                acc = wide_a[k] == 0 ? wide_tot[0] : wide_tot[kItLongCache - 1];
            }
            g[k] = acc;
        }
        if (t > 0) {
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int c = tid + kItThreads * k;
                if (c < na) {
                    float gv = g[k];
                    if (ri[k] >= 1.0f && !(dot_lo_hi(col[k], T.col_ij, h_pre, le) <= 1.0f)) gv = 0.0f;
                    gh_nxt[c] = gv;
                    h_in[c] = slot[k];          // r_{t-2} goes to the row no thread reads in this round
                }
            }
        } else if (grad_r0) {
#pragma unroll
            for (int k = 0; k < K; ++k)
                if (tid + kItThreads * k < na) grad_r0[s * na + tid + kItThreads * k] = g[k];
        }
        if (primed) {
#pragma unroll
            for (int k = 0; k < K; ++k)
                slot[k] = hs[max(t - 2 - kItAhead, 0) * plane + min(tid + kItThreads * k, na - 1)];
        }
        lds_barrier();
        float *sw = gh_cur; gh_cur = gh_nxt; gh_nxt = sw;
        sw = h_cur; h_cur = h_pre; h_pre = h_in; h_in = sw;
    };
    float ring[kItAhead][K];
    int t = rounds - 1;
    for (; (t + 1) % kItAhead != 0; --t) round_body(t, ring[0], false);
    if (t >= 0) {
#pragma unroll
        for (int x = 0; x < kItAhead; ++x)
#pragma unroll
            for (int k = 0; k < K; ++k)
                ring[x][k] = hs[max(t - 2 - x, 0) * plane + min(tid + kItThreads * k, na - 1)];
    }
    for (; t >= 0; t -= kItAhead) {
        round_body(t, ring[0], true);
        round_body(t - 1, ring[1], true);
        round_body(t - 2, ring[2], true);
        round_body(t - 3, ring[3], true);
    }
    if (!grad_e) return;
    // The tuples' shares meet per symbol of e.  Symbols whose row is long (met by most threads) are summed over
    // the workgroup first, two of them; every other share is added to its symbol's entry in LDS.
    int jw[kItLongCache];
#pragma unroll
    for (int l = 0; l < kItLongCache; ++l) {
        const int x = n_long_a + l;
        jw[l] = x < T.n_long ? static_cast<int>(T.long_rows[x]) - na : -1;
    }
    float wide_e[kItLongCache];
#pragma unroll
    for (int l = 0; l < kItLongCache; ++l) wide_e[l] = 0.0f;
    auto deposit = [&](uint32_t tu, float v) {
        const int j = static_cast<int>(tu & 0xffffu);
        if (j >= nb) return;                    // an empty register slot
        if (j == jw[0]) wide_e[0] += v;
        else if (j == jw[kItLongCache - 1]) wide_e[kItLongCache - 1] += v;
        else atomicAdd(&ge[j], v);
    };
#pragma unroll
    for (int k = 0; k < K; ++k)
        if (wide_a[k] < 0)
#pragma unroll
            for (int x = 0; x < kItCacheA; ++x) deposit(rowa[k].t[x], share[k][x]);
#pragma unroll
    for (int l = 0; l < kItLongCache; ++l)
        if (l_on[l])
#pragma unroll
            for (int k = 0; k < kItMaxK; ++k) deposit(ent_l[l][k], share_l[l][k]);
#pragma unroll
    for (int l = 0; l < kItLongCache; ++l) {
        if (jw[l] >= 0) {
            const float tot = block_sum(wide_e[l], red + l * kItWaves);
            if (tid == 0) atomicAdd(&ge[jw[l]], tot);
        }
    }
    lds_barrier();
    for (int j = tid; j < nb; j += kItThreads) grad_e[s * ldge + j] = ge[j];
}

static dol_status check_iterate(const dol_dist *e, const dol_fn_table *f, int32_t rounds, size_t lds_bytes)
{
    if (!e || !f) return fail(DOL_EINVAL, "NULL argument");
    if (rounds < 0) return fail(DOL_EINVAL, "rounds is negative");
    if (e->batch < 0 || e->n_sym != f->nb || e->ld < e->n_sym) return fail(DOL_ESHAPE, "e has %d symbols, the table needs %d", e->n_sym, f->nb);
    if (f->n_out != f->na) return fail(DOL_EUNSUPPORTED, "the table maps %d symbols to %d: not square", f->na, f->n_out);
    if (f->na > kItMaxRow || f->nb > kItMaxRow) return fail(DOL_EUNSUPPORTED, "operands of more than %d symbols", kItMaxRow);
    if (lds_bytes > 64 * 1024) return fail(DOL_EUNSUPPORTED, "the rows need %zu bytes of LDS, more than 65536", lds_bytes);
    if (e->batch > 0 && e->n_sym > 0 && !e->prob) return fail(DOL_EINVAL, "e.prob is NULL");
    return DOL_OK;
}

static int iterate_k(int n) { return n <= kItThreads ? 1 : n <= 2 * kItThreads ? 2 : 4; }

}  // namespace dol

using namespace dol;

extern "C" {

dol_status dol_iterate_apply2(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds, float *hist,
                              void *hip_stream)
{
    if (!r0) return fail(DOL_EINVAL, "r0 is NULL");
    const size_t lds = f ? sizeof(float) * (2 * static_cast<size_t>(f->na) + f->nb + 3) : 0;
    if (dol_status st = check_iterate(e, f, rounds, lds)) return st;
    if (r0->batch != e->batch || r0->n_sym != f->na || r0->ld < r0->n_sym)
        return fail(DOL_ESHAPE, "r0 has %d x %d, the table needs %d x %d", r0->batch, r0->n_sym, e->batch, f->na);
    if (r0->sym_ids)
        for (int32_t c = 0; c < f->na; ++c)
            if (r0->sym_ids[c] != f->out_syms[c])
                return fail(DOL_EUNSUPPORTED, "the table produces symbol %d where r0 has %d: a round's result cannot feed the next", f->out_syms[c], r0->sym_ids[c]);
    if (r0->batch == 0 || f->na == 0) return DOL_OK;
    if (!r0->prob || !hist) return fail(DOL_EINVAL, "r0.prob or hist is NULL");
    const dim3 grid(static_cast<unsigned>(r0->batch)), block(kItThreads);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
#define DOL_IT_FWD(KK)                                                                                              \
    hipLaunchKernelGGL(damp_iterate_fwd_kernel<KK>, grid, block, lds, st, r0->batch, f->na, f->nb, rounds, f->col_ptr.ptr, \
                       f->col_ij.ptr, r0->prob, r0->ld, e->prob, e->ld, hist)
    switch (iterate_k(f->na)) {
    case 1: DOL_IT_FWD(1); break;
    case 2: DOL_IT_FWD(2); break;
    default: DOL_IT_FWD(4); break;
    }
#undef DOL_IT_FWD
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

dol_status dol_iterate_backward(const dol_dist *e, const dol_fn_table *f, int32_t rounds, const float *hist,
                                const float *grad_out, int64_t grad_out_ld, float *grad_r0, float *grad_e,
                                void *hip_stream)
{
    const size_t lds = f ? sizeof(float) * (5 * static_cast<size_t>(f->na) + 2 * static_cast<size_t>(f->nb) + 7 + kItLongCache * kItWaves) : 0;
    if (dol_status st = check_iterate(e, f, rounds, lds)) return st;
    if (e->batch == 0 || f->na == 0 || (!grad_r0 && !grad_e)) return DOL_OK;
    if (!hist || !grad_out) return fail(DOL_EINVAL, "hist or grad_out is NULL");
    if (grad_out_ld < f->na) return fail(DOL_ESHAPE, "grad_out_ld = %lld is smaller than %d", static_cast<long long>(grad_out_ld), f->na);
    const ItTable T{f->col_ptr.ptr, f->col_ij.ptr, f->rowa_ptr.ptr, f->rowa_jc.ptr, f->rowb_ptr.ptr, f->rowb_ic.ptr,
                    f->long_rows.ptr, static_cast<int32_t>(f->long_rows.n)};
    const dim3 grid(static_cast<unsigned>(e->batch)), block(kItThreads);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
#define DOL_IT_BWD(KA)                                                                                              \
    hipLaunchKernelGGL((damp_iterate_bwd_kernel<KA>), grid, block, lds, st, e->batch, f->na, f->nb, rounds, T,            \
                       e->prob, e->ld, hist, grad_out, grad_out_ld, grad_r0, grad_e, e->ld)
    switch (iterate_k(f->na)) {
    case 1: DOL_IT_BWD(1); break;
    case 2: DOL_IT_BWD(2); break;
    default: DOL_IT_BWD(4); break;
    }
#undef DOL_IT_BWD
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

}  // extern "C"
