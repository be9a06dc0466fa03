// Repeated DAMP Apply with feedback (the fixed-round form of the recursion of App. B, Fig. 9):
//     r_{t+1}[c] = min(1, sum over the tuples (i, j) of column c of r_t[i] * e[j]),
// every round in one launch.  One workgroup of 512 threads owns a sample: r_t, r_{t+1} and the second
// operand sit in LDS; the function table never changes between rounds, so every thread keeps the tuples of
// its own columns (rows, for the reverse sweep) in registers and a round is one burst of LDS reads, a short
// fma chain and a barrier.  Tuples beyond the first few of a column are read through the caches; rows with
// more than 64 tuples are summed by the whole workgroup.  Summation order and clamp decisions are those of
// dol_apply2 / dol_backward.
#include "internal.h"
#include "wave_util.h"

namespace dol {

constexpr int kItThreads = 512;
constexpr int kItWaves = kItThreads / kWave;
constexpr int kItMaxK = 4;              // columns per thread: na, nb up to 2048
constexpr int kItMaxRow = kItThreads * kItMaxK;
constexpr int kItCacheA = 6;            // tuples of a column / of a row of the first operand kept in registers
constexpr int kItCacheB = 4;            // tuples of a row of the second operand kept in registers

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
    __syncthreads();
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
        __syncthreads();
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
    __syncthreads();
    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < kItWaves; ++w) tot += red[w];
    return tot;
}

template <int K, int KB>                // columns of a / rows of b per thread
__global__ void __launch_bounds__(kItThreads)
damp_iterate_bwd_kernel(int32_t batch, int32_t na, int32_t nb, int32_t rounds, ItTable T,
                        const float *__restrict__ e, int64_t lde, const float *__restrict__ hist,
                        const float *__restrict__ gout, int64_t ldg, float *__restrict__ grad_r0,
                        float *__restrict__ grad_e, int64_t ldge)
{
    extern __shared__ float lds[];          // H[3], G[2], ghat: rows of na + 1; e, ge: nb + 1; red[2][kItWaves]
    const int na1 = na + 1;                 // operand rows end with a zero entry (see load_cached)
    float *H0 = lds, *H1 = lds + na1, *H2 = lds + 2 * na1, *G0 = lds + 3 * na1, *G1 = lds + 4 * na1, *ghat = lds + 5 * na1;
    float *le = lds + 6 * na1, *ge = le + nb + 1, *red = ge + nb + 1;
    const int tid = threadIdx.x;
    const int64_t s = blockIdx.x;
    const int64_t plane = static_cast<int64_t>(batch) * na;
    const float *hs = hist + s * na;
    float *g_cur = G0, *g_nxt = G1, *h_nxt = H0, *h_cur = H1, *h_pre = H2;
    for (int c = tid; c < na; c += kItThreads) {
        g_cur[c] = gout[s * ldg + c];
        h_nxt[c] = hs[rounds * plane + c];
        if (rounds > 0) h_cur[c] = hs[(rounds - 1) * plane + c];
    }
    for (int j = tid; j < nb; j += kItThreads) { le[j] = e[s * lde + j]; ge[j] = 0.0f; }
    if (tid == 0) { H0[na] = 0.0f; H1[na] = 0.0f; H2[na] = 0.0f; ghat[na] = 0.0f; le[nb] = 0.0f; }
    constexpr int KL = K > KB ? K : KB;
    Cached<kItCacheA> col[K], rowa[K];
    Cached<kItCacheB> rowb[KB];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        load_cached(col[k], T.col_ptr, T.col_ij, tid + kItThreads * k, na, pack16(na, nb));
        load_cached(rowa[k], T.rowa_ptr, T.rowa_jc, tid + kItThreads * k, na, pack16(nb, na));
    }
#pragma unroll
    for (int k = 0; k < KB; ++k) load_cached(rowb[k], T.rowb_ptr, T.rowb_ic, tid + kItThreads * k, nb, pack16(na, na));
    // long rows: which they are, and this thread's share of their tuples, are the same in every round
    int lx[kItLongCache];
    uint32_t len_l[kItLongCache], ent_l[kItLongCache][KL];
#pragma unroll
    for (int l = 0; l < kItLongCache; ++l) {
        lx[l] = l < T.n_long ? static_cast<int>(T.long_rows[l]) : 0;
        const bool is_a = lx[l] < na;
        const int r = is_a ? lx[l] : lx[l] - na;
        const uint32_t *ptr = is_a ? T.rowa_ptr : T.rowb_ptr;
        const uint32_t *ent = is_a ? T.rowa_jc : T.rowb_ic;
        const uint32_t q0 = l < T.n_long ? ptr[r] : 0u;
        len_l[l] = l < T.n_long ? ptr[r + 1] - q0 : 0u;
#pragma unroll
        for (int k = 0; k < KL; ++k)
            ent_l[l][k] = static_cast<uint32_t>(tid + kItThreads * k) < len_l[l] ? ent[q0 + tid + kItThreads * k] : 0u;
    }
    __syncthreads();
    // One round of the reverse sweep.  `slot` carries this thread's piece of r_{t-1} from memory: with `primed`
    // it was requested kItAhead rounds ago and is re-armed here for round t - kItAhead; otherwise it is
    // requested at the start of the round.  The requests are unconditional (indices clamped) so that the
    // wait in front of their use counts exactly the younger requests in flight.
    auto round_body = [&](int t, float (&slot)[K], bool primed) {
        if (!primed) {
#pragma unroll
            for (int k = 0; k < K; ++k)
                slot[k] = hs[max(t - 1, 0) * plane + min(tid + kItThreads * k, na - 1)];
        }
        // gradient reaching the unclamped sums of round t: h_nxt < 1 means the clamp did not act
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int c = tid + kItThreads * k;
            if (c < na) {
                float gv = g_cur[c];
                if (h_nxt[c] >= 1.0f && !(dot_lo_hi(col[k], T.col_ij, h_cur, le) <= 1.0f)) gv = 0.0f;
                ghat[c] = gv;
            }
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int i = tid + kItThreads * k;         // rowa tuples are (j | column << 16)
            if (i < na && rowa[k].q1 - rowa[k].q0 <= kLongTableRow) g_nxt[i] = dot_lo_hi(rowa[k], T.rowa_jc, le, ghat);
        }
#pragma unroll
        for (int k = 0; k < KB; ++k) {
            const int j = tid + kItThreads * k;         // rowb tuples are (i | column << 16)
            if (j < nb && rowb[k].q1 - rowb[k].q0 <= kLongTableRow) ge[j] += dot_lo_hi(rowb[k], T.rowb_ic, h_cur, ghat);
        }
        for (int l = 0; l < T.n_long; ++l) {     // rows with many tuples: the whole workgroup sums one row
            const int x = l < kItLongCache ? lx[l < kItLongCache ? l : 0] : static_cast<int>(T.long_rows[l]);
            const bool is_a = x < na;
            const int r = is_a ? x : x - na;
            const float *other = is_a ? le : h_cur;
            float acc = 0.0f;
            if (l < kItLongCache) {
#pragma unroll
                for (int k = 0; k < KL; ++k) {
                    const uint32_t en = l == 0 ? ent_l[0][k] : ent_l[kItLongCache - 1][k];
                    const uint32_t len = l == 0 ? len_l[0] : len_l[kItLongCache - 1];
                    if (static_cast<uint32_t>(tid + kItThreads * k) < len) acc = __builtin_fmaf(ghat[en >> 16], other[en & 0xffffu], acc);
                }
            } else {
                const uint32_t *ptr = is_a ? T.rowa_ptr : T.rowb_ptr;
                const uint32_t *ent = is_a ? T.rowa_jc : T.rowb_ic;
                for (uint32_t q = ptr[r] + tid, q1 = ptr[r + 1]; q < q1; q += kItThreads) {
                    const uint32_t en = ent[q];
                    acc = __builtin_fmaf(ghat[en >> 16], other[en & 0xffffu], acc);
                }
                __syncthreads();                // rows past the first two share one scratch row
            }
            const float tot = block_sum(acc, red + (l < kItLongCache ? l : kItLongCache - 1) * kItWaves);
            if (tid == 0) {
                if (is_a) g_nxt[r] = tot;
                else ge[r] += tot;
            }
        }
        if (t > 0) {                            // r_{t-1} goes to the buffer no thread reads in this round
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int c = tid + kItThreads * k;
                if (c < na) h_pre[c] = slot[k];
            }
        }
        if (primed) {
#pragma unroll
            for (int k = 0; k < K; ++k)
                slot[k] = hs[max(t - 1 - kItAhead, 0) * plane + min(tid + kItThreads * k, na - 1)];
        }
        __syncthreads();
        float *sw = g_cur; g_cur = g_nxt; g_nxt = sw;
        sw = h_nxt; h_nxt = h_cur; h_cur = h_pre; h_pre = sw;
    };
    float ring[kItAhead][K];
    int t = rounds - 1;
    for (; (t + 1) % kItAhead != 0; --t) round_body(t, ring[0], false);
    if (t >= 0) {
#pragma unroll
        for (int x = 0; x < kItAhead; ++x)
#pragma unroll
            for (int k = 0; k < K; ++k)
                ring[x][k] = hs[max(t - 1 - x, 0) * plane + min(tid + kItThreads * k, na - 1)];
    }
    for (; t >= 0; t -= kItAhead) {
        round_body(t, ring[0], true);
        round_body(t - 1, ring[1], true);
        round_body(t - 2, ring[2], true);
        round_body(t - 3, ring[3], true);
    }
    if (grad_r0)
        for (int c = tid; c < na; c += kItThreads) grad_r0[s * na + c] = g_cur[c];
    if (grad_e)
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
    const size_t lds = f ? sizeof(float) * (6 * static_cast<size_t>(f->na) + 2 * static_cast<size_t>(f->nb) + 8 + kItLongCache * kItWaves) : 0;
    if (dol_status st = check_iterate(e, f, rounds, lds)) return st;
    if (e->batch == 0 || f->na == 0 || (!grad_r0 && !grad_e)) return DOL_OK;
    if (!hist || !grad_out) return fail(DOL_EINVAL, "hist or grad_out is NULL");
    if (grad_out_ld < f->na) return fail(DOL_ESHAPE, "grad_out_ld = %lld is smaller than %d", static_cast<long long>(grad_out_ld), f->na);
    const ItTable T{f->col_ptr.ptr, f->col_ij.ptr, f->rowa_ptr.ptr, f->rowa_jc.ptr, f->rowb_ptr.ptr, f->rowb_ic.ptr,
                    f->long_rows.ptr, static_cast<int32_t>(f->long_rows.n)};
    const dim3 grid(static_cast<unsigned>(e->batch)), block(kItThreads);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
#define DOL_IT_BWD(KA, KB)                                                                                          \
    hipLaunchKernelGGL((damp_iterate_bwd_kernel<KA, KB>), grid, block, lds, st, e->batch, f->na, f->nb, rounds, T,       \
                       e->prob, e->ld, hist, grad_out, grad_out_ld, grad_r0, grad_e, e->ld)
    switch (iterate_k(f->na) * 10 + iterate_k(f->nb)) {
    case 11: DOL_IT_BWD(1, 1); break;
    case 12: DOL_IT_BWD(1, 2); break;
    case 14: DOL_IT_BWD(1, 4); break;
    case 21: DOL_IT_BWD(2, 1); break;
    case 22: DOL_IT_BWD(2, 2); break;
    case 24: DOL_IT_BWD(2, 4); break;
    case 41: DOL_IT_BWD(4, 1); break;
    case 42: DOL_IT_BWD(4, 2); break;
    default: DOL_IT_BWD(4, 4); break;
    }
#undef DOL_IT_BWD
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

}  // extern "C"
