// Apply / ApplyIf over K Distributions, K = 1..DOL_MAX_ARITY, and the unary Apply (Sec. 3.1.2, Eq. 1-3) for gfx950:
// symbol-side plan, DAMP forward and vector-Jacobian product, DTKP-AM forward.
//
// The admitted tuples are kept as 16-bit operand positions, grouped by the output column they land in and, inside a
// column, in ascending index order (the order the float sum of a column is defined in).  For the backward pass every
// operand row lists the tuples it takes part in.  One thread owns one (sample, output symbol) in the forward kernels
// and one (sample, operand symbol) in the backward kernel; lanes run along a row, so stores are coalesced and the
// gathers of neighbouring lanes fall into the same few cache lines of the sample's tag rows.
#include "dtkp_util.h"
#include "element_map.h"
#include "internal.h"
#include "wave_util.h"

#include <algorithm>
#include <cstdio>
#include <memory>
#include <new>
#include <numeric>

struct dol_fnk_table {
    int32_t K = 0;
    int32_t n_sym[DOL_MAX_ARITY] = {};
    int32_t row_base[DOL_MAX_ARITY + 1] = {};   // operand l owns rows row_base[l] .. row_base[l+1] of row_ptr
    int32_t n_out = 0;
    int64_t n_tuples = 0;
    std::vector<int32_t> out_syms;
    dol::DevArray<uint32_t> col_ptr;     // [n_out+1] tuples of a column
    dol::DevArray<uint16_t> tup;         // [n_tuples*K] operand positions, column-grouped
    dol::DevArray<uint32_t> tup_col;     // [n_tuples] column of each grouped tuple
    dol::DevArray<uint32_t> row_ptr;     // [sum n_sym + 1]
    dol::DevArray<uint32_t> row_tup;     // [n_tuples*K] grouped-tuple numbers of each operand row, ascending
    dol::DevArray<uint32_t> long_cols;   // columns with more than dol::kLongTableCol tuples
    dol::DevArray<uint32_t> dtkp_long_cols;   // ... more than dol::kLongDtkpCol: first those above dol::kWaveDtkpCol
    int32_t n_wave_dtkp_cols = 0;             // (one wavefront each), then the shorter ones (four to a wavefront)
    dol::DevArray<uint32_t> col_order;   // all columns in the order of dol::columns_by_length (limit: kLongDtkpCol)
    // unary functions (K = 1): the first eight symbols of every image again, 16 bytes per column (0xFFFF = none), and
    // the column of every symbol (-1: rejected)
    dol::DevArray<uint16_t> unary_head;
    dol::DevArray<uint16_t> unary_head_ord;   // the same, entry r being that of column col_order[r]
    dol::DevArray<int32_t> unary_col;
    int device = 0;
};

namespace dol {

struct KOperands {
    const float *p[DOL_MAX_ARITY];
    int64_t ld[DOL_MAX_ARITY];
};

struct KGrads {
    float *p[DOL_MAX_ARITY];
    int32_t row_base[DOL_MAX_ARITY + 1];
};

struct KProofs {
    const uint64_t *m[DOL_MAX_ARITY];
    const float *p[DOL_MAX_ARITY];
    int32_t n[DOL_MAX_ARITY];
};

// ---------------------------------------------------------------- DAMP

// pre of one column: tuples in ascending index order, one term each (the order fixes the clamp decision).  The
// loads of kGatherK tuples are issued together (positions first, then the tags they name); the adds keep their order.
constexpr int kGatherK = 4;

template <int K>
__device__ __forceinline__ float column_sum_k(const float *const *row, const uint16_t *__restrict__ tup,
                                              uint32_t q0, uint32_t q1)
{
    float acc = 0.0f;
    for (uint32_t q = q0; q < q1; q += kGatherK) {
        uint16_t pos[kGatherK][K];
        float v[kGatherK][K];
#pragma unroll
        for (int u = 0; u < kGatherK; ++u) {
            const uint16_t *t = tup + static_cast<size_t>(min(q + u, q1 - 1)) * K;
#pragma unroll
            for (int l = 0; l < K; ++l) pos[u][l] = t[l];
        }
#pragma unroll
        for (int u = 0; u < kGatherK; ++u)
#pragma unroll
            for (int l = 0; l < K; ++l) v[u][l] = row[l][pos[u][l]];
#pragma unroll
        for (int u = 0; u < kGatherK; ++u) {
            if (q + u >= q1) break;
            float head = v[u][0];
#pragma unroll
            for (int l = 1; l + 1 < K; ++l) head = head * v[u][l];
            if (K == 1) acc = acc + head;
            else acc = __builtin_fmaf(head, v[u][K - 1], acc);
        }
    }
    return acc;
}

template <int K>
__global__ void __launch_bounds__(kThreads)
damp_applyk_fwd_kernel(Rows R, KOperands in, const uint32_t *__restrict__ col_ptr, const uint16_t *__restrict__ tup,
                       float *__restrict__ out, int64_t ldo)
{
    for_each_element(R, [&](int64_t s, int c) {
        const float *row[K];
#pragma unroll
        for (int l = 0; l < K; ++l) row[l] = in.p[l] + s * in.ld[l];
        const uint32_t q0 = col_ptr[c], q1 = col_ptr[c + 1];
        if (q1 - q0 > static_cast<uint32_t>(kLongTableCol)) return;        // left to the wavefront-per-column kernel
        out[s * ldo + c] = fminf(column_sum_k<K>(row, tup, q0, q1), 1.0f);
    });
}

// Unary Apply: out[c] = clamp(sum of the tags of the symbols with image c).  The first eight symbols of a column come
// with one 16-byte load; only a column with more goes on through its list (same order).
__global__ void __launch_bounds__(kThreads)
damp_apply1_fwd_kernel(Rows R, const float *__restrict__ x, int64_t ldx, const uint32_t *__restrict__ col_ptr,
                       const uint16_t *__restrict__ tup, const uint4 *__restrict__ head, float *__restrict__ out,
                       int64_t ldo)
{
    for_each_element(R, [&](int64_t s, int c) {
        const float *xr = x + s * ldx;
        const uint4 h = head[c];
        const uint32_t w[4] = {h.x, h.y, h.z, h.w};
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t pos = (w[u / 2] >> (16 * (u & 1))) & 0xffffu;
            v[u] = pos != 0xffffu ? xr[pos] : 0.0f;
        }
        float acc = 0.0f;
#pragma unroll
        for (int u = 0; u < 8; ++u)
            if (((w[u / 2] >> (16 * (u & 1))) & 0xffffu) != 0xffffu) acc = acc + v[u];
        if ((w[3] >> 16) != 0xffffu) {                                     // eight or more symbols: the rest of the list
            const uint32_t q0 = col_ptr[c], q1 = col_ptr[c + 1];
            if (q1 - q0 > static_cast<uint32_t>(kLongTableCol)) return;    // left to the wavefront-per-column kernel
            for (uint32_t q = q0 + 8; q < q1; q += kGatherK) {
                float t[kGatherK];
#pragma unroll
                for (int u = 0; u < kGatherK; ++u) t[u] = xr[tup[min(q + u, q1 - 1)]];
#pragma unroll
                for (int u = 0; u < kGatherK; ++u)
                    if (q + u < q1) acc = acc + t[u];
            }
        }
        out[s * ldo + c] = fminf(acc, 1.0f);
    });
}

// Its vector-Jacobian product: gx[i] = g[col(i)] where the column is not clamped (0 for a rejected symbol).
__global__ void __launch_bounds__(kThreads)
damp_apply1_bwd_kernel(Rows R, const float *__restrict__ x, int64_t ldx, const int32_t *__restrict__ col_of,
                       const uint32_t *__restrict__ col_ptr, const uint16_t *__restrict__ tup,
                       const float *__restrict__ out, int64_t ldo, const float *__restrict__ g, int64_t ldg,
                       float *__restrict__ gx)
{
    for_each_element(R, [&](int64_t s, int i) {
        const int32_t c = col_of[i];
        float gh = 0.0f;
        if (c >= 0) {
            gh = g[s * ldg + c];
            if (out[s * ldo + c] >= 1.0f) {         // pre == 1 passes, pre > 1 blocks: only pre itself tells
                const float *row[1] = {x + s * ldx};
                if (!(column_sum_k<1>(row, tup, col_ptr[c], col_ptr[c + 1]) <= 1.0f)) gh = 0.0f;
            }
        }
        gx[s * ldx + i] = gh;
    });
}

// The same two for wide rows, staged in LDS (element_map.h).  Forward: the operand row is staged and the symbols of a
// column are gathered from it, in the same order.  Backward: the gradient row, gated by the clamp, is staged and
// every operand symbol picks its column's entry.
__global__ void __launch_bounds__(kStageThreads)
damp_apply1_fwd_staged_kernel(int32_t n_in, int32_t S, int32_t parts, const float *__restrict__ x, int64_t ldx,
                              const uint32_t *__restrict__ order, const uint32_t *__restrict__ col_ptr, const uint16_t *__restrict__ tup,
                              const uint4 *__restrict__ head, float *__restrict__ out, int64_t ldo)
{
    extern __shared__ __align__(16) float xr[];
    const int64_t s = blockIdx.x / static_cast<unsigned>(parts);
    int c0, c1;
    stage_part(S, parts, static_cast<int>(blockIdx.x - s * parts), c0, c1);
    stage_row(xr, x + s * ldx, n_in);
    __syncthreads();
    // kStageUnroll columns per thread and pass, so that their index and head loads are in flight together
    for (int r0 = c0 + threadIdx.x; r0 < c1; r0 += kStageUnroll * kStageThreads) {
        uint32_t c[kStageUnroll];
        uint4 h[kStageUnroll];
#pragma unroll
        for (int v = 0; v < kStageUnroll; ++v) {
            const int r = min(r0 + v * kStageThreads, c1 - 1);
            c[v] = order[r];                                               // lanes of a wavefront: columns of like length
            h[v] = head[r];                                                // (the head table in that order: a coalesced load)
        }
#pragma unroll
        for (int v = 0; v < kStageUnroll; ++v) {
            if (r0 + v * kStageThreads >= c1) continue;
            const uint32_t w[4] = {h[v].x, h[v].y, h[v].z, h[v].w};
            float val[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {                                  // all eight reads at once (slot 0 for "none")
                const uint32_t pos = (w[u / 2] >> (16 * (u & 1))) & 0xffffu;
                val[u] = xr[pos != 0xffffu ? pos : 0u];
            }
            float acc = 0.0f;
#pragma unroll
            for (int u = 0; u < 8; ++u)
                if (((w[u / 2] >> (16 * (u & 1))) & 0xffffu) != 0xffffu) acc = acc + val[u];
            if ((w[3] >> 16) != 0xffffu) {                                 // eight or more symbols: the rest of the list
                const uint32_t q0 = col_ptr[c[v]], q1 = col_ptr[c[v] + 1];
                if (q1 - q0 > static_cast<uint32_t>(kLongTableCol)) continue;   // left to the wavefront-per-column kernel
                for (uint32_t q = q0 + 8; q < q1; q += kGatherK) {
                    uint32_t pos[kGatherK];
#pragma unroll
                    for (int u = 0; u < kGatherK; ++u) pos[u] = tup[min(q + u, q1 - 1)];
#pragma unroll
                    for (int u = 0; u < kGatherK; ++u)
                        if (q + u < q1) acc = acc + xr[pos[u]];
                }
            }
            out[s * ldo + c[v]] = fminf(acc, 1.0f);
        }
    }
}

__global__ void __launch_bounds__(kStageThreads)
damp_apply1_bwd_staged_kernel(int32_t n_in, int32_t S, int32_t parts, const float *__restrict__ x, int64_t ldx,
                              const int32_t *__restrict__ col_of, const uint32_t *__restrict__ col_ptr,
                              const uint16_t *__restrict__ tup, const float *__restrict__ out, int64_t ldo,
                              const float *__restrict__ g, int64_t ldg, float *__restrict__ gx)
{
    extern __shared__ __align__(16) float gh[];
    const int64_t s = blockIdx.x / static_cast<unsigned>(parts);
    int i0, i1;
    stage_part(n_in, parts, static_cast<int>(blockIdx.x - s * parts), i0, i1);
    for (int c = threadIdx.x; c < S; c += kStageThreads) {
        float v = g[s * ldg + c];
        if (out[s * ldo + c] >= 1.0f) {             // pre == 1 passes, pre > 1 blocks: only pre itself tells
            const float *row[1] = {x + s * ldx};
            if (!(column_sum_k<1>(row, tup, col_ptr[c], col_ptr[c + 1]) <= 1.0f)) v = 0.0f;
        }
        gh[c] = v;
    }
    __syncthreads();
    for (int i = i0 + threadIdx.x; i < i1; i += kStageThreads) {
        const int32_t c = col_of[i];
        gx[s * ldx + i] = c >= 0 ? gh[c] : 0.0f;
    }
}

// One wavefront per (sample, long column): lanes stride over the tuples and their partial sums meet by shuffles.
// That is not the order the clamp decision is defined in, so the lanes also add up the terms' magnitudes, which
// bounds how far the two orders can lie apart (about n roundings of relative size 2^-24 each way); only a sum within
// that distance of 1 is taken again in the defining order.
template <int K>
__global__ void __launch_bounds__(kWave)
damp_applyk_fwd_long_kernel(int32_t n_long, const uint32_t *__restrict__ long_cols, KOperands in,
                            const uint32_t *__restrict__ col_ptr, const uint16_t *__restrict__ tup,
                            float *__restrict__ out, int64_t ldo)
{
    const int64_t s = blockIdx.x / n_long;
    const uint32_t c = long_cols[blockIdx.x - s * n_long];
    const float *row[K];
#pragma unroll
    for (int l = 0; l < K; ++l) row[l] = in.p[l] + s * in.ld[l];
    const uint32_t q0 = col_ptr[c], q1 = col_ptr[c + 1];
    float acc = 0.0f, mag = 0.0f;
    for (uint32_t q = q0 + threadIdx.x; q < q1; q += kWave) {
        const uint16_t *t = tup + static_cast<size_t>(q) * K;
        float term = row[0][t[0]];
#pragma unroll
        for (int l = 1; l < K; ++l) term = term * row[l][t[l]];
        acc = acc + term;
        mag = mag + fabsf(term);
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        acc += __shfl_xor(acc, d, kWave);
        mag += __shfl_xor(mag, d, kWave);
    }
    // the per-term products differ from the defining order's by at most K roundings each
    const float slack = mag * (static_cast<float>(q1 - q0 + kWave + 2 * K) * 1.1920929e-7f);
    float pre = acc;
    if (fabsf(acc - 1.0f) <= slack) pre = column_sum_k<K>(row, tup, q0, q1);
    if (threadIdx.x == 0) out[s * ldo + c] = fminf(pre, 1.0f);
}

template <int K>
__global__ void __launch_bounds__(kThreads)
damp_applyk_bwd_kernel(Rows R, KOperands in, KGrads gin, const uint32_t *__restrict__ col_ptr,
                       const uint16_t *__restrict__ tup, const uint32_t *__restrict__ tup_col,
                       const uint32_t *__restrict__ row_ptr, const uint32_t *__restrict__ row_tup,
                       const float *__restrict__ out, int64_t ldo, const float *__restrict__ g, int64_t ldg)
{
    for_each_element(R, [&](int64_t s, int x) {
        int l = 0;
#pragma unroll
        for (int m = 1; m < K; ++m) l = x >= gin.row_base[m] ? m : l;
        float *dst = nullptr;
#pragma unroll
        for (int m = 0; m < K; ++m) dst = l == m ? gin.p[m] : dst;
        if (!dst) return;
        const float *row[K];
#pragma unroll
        for (int m = 0; m < K; ++m) row[m] = in.p[m] + s * in.ld[m];
        float acc = 0.0f;
        for (uint32_t q = row_ptr[x], q1 = row_ptr[x + 1]; q < q1; ++q) {
            const uint32_t tn = row_tup[q], c = tup_col[tn];
            float gh = g[s * ldg + c];
            // out < 1: the clamp did not act; out == 1 leaves pre == 1 (passes) and pre > 1 (blocks) apart only by pre
            if (out[s * ldo + c] >= 1.0f && !(column_sum_k<K>(row, tup, col_ptr[c], col_ptr[c + 1]) <= 1.0f)) gh = 0.0f;
            const uint16_t *t = tup + static_cast<size_t>(tn) * K;
            float others = 1.0f;
#pragma unroll
            for (int m = 0; m < K; ++m)
                if (m != l) others = others * row[m][t[m]];
            acc = __builtin_fmaf(gh, others, acc);
        }
        int64_t ld = 0;
        int32_t base = 0;
#pragma unroll
        for (int m = 0; m < K; ++m)
            if (l == m) { ld = in.ld[m]; base = gin.row_base[m]; }
        dst[s * ld + (x - base)] = acc;
    });
}

// Unary functions over wide rows go through the kernels that stage a row in LDS.
static bool staged_unary_fwd(const dol_fnk_table *f) { return f->K == 1 && stage_fits(f->n_sym[0]); }
static bool staged_unary_bwd(const dol_fnk_table *f)
{
    return f->K == 1 && f->n_sym[0] >= kStageMinRow && sizeof(float) * f->n_out <= kStageMaxBytes;
}

template <int K>
static void launch_fwd_k(const Rows &R, const KOperands &in, const dol_fnk_table *f, float *out, int64_t ldo, hipStream_t st)
{
    if (K == 1 && staged_unary_fwd(f)) {
        const int32_t parts = stage_parts(R.batch, f->n_out);
        (void)allow_dynamic_lds(reinterpret_cast<const void *>(damp_apply1_fwd_staged_kernel), kStageMaxBytes);
        hipLaunchKernelGGL(damp_apply1_fwd_staged_kernel, dim3(static_cast<unsigned>(R.batch) * parts), dim3(kStageThreads),
                           sizeof(float) * f->n_sym[0], st, f->n_sym[0], f->n_out, parts, in.p[0], in.ld[0], f->col_order.ptr,
                           f->col_ptr.ptr, f->tup.ptr, reinterpret_cast<const uint4 *>(f->unary_head_ord.ptr), out, ldo);
    } else if (K == 1)
        hipLaunchKernelGGL(damp_apply1_fwd_kernel, dim3(R.grid), dim3(kThreads), 0, st, R, in.p[0], in.ld[0], f->col_ptr.ptr,
                           f->tup.ptr, reinterpret_cast<const uint4 *>(f->unary_head.ptr), out, ldo);
    else
        hipLaunchKernelGGL(damp_applyk_fwd_kernel<K>, dim3(R.grid), dim3(kThreads), 0, st, R, in, f->col_ptr.ptr, f->tup.ptr,
                           out, ldo);
    const int64_t n_long = static_cast<int64_t>(f->long_cols.n);
    if (n_long > 0)
        hipLaunchKernelGGL(damp_applyk_fwd_long_kernel<K>, dim3(static_cast<unsigned>(R.batch * n_long)), dim3(kWave), 0, st,
                           static_cast<int32_t>(n_long), f->long_cols.ptr, in, f->col_ptr.ptr, f->tup.ptr, out, ldo);
}

template <int K>
static void launch_bwd_k(const Rows &R, const KOperands &in, const KGrads &gin, const dol_fnk_table *f, const float *out,
                         int64_t ldo, const float *g, int64_t ldg, hipStream_t st)
{
    if (K == 1 && staged_unary_bwd(f)) {
        const int32_t parts = stage_parts(R.batch, f->n_sym[0]);
        (void)allow_dynamic_lds(reinterpret_cast<const void *>(damp_apply1_bwd_staged_kernel), kStageMaxBytes);
        hipLaunchKernelGGL(damp_apply1_bwd_staged_kernel, dim3(static_cast<unsigned>(R.batch) * parts), dim3(kStageThreads),
                           sizeof(float) * f->n_out, st, f->n_sym[0], f->n_out, parts, in.p[0], in.ld[0], f->unary_col.ptr,
                           f->col_ptr.ptr, f->tup.ptr, out, ldo, g, ldg, gin.p[0]);
    } else if (K == 1)
        hipLaunchKernelGGL(damp_apply1_bwd_kernel, dim3(R.grid), dim3(kThreads), 0, st, R, in.p[0], in.ld[0], f->unary_col.ptr,
                           f->col_ptr.ptr, f->tup.ptr, out, ldo, g, ldg, gin.p[0]);
    else
        hipLaunchKernelGGL(damp_applyk_bwd_kernel<K>, dim3(R.grid), dim3(kThreads), 0, st, R, in, gin, f->col_ptr.ptr,
                           f->tup.ptr, f->tup_col.ptr, f->row_ptr.ptr, f->row_tup.ptr, out, ldo, g, ldg);
}

#define DOL_DISPATCH_ARITY(K, CALL)  \
    switch (K) {                     \
    case 1: CALL(1); break;          \
    case 2: CALL(2); break;          \
    case 3: CALL(3); break;          \
    case 4: CALL(4); break;          \
    case 5: CALL(5); break;          \
    default: CALL(6); break;         \
    }

// ---------------------------------------------------------------- DTKP-AM

constexpr int kThreadsP = 128;

// Offers the proofs of one tuple's tag to the list: the binary conjunction of Table 1 folded over the operands left
// to right, each intermediate pruned to k proofs.
template <int KP>
__device__ __forceinline__ void offer_tuple_k(TopK<KP> &top, const uint16_t *__restrict__ t, int64_t s, int32_t arity,
                                              const KProofs &in, const GroupMasks &gm, const float *__restrict__ fp)
{
    TopK<KP> cur;
    {
        const int64_t o = (s * in.n[0] + t[0]) * KP;
        load_masks<KP>(in.m[0] + o, cur.m);
        if (in.p[0]) load_probs<KP>(in.p[0] + o, cur.p);
#pragma unroll
        for (int x = 0; x < KP; ++x)
            cur.p[x] = cur.m[x] == kAbsent ? -1.0f : in.p[0] ? cur.p[x] : proof_prob(cur.m[x], fp);
    }
    for (int l = 1; l < arity; ++l) {
        const int64_t o = (s * in.n[l] + t[l]) * KP;
        uint64_t mb[KP];
        float pb[KP];
        load_masks<KP>(in.m[l] + o, mb);
#pragma unroll
        for (int y = 0; y < KP; ++y) pb[y] = -1.0f;
        if (in.p[l]) load_probs<KP>(in.p[l] + o, pb);
        TopK<KP> nxt;
        nxt.clear();
#pragma unroll
        for (int x = 0; x < KP; ++x) {
            if (cur.m[x] == kAbsent) continue;
#pragma unroll
            for (int y = 0; y < KP; ++y) {
                if (mb[y] == kAbsent) continue;
                const uint64_t u = cur.m[x] | mb[y];
                if (proof_conflict(u, gm)) continue;
                nxt.insert(u, union_prob(cur.m[x], cur.p[x], mb[y], pb[y], fp));
            }
        }
        cur = nxt;
    }
#pragma unroll
    for (int x = 0; x < KP; ++x)
        if (cur.m[x] != kAbsent) top.insert(cur.m[x], cur.p[x]);
}

// One thread per (sample, output symbol): the proofs of the column's tuples meet in one k-entry list.
template <int KP>
__global__ void __launch_bounds__(kThreadsP)
dtkp_applyk_kernel(int64_t total, int32_t S, int32_t arity, KProofs in, const uint32_t *__restrict__ order,
                   const uint32_t *__restrict__ col_ptr,
                   const uint16_t *__restrict__ tup, GroupMasks gm, int32_t n_facts, const float *__restrict__ fact_prob,
                   uint64_t *__restrict__ om, float *__restrict__ op, float *__restrict__ oprob, int64_t ldo)
{
    // (each XCD takes a contiguous range of samples: a sample's operand lists then fill one L2 and not all eight)
    const int64_t idx = static_cast<int64_t>(xcd_contiguous(blockIdx.x, gridDim.x)) * kThreadsP + threadIdx.x;
    if (idx >= total) return;
    const int64_t s = idx / S;
    const int32_t r = static_cast<int32_t>(idx - s * S);
    // lanes of a wavefront: columns of like length (not for a unary function under DTKP-AM, whose lists are one
    // gather each: there the neighbouring columns' neighbouring symbols matter more)
    const int32_t c = order ? static_cast<int32_t>(order[r]) : r;
    const float *fp = fact_prob + s * n_facts;
    const uint32_t q0 = col_ptr[c], q1 = col_ptr[c + 1];
    if (q1 - q0 > static_cast<uint32_t>(kLongDtkpCol)) return;             // left to the wavefront-per-column kernel
    TopK<KP> top;
    top.clear();
    for (uint32_t q = q0; q < q1; ++q) {
        offer_tuple_k<KP>(top, tup + static_cast<size_t>(q) * arity, s, arity, in, gm, fp);
    }
    const int64_t o = s * S + c;
    oprob[s * ldo + c] = top.store(om + o * KP, op + o * KP);
}

// One wavefront per (sample, long column): every lane streams a share of the tuples through a list of its own; the
// lists meet by exchange rounds (the list order is total on distinct proofs, so the split does not matter).
template <int KP>
__global__ void __launch_bounds__(kWave)
dtkp_applyk_long_kernel(int32_t n_long, const uint32_t *__restrict__ long_cols, int32_t S, int32_t arity, KProofs in,
                        const uint32_t *__restrict__ col_ptr, const uint16_t *__restrict__ tup, GroupMasks gm,
                        int32_t n_facts, const float *__restrict__ fact_prob, uint64_t *__restrict__ om,
                        float *__restrict__ op, float *__restrict__ oprob, int64_t ldo)
{
    const int64_t wg = xcd_contiguous(blockIdx.x, gridDim.x);       // a sample's columns on one XCD: its lists fill one L2
    const int64_t s = wg / n_long;
    const uint32_t c = long_cols[wg - s * n_long];
    const float *fp = fact_prob + s * n_facts;
    TopK<KP> top;
    top.clear();
    for (uint32_t q = col_ptr[c] + threadIdx.x, q1 = col_ptr[c + 1]; q < q1; q += kWave)
        offer_tuple_k<KP>(top, tup + static_cast<size_t>(q) * arity, s, arity, in, gm, fp);
    merge_lists<KP>(top);
    if (threadIdx.x == 0) {
        const int64_t idx = s * S + c;
        oprob[s * ldo + c] = top.store(om + idx * KP, op + idx * KP);
    }
}

// Columns of a few dozen tuples: four to a wavefront, 16 lanes each.
template <int KP>
__global__ void __launch_bounds__(kWave)
dtkp_applyk_mid_kernel(int32_t n_mid, const uint32_t *__restrict__ cols, int32_t S, int32_t arity, KProofs in,
                       const uint32_t *__restrict__ col_ptr, const uint16_t *__restrict__ tup, GroupMasks gm,
                       int32_t n_facts, const float *__restrict__ fact_prob, uint64_t *__restrict__ om,
                       float *__restrict__ op, float *__restrict__ oprob, int64_t ldo)
{
    const int32_t quads = (n_mid + 3) / 4;
    const int64_t wg = xcd_contiguous(blockIdx.x, gridDim.x);       // a sample's columns on one XCD: its lists fill one L2
    const int64_t s = wg / quads;
    const int32_t ci = static_cast<int32_t>(wg - s * quads) * 4 + static_cast<int32_t>(threadIdx.x / 16);
    if (ci >= n_mid) return;                        // a whole group of 16 lanes at once
    const uint32_t c = cols[ci];
    const float *fp = fact_prob + s * n_facts;
    TopK<KP> top;
    top.clear();
    for (uint32_t q = col_ptr[c] + (threadIdx.x & 15), q1 = col_ptr[c + 1]; q < q1; q += 16)
        offer_tuple_k<KP>(top, tup + static_cast<size_t>(q) * arity, s, arity, in, gm, fp);
    merge_lists<KP, 16>(top);
    if ((threadIdx.x & 15) == 0) {
        const int64_t idx = s * S + c;
        oprob[s * ldo + c] = top.store(om + idx * KP, op + idx * KP);
    }
}

template <int KP>
static void launch_dtkp_k(int64_t total, const dol_fnk_table *f, const KProofs &in, const GroupMasks &gm, int32_t n_facts,
                          const float *fact_prob, uint64_t *om, float *op, float *oprob, int64_t ldo, hipStream_t st)
{
    hipLaunchKernelGGL(dtkp_applyk_kernel<KP>, dim3(static_cast<unsigned>((total + kThreadsP - 1) / kThreadsP)),
                       dim3(kThreadsP), 0, st, total, f->n_out, f->K, in, f->K >= 2 ? f->col_order.ptr : nullptr, f->col_ptr.ptr, f->tup.ptr, gm,
                       n_facts, fact_prob, om, op, oprob, ldo);
    const int64_t n_wave = f->n_wave_dtkp_cols, n_mid = static_cast<int64_t>(f->dtkp_long_cols.n) - n_wave;
    const int64_t batch = total / f->n_out;
    if (n_wave > 0)
        hipLaunchKernelGGL(dtkp_applyk_long_kernel<KP>, dim3(static_cast<unsigned>(batch * n_wave)), dim3(kWave), 0, st,
                           static_cast<int32_t>(n_wave), f->dtkp_long_cols.ptr, f->n_out, f->K, in, f->col_ptr.ptr, f->tup.ptr,
                           gm, n_facts, fact_prob, om, op, oprob, ldo);
    if (n_mid > 0)
        hipLaunchKernelGGL(dtkp_applyk_mid_kernel<KP>, dim3(static_cast<unsigned>(batch * ((n_mid + 3) / 4))), dim3(kWave), 0, st,
                           static_cast<int32_t>(n_mid), f->dtkp_long_cols.ptr + n_wave, f->n_out, f->K, in, f->col_ptr.ptr,
                           f->tup.ptr, gm, n_facts, fact_prob, om, op, oprob, ldo);
}

// ---------------------------------------------------------------- plan

static dol_status build_k(int32_t K, const int32_t *n_sym, int64_t n, const int32_t *idx, const int32_t *out_id,
                          dol_fnk_table **out)
{
    std::unique_ptr<dol_fnk_table> tb(new (std::nothrow) dol_fnk_table);
    if (!tb) return fail(DOL_ENOMEM, "out of host memory");
    tb->K = K;
    for (int l = 0; l < K; ++l) {
        tb->n_sym[l] = n_sym[l];
        tb->row_base[l + 1] = tb->row_base[l] + n_sym[l];
    }
    // admitted tuples in ascending index order; a function has one value per argument tuple
    std::vector<int64_t> order;
    order.reserve(static_cast<size_t>(n));
    for (int64_t t = 0; t < n; ++t) {
        for (int l = 0; l < K; ++l)
            if (idx[t * K + l] < 0 || idx[t * K + l] >= n_sym[l])
                return fail(DOL_ESHAPE, "tuple %lld: position %d outside operand %d with %d symbols",
                            static_cast<long long>(t), idx[t * K + l], l, n_sym[l]);
        if (out_id[t] >= 0) order.push_back(t);
    }
    auto less = [&](int64_t x, int64_t y) { return std::lexicographical_compare(idx + x * K, idx + x * K + K, idx + y * K, idx + y * K + K); };
    std::sort(order.begin(), order.end(), less);
    for (size_t t = 1; t < order.size(); ++t)
        if (!less(order[t - 1], order[t])) return fail(DOL_EINVAL, "the tuple list names one index tuple twice (entries %lld and %lld)",
                                                       static_cast<long long>(order[t - 1]), static_cast<long long>(order[t]));
    const size_t m = order.size();
    if (m * static_cast<size_t>(K) > (size_t(1) << 31)) return fail(DOL_EUNSUPPORTED, "more than 2^31 tuple entries");
    tb->n_tuples = static_cast<int64_t>(m);

    // Eq. 2: the output symbols are the distinct produced ids, ascending
    for (int64_t t : order) tb->out_syms.push_back(out_id[t]);
    std::sort(tb->out_syms.begin(), tb->out_syms.end());
    tb->out_syms.erase(std::unique(tb->out_syms.begin(), tb->out_syms.end()), tb->out_syms.end());
    if (tb->out_syms.size() > DOL_MAX_SYMBOLS)
        return fail(DOL_EUNSUPPORTED, "the function produces %zu symbols, more than %d", tb->out_syms.size(), DOL_MAX_SYMBOLS);
    const int32_t S = tb->n_out = static_cast<int32_t>(tb->out_syms.size());

    // stable counting sort by column
    std::vector<uint32_t> col(m), col_ptr(S + 1, 0);
    for (size_t t = 0; t < m; ++t) {
        col[t] = static_cast<uint32_t>(std::lower_bound(tb->out_syms.begin(), tb->out_syms.end(), out_id[order[t]]) - tb->out_syms.begin());
        col_ptr[col[t] + 1]++;
    }
    for (int32_t c = 0; c < S; ++c) col_ptr[c + 1] += col_ptr[c];
    std::vector<uint16_t> tup(m * K);
    std::vector<uint32_t> tup_col(m);
    {
        std::vector<uint32_t> fill(col_ptr.begin(), col_ptr.end() - 1);
        for (size_t t = 0; t < m; ++t) {
            const uint32_t pos = fill[col[t]]++;
            for (int l = 0; l < K; ++l) tup[static_cast<size_t>(pos) * K + l] = static_cast<uint16_t>(idx[order[t] * K + l]);
            tup_col[pos] = col[t];
        }
    }
    // rows of every operand: the grouped tuples they take part in, ascending
    const int32_t rows = tb->row_base[K];
    std::vector<uint32_t> row_ptr(rows + 1, 0), row_tup(m * K);
    for (size_t t = 0; t < m; ++t)
        for (int l = 0; l < K; ++l) row_ptr[tb->row_base[l] + tup[t * K + l] + 1]++;
    for (int32_t r = 0; r < rows; ++r) row_ptr[r + 1] += row_ptr[r];
    {
        std::vector<uint32_t> fill(row_ptr.begin(), row_ptr.end() - 1);
        for (size_t t = 0; t < m; ++t)
            for (int l = 0; l < K; ++l) row_tup[fill[tb->row_base[l] + tup[t * K + l]]++] = static_cast<uint32_t>(t);
    }

    std::vector<uint32_t> long_cols, dtkp_long_cols, dtkp_mid_cols;
    for (int32_t c = 0; c < S; ++c) {
        const uint32_t len = col_ptr[c + 1] - col_ptr[c];
        if (len > static_cast<uint32_t>(kLongTableCol)) long_cols.push_back(static_cast<uint32_t>(c));
        if (len > static_cast<uint32_t>(kWaveDtkpCol)) dtkp_long_cols.push_back(static_cast<uint32_t>(c));
        else if (len > static_cast<uint32_t>(kLongDtkpCol)) dtkp_mid_cols.push_back(static_cast<uint32_t>(c));
    }
    tb->n_wave_dtkp_cols = static_cast<int32_t>(dtkp_long_cols.size());
    dtkp_long_cols.insert(dtkp_long_cols.end(), dtkp_mid_cols.begin(), dtkp_mid_cols.end());

    const std::vector<uint32_t> col_order = columns_by_length(col_ptr, S, kLongDtkpCol);
    if (K == 1) {
        std::vector<uint16_t> head(static_cast<size_t>(S) * 8, 0xFFFFu);
        std::vector<int32_t> col_of(static_cast<size_t>(n_sym[0]), -1);
        for (int32_t c = 0; c < S; ++c)
            for (uint32_t q = col_ptr[c]; q < col_ptr[c + 1]; ++q) {
                if (q - col_ptr[c] < 8) head[static_cast<size_t>(c) * 8 + (q - col_ptr[c])] = tup[q];
                col_of[tup[q]] = c;
            }
        DOL_HIP(tb->unary_head.upload(head));
        DOL_HIP(tb->unary_col.upload(col_of));
        std::vector<uint16_t> ord(head.size());
        for (int32_t r = 0; r < S; ++r)
            for (int u = 0; u < 8; ++u) ord[static_cast<size_t>(r) * 8 + u] = head[static_cast<size_t>(col_order[r]) * 8 + u];
        DOL_HIP(tb->unary_head_ord.upload(ord));
    }
    DOL_HIP(hipGetDevice(&tb->device));
    DOL_HIP(tb->long_cols.upload(long_cols));
    DOL_HIP(tb->dtkp_long_cols.upload(dtkp_long_cols));
    DOL_HIP(tb->col_order.upload(col_order));
    DOL_HIP(tb->col_ptr.upload(col_ptr));
    DOL_HIP(tb->tup.upload(tup));
    DOL_HIP(tb->tup_col.upload(tup_col));
    DOL_HIP(tb->row_ptr.upload(row_ptr));
    DOL_HIP(tb->row_tup.upload(row_tup));
    *out = tb.release();
    return DOL_OK;
}

static dol_status check_operands(int32_t K, const dol_dist *const *in, const dol_fnk_table *f, bool dtkp)
{
    if (!f) return fail(DOL_EINVAL, "function table is NULL");
    if (K != f->K) return fail(DOL_ESHAPE, "K = %d, the table was built for %d operands", K, f->K);
    if (!in) return fail(DOL_EINVAL, "in is NULL");
    for (int l = 0; l < K; ++l) {
        char name[16];
        snprintf(name, sizeof name, "in[%d]", l);
        if (dol_status st = check_dist(in[l], name, dtkp, false, !dtkp)) return st;
        if (in[l]->batch != in[0]->batch) return fail(DOL_ESHAPE, "batch sizes differ: in[0] has %d, in[%d] has %d", in[0]->batch, l, in[l]->batch);
        if (in[l]->n_sym != f->n_sym[l]) return fail(DOL_ESHAPE, "in[%d] has %d symbols, the table expects %d", l, in[l]->n_sym, f->n_sym[l]);
    }
    return DOL_OK;
}

}  // namespace dol

using namespace dol;

extern "C" {

dol_status dol_fnk_table_create(int32_t K, const int32_t *n_sym, int64_t n, const int32_t *idx, const int32_t *out_id,
                                dol_fnk_table **table)
{
    if (!table) return fail(DOL_EINVAL, "table is NULL");
    *table = nullptr;
    if (K < 1 || K > DOL_MAX_ARITY) return fail(DOL_EINVAL, "K = %d outside 1..%d", K, DOL_MAX_ARITY);
    if (!n_sym) return fail(DOL_EINVAL, "n_sym is NULL");
    for (int l = 0; l < K; ++l)
        if (n_sym[l] < 0 || n_sym[l] > DOL_MAX_SYMBOLS) return fail(DOL_ESHAPE, "n_sym[%d] = %d outside 0..%d", l, n_sym[l], DOL_MAX_SYMBOLS);
    if (n < 0) return fail(DOL_EINVAL, "negative tuple count");
    if (n > 0 && (!idx || !out_id)) return fail(DOL_EINVAL, "tuple arrays are NULL");
    return build_k(K, n_sym, n, idx, out_id, table);
}

int32_t dol_fnk_table_n_out(const dol_fnk_table *table) { return table ? table->n_out : 0; }

const int32_t *dol_fnk_table_out_syms(const dol_fnk_table *table) { return table ? table->out_syms.data() : nullptr; }

const char *dol_fnk_table_kernel(const dol_fnk_table *table, int32_t which)
{
    static thread_local char name[64];
    if (!table) return "";
    if (table->K == 1)
        snprintf(name, sizeof name, "damp_apply1_%s%s_kernel", which ? "bwd" : "fwd",
                 (which ? staged_unary_bwd(table) : staged_unary_fwd(table)) ? "_staged" : "");
    else
        snprintf(name, sizeof name, "damp_applyk_%s_kernel<%d>", which ? "bwd" : "fwd", table->K);
    return name;
}

void dol_fnk_table_destroy(dol_fnk_table *table) { delete table; }

dol_status dol_apply_k(int32_t K, const dol_dist *const *in, const dol_fnk_table *f, const dol_prov *prov, dol_dist *out,
                       void *hip_stream)
{
    const bool dtkp = is_dtkp(prov);
    if (dol_status st = check_operands(K, in, f, dtkp)) return st;
    if (dol_status st = check_dist(out, "out", dtkp, false, true)) return st;
    const int32_t batch = in[0]->batch;
    if (dol_status st = check_prov(prov, batch)) return st;
    if (out->batch != batch) return fail(DOL_ESHAPE, "batch sizes differ: in[0] has %d, out has %d", batch, out->batch);
    if (out->n_sym != f->n_out) return fail(DOL_ESHAPE, "out.n_sym = %d, the table produces %d symbols", out->n_sym, f->n_out);
    if (out->sym_ids)
        for (int32_t c = 0; c < f->n_out; ++c)
            if (out->sym_ids[c] != f->out_syms[c]) return fail(DOL_EINVAL, "out.sym_ids[%d] = %d, the table produces %d there", c, out->sym_ids[c], f->out_syms[c]);
    if (dol_status st = check_work(batch, f->n_out)) return st;
    if (batch == 0 || f->n_out == 0) return DOL_OK;
    if (static_cast<int64_t>(batch) * static_cast<int64_t>(std::max(f->long_cols.n, f->dtkp_long_cols.n)) > 0x7fffffffLL)
        return fail(DOL_EUNSUPPORTED, "batch x long table columns exceeds 2^31");
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (!dtkp) {
        KOperands ops{};
        for (int l = 0; l < K; ++l) { ops.p[l] = in[l]->prob; ops.ld[l] = in[l]->ld; }
        const Rows R = rows_of(batch, f->n_out);
#define CALL(KK) launch_fwd_k<KK>(R, ops, f, out->prob, out->ld, st)
        DOL_DISPATCH_ARITY(K, CALL)
#undef CALL
        DOL_HIP(hipGetLastError());
        return DOL_OK;
    }
    if (!out->proof_prob) return fail(DOL_EINVAL, "out.proof_prob is NULL");
    GroupMasks gm;
    if (dol_status s2 = make_group_masks(prov, &gm)) return s2;
    KProofs pr{};
    for (int l = 0; l < K; ++l) { pr.m[l] = in[l]->proof_mask; pr.p[l] = in[l]->proof_prob; pr.n[l] = in[l]->n_sym; }
    const int64_t total = static_cast<int64_t>(batch) * f->n_out;
    switch (prov->k) {
#define CASE(KP) case KP: launch_dtkp_k<KP>(total, f, pr, gm, prov->n_facts, prov->fact_prob, out->proof_mask, out->proof_prob, out->prob, out->ld, st); break;
        CASE(1) CASE(2) CASE(3) CASE(4) CASE(5) CASE(6) CASE(7) CASE(8)
#undef CASE
    default: return fail(DOL_EINVAL, "k = %d outside 1..%d", prov->k, DOL_MAX_K);
    }
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

dol_status dol_apply_k_backward(int32_t K, const dol_dist *const *in, const dol_fnk_table *f, const dol_dist *out,
                                const float *grad_out, int64_t grad_out_ld, float *const *grad_in, void *hip_stream)
{
    if (dol_status st = check_operands(K, in, f, false)) return st;
    if (dol_status st = check_dist(out, "out", false, false, true)) return st;
    const int32_t batch = in[0]->batch;
    if (out->batch != batch) return fail(DOL_ESHAPE, "batch sizes differ: in[0] has %d, out has %d", batch, out->batch);
    if (out->n_sym != f->n_out) return fail(DOL_ESHAPE, "out.n_sym = %d, the table produces %d symbols", out->n_sym, f->n_out);
    if (!grad_in) return fail(DOL_EINVAL, "grad_in is NULL");
    if (grad_out_ld < f->n_out) return fail(DOL_ESHAPE, "grad_out_ld = %lld smaller than %d symbols", static_cast<long long>(grad_out_ld), f->n_out);
    const int32_t rows = f->row_base[K];
    if (dol_status st = check_work(batch, rows)) return st;
    bool any = false;
    for (int l = 0; l < K; ++l) any |= grad_in[l] != nullptr && f->n_sym[l] > 0;
    if (batch == 0 || rows == 0 || !any) return DOL_OK;
    if (f->n_out > 0 && !grad_out) return fail(DOL_EINVAL, "grad_out is NULL");
    KOperands ops{};
    KGrads gr{};
    for (int l = 0; l < K; ++l) { ops.p[l] = in[l]->prob; ops.ld[l] = in[l]->ld; gr.p[l] = grad_in[l]; }
    for (int l = 0; l <= K; ++l) gr.row_base[l] = f->row_base[l];
    const Rows R = rows_of(batch, rows);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
#define CALL(KK) launch_bwd_k<KK>(R, ops, gr, f, out->prob, out->ld, grad_out, grad_out_ld, st)
    DOL_DISPATCH_ARITY(K, CALL)
#undef CALL
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

}  // extern "C"
