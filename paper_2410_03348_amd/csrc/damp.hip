// DAMP provenance kernels (Sec. 3.2, Table 1: conjunction t*t', disjunction min(1, t+t')) for gfx950.
//
// Thread mapping: one thread per (sample, output element), consecutive lanes on consecutive elements of one
// row, so that every store is coalesced and, for tables with regular structure (sums, grids), lane-adjacent
// gathers touch adjacent addresses.  Rows are short (tens to a few thousand floats) and every operand row is
// re-read only by the threads of the same wavefronts, so gathers are served from L1/L2; HBM sees each
// operand once.
#include "internal.h"

namespace dol {

constexpr int kThreads = 256;

static inline unsigned grid_for(int64_t work) { return static_cast<unsigned>((work + kThreads - 1) / kThreads); }

// ---------------------------------------------------------------- apply2 forward

// pre[c] = sum over the tuples of column c, ascending (i, j), one fma each.  This order is part of the
// operator's contract: the backward pass re-derives the clamp decision [pre <= 1] from it.
__device__ __forceinline__ float column_sum(const float *__restrict__ ar, const float *__restrict__ br,
                                            const uint32_t *__restrict__ col_ij, uint32_t q0, uint32_t q1)
{
    float acc = 0.0f;
    for (uint32_t q = q0; q < q1; ++q) {
        const uint32_t ij = col_ij[q];
        acc = __builtin_fmaf(ar[ij & 0xffffu], br[ij >> 16], acc);
    }
    return acc;
}

__global__ void __launch_bounds__(kThreads)
damp_apply2_fwd_kernel(int64_t total, int32_t S, const uint32_t *__restrict__ col_ptr,
                       const uint32_t *__restrict__ col_ij, const float *__restrict__ a, int64_t lda,
                       const float *__restrict__ b, int64_t ldb, float *__restrict__ out, int64_t ldo)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t s = idx / S;
    const int32_t c = static_cast<int32_t>(idx - s * S);
    const float pre = column_sum(a + s * lda, b + s * ldb, col_ij, col_ptr[c], col_ptr[c + 1]);
    out[s * ldo + c] = fminf(pre, 1.0f);
}

dol_status launch_damp_apply2_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                  int64_t ldb, float *out, int64_t ldo, hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * f->n_out;
    if (total == 0) return DOL_OK;
    if (conv_path_ok(f)) return launch_damp_conv_fwd(f, batch, a, lda, b, ldb, out, ldo, st);
    hipLaunchKernelGGL(damp_apply2_fwd_kernel, dim3(grid_for(total)), dim3(kThreads), 0, st, total, f->n_out,
                       f->col_ptr.ptr, f->col_ij.ptr, a, lda, b, ldb, out, ldo);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// ---------------------------------------------------------------- apply2 backward

// Gradient reaching the unclamped sum of column c.  out < 1 means the clamp did not act (pre = out);
// out == 1 leaves pre == 1 (passes) and pre > 1 (blocks) apart only by recomputing pre.
__device__ __forceinline__ float gated_grad(const float *__restrict__ gr, const float *__restrict__ outr,
                                            const float *__restrict__ ar, const float *__restrict__ br,
                                            const uint32_t *__restrict__ col_ptr,
                                            const uint32_t *__restrict__ col_ij, uint32_t c)
{
    float g = gr[c];
    if (outr[c] >= 1.0f) {
        const float pre = column_sum(ar, br, col_ij, col_ptr[c], col_ptr[c + 1]);
        if (!(pre <= 1.0f)) g = 0.0f;
    }
    return g;
}

__global__ void __launch_bounds__(kThreads)
damp_apply2_bwd_kernel(int64_t total, int32_t na, int32_t nb, const uint32_t *__restrict__ col_ptr,
                       const uint32_t *__restrict__ col_ij, const uint32_t *__restrict__ rowa_ptr,
                       const uint32_t *__restrict__ rowa_jc, const uint32_t *__restrict__ rowb_ptr,
                       const uint32_t *__restrict__ rowb_ic, const float *__restrict__ a, int64_t lda,
                       const float *__restrict__ b, int64_t ldb, const float *__restrict__ out, int64_t ldo,
                       const float *__restrict__ g, int64_t ldg, float *__restrict__ ga, float *__restrict__ gb,
                       int32_t accumulate)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int32_t n = na + nb;
    const int64_t s = idx / n;
    const int32_t x = static_cast<int32_t>(idx - s * n);
    const float *ar = a + s * lda, *br = b + s * ldb, *outr = out + s * ldo, *gr = g + s * ldg;
    if (x < na) {
        if (!ga) return;
        float acc = 0.0f;
        for (uint32_t q = rowa_ptr[x], q1 = rowa_ptr[x + 1]; q < q1; ++q) {
            const uint32_t jc = rowa_jc[q];
            acc = __builtin_fmaf(gated_grad(gr, outr, ar, br, col_ptr, col_ij, jc >> 16), br[jc & 0xffffu], acc);
        }
        ga[s * lda + x] = (accumulate & 1) ? ga[s * lda + x] + acc : acc;
    } else {
        if (!gb) return;
        const int32_t j = x - na;
        float acc = 0.0f;
        for (uint32_t q = rowb_ptr[j], q1 = rowb_ptr[j + 1]; q < q1; ++q) {
            const uint32_t ic = rowb_ic[q];
            acc = __builtin_fmaf(gated_grad(gr, outr, ar, br, col_ptr, col_ij, ic >> 16), ar[ic & 0xffffu], acc);
        }
        gb[s * ldb + j] = (accumulate & 2) ? gb[s * ldb + j] + acc : acc;
    }
}

dol_status launch_damp_apply2_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                  int64_t ldb, const float *out, int64_t ldo, const float *g, int64_t ldg, float *ga,
                                  float *gb, int32_t accumulate, hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * (f->na + f->nb);
    if (total == 0 || (!ga && !gb)) return DOL_OK;
    if (conv_path_ok(f)) return launch_damp_conv_bwd(f, batch, a, lda, b, ldb, g, ldg, ga, gb, accumulate, st);
    hipLaunchKernelGGL(damp_apply2_bwd_kernel, dim3(grid_for(total)), dim3(kThreads), 0, st, total, f->na, f->nb,
                       f->col_ptr.ptr, f->col_ij.ptr, f->rowa_ptr.ptr, f->rowa_jc.ptr, f->rowb_ptr.ptr,
                       f->rowb_ic.ptr, a, lda, b, ldb, out, ldo, g, ldg, ga, gb, accumulate);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// ---------------------------------------------------------------- filter

// x[s, 0..n) = 0 (a fill kernel rather than a memset node, so that callers may capture the stream)
__global__ void __launch_bounds__(kThreads)
zero_rows_kernel(int64_t total, int32_t n, float *__restrict__ x, int64_t ld)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t s = idx / n;
    x[s * ld + (idx - s * n)] = 0.0f;
}

dol_status launch_zero_rows(int32_t batch, int32_t n, float *x, int64_t ld, hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * n;
    if (total == 0) return DOL_OK;
    hipLaunchKernelGGL(zero_rows_kernel, dim3(grid_for(total)), dim3(kThreads), 0, st, total, n, x, ld);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

__global__ void __launch_bounds__(kThreads)
damp_gather_cols_kernel(int64_t total, int32_t n_out, const int32_t *__restrict__ src_col,
                        const float *__restrict__ in, int64_t ldi, float *__restrict__ out, int64_t ldo,
                        int32_t accumulate)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t s = idx / n_out;
    const int32_t c = static_cast<int32_t>(idx - s * n_out);
    const int32_t i = src_col[c];
    const float v = i >= 0 ? in[s * ldi + i] : 0.0f;
    out[s * ldo + c] = accumulate ? out[s * ldo + c] + v : v;
}

dol_status launch_damp_filter_fwd(const FilterPlan *p, int32_t batch, const float *in, int64_t ldi, float *out,
                                  int64_t ldo, hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * p->n_out;
    if (total == 0) return DOL_OK;
    hipLaunchKernelGGL(damp_gather_cols_kernel, dim3(grid_for(total)), dim3(kThreads), 0, st, total, p->n_out,
                       p->d_keep_idx.ptr, in, ldi, out, ldo, 0);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

dol_status launch_damp_filter_bwd(const FilterPlan *p, int32_t batch, const float *g, int64_t ldg, float *gin,
                                  int64_t ldgi, int32_t accumulate, hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * p->n_in;
    if (total == 0) return DOL_OK;
    hipLaunchKernelGGL(damp_gather_cols_kernel, dim3(grid_for(total)), dim3(kThreads), 0, st, total, p->n_in,
                       p->d_pos.ptr, g, ldg, gin, ldgi, accumulate & 1);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// ---------------------------------------------------------------- union

__global__ void __launch_bounds__(kThreads)
damp_union_fwd_kernel(int64_t total, int32_t S, const int32_t *__restrict__ ia, const int32_t *__restrict__ ib,
                      const float *__restrict__ a, int64_t lda, const float *__restrict__ b, int64_t ldb,
                      float *__restrict__ out, int64_t ldo)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t s = idx / S;
    const int32_t c = static_cast<int32_t>(idx - s * S);
    const int32_t i = ia[c], j = ib[c];
    float v;
    if (i >= 0 && j >= 0) v = fminf(a[s * lda + i] + b[s * ldb + j], 1.0f);
    else if (i >= 0) v = a[s * lda + i];
    else v = b[s * ldb + j];
    out[s * ldo + c] = v;
}

dol_status launch_damp_union_fwd(const UnionPlan *p, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, float *out, int64_t ldo, hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * p->n_out;
    if (total == 0) return DOL_OK;
    hipLaunchKernelGGL(damp_union_fwd_kernel, dim3(grid_for(total)), dim3(kThreads), 0, st, total, p->n_out,
                       p->d_ia.ptr, p->d_ib.ptr, a, lda, b, ldb, out, ldo);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// Thread x of a sample handles input position x of a (x < na) or x - na of b.
__global__ void __launch_bounds__(kThreads)
damp_union_bwd_kernel(int64_t total, int32_t na, int32_t nb, const int32_t *__restrict__ ia,
                      const int32_t *__restrict__ ib, const int32_t *__restrict__ ca, const int32_t *__restrict__ cb,
                      const float *__restrict__ a, int64_t lda, const float *__restrict__ b, int64_t ldb,
                      const float *__restrict__ g, int64_t ldg, float *__restrict__ ga, float *__restrict__ gb,
                      int32_t accumulate)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int32_t n = na + nb;
    const int64_t s = idx / n;
    const int32_t x = static_cast<int32_t>(idx - s * n);
    const bool is_a = x < na;
    if (is_a ? !ga : !gb) return;
    const int32_t c = is_a ? ca[x] : cb[x - na];
    const int32_t i = ia[c], j = ib[c];
    float gv = g[s * ldg + c];
    if (i >= 0 && j >= 0 && !(a[s * lda + i] + b[s * ldb + j] <= 1.0f)) gv = 0.0f;
    if (is_a) ga[s * lda + x] = (accumulate & 1) ? ga[s * lda + x] + gv : gv;
    else gb[s * ldb + (x - na)] = (accumulate & 2) ? gb[s * ldb + (x - na)] + gv : gv;
}

dol_status launch_damp_union_bwd(const UnionPlan *p, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                                 hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * (p->na + p->nb);
    if (total == 0 || (!ga && !gb)) return DOL_OK;
    hipLaunchKernelGGL(damp_union_bwd_kernel, dim3(grid_for(total)), dim3(kThreads), 0, st, total, p->na, p->nb,
                       p->d_ia.ptr, p->d_ib.ptr, p->d_ca.ptr, p->d_cb.ptr, a, lda, b, ldb, g, ldg, ga, gb, accumulate);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// ---------------------------------------------------------------- harness helper: gradient of -log p[target]

__global__ void __launch_bounds__(kThreads)
nll_grad_kernel(int64_t total, int32_t n, const float *__restrict__ p, int64_t ld, const int32_t *__restrict__ target,
                float *__restrict__ grad)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (idx >= total) return;
    const int64_t s = idx / n;
    const int32_t c = static_cast<int32_t>(idx - s * n);
    grad[s * ld + c] = c == target[s] ? -1.0f / fmaxf(p[s * ld + c], 1.17549435e-38f) : 0.0f;
}

dol_status launch_nll_grad(int32_t batch, int32_t n, const float *p, int64_t ld, const int32_t *target, float *grad,
                           hipStream_t st)
{
    const int64_t total = static_cast<int64_t>(batch) * n;
    if (total == 0) return DOL_OK;
    hipLaunchKernelGGL(nll_grad_kernel, dim3(grid_for(total)), dim3(kThreads), 0, st, total, n, p, ld, target, grad);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

}  // namespace dol
