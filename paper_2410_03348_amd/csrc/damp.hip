// DAMP provenance kernels (Sec. 3.2, Table 1: conjunction t*t', disjunction min(1, t+t')) for gfx950:
// Apply with an arbitrary function table, Filter, Union and their vector-Jacobian products.
//
// Thread mapping: one thread per (sample, output element), consecutive lanes on consecutive elements of one
// row, so that every store is coalesced and, for tables with regular structure (grids), lane-adjacent gathers
// touch adjacent addresses.  A workgroup owns a chunk of whole rows (about 2048 elements) and splits its
// flat element index into (row, column) with a float reciprocal, which is exact for such small indices.
// Sum-shaped tables take the LDS kernels of damp_conv.hip instead.
#include "element_map.h"
#include "internal.h"
#include "wave_util.h"

namespace dol {

// ---------------------------------------------------------------- apply2 forward

// pre[c] = sum over the tuples of column c, ascending (i, j), one fma each.  This order is part of the
// operator's contract: the backward pass re-derives the clamp decision [pre <= 1] from it.
// The loads of kGather tuples are issued together (index words first, then the tags they name) so that a column
// costs a few memory round trips rather than two per tuple; the adds keep their order.
constexpr int kGather = 4;

__device__ __forceinline__ float column_sum(const float *__restrict__ ar, const float *__restrict__ br,
                                            const uint32_t *__restrict__ col_ij, uint32_t q0, uint32_t q1)
{
    float acc = 0.0f;
    for (uint32_t q = q0; q < q1; q += kGather) {
        uint32_t ij[kGather];
        float x[kGather], y[kGather];
#pragma unroll
        for (int u = 0; u < kGather; ++u) ij[u] = col_ij[min(q + u, q1 - 1)];
#pragma unroll
        for (int u = 0; u < kGather; ++u) {
            x[u] = ar[ij[u] & 0xffffu];
            y[u] = br[ij[u] >> 16];
        }
#pragma unroll
        for (int u = 0; u < kGather; ++u)
            if (q + u < q1) acc = __builtin_fmaf(x[u], y[u], acc);
    }
    return acc;
}

// One thread per (sample, column).  The column's first four tuples come with one 16-byte load of col_head; only a
// column with more tuples goes on through its list (same order).
__global__ void __launch_bounds__(kThreads)
damp_apply2_fwd_kernel(Rows R, const uint32_t *__restrict__ col_ptr, const uint32_t *__restrict__ col_ij,
                       const uint4 *__restrict__ col_head, const float *__restrict__ a, int64_t lda,
                       const float *__restrict__ b, int64_t ldb, float *__restrict__ out, int64_t ldo)
{
    for_each_element(R, [&](int64_t s, int c) {
        const float *ar = a + s * lda, *br = b + s * ldb;
        const uint4 h = col_head[c];
        const uint32_t t[4] = {h.x, h.y, h.z, h.w};
        float x[4], y[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool there = t[u] != 0xFFFFFFFFu;
            x[u] = there ? ar[t[u] & 0xffffu] : 0.0f;
            y[u] = there ? br[t[u] >> 16] : 0.0f;
        }
        float acc = 0.0f;
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (t[u] != 0xFFFFFFFFu) acc = __builtin_fmaf(x[u], y[u], acc);
        if (t[3] != 0xFFFFFFFFu) {                                         // four or more tuples: the rest of the list
            const uint32_t q0 = col_ptr[c], q1 = col_ptr[c + 1];
            if (q1 - q0 > static_cast<uint32_t>(kLongTableCol)) return;    // left to the wavefront-per-column kernel
            for (uint32_t q = q0 + 4; q < q1; q += kGather) {
                uint32_t ij[kGather];
                float xs[kGather], ys[kGather];
#pragma unroll
                for (int u = 0; u < kGather; ++u) ij[u] = col_ij[min(q + u, q1 - 1)];
#pragma unroll
                for (int u = 0; u < kGather; ++u) {
                    xs[u] = ar[ij[u] & 0xffffu];
                    ys[u] = br[ij[u] >> 16];
                }
#pragma unroll
                for (int u = 0; u < kGather; ++u)
                    if (q + u < q1) acc = __builtin_fmaf(xs[u], ys[u], acc);
            }
        }
        out[s * ldo + c] = fminf(acc, 1.0f);
    });
}

// The same for wide operand rows, staged in LDS (element_map.h): both rows of the sample are copied in, then every
// thread walks columns as above with its gathers served by LDS.
__global__ void __launch_bounds__(kStageThreads)
damp_apply2_fwd_staged_kernel(int32_t na, int32_t nb, int32_t S, int32_t parts, const uint32_t *__restrict__ order,
                              const uint32_t *__restrict__ col_ptr, const uint32_t *__restrict__ col_ij,
                              const uint4 *__restrict__ col_head,
                              const float *__restrict__ a, int64_t lda, const float *__restrict__ b, int64_t ldb,
                              float *__restrict__ out, int64_t ldo)
{
    extern __shared__ __align__(16) float lds_rows[];
    float *ar = lds_rows, *br = lds_rows + ((na + 3) & ~3);
    const int64_t s = blockIdx.x / static_cast<unsigned>(parts);
    int c0, c1;
    stage_part(S, parts, static_cast<int>(blockIdx.x - s * parts), c0, c1);
    stage_row(ar, a + s * lda, na);
    stage_row(br, b + s * ldb, nb);
    __syncthreads();
    // kStageUnroll columns per thread and pass, so that their index and head loads are in flight together
    for (int r0 = c0 + threadIdx.x; r0 < c1; r0 += kStageUnroll * kStageThreads) {
        uint32_t c[kStageUnroll];
        uint4 h[kStageUnroll];
#pragma unroll
        for (int v = 0; v < kStageUnroll; ++v) {
            const int r = min(r0 + v * kStageThreads, c1 - 1);
            c[v] = order[r];                                               // lanes of a wavefront: columns of like length
            h[v] = col_head[r];                                            // (the head table in that order: a coalesced load)
        }
#pragma unroll
        for (int v = 0; v < kStageUnroll; ++v) {
            if (r0 + v * kStageThreads >= c1) continue;
            const uint32_t t[4] = {h[v].x, h[v].y, h[v].z, h[v].w};
            float x[4], y[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {                                  // all eight reads at once (tuple (0, 0) for "none")
                const uint32_t ij = t[u] != 0xFFFFFFFFu ? t[u] : 0u;
                x[u] = ar[ij & 0xffffu];
                y[u] = br[ij >> 16];
            }
            float acc = 0.0f;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (t[u] != 0xFFFFFFFFu) acc = __builtin_fmaf(x[u], y[u], acc);
            if (t[3] != 0xFFFFFFFFu) {                                     // four or more tuples: the rest of the list
                const uint32_t q0 = col_ptr[c[v]], q1 = col_ptr[c[v] + 1];
                if (q1 - q0 > static_cast<uint32_t>(kLongTableCol)) continue;   // left to the wavefront-per-column kernel
                for (uint32_t q = q0 + 4; q < q1; q += kGather) {
                    uint32_t ij[kGather];
#pragma unroll
                    for (int u = 0; u < kGather; ++u) ij[u] = col_ij[min(q + u, q1 - 1)];
#pragma unroll
                    for (int u = 0; u < kGather; ++u)
                        if (q + u < q1) acc = __builtin_fmaf(ar[ij[u] & 0xffffu], br[ij[u] >> 16], acc);
                }
            }
            out[s * ldo + c[v]] = fminf(acc, 1.0f);
        }
    }
}

// One workgroup of 1, 4 or 16 wavefronts (by the table's longest column) per (sample, long column).  The lanes stride
// over the column's tuples and their partial sums meet by shuffles and, between wavefronts, through LDS; this is not the order the clamp decision is defined in, so alongside the sum the lanes add up the
// terms' magnitudes, which bounds how far the two orders can lie apart (n roundings of relative size 2^-24 each
// way).  Only a sum within that distance of 1 is taken again in the defining order, by every lane alike.
__global__ void __launch_bounds__(1024)
damp_apply2_fwd_long_kernel(int32_t n_long, const uint32_t *__restrict__ long_cols,
                            const uint32_t *__restrict__ col_ptr, const uint32_t *__restrict__ col_ij,
                            const float *__restrict__ a, int64_t lda, const float *__restrict__ b, int64_t ldb,
                            float *__restrict__ out, int64_t ldo)
{
    const int64_t s = blockIdx.x / n_long;
    const uint32_t c = long_cols[blockIdx.x - s * n_long];
    const float *ar = a + s * lda, *br = b + s * ldb;
    const uint32_t q0 = col_ptr[c], q1 = col_ptr[c + 1];
    __shared__ float part[2][16];
    const uint32_t step = blockDim.x;
    float acc = 0.0f, mag = 0.0f;
    for (uint32_t q = q0 + threadIdx.x; q < q1; q += kGather * step) {
        uint32_t ij[kGather];
        float x[kGather], y[kGather];
#pragma unroll
        for (int u = 0; u < kGather; ++u) ij[u] = col_ij[min(q + u * step, q1 - 1)];
#pragma unroll
        for (int u = 0; u < kGather; ++u) {
            x[u] = ar[ij[u] & 0xffffu];
            y[u] = br[ij[u] >> 16];
        }
#pragma unroll
        for (int u = 0; u < kGather; ++u)
            if (q + u * step < q1) {
                acc = __builtin_fmaf(x[u], y[u], acc);
                mag = __builtin_fmaf(fabsf(x[u]), fabsf(y[u]), mag);
            }
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) {
        acc += __shfl_xor(acc, d, kWave);
        mag += __shfl_xor(mag, d, kWave);
    }
    if (step > kWave) {                             // uniform: the wavefronts' sums, added in wavefront order
        const int wave = threadIdx.x / kWave, n_waves = step / kWave;
        if ((threadIdx.x & (kWave - 1)) == 0) { part[0][wave] = acc; part[1][wave] = mag; }
        __syncthreads();
        if (wave != 0) return;
        acc = 0.0f, mag = 0.0f;
        for (int w = 0; w < n_waves; ++w) { acc += part[0][w]; mag += part[1][w]; }
    }
    const float slack = mag * (static_cast<float>(q1 - q0 + step) * 1.1920929e-7f);
    float pre = acc;
    if (fabsf(acc - 1.0f) <= slack) pre = column_sum(ar, br, col_ij, q0, q1);
    if (threadIdx.x == 0) out[s * ldo + c] = fminf(pre, 1.0f);
}

// Tables with a short second operand: one thread per (sample, column) walks the dense map one j at a time (index
// loads coalesced, the gathers of neighbouring lanes adjacent wherever the function is monotone in i).  That is
// not the order the clamp decision is defined in; the terms' magnitudes bound how far the two sums can lie apart,
// and only a sum within that distance of 1 is taken again in the defining order.
// (The maps have NBP >= nb rows, the extra ones empty.)
template <int NBP>
__global__ void __launch_bounds__(kThreads)
damp_byj_fwd_kernel(Rows R, int32_t nb, const uint16_t *__restrict__ src, const uint32_t *__restrict__ col_ptr,
                    const uint32_t *__restrict__ col_ij, const float *__restrict__ a, int64_t lda,
                    const float *__restrict__ b, int64_t ldb, float *__restrict__ out, int64_t ldo)
{
    float y[NBP];                                   // the short operand's row of the sample at hand
    int64_t s_held = -1;
    for_each_element(R, [&](int64_t s, int c) {
        const float *ar = a + s * lda, *br = b + s * ldb;
        if (s != s_held) {
#pragma unroll
            for (int j = 0; j < NBP; ++j) y[j] = br[j < nb ? j : 0];
            s_held = s;
        }
        uint16_t i[NBP];
        float x[NBP];
#pragma unroll
        for (int j = 0; j < NBP; ++j) i[j] = src[static_cast<size_t>(j) * R.n + c];
        if (i[0] == kByJWave) return;                                     // left to the wavefront-per-column kernel
        if (i[0] == kByJList) {                                           // some j twice: the tuple list itself
            out[s * ldo + c] = fminf(column_sum(ar, br, col_ij, col_ptr[c], col_ptr[c + 1]), 1.0f);
            return;
        }
#pragma unroll
        for (int j = 0; j < NBP; ++j) x[j] = i[j] != kByJNone ? ar[i[j]] : 0.0f;
        float acc = 0.0f, mag = 0.0f;
#pragma unroll
        for (int j = 0; j < NBP; ++j) {
            acc = __builtin_fmaf(x[j], y[j], acc);
            mag = __builtin_fmaf(fabsf(x[j]), fabsf(y[j]), mag);
        }
        float pre = acc;
        if (fabsf(acc - 1.0f) <= mag * (static_cast<float>(NBP + 2) * 1.1920929e-7f))
            pre = column_sum(ar, br, col_ij, col_ptr[c], col_ptr[c + 1]);
        out[s * ldo + c] = fminf(pre, 1.0f);
    });
}

// The same with the first operand's row staged in LDS (element_map.h), for rows of thousands of tags: one workgroup
// per (sample, part of the output row); the map is still read coalesced and the gathers become LDS reads (an empty
// entry reads element 0 and counts as 0).
template <int NBP>
__global__ void __launch_bounds__(kStageThreads)
damp_byj_fwd_staged_kernel(int32_t na, int32_t nb, int32_t S, int32_t parts, const uint16_t *__restrict__ src,
                           const uint32_t *__restrict__ col_ptr, const uint32_t *__restrict__ col_ij,
                           const float *__restrict__ a, int64_t lda, const float *__restrict__ b, int64_t ldb,
                           float *__restrict__ out, int64_t ldo)
{
    extern __shared__ __align__(16) float a_row[];
    const int64_t s = blockIdx.x / static_cast<unsigned>(parts);
    int c0, c1;
    stage_part(S, parts, static_cast<int>(blockIdx.x - s * parts), c0, c1);
    const float *ar = a + s * lda, *br = b + s * ldb;
    stage_row(a_row, ar, na);
    float y[NBP];
#pragma unroll
    for (int j = 0; j < NBP; ++j) y[j] = br[j < nb ? j : 0];
    __syncthreads();
    for (int c = c0 + threadIdx.x; c < c1; c += kStageThreads) {
        uint16_t i[NBP];
        float x[NBP];
#pragma unroll
        for (int j = 0; j < NBP; ++j) i[j] = src[static_cast<size_t>(j) * S + c];
        if (i[0] == kByJWave) continue;                                   // left to the wavefront-per-column kernel
        if (i[0] == kByJList) {                                           // some j twice: the tuple list itself
            out[s * ldo + c] = fminf(column_sum(ar, br, col_ij, col_ptr[c], col_ptr[c + 1]), 1.0f);
            continue;
        }
#pragma unroll
        for (int j = 0; j < NBP; ++j) {
            const float v = a_row[i[j] != kByJNone ? i[j] : 0];
            x[j] = i[j] != kByJNone ? v : 0.0f;
        }
        float acc = 0.0f, mag = 0.0f;
#pragma unroll
        for (int j = 0; j < NBP; ++j) {
            acc = __builtin_fmaf(x[j], y[j], acc);
            mag = __builtin_fmaf(fabsf(x[j]), fabsf(y[j]), mag);
        }
        float pre = acc;
        if (fabsf(acc - 1.0f) <= mag * (static_cast<float>(NBP + 2) * 1.1920929e-7f))
            pre = column_sum(ar, br, col_ij, col_ptr[c], col_ptr[c + 1]);
        out[s * ldo + c] = fminf(pre, 1.0f);
    }
}

#define DOL_DISPATCH_NBP(nbp, CALL) \
    switch (nbp) {                  \
    case 4: CALL(4); break;         \
    case 8: CALL(8); break;         \
    case 10: CALL(10); break;       \
    default: CALL(16); break;       \
    }

static dol_status launch_fwd_waves(const dol_fn_table *f, const DevArray<uint32_t> &cols, int32_t n_huge, int32_t batch,
                                   const float *a, int64_t lda, const float *b, int64_t ldb, float *out, int64_t ldo,
                                   hipStream_t st)
{
    const int64_t n_long = static_cast<int64_t>(cols.n);
    if (n_long == 0) return DOL_OK;
    if (batch * n_long > 0x7fffffffLL)
        return fail(DOL_EUNSUPPORTED, "batch x long table columns = %lld exceeds 2^31", static_cast<long long>(batch * n_long));
    if (n_huge > 0)                                  // the list's first n_huge columns: 16 wavefronts each
        hipLaunchKernelGGL(damp_apply2_fwd_long_kernel, dim3(static_cast<unsigned>(batch) * n_huge), dim3(1024), 0, st, n_huge,
                           cols.ptr, f->col_ptr.ptr, f->col_ij.ptr, a, lda, b, ldb, out, ldo);
    if (n_long > n_huge)
        hipLaunchKernelGGL(damp_apply2_fwd_long_kernel, dim3(static_cast<unsigned>(batch * (n_long - n_huge))), dim3(kWave), 0,
                           st, static_cast<int32_t>(n_long - n_huge), cols.ptr + n_huge, f->col_ptr.ptr, f->col_ij.ptr, a, lda,
                           b, ldb, out, ldo);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

dol_status launch_damp_apply2_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                  int64_t ldb, float *out, int64_t ldo, hipStream_t st)
{
    if (batch == 0 || f->n_out == 0) return DOL_OK;
    {   // shape limits before anything is launched (a failing call leaves the outputs untouched)
        const int64_t most = static_cast<int64_t>(std::max(f->long_cols.n, f->byj_wave_cols.n));
        if (batch * most > 0x7fffffffLL)
            return fail(DOL_EUNSUPPORTED, "batch x long table columns = %lld exceeds 2^31", static_cast<long long>(batch * most));
    }
    if (conv_path_ok(f)) return launch_damp_conv_fwd(f, batch, a, lda, b, ldb, out, ldo, st);
    bool done = false;
    if (dol_status s2 = launch_damp_table_fwd(f, batch, a, lda, b, ldb, out, ldo, st, &done)) return s2;
    if (done) return DOL_OK;
    if (dol_status s2 = launch_damp_lds_fwd(f, batch, a, lda, b, ldb, out, ldo, st, &done)) return s2;
    if (done) return DOL_OK;
    const Rows R = rows_of(batch, f->n_out);
    if (f->byj_fwd && byj_fwd_staged_ok(f)) {
        const int32_t parts = stage_parts(batch, f->n_out);
#define CALL(N)                                                                                                           \
    {                                                                                                                     \
        DOL_HIP(allow_dynamic_lds(reinterpret_cast<const void *>(damp_byj_fwd_staged_kernel<N>), kStageMaxBytes));                    \
        hipLaunchKernelGGL(damp_byj_fwd_staged_kernel<N>, dim3(static_cast<unsigned>(batch) * parts), dim3(kStageThreads), \
                           sizeof(float) * f->na, st, f->na, f->nb, f->n_out, parts, f->byj_src.ptr, f->col_ptr.ptr,      \
                           f->col_ij.ptr, a, lda, b, ldb, out, ldo);                                                      \
    }
        DOL_DISPATCH_NBP(f->byj_nbp, CALL)
#undef CALL
        DOL_HIP(hipGetLastError());
        return launch_fwd_waves(f, f->byj_wave_cols, f->n_huge_byj_cols, batch, a, lda, b, ldb, out, ldo, st);
    }
    if (f->byj_fwd) {
#define CALL(N) hipLaunchKernelGGL(damp_byj_fwd_kernel<N>, dim3(R.grid), dim3(kThreads), 0, st, R, f->nb, f->byj_src.ptr, \
                                   f->col_ptr.ptr, f->col_ij.ptr, a, lda, b, ldb, out, ldo)
        DOL_DISPATCH_NBP(f->byj_nbp, CALL)
#undef CALL
        DOL_HIP(hipGetLastError());
        return launch_fwd_waves(f, f->byj_wave_cols, f->n_huge_byj_cols, batch, a, lda, b, ldb, out, ldo, st);
    }
    if (staged_fwd_ok(f)) {
        const int32_t parts = stage_parts(batch, f->n_out);
        DOL_HIP(allow_dynamic_lds(reinterpret_cast<const void *>(damp_apply2_fwd_staged_kernel), kStageMaxBytes));
        hipLaunchKernelGGL(damp_apply2_fwd_staged_kernel, dim3(static_cast<unsigned>(batch) * parts), dim3(kStageThreads),
                           sizeof(float) * (((f->na + 3) & ~3) + f->nb), st, f->na, f->nb, f->n_out, parts, f->col_order.ptr,
                           f->col_ptr.ptr, f->col_ij.ptr, reinterpret_cast<const uint4 *>(f->col_head_ord.ptr), a, lda, b, ldb, out, ldo);
    } else {
        hipLaunchKernelGGL(damp_apply2_fwd_kernel, dim3(R.grid), dim3(kThreads), 0, st, R, f->col_ptr.ptr, f->col_ij.ptr,
                           reinterpret_cast<const uint4 *>(f->col_head.ptr), a, lda, b, ldb, out, ldo);
    }
    DOL_HIP(hipGetLastError());
    return launch_fwd_waves(f, f->long_cols, f->n_huge_cols, batch, a, lda, b, ldb, out, ldo, st);
}

// ---------------------------------------------------------------- apply2 backward

// Gradient reaching the unclamped sum of column c.  out < 1 means the clamp did not act (pre = out);
// out == 1 leaves pre == 1 (passes) and pre > 1 (blocks) apart only by recomputing pre.
__device__ __forceinline__ float gated_grad(float g, float out_c, const float *__restrict__ ar,
                                            const float *__restrict__ br, const uint32_t *__restrict__ col_ptr,
                                            const uint32_t *__restrict__ col_ij, uint32_t c)
{
    if (out_c >= 1.0f) {
        const float pre = column_sum(ar, br, col_ij, col_ptr[c], col_ptr[c + 1]);
        if (!(pre <= 1.0f)) g = 0.0f;
    }
    return g;
}

// acc += sum over entries q0 + k * stride < q1 of gated gradient of the entry's column times the other operand's
// tag, in entry order; the loads of kGather entries are issued together.
__device__ __forceinline__ float row_sum(float acc, const uint32_t *__restrict__ ent, uint32_t q0, uint32_t q1,
                                         uint32_t stride, const float *__restrict__ gr, const float *__restrict__ outr,
                                         const float *__restrict__ other, const float *__restrict__ ar,
                                         const float *__restrict__ br, const uint32_t *__restrict__ col_ptr,
                                         const uint32_t *__restrict__ col_ij)
{
    for (uint32_t q = q0; q < q1; q += kGather * stride) {
        uint32_t e[kGather];
        float gv[kGather], ov[kGather], xv[kGather];
#pragma unroll
        for (int u = 0; u < kGather; ++u) e[u] = ent[min(q + u * stride, q1 - 1)];
#pragma unroll
        for (int u = 0; u < kGather; ++u) {
            gv[u] = gr[e[u] >> 16];
            ov[u] = outr[e[u] >> 16];
            xv[u] = other[e[u] & 0xffffu];
        }
#pragma unroll
        for (int u = 0; u < kGather; ++u)
            if (q + u * stride < q1)
                acc = __builtin_fmaf(gated_grad(gv[u], ov[u], ar, br, col_ptr, col_ij, e[u] >> 16), xv[u], acc);
    }
    return acc;
}

struct BwdTable {
    const uint32_t *col_ptr, *col_ij, *rowa_ptr, *rowa_jc, *rowb_ptr, *rowb_ic;
    int32_t na, nb;
};

// Element x of a sample is position x of a (x < na) or x - na of b.  Rows of the table with more than
// kLongTableRow tuples are left to damp_apply2_bwd_long_kernel.
__global__ void __launch_bounds__(kThreads)
damp_apply2_bwd_kernel(Rows R, BwdTable T, const float *__restrict__ a, int64_t lda, const float *__restrict__ b,
                       int64_t ldb, const float *__restrict__ out, int64_t ldo, const float *__restrict__ g,
                       int64_t ldg, float *__restrict__ ga, float *__restrict__ gb, int32_t accumulate)
{
    for_each_element(R, [&](int64_t s, int x) {
        const float *ar = a + s * lda, *br = b + s * ldb, *outr = out + s * ldo, *gr = g + s * ldg;
        const bool is_a = x < T.na;
        if (is_a ? !ga : !gb) return;
        const int r = is_a ? x : x - T.na;
        const uint32_t *ptr = is_a ? T.rowa_ptr : T.rowb_ptr;
        const uint32_t *ent = is_a ? T.rowa_jc : T.rowb_ic;
        const float *other = is_a ? br : ar;
        const uint32_t q0 = ptr[r], q1 = ptr[r + 1];
        if (q1 - q0 > kLongTableRow) return;
        const float acc = row_sum(0.0f, ent, q0, q1, 1, gr, outr, other, ar, br, T.col_ptr, T.col_ij);
        float *dst = is_a ? ga + s * lda + r : gb + s * ldb + r;
        const bool add = is_a ? (accumulate & 1) : (accumulate & 2);
        *dst = add ? *dst + acc : acc;
    });
}

// The same with the gated gradient row in LDS: one workgroup per sample first works out gh[c] = g[c] * [pre(c) <= 1] for
// every column ONCE (a column's sum is re-derived only where out == 1), then every symbol of a and b adds up its tuples
// from that row, in the order of its list.  The kernel above re-derives a column's decision for every tuple that reads
// it: with many results at the clamp (the later rounds of a reachability sweep) that is most of its time.  Rows of more
// than kLongTableRow tuples are summed by the whole workgroup: strided partial sums in list order, then the
// wavefronts' totals in a fixed order.
constexpr int kBwdStagedThreads = 1024;

__global__ void __launch_bounds__(kBwdStagedThreads)
damp_apply2_bwd_staged_kernel(BwdTable T, int32_t S, int32_t n_long, const uint32_t *__restrict__ long_rows,
                              const float *__restrict__ a, int64_t lda, const float *__restrict__ b, int64_t ldb,
                              const float *__restrict__ out, int64_t ldo, const float *__restrict__ g, int64_t ldg,
                              float *__restrict__ ga, float *__restrict__ gb, int32_t accumulate)
{
    extern __shared__ float gh[];           // [S], then one float per wavefront
    float *red = gh + S;
    const int tid = threadIdx.x;
    const int64_t s = blockIdx.x;
    const float *ar = a + s * lda, *br = b + s * ldb, *outr = out + s * ldo, *gr = g + s * ldg;
    for (int c = tid; c < S; c += kBwdStagedThreads)
        gh[c] = gated_grad(gr[c], outr[c], ar, br, T.col_ptr, T.col_ij, static_cast<uint32_t>(c));
    __syncthreads();
    for (int x = tid; x < T.na + T.nb; x += kBwdStagedThreads) {
        const bool is_a = x < T.na;
        if (is_a ? !ga : !gb) continue;
        const int r = is_a ? x : x - T.na;
        const uint32_t *ent = is_a ? T.rowa_jc : T.rowb_ic;
        const float *other = is_a ? br : ar;
        const uint32_t q0 = (is_a ? T.rowa_ptr : T.rowb_ptr)[r], q1 = (is_a ? T.rowa_ptr : T.rowb_ptr)[r + 1];
        if (q1 - q0 > static_cast<uint32_t>(kLongTableRow)) continue;
        float acc = 0.0f;
        for (uint32_t q = q0; q < q1; ++q) {
            const uint32_t e = ent[q];
            acc = __builtin_fmaf(gh[e >> 16], other[e & 0xffffu], acc);
        }
        float *dst = is_a ? ga + s * lda + r : gb + s * ldb + r;
        *dst = (is_a ? (accumulate & 1) : (accumulate & 2)) ? *dst + acc : acc;
    }
    for (int l = 0; l < n_long; ++l) {
        const int x = static_cast<int>(long_rows[l]);
        const bool is_a = x < T.na;
        if (is_a ? !ga : !gb) continue;     // (the same for every thread)
        const int r = is_a ? x : x - T.na;
        const uint32_t *ent = is_a ? T.rowa_jc : T.rowb_ic;
        const float *other = is_a ? br : ar;
        const uint32_t q0 = (is_a ? T.rowa_ptr : T.rowb_ptr)[r], q1 = (is_a ? T.rowa_ptr : T.rowb_ptr)[r + 1];
        float acc = 0.0f;
        for (uint32_t q = q0 + tid; q < q1; q += kBwdStagedThreads) {
            const uint32_t e = ent[q];
            acc = __builtin_fmaf(gh[e >> 16], other[e & 0xffffu], acc);
        }
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, kWave);
        __syncthreads();                    // (the last row's totals have been read)
        if ((tid & (kWave - 1)) == 0) red[tid / kWave] = acc;
        __syncthreads();
        if (tid == 0) {
            float tot = 0.0f;
            for (int w = 0; w < kBwdStagedThreads / kWave; ++w) tot += red[w];
            float *dst = is_a ? ga + s * lda + r : gb + s * ldb + r;
            *dst = (is_a ? (accumulate & 1) : (accumulate & 2)) ? *dst + tot : tot;
        }
    }
}

// Tables the staged kernel takes: enough symbols to give a workgroup per sample its work, a result row that fits LDS.
bool apply2_bwd_staged(const dol_fn_table *f)
{
    return f->n_out >= 256 && f->na + f->nb >= 1024 && sizeof(float) * (f->n_out + kBwdStagedThreads / kWave) <= kStageMaxBytes;
}

// Gradient of row i of a from the dense map, one j at a time (ascending j, the order of the row's tuple list), and
// the row's shares gh * a[i] of the gradient of b (added to pb where SHARES).  `clamped`: some column of the sample may
// sit at the clamp, so `out` has to be looked at.  Empty map entries read element 0 and count as 0.
template <int NBP, bool SHARES>
__device__ __forceinline__ float byj_row(const uint16_t *__restrict__ col_of, int32_t na, int i, bool clamped,
                                         const float *__restrict__ gr, const float *__restrict__ outr,
                                         const float *__restrict__ ar, const float *__restrict__ br,
                                         const float (&bj)[NBP], const BwdTable &T, float (&pb)[NBP])
{
    uint16_t c[NBP];
    float gv[NBP];
#pragma unroll
    for (int j = 0; j < NBP; ++j) c[j] = col_of[static_cast<size_t>(j) * na + i];
#pragma unroll
    for (int j = 0; j < NBP; ++j) gv[j] = gr[c[j] == kByJNone ? 0 : c[j]];
    if (clamped) {
#pragma unroll
        for (int j = 0; j < NBP; ++j)
            if (c[j] != kByJNone) gv[j] = gated_grad(gv[j], outr[c[j]], ar, br, T.col_ptr, T.col_ij, c[j]);
    }
    const float ai = SHARES ? ar[i] : 0.0f;
    float acc = 0.0f;
#pragma unroll
    for (int j = 0; j < NBP; ++j) {
        const float gh = c[j] == kByJNone ? 0.0f : gv[j];
        acc = __builtin_fmaf(gh, bj[j], acc);
        if (SHARES) pb[j] = __builtin_fmaf(gh, ai, pb[j]);
    }
    return acc;
}

// Backward for tables with a short second operand: a row i of a reads its columns from the dense map; rows of b walk
// their lists as above.
template <int NBP>
__global__ void __launch_bounds__(kThreads)
damp_byj_bwd_kernel(Rows R, BwdTable T, const uint16_t *__restrict__ col_of, const float *__restrict__ a, int64_t lda,
                    const float *__restrict__ b, int64_t ldb, const float *__restrict__ out, int64_t ldo,
                    const float *__restrict__ g, int64_t ldg, float *__restrict__ ga, float *__restrict__ gb,
                    int32_t accumulate)
{
    float bj[NBP];                                  // the short operand's row of the sample at hand
    int64_t s_held = -1;
    for_each_element(R, [&](int64_t s, int x) {
        const float *ar = a + s * lda, *br = b + s * ldb, *outr = out + s * ldo, *gr = g + s * ldg;
        if (x < T.na) {
            if (!ga) return;
            float none[NBP];
            if (s != s_held) {
#pragma unroll
                for (int j = 0; j < NBP; ++j) bj[j] = j < T.nb ? br[j] : 0.0f;
                s_held = s;
            }
            const float acc = byj_row<NBP, false>(col_of, T.na, x, true, gr, outr, ar, br, bj, T, none);
            float *dst = ga + s * lda + x;
            *dst = (accumulate & 1) ? *dst + acc : acc;
            return;
        }
        if (!gb) return;
        const int r = x - T.na;
        const uint32_t q0 = T.rowb_ptr[r], q1 = T.rowb_ptr[r + 1];
        if (q1 - q0 > kLongTableRow) return;
        const float acc = row_sum(0.0f, T.rowb_ic, q0, q1, 1, gr, outr, ar, ar, br, T.col_ptr, T.col_ij);
        float *dst = gb + s * ldb + r;
        *dst = (accumulate & 2) ? *dst + acc : acc;
    });
}

// The same for wide operands (na + nb > 1024): one workgroup of 1024 threads owns a whole sample.  STAGED (the result
// row fits LDS): a first pass copies the sample's gradient row into LDS, gated by the clamp (a column with out == 1 has
// its sum taken again), and the rows then gather from LDS alone.  Otherwise a first pass over the sample's result row
// tells whether any column sits at the clamp; if none does, the gate is open everywhere and `out` is not gathered
// again.  Each thread also adds its rows' shares g^[col(i, j)] * a[i] of the gradient w.r.t. b[j] into registers; the
// workgroup sums them, so the long rows of b need no launch of their own.
constexpr int kByJRowThreads = 1024;

template <int NBP, bool STAGED>
__global__ void __launch_bounds__(kByJRowThreads)
damp_byj_bwd_row_kernel(BwdTable T, int32_t S, const uint16_t *__restrict__ col_of, const float *__restrict__ a,
                        int64_t lda, const float *__restrict__ b, int64_t ldb, const float *__restrict__ out, int64_t ldo,
                        const float *__restrict__ g, int64_t ldg, float *__restrict__ ga, float *__restrict__ gb,
                        int32_t accumulate)
{
    extern __shared__ __align__(16) float gh_row[];                 // STAGED: [S] gated gradient
    __shared__ float red[NBP][kByJRowThreads / kWave];
    const int64_t s = blockIdx.x;
    const float *ar = a + s * lda, *br = b + s * ldb, *outr = out + s * ldo, *gr = g + s * ldg;
    bool clamped = false;
    if (STAGED) {
        for (int c = threadIdx.x; c < S; c += kByJRowThreads) {
            const float o = outr[c];
            float v = gr[c];
            if (o >= 1.0f) v = gated_grad(v, o, ar, br, T.col_ptr, T.col_ij, c);
            gh_row[c] = v;
        }
        __syncthreads();
    } else {
        int hit = 0;
        for (int c = threadIdx.x; c < S; c += kByJRowThreads) hit |= outr[c] >= 1.0f;
        clamped = __syncthreads_or(hit) != 0;
    }
    float bj[NBP], pb[NBP];
#pragma unroll
    for (int j = 0; j < NBP; ++j) {
        bj[j] = j < T.nb ? br[j] : 0.0f;
        pb[j] = 0.0f;
    }
    for (int i = threadIdx.x; i < T.na; i += kByJRowThreads) {
        const float acc = STAGED ? byj_row<NBP, true>(col_of, T.na, i, false, gh_row, outr, ar, br, bj, T, pb)
                                 : byj_row<NBP, true>(col_of, T.na, i, clamped, gr, outr, ar, br, bj, T, pb);
        if (ga) {
            float *dst = ga + s * lda + i;
            *dst = (accumulate & 1) ? *dst + acc : acc;
        }
    }
    if (!gb) return;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
#pragma unroll
    for (int j = 0; j < NBP; ++j) {
        float v = pb[j];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, kWave);
        if (lane == 0) red[j][wave] = v;
    }
    __syncthreads();
    if (threadIdx.x < static_cast<unsigned>(T.nb)) {
        float tot = 0.0f;
        for (int w = 0; w < kByJRowThreads / kWave; ++w) tot = tot + red[threadIdx.x][w];
        float *dst = gb + s * ldb + threadIdx.x;
        *dst = (accumulate & 2) ? *dst + tot : tot;
    }
}

// One wavefront per (sample, long row): lanes stride over the row's tuples, the partial sums meet by shuffles.
__global__ void __launch_bounds__(kWave)
damp_apply2_bwd_long_kernel(int32_t n_long, const uint32_t *__restrict__ long_rows, BwdTable T,
                            const float *__restrict__ a, int64_t lda, const float *__restrict__ b, int64_t ldb,
                            const float *__restrict__ out, int64_t ldo, const float *__restrict__ g, int64_t ldg,
                            float *__restrict__ ga, float *__restrict__ gb, int32_t accumulate)
{
    const int64_t s = blockIdx.x / n_long;
    const int x = static_cast<int>(long_rows[blockIdx.x - s * n_long]);
    const float *ar = a + s * lda, *br = b + s * ldb, *outr = out + s * ldo, *gr = g + s * ldg;
    const bool is_a = x < T.na;
    if (is_a ? !ga : !gb) return;
    const int r = is_a ? x : x - T.na;
    const uint32_t *ptr = is_a ? T.rowa_ptr : T.rowb_ptr;
    const uint32_t *ent = is_a ? T.rowa_jc : T.rowb_ic;
    const float *other = is_a ? br : ar;
    float acc = row_sum(0.0f, ent, ptr[r] + threadIdx.x, ptr[r + 1], kWave, gr, outr, other, ar, br, T.col_ptr, T.col_ij);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, kWave);
    if (threadIdx.x == 0) {
        float *dst = is_a ? ga + s * lda + r : gb + s * ldb + r;
        const bool add = is_a ? (accumulate & 1) : (accumulate & 2);
        *dst = add ? *dst + acc : acc;
    }
}

// The workgroup-per-sample backward stages the gated gradient row in LDS when it fits beside the reduction scratch.
static bool byj_bwd_staged(const dol_fn_table *f) { return sizeof(float) * f->n_out + 2048 <= kStageMaxBytes; }

dol_status launch_damp_apply2_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                  int64_t ldb, const float *out, int64_t ldo, const float *g, int64_t ldg, float *ga,
                                  float *gb, int32_t accumulate, hipStream_t st)
{
    if (batch == 0 || f->na + f->nb == 0 || (!ga && !gb)) return DOL_OK;
    if (batch * static_cast<int64_t>(f->long_rows.n) > 0x7fffffffLL)      // before anything is launched
        return fail(DOL_EUNSUPPORTED, "batch x long table rows = %lld exceeds 2^31",
                    static_cast<long long>(batch * static_cast<int64_t>(f->long_rows.n)));
    if (conv_path_ok(f)) return launch_damp_conv_bwd(f, batch, a, lda, b, ldb, g, ldg, ga, gb, accumulate, st);
    bool done = false;
    if (dol_status s2 = launch_damp_table_bwd(f, batch, a, lda, b, ldb, g, ldg, ga, gb, accumulate, st, &done)) return s2;
    if (done) return DOL_OK;
    if (dol_status s2 = launch_damp_lds_bwd(f, batch, a, lda, b, ldb, out, ldo, g, ldg, ga, gb, accumulate, st, &done)) return s2;
    if (done) return DOL_OK;
    const BwdTable T{f->col_ptr.ptr, f->col_ij.ptr, f->rowa_ptr.ptr, f->rowa_jc.ptr, f->rowb_ptr.ptr, f->rowb_ic.ptr,
                     f->na, f->nb};
    const Rows R = rows_of(batch, f->na + f->nb);
    if (f->byj_ok && R.rpb == 1) {
        if (byj_bwd_staged(f)) {
#define CALL(N)                                                                                                           \
    {                                                                                                                     \
        DOL_HIP(allow_dynamic_lds(reinterpret_cast<const void *>(damp_byj_bwd_row_kernel<N, true>), kStageMaxBytes));                    \
        hipLaunchKernelGGL((damp_byj_bwd_row_kernel<N, true>), dim3(static_cast<unsigned>(batch)), dim3(kByJRowThreads),  \
                           sizeof(float) * f->n_out, st, T, f->n_out, f->byj_col.ptr, a, lda, b, ldb, out, ldo, g, ldg,   \
                           ga, gb, accumulate);                                                                           \
    }
            DOL_DISPATCH_NBP(f->byj_nbp, CALL)
#undef CALL
        } else {
#define CALL(N) hipLaunchKernelGGL((damp_byj_bwd_row_kernel<N, false>), dim3(static_cast<unsigned>(batch)), dim3(kByJRowThreads), 0, \
                                   st, T, f->n_out, f->byj_col.ptr, a, lda, b, ldb, out, ldo, g, ldg, ga, gb, accumulate)
            DOL_DISPATCH_NBP(f->byj_nbp, CALL)
#undef CALL
        }
        DOL_HIP(hipGetLastError());
        return DOL_OK;
    }
    if (f->byj_ok) {
#define CALL(N) hipLaunchKernelGGL(damp_byj_bwd_kernel<N>, dim3(R.grid), dim3(kThreads), 0, st, R, T, f->byj_col.ptr, a, lda, \
                                   b, ldb, out, ldo, g, ldg, ga, gb, accumulate)
        DOL_DISPATCH_NBP(f->byj_nbp, CALL)
#undef CALL
    }
    else if (apply2_bwd_staged(f)) {
        const size_t lds = sizeof(float) * (f->n_out + kBwdStagedThreads / kWave);
        if (lds > 64 * 1024) DOL_HIP(allow_dynamic_lds(reinterpret_cast<const void *>(damp_apply2_bwd_staged_kernel), kStageMaxBytes));
        hipLaunchKernelGGL(damp_apply2_bwd_staged_kernel, dim3(static_cast<unsigned>(batch)), dim3(kBwdStagedThreads), lds, st, T,
                           f->n_out, static_cast<int32_t>(f->long_rows.n), f->long_rows.ptr, a, lda, b, ldb, out, ldo, g, ldg, ga, gb,
                           accumulate);
        DOL_HIP(hipGetLastError());
        return DOL_OK;
    }
    else
        hipLaunchKernelGGL(damp_apply2_bwd_kernel, dim3(R.grid), dim3(kThreads), 0, st, R, T, a, lda, b, ldb, out, ldo, g,
                           ldg, ga, gb, accumulate);
    DOL_HIP(hipGetLastError());
    const int64_t n_long = static_cast<int64_t>(f->long_rows.n);
    if (n_long > 0) {
        if (batch * n_long > 0x7fffffffLL)
            return fail(DOL_EUNSUPPORTED, "batch x long table rows = %lld exceeds 2^31", static_cast<long long>(batch * n_long));
        hipLaunchKernelGGL(damp_apply2_bwd_long_kernel, dim3(static_cast<unsigned>(batch * n_long)), dim3(kWave), 0, st,
                           static_cast<int32_t>(n_long), f->long_rows.ptr, T, a, lda, b, ldb, out, ldo, g, ldg, ga, gb,
                           accumulate);
        DOL_HIP(hipGetLastError());
    }
    return DOL_OK;
}

// ---------------------------------------------------------------- filter

// x[s, 0..n) = 0 (a fill kernel rather than a memset node, so that callers may capture the stream)
__global__ void __launch_bounds__(kThreads)
zero_rows_kernel(Rows R, float *__restrict__ x, int64_t ld)
{
    for_each_element(R, [&](int64_t s, int c) { x[s * ld + c] = 0.0f; });
}

dol_status launch_zero_rows(int32_t batch, int32_t n, float *x, int64_t ld, hipStream_t st)
{
    if (batch == 0 || n == 0) return DOL_OK;
    const Rows R = rows_of(batch, n);
    hipLaunchKernelGGL(zero_rows_kernel, dim3(R.grid), dim3(kThreads), 0, st, R, x, ld);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// out[s, c] = in[s, src_col[c]], or 0 where src_col[c] < 0: Filter forward (src_col = kept positions) and its
// transpose (src_col = position in the filtered row or -1).
__global__ void __launch_bounds__(kThreads)
damp_gather_cols_kernel(Rows R, const int32_t *__restrict__ src_col, const float *__restrict__ in, int64_t ldi,
                        float *__restrict__ out, int64_t ldo, int32_t accumulate)
{
    for_each_element(R, [&](int64_t s, int c) {
        const int32_t i = src_col[c];
        const float v = i >= 0 ? in[s * ldi + i] : 0.0f;
        out[s * ldo + c] = accumulate ? out[s * ldo + c] + v : v;
    });
}

dol_status launch_damp_filter_fwd(const FilterPlan *p, int32_t batch, const float *in, int64_t ldi, float *out,
                                  int64_t ldo, hipStream_t st)
{
    if (batch == 0 || p->n_out == 0) return DOL_OK;
    bool done = false;
    if (dol_status s2 = launch_rows_gather(batch, p->n_in, p->n_out, p->d_keep_idx.ptr, in, ldi, out, ldo, 0, st, &done)) return s2;
    if (done) return DOL_OK;
    const Rows R = rows_of(batch, p->n_out);
    hipLaunchKernelGGL(damp_gather_cols_kernel, dim3(R.grid), dim3(kThreads), 0, st, R, p->d_keep_idx.ptr, in, ldi, out,
                       ldo, 0);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

dol_status launch_damp_filter_bwd(const FilterPlan *p, int32_t batch, const float *g, int64_t ldg, float *gin,
                                  int64_t ldgi, int32_t accumulate, hipStream_t st)
{
    if (batch == 0 || p->n_in == 0) return DOL_OK;
    bool done = false;
    if (p->n_out > 0)
        if (dol_status s2 = launch_rows_gather(batch, p->n_out, p->n_in, p->d_pos.ptr, g, ldg, gin, ldgi, accumulate & 1, st, &done)) return s2;
    if (done) return DOL_OK;
    const Rows R = rows_of(batch, p->n_in);
    hipLaunchKernelGGL(damp_gather_cols_kernel, dim3(R.grid), dim3(kThreads), 0, st, R, p->d_pos.ptr, g, ldg, gin, ldgi,
                       accumulate & 1);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// ---------------------------------------------------------------- union

__global__ void __launch_bounds__(kThreads)
damp_union_fwd_kernel(Rows R, const int32_t *__restrict__ ia, const int32_t *__restrict__ ib,
                      const float *__restrict__ a, int64_t lda, const float *__restrict__ b, int64_t ldb,
                      float *__restrict__ out, int64_t ldo)
{
    for_each_element(R, [&](int64_t s, int c) {
        const int32_t i = ia[c], j = ib[c];
        float v;
        if (i >= 0 && j >= 0) v = fminf(a[s * lda + i] + b[s * ldb + j], 1.0f);
        else if (i >= 0) v = a[s * lda + i];
        else v = b[s * ldb + j];
        out[s * ldo + c] = v;
    });
}

dol_status launch_damp_union_fwd(const UnionPlan *p, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, float *out, int64_t ldo, hipStream_t st)
{
    if (batch == 0 || p->n_out == 0) return DOL_OK;
    bool done = false;
    if (dol_status s2 = launch_rows_union_fwd(p, batch, a, lda, b, ldb, out, ldo, st, &done)) return s2;
    if (done) return DOL_OK;
    const Rows R = rows_of(batch, p->n_out);
    hipLaunchKernelGGL(damp_union_fwd_kernel, dim3(R.grid), dim3(kThreads), 0, st, R, p->d_ia.ptr, p->d_ib.ptr, a, lda, b,
                       ldb, out, ldo);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// Element x of a sample is input position x of a (x < na) or x - na of b.
__global__ void __launch_bounds__(kThreads)
damp_union_bwd_kernel(Rows R, int32_t na, const int32_t *__restrict__ ia, const int32_t *__restrict__ ib,
                      const int32_t *__restrict__ ca, const int32_t *__restrict__ cb, const float *__restrict__ a,
                      int64_t lda, const float *__restrict__ b, int64_t ldb, const float *__restrict__ g, int64_t ldg,
                      float *__restrict__ ga, float *__restrict__ gb, int32_t accumulate)
{
    for_each_element(R, [&](int64_t s, int x) {
        const bool is_a = x < na;
        if (is_a ? !ga : !gb) return;
        const int32_t c = is_a ? ca[x] : cb[x - na];
        float gv = 0.0f;
        if (c >= 0) {                       // -1: a symbol the fused filter drops
            const int32_t i = ia[c], j = ib[c];
            gv = g[s * ldg + c];
            if (i >= 0 && j >= 0 && !(a[s * lda + i] + b[s * ldb + j] <= 1.0f)) gv = 0.0f;
        }
        if (is_a) ga[s * lda + x] = (accumulate & 1) ? ga[s * lda + x] + gv : gv;
        else gb[s * ldb + (x - na)] = (accumulate & 2) ? gb[s * ldb + (x - na)] + gv : gv;
    });
}

dol_status launch_damp_union_bwd(const UnionPlan *p, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                                 hipStream_t st)
{
    if (batch == 0 || p->na + p->nb == 0 || (!ga && !gb)) return DOL_OK;
    bool done = false;
    if (dol_status s2 = launch_rows_union_bwd(p, batch, a, lda, b, ldb, g, ldg, ga, gb, accumulate, st, &done)) return s2;
    if (done) return DOL_OK;
    const Rows R = rows_of(batch, p->na + p->nb);
    hipLaunchKernelGGL(damp_union_bwd_kernel, dim3(R.grid), dim3(kThreads), 0, st, R, p->na, p->d_ia.ptr, p->d_ib.ptr,
                       p->d_ca.ptr, p->d_cb.ptr, a, lda, b, ldb, g, ldg, ga, gb, accumulate);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// ---------------------------------------------------------------- harness helper: gradient of -log p[target]

__global__ void __launch_bounds__(kThreads)
nll_grad_kernel(Rows R, const float *__restrict__ p, int64_t ld, const int32_t *__restrict__ target,
                float *__restrict__ grad)
{
    for_each_element(R, [&](int64_t s, int c) {
        grad[s * ld + c] = c == target[s] ? -1.0f / fmaxf(p[s * ld + c], 1.17549435e-38f) : 0.0f;
    });
}

// The same over a contiguous [batch, n] gradient, 16 bytes per store: a workgroup owns `rows` whole rows (a multiple of
// four, so its piece starts on a 16-byte boundary; at most kNllRows), first puts every row's target and value in LDS
// and then walks its piece without a division and without a load between the stores (a load's wait would also wait for
// the stores before it).
constexpr int kNllRows = 2048;

__global__ void __launch_bounds__(kThreads)
nll_grad_flat_kernel(int32_t batch, int32_t n, int32_t rows, const float *__restrict__ p, const int32_t *__restrict__ target,
                     float *__restrict__ grad)
{
    __shared__ int32_t tg[kNllRows];
    __shared__ float val[kNllRows];
    const int64_t s0 = static_cast<int64_t>(blockIdx.x) * rows;
    const int32_t rows_here = static_cast<int32_t>(min(static_cast<int64_t>(rows), batch - s0));
    const int32_t n_here = rows_here * n;           // floats of this piece
    const float *pp = p + s0 * n;
    float *gg = grad + s0 * n;
    for (int r = threadIdx.x; r < rows_here; r += kThreads) {
        const int32_t t = target[s0 + r];
        tg[r] = t;
        val[r] = t >= 0 && t < n ? -1.0f / fmaxf(pp[static_cast<int64_t>(r) * n + t], 1.17549435e-38f) : 0.0f;
    }
    __syncthreads();
    constexpr int kStep = 4 * kThreads;
    const int32_t dr = kStep / n, dc = kStep - dr * n;
    int32_t e = 4 * static_cast<int32_t>(threadIdx.x);
    int32_t r = e / n, c = e - r * n;
    for (; e < n_here; e += kStep) {
        int32_t rr = r, cc = c;
        float v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            while (cc >= n) { cc -= n; ++rr; }      // (once at most per element, n >= 1)
            v[k] = e + k < n_here && cc == tg[rr] ? val[rr] : 0.0f;
            ++cc;
        }
        if (e + 3 < n_here) *reinterpret_cast<float4 *>(gg + e) = make_float4(v[0], v[1], v[2], v[3]);
        else
            for (int k = 0; e + k < n_here; ++k) gg[e + k] = v[k];
        r += dr; c += dc;
        if (c >= n) { c -= n; ++r; }
    }
}

dol_status launch_nll_grad(int32_t batch, int32_t n, const float *p, int64_t ld, const int32_t *target, float *grad,
                           hipStream_t st)
{
    if (batch == 0 || n == 0) return DOL_OK;
    if (ld == n && reinterpret_cast<uintptr_t>(grad) % 16 == 0) {
        const int32_t rows = std::min(kNllRows, std::max(4, (8192 / n + 3) / 4 * 4));
        if (static_cast<int64_t>(rows) * n < (int64_t{1} << 30)) {
            const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(batch) + rows - 1) / rows);
            hipLaunchKernelGGL(nll_grad_flat_kernel, dim3(grid), dim3(kThreads), 0, st, batch, n, rows, p, target, grad);
            DOL_HIP(hipGetLastError());
            return DOL_OK;
        }
    }
    const Rows R = rows_of(batch, n);
    hipLaunchKernelGGL(nll_grad_kernel, dim3(R.grid), dim3(kThreads), 0, st, R, p, ld, target, grad);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

}  // namespace dol
