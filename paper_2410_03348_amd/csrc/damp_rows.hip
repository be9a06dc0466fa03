// DAMP Filter and Union (Sec. 3.1.2) and their vector-Jacobian products for contiguous tensors: every global
// access is a coalesced 16-byte one.
//
// A workgroup takes tiles of whole rows (a multiple of four, so that a tile of any row length starts on a
// 16-byte boundary), copies the input tiles flat into LDS, and then walks the flat output tile four elements per
// lane: the column maps (kept positions, merge positions) and the irregular reads they cause are served by LDS,
// the results leave as 16-byte stores.  Column maps are staged once per workgroup; workgroups loop over tiles.
// Tensors with padded rows or unaligned bases take the element-wise kernels of damp.hip.
#include "internal.h"
#include "wave_util.h"

namespace dol {

constexpr int kRowsWG = 256;
constexpr int kRowsTileFloats = 2048;          // floats of the widest tensor in one tile
constexpr size_t kRowsLdsMax = 64 * 1024;

// Copies `total` floats (src 16-byte aligned) into LDS: 16-byte pieces, four in flight per lane, then the tail.
__device__ __forceinline__ void stage_flat(float *dst, const float *__restrict__ src, int total)
{
    const int n4 = total >> 2;
    const float4 *src4 = reinterpret_cast<const float4 *>(src);
    float4 *dst4 = reinterpret_cast<float4 *>(dst);
    for (int f0 = 0; f0 < n4; f0 += 4 * kRowsWG) {
        const int f = f0 + threadIdx.x;
        float4 v0, v1, v2, v3;
        if (f < n4) v0 = src4[f];
        if (f + kRowsWG < n4) v1 = src4[f + kRowsWG];
        if (f + 2 * kRowsWG < n4) v2 = src4[f + 2 * kRowsWG];
        if (f + 3 * kRowsWG < n4) v3 = src4[f + 3 * kRowsWG];
        if (f < n4) dst4[f] = v0;
        if (f + kRowsWG < n4) dst4[f + kRowsWG] = v1;
        if (f + 2 * kRowsWG < n4) dst4[f + 2 * kRowsWG] = v2;
        if (f + 3 * kRowsWG < n4) dst4[f + 3 * kRowsWG] = v3;
    }
    const int t = (n4 << 2) + threadIdx.x;
    if (t < total) dst[t] = src[t];
}

__device__ __forceinline__ void stage_ints(int32_t *dst, const int32_t *__restrict__ src, int n)
{
    for (int e = threadIdx.x; e < n; e += kRowsWG) dst[e] = src[e];
}

// out[0 .. rows * n) = f(row, column) (+ what is there), flat, four elements per lane and step.
template <typename F>
__device__ __forceinline__ void emit_flat(float *__restrict__ out, int rows, int n, float inv_n, bool add, F f)
{
    const int total = rows * n, n4 = total >> 2;
    float4 *out4 = reinterpret_cast<float4 *>(out);
    for (int q = threadIdx.x; q < n4; q += kRowsWG) {
        const int e = q << 2;
        int r = static_cast<int>(static_cast<float>(e) * inv_n);
        int c = e - r * n;
        if (c < 0) { c += n; --r; } else if (c >= n) { c -= n; ++r; }
        float4 v;
        v.x = f(r, c);
        if (++c == n) { c = 0; ++r; }
        v.y = f(r, c);
        if (++c == n) { c = 0; ++r; }
        v.z = f(r, c);
        if (++c == n) { c = 0; ++r; }
        v.w = f(r, c);
        if (add) {
            const float4 o = out4[q];
            v.x += o.x, v.y += o.y, v.z += o.z, v.w += o.w;
        }
        out4[q] = v;
    }
    const int t = (n4 << 2) + threadIdx.x;
    if (t < total) {
        const int r = t / n, c = t - r * n;
        const float v = f(r, c);
        out[t] = add ? out[t] + v : v;
    }
}

struct RowTiles {
    int32_t batch, rows_per_tile, n_tiles;
};

// ---------------------------------------------------------------- filter (both directions)

// out[s, c] = in[s, src_col[c]], or 0 where src_col[c] < 0
__global__ void __launch_bounds__(kRowsWG)
damp_rows_gather_kernel(RowTiles T, int32_t n_in, int32_t n_out, float inv_n_out, const int32_t *__restrict__ src_col,
                        const float *__restrict__ in, float *__restrict__ out, int32_t accumulate)
{
    extern __shared__ __align__(16) float lds[];
    float *tin = lds;
    int32_t *col = reinterpret_cast<int32_t *>(lds + ((T.rows_per_tile * n_in + 3) & ~3));
    stage_ints(col, src_col, n_out);
    for (int tile = blockIdx.x; tile < T.n_tiles; tile += gridDim.x) {
        const int64_t s0 = static_cast<int64_t>(tile) * T.rows_per_tile;
        const int rows = static_cast<int>(min(static_cast<int64_t>(T.rows_per_tile), T.batch - s0));
        lds_barrier();
        stage_flat(tin, in + s0 * n_in, rows * n_in);
        lds_barrier();
        emit_flat(out + s0 * n_out, rows, n_out, inv_n_out, accumulate != 0, [&](int r, int c) {
            const int32_t i = col[c];
            return i >= 0 ? tin[r * n_in + i] : 0.0f;
        });
    }
}

// ---------------------------------------------------------------- union

__global__ void __launch_bounds__(kRowsWG)
damp_rows_union_fwd_kernel(RowTiles T, int32_t na, int32_t nb, int32_t n_out, float inv_n_out,
                           const int32_t *__restrict__ g_ia, const int32_t *__restrict__ g_ib,
                           const float *__restrict__ a, const float *__restrict__ b, float *__restrict__ out)
{
    extern __shared__ __align__(16) float lds[];
    float *ta = lds, *tb = ta + ((T.rows_per_tile * na + 3) & ~3);
    int32_t *ia = reinterpret_cast<int32_t *>(tb + ((T.rows_per_tile * nb + 3) & ~3)), *ib = ia + n_out;
    stage_ints(ia, g_ia, n_out);
    stage_ints(ib, g_ib, n_out);
    for (int tile = blockIdx.x; tile < T.n_tiles; tile += gridDim.x) {
        const int64_t s0 = static_cast<int64_t>(tile) * T.rows_per_tile;
        const int rows = static_cast<int>(min(static_cast<int64_t>(T.rows_per_tile), T.batch - s0));
        lds_barrier();
        stage_flat(ta, a + s0 * na, rows * na);
        stage_flat(tb, b + s0 * nb, rows * nb);
        lds_barrier();
        emit_flat(out + s0 * n_out, rows, n_out, inv_n_out, false, [&](int r, int c) {
            const int32_t i = ia[c], j = ib[c];
            if (i >= 0 && j >= 0) return fminf(ta[r * na + i] + tb[r * nb + j], 1.0f);
            return i >= 0 ? ta[r * na + i] : tb[r * nb + j];
        });
    }
}

__global__ void __launch_bounds__(kRowsWG)
damp_rows_union_bwd_kernel(RowTiles T, int32_t na, int32_t nb, int32_t n_out, float inv_na, float inv_nb,
                           const int32_t *__restrict__ g_ia, const int32_t *__restrict__ g_ib,
                           const int32_t *__restrict__ g_ca, const int32_t *__restrict__ g_cb,
                           const float *__restrict__ a, const float *__restrict__ b, const float *__restrict__ g,
                           float *__restrict__ ga, float *__restrict__ gb, int32_t accumulate)
{
    extern __shared__ __align__(16) float lds[];
    float *ta = lds, *tb = ta + ((T.rows_per_tile * na + 3) & ~3), *tg = tb + ((T.rows_per_tile * nb + 3) & ~3);
    int32_t *ia = reinterpret_cast<int32_t *>(tg + ((T.rows_per_tile * n_out + 3) & ~3));
    int32_t *ib = ia + n_out, *ca = ib + n_out, *cb = ca + na;
    stage_ints(ia, g_ia, n_out);
    stage_ints(ib, g_ib, n_out);
    stage_ints(ca, g_ca, na);
    stage_ints(cb, g_cb, nb);
    for (int tile = blockIdx.x; tile < T.n_tiles; tile += gridDim.x) {
        const int64_t s0 = static_cast<int64_t>(tile) * T.rows_per_tile;
        const int rows = static_cast<int>(min(static_cast<int64_t>(T.rows_per_tile), T.batch - s0));
        lds_barrier();
        stage_flat(ta, a + s0 * na, rows * na);
        stage_flat(tb, b + s0 * nb, rows * nb);
        stage_flat(tg, g + s0 * n_out, rows * n_out);
        lds_barrier();
        // the gradient of column c passes unless both operands are present and their sum exceeds 1
        auto gated = [&](int r, int c) {
            const int32_t i = ia[c], j = ib[c];
            const float gv = tg[r * n_out + c];
            return i >= 0 && j >= 0 && !(ta[r * na + i] + tb[r * nb + j] <= 1.0f) ? 0.0f : gv;
        };
        if (ga) emit_flat(ga + s0 * na, rows, na, inv_na, (accumulate & 1) != 0, [&](int r, int x) {
            const int32_t c = ca[x];                // -1: a symbol the fused filter drops
            return c >= 0 ? gated(r, c) : 0.0f;
        });
        if (gb) emit_flat(gb + s0 * nb, rows, nb, inv_nb, (accumulate & 2) != 0, [&](int r, int x) { return gated(r, cb[x]); });
    }
}

// ---------------------------------------------------------------- launchers

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Cuts the batch into tiles of whole rows; false when one tile of four rows does not fit in LDS.
static bool make_tiles(int32_t batch, int32_t widest, size_t floats_per_row, size_t extra_bytes, RowTiles *T, size_t *lds,
                       unsigned *grid)
{
    int rows = (kRowsTileFloats / (widest > 0 ? widest : 1)) & ~3;
    if (rows < 4) rows = 4;
    // each staged tensor is padded to a multiple of four floats: at most 3 floats each, 16 covers them
    size_t bytes = sizeof(float) * (rows * floats_per_row + 16) + extra_bytes;
    while (bytes > kRowsLdsMax && rows > 4) {
        rows -= 4;
        bytes = sizeof(float) * (rows * floats_per_row + 16) + extra_bytes;
    }
    if (bytes > kRowsLdsMax) return false;
    T->batch = batch;
    T->rows_per_tile = rows;
    T->n_tiles = static_cast<int32_t>((static_cast<int64_t>(batch) + rows - 1) / rows);
    *lds = bytes;
    const int cap = 8192;                        // beyond this workgroups loop (the column maps are staged once each)
    *grid = static_cast<unsigned>(T->n_tiles < cap ? T->n_tiles : cap);
    return true;
}

// Each launcher sets *done when it took the call; otherwise the caller uses the element-wise kernels.
dol_status launch_rows_gather(int32_t batch, int32_t n_in, int32_t n_out, const int32_t *src_col, const float *in,
                              int64_t ldi, float *out, int64_t ldo, int32_t accumulate, hipStream_t st, bool *done)
{
    *done = false;
    RowTiles T;
    size_t lds;
    unsigned grid;
    if (ldi != n_in || ldo != n_out || !aligned16(in) || !aligned16(out) || n_in == 0 || n_out == 0 ||
        !make_tiles(batch, n_in > n_out ? n_in : n_out, n_in, sizeof(int32_t) * n_out, &T, &lds, &grid))
        return DOL_OK;
    hipLaunchKernelGGL(damp_rows_gather_kernel, dim3(grid), dim3(kRowsWG), lds, st, T, n_in, n_out,
                       1.0f / static_cast<float>(n_out), src_col, in, out, accumulate);
    DOL_HIP(hipGetLastError());
    *done = true;
    return DOL_OK;
}

dol_status launch_rows_union_fwd(const UnionPlan *p, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, float *out, int64_t ldo, hipStream_t st, bool *done)
{
    *done = false;
    RowTiles T;
    size_t lds;
    unsigned grid;
    if (lda != p->na || ldb != p->nb || ldo != p->n_out || !aligned16(a) || !aligned16(b) || !aligned16(out) ||
        !make_tiles(batch, p->n_out, static_cast<size_t>(p->na) + p->nb, sizeof(int32_t) * 2 * p->n_out, &T, &lds, &grid))
        return DOL_OK;
    hipLaunchKernelGGL(damp_rows_union_fwd_kernel, dim3(grid), dim3(kRowsWG), lds, st, T, p->na, p->nb, p->n_out,
                       1.0f / static_cast<float>(p->n_out), p->d_ia.ptr, p->d_ib.ptr, a, b, out);
    DOL_HIP(hipGetLastError());
    *done = true;
    return DOL_OK;
}

dol_status launch_rows_union_bwd(const UnionPlan *p, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                                 hipStream_t st, bool *done)
{
    *done = false;
    RowTiles T;
    size_t lds;
    unsigned grid;
    if (lda != p->na || ldb != p->nb || ldg != p->n_out || p->na == 0 || p->nb == 0 || !aligned16(a) || !aligned16(b) ||
        !aligned16(g) || !aligned16(ga) || !aligned16(gb) ||
        !make_tiles(batch, p->n_out, static_cast<size_t>(p->na) + p->nb + p->n_out,
                    sizeof(int32_t) * (2 * p->n_out + p->na + p->nb), &T, &lds, &grid))
        return DOL_OK;
    hipLaunchKernelGGL(damp_rows_union_bwd_kernel, dim3(grid), dim3(kRowsWG), lds, st, T, p->na, p->nb, p->n_out,
                       1.0f / static_cast<float>(p->na), 1.0f / static_cast<float>(p->nb), p->d_ia.ptr, p->d_ib.ptr,
                       p->d_ca.ptr, p->d_cb.ptr, a, b, g, ga, gb, accumulate);
    DOL_HIP(hipGetLastError());
    *done = true;
    return DOL_OK;
}

}  // namespace dol
