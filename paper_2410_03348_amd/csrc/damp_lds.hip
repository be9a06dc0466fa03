// DAMP apply2 for arbitrary (hashed, dense) function tables whose operand rows fit in LDS.
//
//     out[s, c] = min(1, sum over the tuples (i, j) of column c, ascending (i, j), of a[s, i] * b[s, j])
//     ga[s, i]  = sum_j gh[s, col(i, j)] * b[s, j],    gb[s, j] = sum_i gh[s, col(i, j)] * a[s, i]
//
// A workgroup (256 threads forward, 512 backward) owns a tile of 64 samples.  The operand rows are staged TRANSPOSED in LDS
// (one 256-byte row of 64 samples per symbol), so that a lane can pull four samples of one symbol with a
// single 16-byte read; 16 lanes cover the 64 samples, and the 16 groups of 16 lanes of the workgroup each
// own a share of the output columns and walk their tuple lists.  Every tuple costs two 16-byte LDS reads and
// four fma per lane; the 16-byte chunks of a row are XOR-swizzled by the row number so that both the
// transposing writes and the reads are free of bank conflicts.  Tuple lists live in LDS too, as packets of
// four tuples (one 16-byte broadcast read), each tuple being the pre-swizzled addresses of its two rows;
// short lists are padded with a tuple that points at a row of zeros, whose product is an exact +0.
#include "internal.h"
#include "wave_util.h"

#include <algorithm>

namespace dol {

constexpr int kLdsFwdWG = 1024, kLdsBwdWG = 1024;   // threads per workgroup
constexpr int kLdsTile = 64;                     // samples per tile = floats per LDS row
constexpr size_t kLdsBytesMax = 160 * 1024;
constexpr int kLdsMaxSym = 128;                  // most symbols of one operand


// Row number -> 16-bit address word: row * 16 chunks, with the swizzle term in the low four bits.
// A lane that wants chunk q of the row reads 16 bytes at ((word ^ q) << 4).
static inline uint32_t row_word(uint32_t row) { return row * 16u | ((row >> 2) & 15u); }

static void make_packets(int32_t n_cols, const std::vector<uint32_t> &ptr, const std::vector<uint32_t> &words,
                         uint32_t dummy, std::vector<uint32_t> &pk, std::vector<uint32_t> &pk_ptr)
{
    pk_ptr.assign(static_cast<size_t>(n_cols) + 1, 0);
    pk.clear();
    for (int32_t c = 0; c < n_cols; ++c) {
        for (uint32_t q = ptr[c]; q < ptr[c + 1]; ++q) pk.push_back(words[q]);
        while (pk.size() % 4) pk.push_back(dummy);
        pk_ptr[c + 1] = static_cast<uint32_t>(pk.size() / 4);
    }
}

// Builds the packet lists of the three gather products.  Leaves tb->lds_ok false when the table does not
// qualify (operand sizes not multiples of four, rows or lists too large for LDS): the direct kernels serve it.
dol_status lds_plan_build(dol_fn_table *tb, const std::vector<uint32_t> &col_ptr, const std::vector<uint32_t> &col_ij,
                          const std::vector<uint32_t> &rowa_ptr, const std::vector<uint32_t> &rowa_jc,
                          const std::vector<uint32_t> &rowb_ptr, const std::vector<uint32_t> &rowb_ic)
{
    const int32_t na = tb->na, nb = tb->nb, S = tb->n_out;
    tb->lds_ok = false;
    if (na < 4 || nb < 4 || S < 4 || na % 4 || nb % 4 || S % 4) return DOL_OK;
    if (na > kLdsMaxSym || nb > kLdsMaxSym || S + na + nb + 1 > 4095) return DOL_OK;
    std::vector<uint32_t> w(col_ij.size()), pk, pk_ptr, pka, pka_ptr, pkb, pkb_ptr;
    // forward: rows [a: na][b: nb][zeros]
    for (size_t q = 0; q < col_ij.size(); ++q)
        w[q] = pack16(row_word(col_ij[q] & 0xffffu), row_word(na + (col_ij[q] >> 16)));
    make_packets(S, col_ptr, w, pack16(row_word(na + nb), row_word(na + nb)), pk, pk_ptr);
    // backward: rows [gh: S][a: na][b: nb][zeros]
    const uint32_t zero = row_word(S + na + nb);
    for (size_t q = 0; q < rowa_jc.size(); ++q)      // (j | column << 16): gh[column] * b[j]
        w[q] = pack16(row_word(rowa_jc[q] >> 16), row_word(S + na + (rowa_jc[q] & 0xffffu)));
    make_packets(na, rowa_ptr, w, pack16(zero, zero), pka, pka_ptr);
    for (size_t q = 0; q < rowb_ic.size(); ++q)      // (i | column << 16): gh[column] * a[i]
        w[q] = pack16(row_word(rowb_ic[q] >> 16), row_word(S + (rowb_ic[q] & 0xffffu)));
    make_packets(nb, rowb_ptr, w, pack16(zero, zero), pkb, pkb_ptr);

    tb->lds_fwd_bytes = sizeof(float) * kLdsTile * static_cast<size_t>(na + nb + 1) + sizeof(uint32_t) * (pk.size() + pk_ptr.size());
    tb->lds_bwd_bytes = sizeof(float) * kLdsTile * static_cast<size_t>(S + na + nb + 1) +
                        sizeof(uint32_t) * (pka.size() + pka_ptr.size() + pkb.size() + pkb_ptr.size());
    if (tb->lds_fwd_bytes > kLdsBytesMax || tb->lds_bwd_bytes > kLdsBytesMax) return DOL_OK;
    hipError_t e;
    if ((e = tb->lds_pk.upload(pk)) != hipSuccess || (e = tb->lds_pk_ptr.upload(pk_ptr)) != hipSuccess ||
        (e = tb->lds_pka.upload(pka)) != hipSuccess || (e = tb->lds_pka_ptr.upload(pka_ptr)) != hipSuccess ||
        (e = tb->lds_pkb.upload(pkb)) != hipSuccess || (e = tb->lds_pkb_ptr.upload(pkb_ptr)) != hipSuccess)
        return hip_fail(e, "uploading the LDS packet lists");
    tb->lds_ok = true;
    return DOL_OK;
}

bool lds_path_ok(const dol_fn_table *f) { return f->lds_ok; }

// ---------------------------------------------------------------- device helpers

// Copies n words from global memory into LDS (all threads of the workgroup).
template <int WG>
__device__ __forceinline__ void copy_words(uint32_t *dst, const uint32_t *__restrict__ src, int n)
{
    for (int e = threadIdx.x; e < n; e += WG) dst[e] = src[e];
}

// Transposing store of four consecutive symbols (i .. i+3, i % 4 == 0) of sample s into rows row0 + i ..
__device__ __forceinline__ void store_transposed(float *rows, int row0, int i, int s, const float4 &v)
{
    const float e[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int row = row0 + i + k;
        rows[row * kLdsTile + ((((s >> 2) ^ (row >> 2)) & 15) << 2) + (s & 3)] = e[k];
    }
}

__device__ __forceinline__ float4 read_chunk(const float *rows, uint32_t word, uint32_t q)
{
    return *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(rows) + ((word ^ q) << 4));
}

// One float of the transposed rows (slow path of the clamp gate).
__device__ __forceinline__ float read_one(const float *rows, int row, int s)
{
    return rows[row * kLdsTile + ((((s >> 2) ^ (row >> 2)) & 15) << 2) + (s & 3)];
}

// acc += x * y for the four samples of this lane, over the packets [p0, p1) of one output column.
__device__ __forceinline__ float4 gather_dot(const float *rows, const uint4 *packets, uint32_t p0, uint32_t p1,
                                             uint32_t q)
{
    float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (uint32_t p = p0; p < p1; ++p) {
        const uint4 t = packets[p];
        const uint32_t tw[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const float4 x = read_chunk(rows, tw[k] & 0xffffu, q);
            const float4 y = read_chunk(rows, tw[k] >> 16, q);
            acc.x = __builtin_fmaf(x.x, y.x, acc.x);
            acc.y = __builtin_fmaf(x.y, y.y, acc.y);
            acc.z = __builtin_fmaf(x.z, y.z, acc.z);
            acc.w = __builtin_fmaf(x.w, y.w, acc.w);
        }
    }
    return acc;
}

// Stages the [kLdsTile x n] tile of a contiguous [batch, n] tensor (n % 4 == 0, n <= kLdsMaxSym) into rows
// row0 .. row0 + n - 1.  Every thread issues all of its loads before the first transposing store.
template <int WG>
__device__ __forceinline__ void stage_tile(float *rows, int row0, const float *__restrict__ src, int n)
{
    const int n4 = n >> 2, total = kLdsTile * n4;
    const float4 *src4 = reinterpret_cast<const float4 *>(src);
    constexpr int kQ = kLdsTile * (kLdsMaxSym / 4) / WG;
    float4 v[kQ];
#pragma unroll
    for (int x = 0; x < kQ; ++x) {
        const int f = threadIdx.x + WG * x;
        if (f < total) v[x] = src4[f];
    }
#pragma unroll
    for (int x = 0; x < kQ; ++x) {
        const int f = threadIdx.x + WG * x;
        if (f < total) {
            const int s = f / n4;
            store_transposed(rows, row0, (f - s * n4) << 2, s, v[x]);
        }
    }
}

// ---------------------------------------------------------------- forward

__global__ void __launch_bounds__(kLdsFwdWG)
damp_lds_fwd_kernel(int32_t n_tiles, int32_t na, int32_t nb, int32_t S, int32_t n_pk, const uint32_t *__restrict__ g_pk,
                    const uint32_t *__restrict__ g_pk_ptr, const float *__restrict__ a, const float *__restrict__ b,
                    float *__restrict__ out)
{
    extern __shared__ __align__(16) float lds[];     // rows [a][b][zeros], packets, packet pointers
    float *rows = lds;
    uint32_t *pk = reinterpret_cast<uint32_t *>(rows + kLdsTile * (na + nb + 1));
    uint32_t *pk_ptr = pk + 4 * n_pk;
    copy_words<kLdsFwdWG>(pk, g_pk, 4 * n_pk);
    copy_words<kLdsFwdWG>(pk_ptr, g_pk_ptr, S + 1);
    for (int e = threadIdx.x; e < kLdsTile; e += kLdsFwdWG) rows[(na + nb) * kLdsTile + e] = 0.0f;
    const uint32_t q = threadIdx.x & 15u;
    const int group = threadIdx.x >> 4;
    const int n_blocks = S >> 2;
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t s0 = static_cast<int64_t>(tile) * kLdsTile;
        __syncthreads();                             // the previous tile's readers are done (and the lists are in)
        stage_tile<kLdsFwdWG>(rows, 0, a + s0 * na, na);
        stage_tile<kLdsFwdWG>(rows, na, b + s0 * nb, nb);
        __syncthreads();
        for (int blk = group; blk < n_blocks; blk += (kLdsFwdWG / 16)) {
            float4 o[4];
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const int c = 4 * blk + cc;
                o[cc] = gather_dot(rows, reinterpret_cast<const uint4 *>(pk), pk_ptr[c], pk_ptr[c + 1], q);
            }
            // lane holds [4 samples][4 columns]: one 16-byte store per sample
            float *dst = out + (s0 + 4 * q) * S + 4 * blk;
            *reinterpret_cast<float4 *>(dst) = make_float4(fminf(o[0].x, 1.0f), fminf(o[1].x, 1.0f), fminf(o[2].x, 1.0f), fminf(o[3].x, 1.0f));
            *reinterpret_cast<float4 *>(dst + S) = make_float4(fminf(o[0].y, 1.0f), fminf(o[1].y, 1.0f), fminf(o[2].y, 1.0f), fminf(o[3].y, 1.0f));
            *reinterpret_cast<float4 *>(dst + 2 * S) = make_float4(fminf(o[0].z, 1.0f), fminf(o[1].z, 1.0f), fminf(o[2].z, 1.0f), fminf(o[3].z, 1.0f));
            *reinterpret_cast<float4 *>(dst + 3 * S) = make_float4(fminf(o[0].w, 1.0f), fminf(o[1].w, 1.0f), fminf(o[2].w, 1.0f), fminf(o[3].w, 1.0f));
        }
    }
}

// ---------------------------------------------------------------- backward

// Stages gh = g gated by the clamp: out < 1 means the clamp did not act.  Elements with out == 1 are decided
// afterwards from pre (see the kernel); their positions are counted in *n_flag.
template <int WG>
__device__ __forceinline__ void stage_gated(float *rows, const float *__restrict__ g, const float *__restrict__ out,
                                            int S, int *n_flag)
{
    const int n4 = S >> 2, total = kLdsTile * n4;
    const float4 *g4 = reinterpret_cast<const float4 *>(g), *o4 = reinterpret_cast<const float4 *>(out);
    int flagged = 0;
    for (int f0 = 0; f0 < total; f0 += WG * 4) {     // four pieces of g and of out in flight per thread
        float4 vg[4], vo[4];
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int f = f0 + threadIdx.x + WG * x;
            if (f < total) { vg[x] = g4[f]; vo[x] = o4[f]; }
        }
#pragma unroll
        for (int x = 0; x < 4; ++x) {
            const int f = f0 + threadIdx.x + WG * x;
            if (f < total) {
                const int s = f / n4;
                flagged |= !(vo[x].x < 1.0f) | !(vo[x].y < 1.0f) | !(vo[x].z < 1.0f) | !(vo[x].w < 1.0f);
                store_transposed(rows, 0, (f - s * n4) << 2, s, vg[x]);
            }
        }
    }
    if (flagged) atomicOr(n_flag, 1);
}

__global__ void __launch_bounds__(kLdsBwdWG)
damp_lds_bwd_kernel(int32_t n_tiles, int32_t na, int32_t nb, int32_t S, int32_t n_pka, int32_t n_pkb,
                    const uint32_t *__restrict__ g_pka, const uint32_t *__restrict__ g_pka_ptr,
                    const uint32_t *__restrict__ g_pkb, const uint32_t *__restrict__ g_pkb_ptr,
                    const uint32_t *__restrict__ col_ptr, const uint32_t *__restrict__ col_ij,
                    const float *__restrict__ a, const float *__restrict__ b, const float *__restrict__ out,
                    const float *__restrict__ g, float *__restrict__ ga, float *__restrict__ gb, int32_t accumulate)
{
    extern __shared__ __align__(16) float lds[];     // rows [gh: S][a: na][b: nb][zeros], lists, flag
    float *rows = lds;
    const int n_rows = S + na + nb + 1;
    uint32_t *pka = reinterpret_cast<uint32_t *>(rows + kLdsTile * n_rows);
    uint32_t *pkb = pka + 4 * n_pka;
    uint32_t *pka_ptr = pkb + 4 * n_pkb;
    uint32_t *pkb_ptr = pka_ptr + na + 1;
    int *flag = reinterpret_cast<int *>(pkb_ptr + nb + 1);
    copy_words<kLdsBwdWG>(pka, g_pka, 4 * n_pka);
    copy_words<kLdsBwdWG>(pka_ptr, g_pka_ptr, na + 1);
    copy_words<kLdsBwdWG>(pkb, g_pkb, 4 * n_pkb);
    copy_words<kLdsBwdWG>(pkb_ptr, g_pkb_ptr, nb + 1);
    for (int e = threadIdx.x; e < kLdsTile; e += kLdsBwdWG) rows[(n_rows - 1) * kLdsTile + e] = 0.0f;
    const uint32_t q = threadIdx.x & 15u;
    const int group = threadIdx.x >> 4;
    const int blocks_a = na >> 2, n_blocks = (na + nb) >> 2;
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t s0 = static_cast<int64_t>(tile) * kLdsTile;
        __syncthreads();
        if (threadIdx.x == 0) *flag = 0;
        __syncthreads();
        stage_gated<kLdsBwdWG>(rows, g + s0 * S, out + s0 * S, S, flag);
        stage_tile<kLdsBwdWG>(rows, S, a + s0 * na, na);
        stage_tile<kLdsBwdWG>(rows, S + na, b + s0 * nb, nb);
        __syncthreads();
        if (*flag) {                                 // rare: some output of this tile sits on the clamp
            for (int e = threadIdx.x; e < kLdsTile * S; e += kLdsBwdWG) {
                const int s = e / S, c = e - s * S;
                if (!(out[(s0 + s) * S + c] < 1.0f)) {
                    float pre = 0.0f;
                    for (uint32_t t = col_ptr[c], t1 = col_ptr[c + 1]; t < t1; ++t) {
                        const uint32_t ij = col_ij[t];
                        pre = __builtin_fmaf(read_one(rows, S + (ij & 0xffffu), s), read_one(rows, S + na + (ij >> 16), s), pre);
                    }
                    if (!(pre <= 1.0f)) rows[c * kLdsTile + ((((s >> 2) ^ (c >> 2)) & 15) << 2) + (s & 3)] = 0.0f;
                }
            }
            __syncthreads();
        }
        for (int blk = group; blk < n_blocks; blk += (kLdsBwdWG / 16)) {
            const bool is_a = blk < blocks_a;
            const int col0 = is_a ? 4 * blk : 4 * (blk - blocks_a);
            const uint4 *packets = reinterpret_cast<const uint4 *>(is_a ? pka : pkb);
            const uint32_t *ptr = is_a ? pka_ptr : pkb_ptr;
            float *base = is_a ? ga : gb;
            if (!base) continue;
            float4 o[4];
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) o[cc] = gather_dot(rows, packets, ptr[col0 + cc], ptr[col0 + cc + 1], q);
            const int n = is_a ? na : nb;
            const bool add = is_a ? (accumulate & 1) : (accumulate & 2);
            float *dst = base + (s0 + 4 * q) * n + col0;
            float4 r[4] = {make_float4(o[0].x, o[1].x, o[2].x, o[3].x), make_float4(o[0].y, o[1].y, o[2].y, o[3].y),
                           make_float4(o[0].z, o[1].z, o[2].z, o[3].z), make_float4(o[0].w, o[1].w, o[2].w, o[3].w)};
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float4 *p = reinterpret_cast<float4 *>(dst + k * n);
                if (add) { const float4 old = *p; r[k].x += old.x; r[k].y += old.y; r[k].z += old.z; r[k].w += old.w; }
                *p = r[k];
            }
        }
    }
}

// ---------------------------------------------------------------- launchers

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static unsigned lds_grid(int n_tiles, size_t lds_bytes)
{
    const int per_cu = static_cast<int>(kLdsBytesMax / lds_bytes) > 0 ? static_cast<int>(kLdsBytesMax / lds_bytes) : 1;
    const int cap = 256 * per_cu;
    return static_cast<unsigned>(n_tiles < cap ? n_tiles : cap);
}

// Number of samples the LDS forward kernel took (a multiple of the tile), 0 when the call does not qualify.
dol_status launch_damp_lds_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                               int64_t ldb, float *out, int64_t ldo, hipStream_t st, int32_t *done)
{
    *done = 0;
    const int n_tiles = batch / kLdsTile;
    if (!f->lds_ok || n_tiles == 0 || lda != f->na || ldb != f->nb || ldo != f->n_out || !aligned16(a) || !aligned16(b) ||
        !aligned16(out))
        return DOL_OK;
    static bool attr_set = false;
    if (!attr_set) {
        DOL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(damp_lds_fwd_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kLdsBytesMax)));
        attr_set = true;
    }
    const int32_t n_pk = static_cast<int32_t>(f->lds_pk.n / 4);
    hipLaunchKernelGGL(damp_lds_fwd_kernel, dim3(lds_grid(n_tiles, f->lds_fwd_bytes)), dim3(kLdsFwdWG), f->lds_fwd_bytes, st,
                       n_tiles, f->na, f->nb, f->n_out, n_pk, f->lds_pk.ptr, f->lds_pk_ptr.ptr, a, b, out);
    DOL_HIP(hipGetLastError());
    *done = n_tiles * kLdsTile;
    return DOL_OK;
}

dol_status launch_damp_lds_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                               int64_t ldb, const float *out, int64_t ldo, const float *g, int64_t ldg, float *ga,
                               float *gb, int32_t accumulate, hipStream_t st, int32_t *done)
{
    *done = 0;
    const int n_tiles = batch / kLdsTile;
    if (!f->lds_ok || n_tiles == 0 || lda != f->na || ldb != f->nb || ldo != f->n_out || ldg != f->n_out ||
        ga == gb || !aligned16(a) || !aligned16(b) || !aligned16(out) || !aligned16(g) || !aligned16(ga) || !aligned16(gb))
        return DOL_OK;
    static bool attr_set = false;
    if (!attr_set) {
        DOL_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(damp_lds_bwd_kernel),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(kLdsBytesMax)));
        attr_set = true;
    }
    const size_t lds = f->lds_bwd_bytes + 16;
    hipLaunchKernelGGL(damp_lds_bwd_kernel, dim3(lds_grid(n_tiles, lds)), dim3(kLdsBwdWG), lds, st, n_tiles, f->na, f->nb,
                       f->n_out, static_cast<int32_t>(f->lds_pka.n / 4), static_cast<int32_t>(f->lds_pkb.n / 4),
                       f->lds_pka.ptr, f->lds_pka_ptr.ptr, f->lds_pkb.ptr, f->lds_pkb_ptr.ptr, f->col_ptr.ptr,
                       f->col_ij.ptr, a, b, out, g, ga, gb, accumulate);
    DOL_HIP(hipGetLastError());
    *done = n_tiles * kLdsTile;
    return DOL_OK;
}

}  // namespace dol
