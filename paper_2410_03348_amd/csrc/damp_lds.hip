// DAMP apply2 for arbitrary (hashed, dense or sparse) function tables whose operand rows fit in LDS.
//
//     out[s, c] = min(1, sum over the tuples (i, j) of column c, ascending (i, j), of a[s, i] * b[s, j])
//     ga[s, i]  = sum_j gh[s, col(i, j)] * b[s, j],    gb[s, j] = sum_i gh[s, col(i, j)] * a[s, i]
//
// A workgroup owns a tile of 64 samples.  The operand rows are staged TRANSPOSED in LDS (one 256-byte row of
// 64 samples per symbol), so that a lane can pull four samples of one symbol with a single 16-byte read; 16
// lanes cover the 64 samples, and the groups of 16 lanes of the workgroup each own a share of the output columns
// and walk their tuple lists.  Every tuple costs two 16-byte LDS reads and four fma per lane; the 16-byte chunks
// of a row are XOR-swizzled by the row number so that the reads are free of bank conflicts.  Tuple lists live in
// LDS too, as packets of four tuples (one 16-byte broadcast read), each tuple being the pre-swizzled addresses of
// its two rows; short lists are padded with a tuple that points at a row of zeros, whose product is an exact +0.
//
// Any shape is taken: symbol counts need not be multiples of four, rows may be padded (ld > n_sym), the batch
// need not be a multiple of the tile.  Contiguous 16-byte aligned tensors are staged with 16-byte loads and
// written with 16-byte stores; others element by element.
#include "internal.h"
#include "wave_util.h"

#include <algorithm>

namespace dol {

constexpr int kLdsFwdWG = 1024, kLdsBwdWG = 1024;   // threads per workgroup
constexpr int kLdsTile = 64;                     // samples per tile = floats per LDS row
constexpr size_t kLdsBytesMax = 160 * 1024;

// Row number -> 16-bit address word: row * 16 chunks, with the swizzle term in the low four bits.
// A lane that wants chunk q of the row reads 16 bytes at ((word ^ q) << 4).
static inline uint32_t row_word(uint32_t row) { return row * 16u | ((row >> 2) & 15u); }

// Packet lists of n_cols columns, padded with empty columns to a multiple of four.
static void make_packets(int32_t n_cols, const std::vector<uint32_t> &ptr, const std::vector<uint32_t> &words,
                         uint32_t dummy, std::vector<uint32_t> &pk, std::vector<uint32_t> &pk_ptr)
{
    const int32_t padded = (n_cols + 3) & ~3;
    pk_ptr.assign(static_cast<size_t>(padded) + 1, 0);
    pk.clear();
    for (int32_t c = 0; c < padded; ++c) {
        if (c < n_cols) {
            for (uint32_t q = ptr[c]; q < ptr[c + 1]; ++q) pk.push_back(words[q]);
            while (pk.size() % 4) pk.push_back(dummy);
        }
        pk_ptr[c + 1] = static_cast<uint32_t>(pk.size() / 4);
    }
}

// Builds the packet lists of the three gather products.  Leaves tb->lds_fwd_ok / lds_bwd_ok false when the rows
// and lists are too large for LDS: the direct kernels serve those.
dol_status lds_plan_build(dol_fn_table *tb, const std::vector<uint32_t> &col_ptr, const std::vector<uint32_t> &col_ij,
                          const std::vector<uint32_t> &rowa_ptr, const std::vector<uint32_t> &rowa_jc,
                          const std::vector<uint32_t> &rowb_ptr, const std::vector<uint32_t> &rowb_ic)
{
    const int32_t na = tb->na, nb = tb->nb, S = tb->n_out;
    tb->lds_fwd_ok = tb->lds_bwd_ok = false;
    if (na < 1 || nb < 1 || S < 1 || col_ij.empty()) return DOL_OK;
    std::vector<uint32_t> w(col_ij.size()), pk, pk_ptr, pka, pka_ptr, pkb, pkb_ptr;
    hipError_t e;
    // forward: rows [a: na][b: nb][zeros]
    const size_t fwd_rows = sizeof(float) * kLdsTile * (static_cast<size_t>(na) + nb + 1);
    if (fwd_rows + sizeof(uint32_t) * (col_ij.size() + S + 8) <= kLdsBytesMax) {
        for (size_t q = 0; q < col_ij.size(); ++q)
            w[q] = pack16(row_word(col_ij[q] & 0xffffu), row_word(na + (col_ij[q] >> 16)));
        make_packets(S, col_ptr, w, pack16(row_word(na + nb), row_word(na + nb)), pk, pk_ptr);
        tb->lds_fwd_bytes = fwd_rows + sizeof(uint32_t) * (pk.size() + pk_ptr.size());
        if (tb->lds_fwd_bytes <= kLdsBytesMax) {
            if ((e = tb->lds_pk.upload(pk)) != hipSuccess || (e = tb->lds_pk_ptr.upload(pk_ptr)) != hipSuccess)
                return hip_fail(e, "uploading the LDS packet lists");
            tb->lds_fwd_ok = true;
        }
    }
    // backward: rows [gh: S][a: na][b: nb][zeros]
    const size_t bwd_rows = sizeof(float) * kLdsTile * (static_cast<size_t>(S) + na + nb + 1);
    if (bwd_rows + sizeof(uint32_t) * (2 * col_ij.size() + na + nb + 16) <= kLdsBytesMax) {
        const uint32_t zero = row_word(S + na + nb);
        for (size_t q = 0; q < rowa_jc.size(); ++q)      // (j | column << 16): gh[column] * b[j]
            w[q] = pack16(row_word(rowa_jc[q] >> 16), row_word(S + na + (rowa_jc[q] & 0xffffu)));
        make_packets(na, rowa_ptr, w, pack16(zero, zero), pka, pka_ptr);
        for (size_t q = 0; q < rowb_ic.size(); ++q)      // (i | column << 16): gh[column] * a[i]
            w[q] = pack16(row_word(rowb_ic[q] >> 16), row_word(S + (rowb_ic[q] & 0xffffu)));
        make_packets(nb, rowb_ptr, w, pack16(zero, zero), pkb, pkb_ptr);
        tb->lds_bwd_bytes = bwd_rows + sizeof(uint32_t) * (pka.size() + pka_ptr.size() + pkb.size() + pkb_ptr.size()) + 16;
        if (tb->lds_bwd_bytes <= kLdsBytesMax) {
            if ((e = tb->lds_pka.upload(pka)) != hipSuccess || (e = tb->lds_pka_ptr.upload(pka_ptr)) != hipSuccess ||
                (e = tb->lds_pkb.upload(pkb)) != hipSuccess || (e = tb->lds_pkb_ptr.upload(pkb_ptr)) != hipSuccess)
                return hip_fail(e, "uploading the LDS packet lists");
            tb->lds_bwd_ok = true;
        }
    }
    return DOL_OK;
}

// ---------------------------------------------------------------- device helpers

// A [batch, n] tensor with row stride ld; vec: rows are contiguous (ld == n) and the base is 16-byte aligned.
struct Rows2D {
    const float *p;
    int64_t ld;
    int32_t n;
    int32_t vec;
    float inv_n;
};

// Copies n words from global memory into LDS (all threads of the workgroup).
template <int WG>
__device__ __forceinline__ void copy_words(uint32_t *dst, const uint32_t *__restrict__ src, int n)
{
    for (int e = threadIdx.x; e < n; e += WG) dst[e] = src[e];
}

// Position of (row, sample) inside the transposed, swizzled rows.
__device__ __forceinline__ int slot_of(int row, int s)
{
    return row * kLdsTile + ((((s >> 2) ^ (row >> 2)) & 15) << 2) + (s & 3);
}

__device__ __forceinline__ float4 read_chunk(const float *rows, uint32_t word, uint32_t q)
{
    return *reinterpret_cast<const float4 *>(reinterpret_cast<const char *>(rows) + ((word ^ q) << 4));
}

// acc += x * y for the four samples of this lane, over the packets [p0, p1) of one output column.
__device__ __forceinline__ float4 gather_dot(const float *rows, const uint4 *packets, uint32_t p0, uint32_t p1,
                                             uint32_t q)
{
    float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (uint32_t p = p0; p < p1; ++p) {
        const uint4 t = packets[p];
        const uint32_t tw[4] = {t.x, t.y, t.z, t.w};
        float4 x[4], y[4];                  // all eight reads of the packet are requested before the first fma
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            x[k] = read_chunk(rows, tw[k] & 0xffffu, q);
            y[k] = read_chunk(rows, tw[k] >> 16, q);
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            acc.x = __builtin_fmaf(x[k].x, y[k].x, acc.x);
            acc.y = __builtin_fmaf(x[k].y, y[k].y, acc.y);
            acc.z = __builtin_fmaf(x[k].z, y[k].z, acc.z);
            acc.w = __builtin_fmaf(x[k].w, y[k].w, acc.w);
        }
    }
    return acc;
}

// Element e of a flat [valid x n] tile -> (sample, symbol); exact for the small integers involved.
__device__ __forceinline__ void split(int e, int n, float inv_n, int &s, int &i)
{
    s = static_cast<int>(static_cast<float>(e) * inv_n);
    i = e - s * n;
    const int d = (i >= n ? 1 : 0) - (i < 0 ? 1 : 0);   // the float quotient may be off by one: fix without a branch
    s += d;
    i -= d * n;
}

// 16-byte pieces of a tile (and of its companion tensor) on their way from memory to one lane.
template <bool AUX>
struct Chunk {
    static constexpr int kPieces = AUX ? 2 : 1;
    float4 v[kPieces], u[AUX ? kPieces : 1];
};

// Requests the pieces f0 + lane + WG * x of the flat tile (contiguous tensors only; indices clamped, no branch).
template <int WG, bool AUX, bool FAST>
__device__ __forceinline__ void stage_request(Chunk<AUX> &c, const Rows2D &T, const Rows2D &X, int64_t s0, int valid, int f0)
{
    const int n4 = (valid * T.n) >> 2;
    if (!(FAST || (T.vec && (!AUX || X.vec))) || n4 == 0) return;
    const float4 *src4 = reinterpret_cast<const float4 *>(T.p + s0 * T.n);
    const float4 *aux4 = reinterpret_cast<const float4 *>(X.p + s0 * T.n);
#pragma unroll
    for (int x = 0; x < Chunk<AUX>::kPieces; ++x) {
        const int q = min(f0 + static_cast<int>(threadIdx.x) + WG * x, n4 - 1);
        c.v[x] = src4[q];
        if (AUX) c.u[x] = aux4[q];
    }
}

// Stages samples s0 .. s0 + valid - 1 of T into rows row0 .. row0 + T.n - 1 as f(value, aux value, s, i); X is a
// second tensor of the same shape read in step with T (AUX), e.g. the forward result beside the upstream gradient.
// Contiguous tensors: the tile is one flat run of valid * n floats starting on a 16-byte boundary (64 samples per
// tile), read in 16-byte pieces; the caller has already requested the first chunk (stage_request with f0 = 0), so
// that the requests of all tensors of a tile are in flight together.
// FAST: the caller vouches for contiguous aligned tensors, n % 4 == 0 and a full tile; only that path is compiled.
template <int WG, bool AUX, bool FAST, typename F>
__device__ __forceinline__ void stage_tile(float *rows, int row0, const Rows2D &T, const Rows2D &X, int64_t s0, int valid,
                                           Chunk<AUX> &c, F f)
{
    const int n = T.n, total = valid * n;
    constexpr int kPieces = Chunk<AUX>::kPieces;
    if (FAST || (T.vec && (!AUX || X.vec))) {
        const int n4 = total >> 2;
        for (int f0 = 0; f0 < n4; f0 += kPieces * WG) {
            if (f0 > 0) stage_request<WG, AUX, FAST>(c, T, X, s0, valid, f0);
#pragma unroll
            for (int x = 0; x < kPieces; ++x) {
                const int q = f0 + threadIdx.x + WG * x;
                if (q < n4) {
                    int s, i;
                    split(q << 2, n, T.inv_n, s, i);
                    const float e[4] = {c.v[x].x, c.v[x].y, c.v[x].z, c.v[x].w};
                    const float a[4] = {AUX ? c.u[x].x : 0.0f, AUX ? c.u[x].y : 0.0f, AUX ? c.u[x].z : 0.0f, AUX ? c.u[x].w : 0.0f};
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        rows[slot_of(row0 + i, s)] = f(e[k], a[k], s, i);
                        ++i;
                        if (!FAST && i == n) { i = 0; ++s; }     // n % 4 != 0: the piece may span two samples
                    }
                }
            }
        }
        if (FAST) return;
        for (int e = (n4 << 2) + threadIdx.x; e < total; e += WG) {
            int s, i;
            split(e, n, T.inv_n, s, i);
            rows[slot_of(row0 + i, s)] = f(T.p[s0 * n + e], AUX ? X.p[s0 * n + e] : 0.0f, s, i);
        }
    } else {
        for (int e = threadIdx.x; e < total; e += WG) {
            int s, i;
            split(e, n, T.inv_n, s, i);
            rows[slot_of(row0 + i, s)] = f(T.p[(s0 + s) * T.ld + i], AUX ? X.p[(s0 + s) * X.ld + i] : 0.0f, s, i);
        }
    }
}

// Writes the lane's block: o[cc] holds columns col0 + cc of samples 4q .. 4q + 3 (in x, y, z, w).
template <bool CLAMP, bool FAST>
__device__ __forceinline__ void store_block(float *__restrict__ base, int64_t ld, int32_t n, int32_t vec, int64_t s0, int valid,
                                            uint32_t q, int col0, const float4 (&o)[4], bool add)
{
    float r[4][4] = {{o[0].x, o[1].x, o[2].x, o[3].x}, {o[0].y, o[1].y, o[2].y, o[3].y},
                     {o[0].z, o[1].z, o[2].z, o[3].z}, {o[0].w, o[1].w, o[2].w, o[3].w}};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int s = 4 * static_cast<int>(q) + k;
        if (!FAST && s >= valid) continue;
        float *dst = base + (s0 + s) * ld + col0;
        if (CLAMP) {
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) r[k][cc] = fminf(r[k][cc], 1.0f);
        }
        if (FAST || (vec && col0 + 3 < n)) {
            float4 v = make_float4(r[k][0], r[k][1], r[k][2], r[k][3]);
            if (add) { const float4 old = *reinterpret_cast<float4 *>(dst); v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w; }
            *reinterpret_cast<float4 *>(dst) = v;
        } else {
#pragma unroll
            for (int cc = 0; cc < 4; ++cc)
                if (col0 + cc < n) dst[cc] = add ? dst[cc] + r[k][cc] : r[k][cc];
        }
    }
}

// ---------------------------------------------------------------- forward

// (16 wavefronts per workgroup and one workgroup or two per CU: at most 4 wavefronts per SIMD can be resident, so
// the register allocator is told not to save registers for more, which would serialise the LDS reads of a packet)
template <bool FAST>
__global__ void __launch_bounds__(kLdsFwdWG) __attribute__((amdgpu_waves_per_eu(1, 4)))
damp_lds_fwd_kernel(int32_t batch, int32_t n_tiles, int32_t S, int32_t n_pk, const uint32_t *__restrict__ g_pk,
                    const uint32_t *__restrict__ g_pk_ptr, Rows2D A, Rows2D B, float *__restrict__ out, int64_t ldo,
                    int32_t vec_out)
{
    extern __shared__ __align__(16) float lds[];     // rows [a][b][zeros], packets, packet pointers
    const int na = A.n, nb = B.n, n_blocks = (S + 3) >> 2;
    float *rows = lds;
    uint32_t *pk = reinterpret_cast<uint32_t *>(rows + kLdsTile * (na + nb + 1));
    uint32_t *pk_ptr = pk + 4 * n_pk;
    copy_words<kLdsFwdWG>(pk, g_pk, 4 * n_pk);
    copy_words<kLdsFwdWG>(pk_ptr, g_pk_ptr, 4 * n_blocks + 1);
    for (int e = threadIdx.x; e < kLdsTile; e += kLdsFwdWG) rows[(na + nb) * kLdsTile + e] = 0.0f;
    const uint32_t q = threadIdx.x & 15u;
    const int group = threadIdx.x >> 4;
    auto plain = [](float v, float, int, int) { return v; };
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t s0 = static_cast<int64_t>(tile) * kLdsTile;
        const int valid = FAST ? kLdsTile : static_cast<int>(min(static_cast<int64_t>(kLdsTile), batch - s0));
        Chunk<false> ca, cb;
        stage_request<kLdsFwdWG, false, FAST>(ca, A, A, s0, valid, 0);
        stage_request<kLdsFwdWG, false, FAST>(cb, B, B, s0, valid, 0);
        lds_barrier();                             // the previous tile's readers are done (and the lists are in)
        stage_tile<kLdsFwdWG, false, FAST>(rows, 0, A, A, s0, valid, ca, plain);
        stage_tile<kLdsFwdWG, false, FAST>(rows, na, B, B, s0, valid, cb, plain);
        lds_barrier();
        for (int blk = group; blk < n_blocks; blk += kLdsFwdWG / 16) {
            float4 o[4];
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) {
                const int c = 4 * blk + cc;
                o[cc] = gather_dot(rows, reinterpret_cast<const uint4 *>(pk), pk_ptr[c], pk_ptr[c + 1], q);
            }
            store_block<true, FAST>(out, ldo, S, vec_out, s0, valid, q, 4 * blk, o, false);
        }
    }
}

// ---------------------------------------------------------------- backward

template <bool FAST>
__global__ void __launch_bounds__(kLdsBwdWG) __attribute__((amdgpu_waves_per_eu(1, 4)))
damp_lds_bwd_kernel(int32_t batch, int32_t n_tiles, int32_t n_pka, int32_t n_pkb,
                    const uint32_t *__restrict__ g_pka, const uint32_t *__restrict__ g_pka_ptr,
                    const uint32_t *__restrict__ g_pkb, const uint32_t *__restrict__ g_pkb_ptr,
                    const uint32_t *__restrict__ col_ptr, const uint32_t *__restrict__ col_ij, Rows2D A, Rows2D B,
                    Rows2D G, Rows2D O, float *__restrict__ ga, float *__restrict__ gb,
                    int32_t vec_ga, int32_t vec_gb, int32_t accumulate)
{
    extern __shared__ __align__(16) float lds[];     // rows [gh: S][a: na][b: nb][zeros], lists, flag
    const int na = A.n, nb = B.n, S = G.n;
    const int blocks_a = (na + 3) >> 2, blocks_b = (nb + 3) >> 2;
    float *rows = lds;
    const int n_rows = S + na + nb + 1;
    uint32_t *pka = reinterpret_cast<uint32_t *>(rows + kLdsTile * n_rows);
    uint32_t *pkb = pka + 4 * n_pka;
    uint32_t *pka_ptr = pkb + 4 * n_pkb;
    uint32_t *pkb_ptr = pka_ptr + 4 * blocks_a + 1;
    int *flag = reinterpret_cast<int *>(pkb_ptr + 4 * blocks_b + 1);
    copy_words<kLdsBwdWG>(pka, g_pka, 4 * n_pka);
    copy_words<kLdsBwdWG>(pka_ptr, g_pka_ptr, 4 * blocks_a + 1);
    copy_words<kLdsBwdWG>(pkb, g_pkb, 4 * n_pkb);
    copy_words<kLdsBwdWG>(pkb_ptr, g_pkb_ptr, 4 * blocks_b + 1);
    for (int e = threadIdx.x; e < kLdsTile; e += kLdsBwdWG) rows[(n_rows - 1) * kLdsTile + e] = 0.0f;
    const uint32_t q = threadIdx.x & 15u;
    const int group = threadIdx.x >> 4;
    auto plain = [](float v, float, int, int) { return v; };
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t s0 = static_cast<int64_t>(tile) * kLdsTile;
        const int valid = FAST ? kLdsTile : static_cast<int>(min(static_cast<int64_t>(kLdsTile), batch - s0));
        Chunk<true> cg;
        Chunk<false> ca, cb;
        stage_request<kLdsBwdWG, true, FAST>(cg, G, O, s0, valid, 0);
        stage_request<kLdsBwdWG, false, FAST>(ca, A, A, s0, valid, 0);
        stage_request<kLdsBwdWG, false, FAST>(cb, B, B, s0, valid, 0);
        lds_barrier();
        if (threadIdx.x == 0) *flag = 0;
        lds_barrier();
        // gh = g gated by the clamp: out < 1 means the clamp did not act; elements with out == 1 are decided below
        int flagged = 0;
        stage_tile<kLdsBwdWG, true, FAST>(rows, 0, G, O, s0, valid, cg, [&](float v, float o, int, int) {
            flagged |= !(o < 1.0f);
            return v;
        });
        if (flagged) atomicOr(flag, 1);
        stage_tile<kLdsBwdWG, false, FAST>(rows, S, A, A, s0, valid, ca, plain);
        stage_tile<kLdsBwdWG, false, FAST>(rows, S + na, B, B, s0, valid, cb, plain);
        lds_barrier();
        if (*flag) {                                 // rare: some output of this tile sits on the clamp
            for (int e = threadIdx.x; e < valid * S; e += kLdsBwdWG) {
                int s, c;
                split(e, S, G.inv_n, s, c);
                if (!(O.p[(s0 + s) * O.ld + c] < 1.0f)) {
                    float pre = 0.0f;
                    for (uint32_t t = col_ptr[c], t1 = col_ptr[c + 1]; t < t1; ++t) {
                        const uint32_t ij = col_ij[t];
                        pre = __builtin_fmaf(rows[slot_of(S + (ij & 0xffffu), s)], rows[slot_of(S + na + (ij >> 16), s)], pre);
                    }
                    if (!(pre <= 1.0f)) rows[slot_of(c, s)] = 0.0f;
                }
            }
            lds_barrier();
        }
        for (int blk = group; blk < blocks_a + blocks_b; blk += kLdsBwdWG / 16) {
            const bool is_a = blk < blocks_a;
            float *base = is_a ? ga : gb;
            if (!base) continue;
            const int col0 = is_a ? 4 * blk : 4 * (blk - blocks_a);
            const uint4 *packets = reinterpret_cast<const uint4 *>(is_a ? pka : pkb);
            const uint32_t *ptr = is_a ? pka_ptr : pkb_ptr;
            float4 o[4];
#pragma unroll
            for (int cc = 0; cc < 4; ++cc) o[cc] = gather_dot(rows, packets, ptr[col0 + cc], ptr[col0 + cc + 1], q);
            store_block<false, FAST>(base, is_a ? A.ld : B.ld, is_a ? na : nb, is_a ? vec_ga : vec_gb, s0, valid, q, col0, o,
                               is_a ? (accumulate & 1) : (accumulate & 2));
        }
    }
}

// ---------------------------------------------------------------- launchers

static bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static Rows2D rows2d(const float *p, int64_t ld, int32_t n)
{
    Rows2D r;
    r.p = p;
    r.ld = ld;
    r.n = n;
    r.vec = ld == n && aligned16(p);
    r.inv_n = 1.0f / static_cast<float>(n);
    return r;
}

static unsigned lds_grid(int n_tiles, size_t lds_bytes)
{
    const int per_cu = static_cast<int>(kLdsBytesMax / lds_bytes) > 0 ? static_cast<int>(kLdsBytesMax / lds_bytes) : 1;
    const int cap = 256 * per_cu;
    return static_cast<unsigned>(n_tiles < cap ? n_tiles : cap);
}

// *done = the call was taken (otherwise the caller uses the direct kernels).
dol_status launch_damp_lds_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                               int64_t ldb, float *out, int64_t ldo, hipStream_t st, bool *done)
{
    *done = false;
    if (!f->lds_fwd_ok || batch < 1) return DOL_OK;
    const int n_tiles = (batch + kLdsTile - 1) / kLdsTile;
    DOL_HIP(allow_dynamic_lds(reinterpret_cast<const void *>(damp_lds_fwd_kernel<true>), kLdsBytesMax));
    DOL_HIP(allow_dynamic_lds(reinterpret_cast<const void *>(damp_lds_fwd_kernel<false>), kLdsBytesMax));
    const int32_t n_pk = static_cast<int32_t>(f->lds_pk.n / 4);
    const int32_t vec_out = (ldo % 4 == 0) && aligned16(out);
    const Rows2D A = rows2d(a, lda, f->na), B = rows2d(b, ldb, f->nb);
    const dim3 grid(lds_grid(n_tiles, f->lds_fwd_bytes)), block(kLdsFwdWG);
    // whole tiles of contiguous aligned tensors whose sizes are multiples of four take the specialised build
    if (A.vec && B.vec && vec_out && ldo == f->n_out && !((f->na | f->nb | f->n_out) & 3) && batch % kLdsTile == 0)
        hipLaunchKernelGGL(damp_lds_fwd_kernel<true>, grid, block, f->lds_fwd_bytes, st, batch, n_tiles, f->n_out, n_pk,
                           f->lds_pk.ptr, f->lds_pk_ptr.ptr, A, B, out, ldo, vec_out);
    else
        hipLaunchKernelGGL(damp_lds_fwd_kernel<false>, grid, block, f->lds_fwd_bytes, st, batch, n_tiles, f->n_out, n_pk,
                           f->lds_pk.ptr, f->lds_pk_ptr.ptr, A, B, out, ldo, vec_out);
    DOL_HIP(hipGetLastError());
    *done = true;
    return DOL_OK;
}

dol_status launch_damp_lds_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                               int64_t ldb, const float *out, int64_t ldo, const float *g, int64_t ldg, float *ga,
                               float *gb, int32_t accumulate, hipStream_t st, bool *done)
{
    *done = false;
    if (!f->lds_bwd_ok || batch < 1 || (ga && ga == gb)) return DOL_OK;
    const int n_tiles = (batch + kLdsTile - 1) / kLdsTile;
    DOL_HIP(allow_dynamic_lds(reinterpret_cast<const void *>(damp_lds_bwd_kernel<true>), kLdsBytesMax));
    DOL_HIP(allow_dynamic_lds(reinterpret_cast<const void *>(damp_lds_bwd_kernel<false>), kLdsBytesMax));
    const int32_t vec_ga = (lda % 4 == 0) && aligned16(ga), vec_gb = (ldb % 4 == 0) && aligned16(gb);
    const Rows2D A = rows2d(a, lda, f->na), B = rows2d(b, ldb, f->nb), G = rows2d(g, ldg, f->n_out), O = rows2d(out, ldo, f->n_out);
    const dim3 grid(lds_grid(n_tiles, f->lds_bwd_bytes)), block(kLdsBwdWG);
    const int32_t n_pka = static_cast<int32_t>(f->lds_pka.n / 4), n_pkb = static_cast<int32_t>(f->lds_pkb.n / 4);
    if (A.vec && B.vec && G.vec && O.vec && vec_ga && vec_gb && !((f->na | f->nb | f->n_out) & 3) && batch % kLdsTile == 0)
        hipLaunchKernelGGL(damp_lds_bwd_kernel<true>, grid, block, f->lds_bwd_bytes, st, batch, n_tiles, n_pka, n_pkb,
                           f->lds_pka.ptr, f->lds_pka_ptr.ptr, f->lds_pkb.ptr, f->lds_pkb_ptr.ptr, f->col_ptr.ptr,
                           f->col_ij.ptr, A, B, G, O, ga, gb, vec_ga, vec_gb, accumulate);
    else
        hipLaunchKernelGGL(damp_lds_bwd_kernel<false>, grid, block, f->lds_bwd_bytes, st, batch, n_tiles, n_pka, n_pkb,
                           f->lds_pka.ptr, f->lds_pka_ptr.ptr, f->lds_pkb.ptr, f->lds_pkb_ptr.ptr, f->col_ptr.ptr,
                           f->col_ij.ptr, A, B, G, O, ga, gb, vec_ga, vec_gb, accumulate);
    DOL_HIP(hipGetLastError());
    *done = true;
    return DOL_OK;
}

}  // namespace dol
