// DAMP apply2 for convolution-shaped function tables (tuple (i, j) lands in column i + j, every tuple
// admitted: the SumN program of Fig. 2) with a short second operand (nb <= 16):
//     out[c] = min(1, sum_j a[c-j] * b[j]),
//     ga[i]  = sum_j gh[i+j] * b[j],   gb[j] = sum_i gh[i+j] * a[i],   gh = g * [pre <= 1].
//
// Tile kernels (contiguous rows, first operand up to 192 symbols): 32 lanes own a sample, a wavefront two,
// a workgroup of 256 threads a tile of 8 or 16 samples.  The lanes first issue every load of their samples'
// rows (many KB in flight per workgroup), park the rows in LDS with a zero halo, and then slide over them:
// lane c reads a[c-9..c] at immediate offsets (conflict-free, rows are spaced so that the two samples of a
// wavefront hit different banks) while the sample's short row sits in registers.  Nothing crosses
// wavefronts, so the tile loop has no workgroup barrier.  Summation runs over ascending i (descending j), one fma per tuple,
// which is the order the operator's contract fixes; halo and padding terms are exact no-ops.
//
// Loop kernels (any leading dimension, rows up to 6000, batch remainders): one wavefront per sample.
#include "internal.h"
#include "wave_util.h"

namespace dol {

constexpr int kConvMaxNb = 16;
constexpr int kConvMaxRow = 6000;       // longest first operand (backward keeps two rows, 48 KB of LDS)

constexpr int kWG = 256;                // tile kernels: threads per workgroup
constexpr int kTC = 32;                 // lanes per sample
constexpr int kSlab = kWG / kTC;        // samples computed side by side
constexpr int kTileMaxM = 192;          // longest first operand of the tile kernels
constexpr int kPA = kTileMaxM / kTC;                                   // row pieces per lane: a
constexpr int kPG = (kTileMaxM + kConvMaxNb - 1 + kTC - 1) / kTC;      // and g

static int padded_nb(int nb) { return nb <= 4 ? 4 : nb <= 8 ? 8 : nb <= 10 ? 10 : 16; }

// Smallest row stride >= n with stride % 64 == 32: the two samples of a wavefront then use disjoint banks.
static int pad_row(int n) { return ((n + 31) / 64) * 64 + 32; }

// Tables served by the thread-per-column forward kernel whose operand rows are wide enough to be worth staging in
// LDS and narrow enough to fit.
bool staged_fwd_ok(const dol_fn_table *f)
{
    // (rows of a thousand tags already: one round of reachability over a 32 x 32 grid, 1 024 x 1 985 symbols, at B=256
    // takes 7.6 us through LDS against 9.7 us with cached gathers)
    return std::max(f->na, f->nb) >= kStageMinRow / 2 && sizeof(float) * (static_cast<size_t>(f->na) + f->nb + 4) <= kStageMaxBytes;
}

// Tables walked through their per-j map whose first operand's row is worth staging in LDS, and fits.
bool byj_fwd_staged_ok(const dol_fn_table *f)
{
    return f->na >= kStageMinRow && sizeof(float) * static_cast<size_t>(f->na) <= kStageMaxBytes;
}

bool conv_path_ok(const dol_fn_table *f)
{
    return f->conv_like && f->nb <= kConvMaxNb && f->na + 3 * kConvMaxNb <= kConvMaxRow;
}

std::string damp_kernel_name(const dol_fn_table *f, bool backward, int64_t batch)
{
    if (!conv_path_ok(f)) {
        if (table_code_ok(f)) return backward ? "damp_table_bwd_kernel" : "damp_table_fwd_kernel";
        if (backward) return f->lds_bwd_ok ? "damp_lds_bwd_kernel" : !f->byj_ok ? (apply2_bwd_staged(f) ? "damp_apply2_bwd_staged_kernel" : "damp_apply2_bwd_kernel") : f->na + f->nb > 1024 ? "damp_byj_bwd_row_kernel" : "damp_byj_bwd_kernel";
        return f->lds_fwd_ok ? "damp_lds_fwd_kernel" : f->byj_fwd ? (byj_fwd_staged_ok(f) ? "damp_byj_fwd_staged_kernel" : "damp_byj_fwd_kernel") :
               staged_fwd_ok(f) ? "damp_apply2_fwd_staged_kernel" : "damp_apply2_fwd_kernel";
    }
    char buf[96];
    snprintf(buf, sizeof buf, "damp_conv_%s_%s_kernel<%d", backward ? "bwd" : "fwd",
             !backward && f->na <= 16 ? "small" : conv_rows_ok(f, batch, backward) ? "rows" : f->na <= kTileMaxM ? "tile" : "loop",
             padded_nb(f->nb));   // a prefix
    return buf;
}

// Samples per tile: 16 for large batches, 8 so that a small batch still covers the chip.
static int tile_samples(int32_t batch) { return batch >= 16 * 1024 ? 16 : 8; }

static unsigned loop_grid(int32_t batch) { return static_cast<unsigned>(batch < 8192 ? batch : 8192); }

// ---------------------------------------------------------------- forward, tiles of 8 * U samples

template <int NBP, int U>
__global__ void __launch_bounds__(kWG)
damp_conv_fwd_tile_kernel(int32_t n_tiles, int32_t m, int32_t nb, int32_t rs, const float *__restrict__ a,
                          const float *__restrict__ b, float *__restrict__ out)
{
    extern __shared__ float lds[];          // TILE rows [H zeros][m][zeros to rs], then TILE rows of NBP
    constexpr int H = NBP - 1, TILE = kSlab * U;
    float *lds_b = lds + TILE * rs;
    const int tid = threadIdx.x, tc = tid & (kTC - 1), ts = tid / kTC;
    const int S = m + nb - 1;
    for (int e = tid; e < TILE * (rs + NBP); e += kWG) lds[e] = 0.0f;
    __syncthreads();
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t s0 = static_cast<int64_t>(tile) * TILE;
        float va[U][kPA], vb[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float *ar = a + (s0 + ts + kSlab * u) * m;
#pragma unroll
            for (int p = 0; p < kPA; ++p)
                if (tc + kTC * p < m) va[u][p] = ar[tc + kTC * p];
            if (tc < nb) vb[u] = b[(s0 + ts + kSlab * u) * nb + tc];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float *row = lds + (ts + kSlab * u) * rs + H;
#pragma unroll
            for (int p = 0; p < kPA; ++p)
                if (tc + kTC * p < m) row[tc + kTC * p] = va[u][p];
            if (tc < nb) lds_b[(ts + kSlab * u) * NBP + tc] = vb[u];
        }
        wave_lds_fence();
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int sl = ts + kSlab * u;
            const float *row = lds + sl * rs + H;
            float bj[NBP];
#pragma unroll
            for (int j = 0; j < NBP; ++j) bj[j] = lds_b[sl * NBP + j];
            float *os = out + (s0 + sl) * S;
            for (int c = tc; c < S; c += kTC) {
                float acc = 0.0f;
#pragma unroll
                for (int j = NBP - 1; j >= 0; --j) acc = __builtin_fmaf(row[c - j], bj[j], acc);
                os[c] = fminf(acc, 1.0f);
            }
        }
        wave_lds_fence();
    }
}

// ---------------------------------------------------------------- forward, short first operand: a thread per sample

// First operand of at most kSmallM symbols (the first apply of a Sum-N program: two digit Distributions), contiguous
// tensors.  A workgroup owns 256 consecutive samples: their rows are one contiguous block of each tensor, copied flat
// (16 bytes per lane) into LDS; each thread then takes its sample's two rows into registers, zero-padded so that
// every column is the same chain of fma over ascending i (padding terms are exact no-ops), writes its result row back
// to LDS, and the block leaves as flat 16-byte stores.
constexpr int kSmallM = 16;
constexpr int kSmallTile = 256;

template <int NBP>
__global__ void __launch_bounds__(kSmallTile)
damp_conv_fwd_small_kernel(int32_t batch, int32_t m, int32_t nb, const float *__restrict__ a, const float *__restrict__ b,
                           float *__restrict__ out)
{
    extern __shared__ __align__(16) float lds[];    // a block, b block, out block
    const int S = m + nb - 1, tid = threadIdx.x;
    const int64_t s0 = static_cast<int64_t>(blockIdx.x) * kSmallTile;
    const int n = static_cast<int>(min(static_cast<int64_t>(kSmallTile), batch - s0));
    float *la = lds, *lb = la + kSmallTile * m, *lo = lb + kSmallTile * nb;
    auto copy_in = [&](float *dst, const float *src, int count) {
        if (count % 4 == 0) {                       // whole tiles of 256 samples always are
            for (int e = tid; e < count / 4; e += kSmallTile)
                reinterpret_cast<float4 *>(dst)[e] = reinterpret_cast<const float4 *>(src)[e];
        } else {
            for (int e = tid; e < count; e += kSmallTile) dst[e] = src[e];
        }
    };
    copy_in(la, a + s0 * m, n * m);
    copy_in(lb, b + s0 * nb, n * nb);
    __syncthreads();
    if (tid < n) {
        float ar[kSmallM + 2 * (NBP - 1)], br[NBP];  // ar[NBP - 1 + i] = a[i], zeros around
#pragma unroll
        for (int i = 0; i < kSmallM + 2 * (NBP - 1); ++i) {
            const int k = i - (NBP - 1);
            ar[i] = k >= 0 && k < m ? la[tid * m + k] : 0.0f;
        }
#pragma unroll
        for (int j = 0; j < NBP; ++j) br[j] = j < nb ? lb[tid * nb + j] : 0.0f;
#pragma unroll
        for (int c = 0; c < kSmallM + NBP - 1; ++c) {
            float acc = 0.0f;
#pragma unroll
            for (int j = NBP - 1; j >= 0; --j) acc = __builtin_fmaf(ar[NBP - 1 + c - j], br[j], acc);
            if (c < S) lo[tid * S + c] = fminf(acc, 1.0f);
        }
    }
    __syncthreads();
    float *dst = out + s0 * S;
    if ((n * S) % 4 == 0) {
        for (int e = tid; e < n * S / 4; e += kSmallTile) reinterpret_cast<float4 *>(dst)[e] = reinterpret_cast<const float4 *>(lo)[e];
    } else {
        for (int e = tid; e < n * S; e += kSmallTile) dst[e] = lo[e];
    }
}

// ---------------------------------------------------------------- forward, one wavefront per sample

template <int NBP>
__global__ void __launch_bounds__(kWave)
damp_conv_fwd_loop_kernel(int32_t batch, int32_t m, int32_t nb, const float *__restrict__ a, int64_t lda,
                          const float *__restrict__ b, int64_t ldb, float *__restrict__ out, int64_t ldo)
{
    extern __shared__ float lds[];          // [H zeros][m values][H zeros]
    constexpr int H = NBP - 1;
    const int lane = threadIdx.x;
    const int S = m + nb - 1;
    float *row = lds + H;
    if (lane < H) { lds[lane] = 0.0f; row[m + lane] = 0.0f; }
    for (int s = blockIdx.x; s < batch; s += gridDim.x) {
        const float *as = a + static_cast<int64_t>(s) * lda;
        const float *bs = b + static_cast<int64_t>(s) * ldb;
        float bj[NBP];
#pragma unroll
        for (int j = 0; j < NBP; ++j) bj[j] = j < nb ? bs[j] : 0.0f;
        for (int i = lane; i < m; i += kWave) row[i] = as[i];
        __syncthreads();
        float *os = out + static_cast<int64_t>(s) * ldo;
        for (int c = lane; c < S; c += kWave) {
            float acc = 0.0f;
#pragma unroll
            for (int j = NBP - 1; j >= 0; --j) acc = __builtin_fmaf(row[c - j], bj[j], acc);
            os[c] = fminf(acc, 1.0f);
        }
        __syncthreads();
    }
}

template <int NBP>
static void launch_fwd_nbp(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                           int64_t ldb, float *out, int64_t ldo, hipStream_t st)
{
    const int m = f->na, nb = f->nb, S = m + nb - 1;
    if (m <= kSmallM && lda == m && ldb == nb && ldo == S && (reinterpret_cast<uintptr_t>(a) | reinterpret_cast<uintptr_t>(b) |
                                                            reinterpret_cast<uintptr_t>(out)) % 16 == 0) {
        // the offsets of the tile's blocks: multiples of 256 samples, hence of 16 bytes
        const size_t lds = sizeof(float) * kSmallTile * static_cast<size_t>(m + nb + S);
        const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(batch) + kSmallTile - 1) / kSmallTile);
        hipLaunchKernelGGL(damp_conv_fwd_small_kernel<NBP>, dim3(grid), dim3(kSmallTile), lds, st, batch, m, nb, a, b, out);
        return;
    }
    int32_t done = 0;
    const int tile_s = tile_samples(batch);
    if (m <= kTileMaxM && batch >= tile_s && lda == m && ldb == nb && ldo == S) {
        const int n_tiles = batch / tile_s;
        const int rs = pad_row(m + 2 * (NBP - 1));
        const size_t lds = sizeof(float) * static_cast<size_t>(tile_s) * (rs + NBP);
        const unsigned grid = static_cast<unsigned>(n_tiles < 4096 ? n_tiles : 4096);
        if (tile_s == 16)
            hipLaunchKernelGGL((damp_conv_fwd_tile_kernel<NBP, 2>), dim3(grid), dim3(kWG), lds, st, n_tiles, m, nb, rs,
                               a, b, out);
        else
            hipLaunchKernelGGL((damp_conv_fwd_tile_kernel<NBP, 1>), dim3(grid), dim3(kWG), lds, st, n_tiles, m, nb, rs,
                               a, b, out);
        done = n_tiles * tile_s;
    }
    if (done < batch) {
        const size_t lds = sizeof(float) * static_cast<size_t>(m + 2 * (NBP - 1));
        hipLaunchKernelGGL(damp_conv_fwd_loop_kernel<NBP>, dim3(loop_grid(batch - done)), dim3(kWave), lds, st,
                           batch - done, m, nb, a + done * lda, lda, b + done * ldb, ldb, out + done * ldo, ldo);
    }
}

dol_status launch_damp_conv_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                int64_t ldb, float *out, int64_t ldo, hipStream_t st)
{
    if (batch == 0) return DOL_OK;
    dol_status taken = DOL_OK;
    if (launch_damp_conv_rows_fwd(f, batch, a, lda, b, ldb, out, ldo, st, &taken)) return taken;
    switch (padded_nb(f->nb)) {
    case 4: launch_fwd_nbp<4>(f, batch, a, lda, b, ldb, out, ldo, st); break;
    case 8: launch_fwd_nbp<8>(f, batch, a, lda, b, ldb, out, ldo, st); break;
    case 10: launch_fwd_nbp<10>(f, batch, a, lda, b, ldb, out, ldo, st); break;
    default: launch_fwd_nbp<16>(f, batch, a, lda, b, ldb, out, ldo, st); break;
    }
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// ---------------------------------------------------------------- backward
//
// The clamp decision needs pre only where it can exceed 1: pre[c] <= max(a) * sum(b) for non-negative tags,
// so a sample whose bound stays below 1 passes g through; the others recompute pre in the forward order.

template <int NBP, int U>
__global__ void __launch_bounds__(kWG)
damp_conv_bwd_tile_kernel(int32_t n_tiles, int32_t m, int32_t nb, int32_t rs_a, int32_t rs_g,
                          const float *__restrict__ a, const float *__restrict__ b, const float *__restrict__ g,
                          float *__restrict__ ga, float *__restrict__ gb, int32_t accumulate)
{
    extern __shared__ float lds[];          // a rows (halo on both sides), g rows (zero tail), b rows of NBP
    constexpr int H = NBP - 1, TILE = kSlab * U;
    float *lds_g = lds + TILE * rs_a;
    float *lds_b = lds_g + TILE * rs_g;
    const int tid = threadIdx.x, tc = tid & (kTC - 1), ts = tid / kTC;
    const int S = m + nb - 1;
    for (int e = tid; e < TILE * (rs_a + rs_g + NBP); e += kWG) lds[e] = 0.0f;
    __syncthreads();
    for (int tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const int64_t s0 = static_cast<int64_t>(tile) * TILE;
        float va[U][kPA], vg[U][kPG], vb[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const float *ar = a + (s0 + ts + kSlab * u) * m;
            const float *gr = g + (s0 + ts + kSlab * u) * S;
#pragma unroll
            for (int p = 0; p < kPA; ++p)
                if (tc + kTC * p < m) va[u][p] = ar[tc + kTC * p];
#pragma unroll
            for (int p = 0; p < kPG; ++p)
                if (tc + kTC * p < S) vg[u][p] = gr[tc + kTC * p];
            if (tc < nb) vb[u] = b[(s0 + ts + kSlab * u) * nb + tc];
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float *row_a = lds + (ts + kSlab * u) * rs_a + H;
            float *row_g = lds_g + (ts + kSlab * u) * rs_g;
#pragma unroll
            for (int p = 0; p < kPA; ++p)
                if (tc + kTC * p < m) row_a[tc + kTC * p] = va[u][p];
#pragma unroll
            for (int p = 0; p < kPG; ++p)
                if (tc + kTC * p < S) row_g[tc + kTC * p] = vg[u][p];
            if (tc < nb) lds_b[(ts + kSlab * u) * NBP + tc] = vb[u];
        }
        wave_lds_fence();
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int sl = ts + kSlab * u;
            const float *row_a = lds + sl * rs_a + H;
            float *row_g = lds_g + sl * rs_g;
            float bj[NBP];
            float sum_b = 0.0f;
#pragma unroll
            for (int j = 0; j < NBP; ++j) { bj[j] = lds_b[sl * NBP + j]; sum_b += bj[j]; }
            float amax = 0.0f;
#pragma unroll
            for (int p = 0; p < kPA; ++p)
                if (tc + kTC * p < m) amax = fmaxf(amax, va[u][p]);
            amax = reduce32<MaxOp>(amax);
            if (!(amax * sum_b <= 0.9999f)) {    // some column of this sample may have been clamped
                for (int c = tc; c < S; c += kTC) {
                    float pre = 0.0f;
#pragma unroll
                    for (int j = NBP - 1; j >= 0; --j) pre = __builtin_fmaf(row_a[c - j], bj[j], pre);
                    if (!(pre <= 1.0f)) row_g[c] = 0.0f;
                }
                wave_lds_fence();
            }
            float pj[NBP];
#pragma unroll
            for (int j = 0; j < NBP; ++j) pj[j] = 0.0f;
            float *gas = ga ? ga + (s0 + sl) * m : nullptr;
            for (int i = tc; i < m; i += kTC) {
                float gv[NBP];
#pragma unroll
                for (int j = 0; j < NBP; ++j) gv[j] = row_g[i + j];
                if (gas) {
                    float acc = 0.0f;
#pragma unroll
                    for (int j = 0; j < NBP; ++j) acc = __builtin_fmaf(gv[j], bj[j], acc);
                    gas[i] = (accumulate & 1) ? gas[i] + acc : acc;
                }
                const float ai = row_a[i];
#pragma unroll
                for (int j = 0; j < NBP; ++j) pj[j] = __builtin_fmaf(gv[j], ai, pj[j]);
            }
            if (gb) {
                float mine = 0.0f;
#pragma unroll
                for (int j = 0; j < NBP; ++j) {
                    const float tot = reduce32<AddOp>(pj[j]);
                    if (tc == j) mine = tot;
                }
                if (tc < nb) {
                    float *dst = gb + (s0 + sl) * nb + tc;
                    *dst = (accumulate & 2) ? *dst + mine : mine;
                }
            }
        }
        wave_lds_fence();
    }
}

template <int NBP>
__global__ void __launch_bounds__(kWave)
damp_conv_bwd_loop_kernel(int32_t batch, int32_t m, int32_t nb, const float *__restrict__ a, int64_t lda,
                          const float *__restrict__ b, int64_t ldb, const float *__restrict__ g, int64_t ldg,
                          float *__restrict__ ga, float *__restrict__ gb, int32_t accumulate)
{
    extern __shared__ float lds[];          // [H zeros][m: a][H zeros] [S: g][NBP zeros] [64: partial sums]
    constexpr int H = NBP - 1;
    constexpr int Q = kWave / NBP;          // chunks of the gb reduction: lane (j, q) sums chunk q for its j
    const int lane = threadIdx.x;
    const int S = m + nb - 1;
    float *row_a = lds + H;
    float *row_g = lds + m + 2 * H;
    float *part = row_g + S + NBP;
    if (lane < H) { lds[lane] = 0.0f; row_a[m + lane] = 0.0f; }
    if (lane < NBP) row_g[S + lane] = 0.0f;
    const int jq = lane % NBP, q = lane / NBP;
    const int chunk = (m + Q - 1) / Q;
    for (int s = blockIdx.x; s < batch; s += gridDim.x) {
        const float *as = a + static_cast<int64_t>(s) * lda;
        const float *bs = b + static_cast<int64_t>(s) * ldb;
        const float *gs = g + static_cast<int64_t>(s) * ldg;
        float bj[NBP];
        float sum_b = 0.0f;
#pragma unroll
        for (int j = 0; j < NBP; ++j) { bj[j] = j < nb ? bs[j] : 0.0f; sum_b += bj[j]; }
        float amax = 0.0f;
        for (int i = lane; i < m; i += kWave) { const float v = as[i]; row_a[i] = v; amax = fmaxf(amax, v); }
        for (int c = lane; c < S; c += kWave) row_g[c] = gs[c];
        amax = wave_max(amax);
        __syncthreads();
        if (!(amax * sum_b <= 0.9999f)) {    // uniform: some column of this sample may have been clamped
            for (int c = lane; c < S; c += kWave) {
                float pre = 0.0f;
#pragma unroll
                for (int j = NBP - 1; j >= 0; --j) pre = __builtin_fmaf(row_a[c - j], bj[j], pre);
                if (!(pre <= 1.0f)) row_g[c] = 0.0f;
            }
            __syncthreads();
        }
        if (ga) {
            float *gas = ga + static_cast<int64_t>(s) * lda;
            for (int i = lane; i < m; i += kWave) {
                float acc = 0.0f;
#pragma unroll
                for (int j = 0; j < NBP; ++j) acc = __builtin_fmaf(row_g[i + j], bj[j], acc);
                gas[i] = (accumulate & 1) ? gas[i] + acc : acc;
            }
        }
        if (gb) {
            if (q < Q) {
                float acc = 0.0f;
                const int i1 = min(m, (q + 1) * chunk);
                for (int i = q * chunk; i < i1; ++i) acc = __builtin_fmaf(row_g[i + jq], row_a[i], acc);
                part[lane] = acc;
            }
            __syncthreads();
            if (lane < nb) {
                float tot = 0.0f;
#pragma unroll
                for (int x = 0; x < Q; ++x) tot += part[x * NBP + lane];
                float *gbs = gb + static_cast<int64_t>(s) * ldb;
                gbs[lane] = (accumulate & 2) ? gbs[lane] + tot : tot;
            }
        }
        __syncthreads();
    }
}

template <int NBP>
static void launch_bwd_nbp(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                           int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                           hipStream_t st)
{
    const int m = f->na, nb = f->nb, S = m + nb - 1;
    int32_t done = 0;
    const int tile_s = tile_samples(batch);
    if (m <= kTileMaxM && batch >= tile_s && lda == m && ldb == nb && ldg == S) {
        const int n_tiles = batch / tile_s;
        const int rs_a = pad_row(m + 2 * (NBP - 1)), rs_g = pad_row(S + NBP);
        const size_t lds = sizeof(float) * static_cast<size_t>(tile_s) * (rs_a + rs_g + NBP);
        const unsigned grid = static_cast<unsigned>(n_tiles < 4096 ? n_tiles : 4096);
        if (tile_s == 16)
            hipLaunchKernelGGL((damp_conv_bwd_tile_kernel<NBP, 2>), dim3(grid), dim3(kWG), lds, st, n_tiles, m, nb, rs_a,
                               rs_g, a, b, g, ga, gb, accumulate);
        else
            hipLaunchKernelGGL((damp_conv_bwd_tile_kernel<NBP, 1>), dim3(grid), dim3(kWG), lds, st, n_tiles, m, nb, rs_a,
                               rs_g, a, b, g, ga, gb, accumulate);
        done = n_tiles * tile_s;
    }
    if (done < batch) {
        const size_t lds = sizeof(float) * static_cast<size_t>(m + 2 * (NBP - 1) + S + NBP + kWave);
        hipLaunchKernelGGL(damp_conv_bwd_loop_kernel<NBP>, dim3(loop_grid(batch - done)), dim3(kWave), lds, st,
                           batch - done, m, nb, a + done * lda, lda, b + done * ldb, ldb, g + done * ldg, ldg,
                           ga ? ga + done * lda : nullptr, gb ? gb + done * ldb : nullptr, accumulate);
    }
}

dol_status launch_damp_conv_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                                hipStream_t st)
{
    if (batch == 0 || (!ga && !gb)) return DOL_OK;
    dol_status taken = DOL_OK;
    if (launch_damp_conv_rows_bwd(f, batch, a, lda, b, ldb, g, ldg, ga, gb, accumulate, st, &taken)) return taken;
    switch (padded_nb(f->nb)) {
    case 4: launch_bwd_nbp<4>(f, batch, a, lda, b, ldb, g, ldg, ga, gb, accumulate, st); break;
    case 8: launch_bwd_nbp<8>(f, batch, a, lda, b, ldb, g, ldg, ga, gb, accumulate, st); break;
    case 10: launch_bwd_nbp<10>(f, batch, a, lda, b, ldb, g, ldg, ga, gb, accumulate, st); break;
    default: launch_bwd_nbp<16>(f, batch, a, lda, b, ldb, g, ldg, ga, gb, accumulate, st); break;
    }
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

}  // namespace dol
