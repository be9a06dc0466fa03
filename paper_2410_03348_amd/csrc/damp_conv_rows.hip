// DAMP apply2 for convolution-shaped function tables (the SumN program of Fig. 2: tuple (i, j) lands in column i + j)
// at large batches, contiguous 16-byte aligned tensors, first operand of up to 192 symbols, second of at most 16:
//     out[c] = min(1, sum_j a[c-j] * b[j]),
//     ga[i]  = sum_j gh[i+j] * b[j],   gb[j] = sum_i gh[i+j] * a[i],   gh = g * [pre <= 1].
//
// A lane owns a sample.  A workgroup of four or eight wavefronts owns a tile of 64 consecutive samples, whose rows are one
// contiguous block of each tensor: the block comes in as flat 16-byte loads (every lane of every load instruction
// carries data, whatever the row length) and is spread over LDS rows of odd pitch, so that the 64 lanes, which all
// read the same column of their own rows, hit 64 different banks.  The wavefronts split the columns; each lane
// slides a window of the long operand through registers (one LDS read per column) with the short operand's row in
// registers, one fma per tuple over ascending i, which is the order the operator's contract fixes (padding terms are
// exact no-ops).  Results are parked in LDS, over the operand they were made from, and leave as flat 16-byte stores.  The backward pass keeps the NBP sums of
// gb in registers, so nothing is reduced across lanes; the wavefronts' partial sums meet in LDS in a fixed order.
//
// The clamp decision needs pre only where it can exceed 1: pre[c] <= max(a) * sum(b) for non-negative tags, so a
// sample whose bound stays below 1 passes g through; tiles with other samples recompute pre in the forward order.
#include "internal.h"
#include "wave_util.h"

namespace dol {

namespace {

constexpr int kRowsTile = 64;           // samples per workgroup
constexpr size_t kRowsFewLdsFwd = 30 * 1024, kRowsFewLds = 40 * 1024;       // tiles of up to this much LDS run four wavefronts (several tiles
                                                // share a compute unit), larger ones eight
constexpr int kRowsMinBatch = 16384;    // below, 64-sample tiles leave most of the chip idle
constexpr int kRowsMinM = 17, kRowsMaxM = 192;
constexpr size_t kRowsMaxLds = 156 * 1024;    // the workgroup-wide "or" keeps a few static bytes of its own

int padded_nb(int nb) { return nb <= 4 ? 4 : nb <= 8 ? 8 : nb <= 10 ? 10 : 16; }

// Copies `count` floats, the rows of length n of consecutive samples (global memory, 16-byte aligned), into LDS rows
// of pitch P at column offset off.  16-byte loads, several in flight per lane; a count that is no multiple of four
// (only the last tile of a batch) ends in scalar copies.
template <int WG>
__device__ __forceinline__ void rows_in(float *dst, int P, int off, const float *__restrict__ src, int n, int count, int tid)
{
    const int pieces = count >> 2;
    const float4 *src4 = reinterpret_cast<const float4 *>(src);
    const int step_s = (4 * WG) / n, step_c = (4 * WG) - step_s * n;
    int s = (4 * tid) / n, col = 4 * tid - s * n;
    for (int p0 = 0; p0 < pieces; p0 += 4 * WG) {
        float4 v[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = src4[min(p0 + k * WG + tid, pieces - 1)];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (p0 + k * WG + tid < pieces) {
                int ss = s, cc = col;
                float *d = dst + off;
                d[ss * P + cc] = v[k].x; if (++cc == n) { cc = 0; ++ss; }
                d[ss * P + cc] = v[k].y; if (++cc == n) { cc = 0; ++ss; }
                d[ss * P + cc] = v[k].z; if (++cc == n) { cc = 0; ++ss; }
                d[ss * P + cc] = v[k].w;
            }
            s += step_s; col += step_c;
            if (col >= n) { col -= n; ++s; }
        }
    }
    for (int e = 4 * pieces + tid; e < count; e += WG) {
        const int ss = e / n;
        dst[ss * P + off + (e - ss * n)] = src[e];
    }
}

// The inverse: LDS rows of pitch P to a flat block of global memory, added to what is there if `add`.
template <int WG>
__device__ __forceinline__ void rows_out(float *__restrict__ dst, const float *src, int P, int n, int count, int tid, bool add)
{
    const int pieces = count >> 2;
    float4 *dst4 = reinterpret_cast<float4 *>(dst);
    const int step_s = WG * 4 / n, step_c = WG * 4 - step_s * n;
    int s = (4 * tid) / n, col = 4 * tid - s * n;
    for (int p = tid; p < pieces; p += WG) {
        int ss = s, cc = col;
        float4 v;
        v.x = src[ss * P + cc]; if (++cc == n) { cc = 0; ++ss; }
        v.y = src[ss * P + cc]; if (++cc == n) { cc = 0; ++ss; }
        v.z = src[ss * P + cc]; if (++cc == n) { cc = 0; ++ss; }
        v.w = src[ss * P + cc];
        if (add) {
            const float4 o = dst4[p];
            v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w;
        }
        dst4[p] = v;
        s += step_s; col += step_c;
        if (col >= n) { col -= n; ++s; }
    }
    for (int e = 4 * pieces + tid; e < count; e += WG) {
        const int ss = e / n;
        const float v = src[ss * P + (e - ss * n)];
        dst[e] = add ? dst[e] + v : v;
    }
}

// Columns [c_lo, c_hi) of one sample's pre, c_lo and c_hi multiples of NBP: row[i] = a[i] with NBP - 1 zeros in front
// and zeros behind, bj the short operand padded with zeros.  The window win[(c - j) mod NBP] = a[c - j] moves on by one
// LDS read per column; every index below is a constant after unrolling.
template <int NBP, typename Sink>
__device__ __forceinline__ void conv_columns(const float *row, const float (&bj)[NBP], int c_lo, int c_hi, Sink &&sink)
{
    float win[NBP];
#pragma unroll
    for (int k = 1; k < NBP; ++k) win[NBP - k] = row[c_lo - k];
    for (int c = c_lo; c < c_hi; c += NBP) {
#pragma unroll
        for (int u = 0; u < NBP; ++u) {
            win[u] = row[c + u];
            float acc = 0.0f;
#pragma unroll
            for (int j = NBP - 1; j >= 0; --j) acc = __builtin_fmaf(win[(u - j + NBP) % NBP], bj[j], acc);
            sink(c + u, u, acc);
        }
    }
}

// Splits `count` units into chunks of NBP and hands wavefront `wave` of WV a contiguous run of chunks.
template <int NBP, int WV>
__device__ __forceinline__ void wave_range(int count, int wave, int &lo, int &hi)
{
    const int chunks = (count + NBP - 1) / NBP, per = (chunks + WV - 1) / WV;
    lo = min(wave * per, chunks) * NBP;
    hi = min((wave + 1) * per, chunks) * NBP;
}

struct RowsLayout {
    int pa, pb, pc;             // LDS pitches: long operand rows, short operand rows, gradient rows
    int waves;                  // wavefronts per workgroup
    size_t floats;
};

// Forward: a rows [H zeros][m][zeros up to the last column any chunk touches] (the result is written over them) and
// b rows.
RowsLayout layout_fwd(int m, int nb, int nbp)
{
    RowsLayout L;
    L.pa = (m + 3 * nbp - 3) | 1;
    L.pb = nbp | 1;
    L.pc = 0;
    L.floats = static_cast<size_t>(kRowsTile) * (L.pa + L.pb);
    L.waves = L.floats * sizeof(float) <= kRowsFewLdsFwd ? 4 : 8;
    return L;
}

// Backward: a rows as in forward (ga is written over them), g rows [S][zeros], b rows (gb is written over them), and
// one float per thread for the row maxima.  The g rows later hold the wavefronts' partial sums of gb.
RowsLayout layout_bwd(int m, int nb, int nbp)
{
    RowsLayout L;
    L.pa = (m + 3 * nbp - 3) | 1;
    L.pb = nbp | 1;
    L.pc = (m + 2 * nbp - 2) | 1;
    L.waves = static_cast<size_t>(kRowsTile) * (L.pa + L.pb + L.pc) * sizeof(float) <= kRowsFewLds ? 4 : 8;
    L.pc = std::max(L.pc, L.waves * L.pb) | 1;
    L.floats = static_cast<size_t>(kRowsTile) * (L.pa + L.pb + L.pc) + 64 * L.waves;
    return L;
}

template <int NBP, int WV>
__global__ void __launch_bounds__(64 * WV)
damp_conv_fwd_rows_kernel(int32_t batch, int32_t m, int32_t nb, int32_t pa, const float *__restrict__ a,
                          const float *__restrict__ b, float *__restrict__ out)
{
    extern __shared__ __align__(16) float lds[];
    constexpr int H = NBP - 1, PB = NBP | 1, WG = 64 * WV;
    const int S = m + nb - 1, tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    float *la = lds, *lb = la + kRowsTile * pa;
    const int64_t s0 = static_cast<int64_t>(blockIdx.x) * kRowsTile;
    const int n = static_cast<int>(min(static_cast<int64_t>(kRowsTile), batch - s0));
    for (int k = wave; k < pa - m; k += WV) la[lane * pa + (k < H ? k : m + k)] = 0.0f;
    for (int k = nb + wave; k < PB; k += WV) lb[lane * PB + k] = 0.0f;
    rows_in<WG>(la, pa, H, a + s0 * m, m, n * m, tid);
    rows_in<WG>(lb, PB, 0, b + s0 * nb, nb, n * nb, tid);
    __syncthreads();
    float bj[NBP];
#pragma unroll
    for (int j = 0; j < NBP; ++j) bj[j] = lb[lane * PB + j];
    int c_lo, c_hi;
    wave_range<NBP, WV>(S, wave, c_lo, c_hi);
    // The result takes the place of the operand: out[c] goes where a[c - H] sat, which this lane's window has left
    // behind by then.  The wavefront that owns the columns before c_lo still reads a[c_lo - H .. c_lo - 1], so the
    // first NBP columns of a run wait in registers until every wavefront is through.
    float *orow = la + lane * pa;
    const float *arow = orow + H;
    float first[NBP];
#pragma unroll
    for (int u = 0; u < NBP; ++u) first[u] = 0.0f;
    if (c_lo < c_hi) {
        conv_columns<NBP>(arow, bj, c_lo, c_lo + NBP, [&](int, int u, float pre) { first[u] = fminf(pre, 1.0f); });
        conv_columns<NBP>(arow, bj, c_lo + NBP, c_hi, [&](int c, int, float pre) {
            if (c < S) orow[c] = fminf(pre, 1.0f);
        });
    }
    __syncthreads();
    if (c_lo < c_hi) {
#pragma unroll
        for (int u = 0; u < NBP; ++u)
            if (c_lo + u < S) orow[c_lo + u] = first[u];
    }
    __syncthreads();
    rows_out<WG>(out + s0 * S, la, pa, S, n * S, tid, false);
}

template <int NBP, int WV>
__global__ void __launch_bounds__(64 * WV)
damp_conv_bwd_rows_kernel(int32_t batch, int32_t m, int32_t nb, int32_t pa, int32_t pg, const float *__restrict__ a,
                          const float *__restrict__ b, const float *__restrict__ g, float *__restrict__ ga,
                          float *__restrict__ gb, int32_t accumulate)
{
    extern __shared__ __align__(16) float lds[];
    constexpr int H = NBP - 1, PB = NBP | 1, WG = 64 * WV;
    const int S = m + nb - 1, tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    float *la = lds, *lg = la + kRowsTile * pa, *lb = lg + kRowsTile * pg, *lmax = lb + kRowsTile * PB;
    const int64_t s0 = static_cast<int64_t>(blockIdx.x) * kRowsTile;
    const int n = static_cast<int>(min(static_cast<int64_t>(kRowsTile), batch - s0));
    for (int k = wave; k < pa - m; k += WV) la[lane * pa + (k < H ? k : m + k)] = 0.0f;
    for (int k = S + wave; k < pg; k += WV) lg[lane * pg + k] = 0.0f;
    for (int k = nb + wave; k < PB; k += WV) lb[lane * PB + k] = 0.0f;
    rows_in<WG>(la, pa, H, a + s0 * m, m, n * m, tid);
    rows_in<WG>(lg, pg, 0, g + s0 * S, S, n * S, tid);
    rows_in<WG>(lb, PB, 0, b + s0 * nb, nb, n * nb, tid);
    __syncthreads();
    float *arow = la + lane * pa + H, *grow = lg + lane * pg;
    float bj[NBP];
    float sum_b = 0.0f;
#pragma unroll
    for (int j = 0; j < NBP; ++j) { bj[j] = lb[lane * PB + j]; sum_b += bj[j]; }
    int i_lo, i_hi;
    wave_range<NBP, WV>(m, wave, i_lo, i_hi);

    // may any column of this sample have been clamped?  (samples beyond the batch hold whatever LDS held: their
    // lanes may ask for the recomputation, which then touches their own rows only)
    float amax = 0.0f;
    for (int i = i_lo; i < i_hi; ++i) amax = fmaxf(amax, arow[i]);
    lmax[tid] = amax;
    __syncthreads();
    amax = lmax[lane];
#pragma unroll
    for (int w = 1; w < WV; ++w) amax = fmaxf(amax, lmax[64 * w + lane]);
    const bool gate = lane < n && !(amax * sum_b <= 0.9999f);
    if (__syncthreads_or(gate)) {
        if (__builtin_amdgcn_ballot_w64(gate)) {
            int c_lo, c_hi;
            wave_range<NBP, WV>(S, wave, c_lo, c_hi);
            conv_columns<NBP>(arow, bj, c_lo, c_hi, [&](int c, int, float pre) {
                if (gate && c < S && !(pre <= 1.0f)) grow[c] = 0.0f;
            });
        }
        __syncthreads();
    }

    // rows [i_lo, i_hi): gw[(i + j - i_lo) mod NBP] = gh[i + j]
    float gw[NBP], pj[NBP];
#pragma unroll
    for (int j = 0; j < NBP; ++j) pj[j] = 0.0f;
#pragma unroll
    for (int k = 0; k < H; ++k) gw[k] = grow[i_lo + k];
    for (int i = i_lo; i < i_hi; i += NBP) {
#pragma unroll
        for (int u = 0; u < NBP; ++u) {
            gw[(u + H) % NBP] = grow[i + u + H];
            const float ai = arow[i + u];
            float acc = 0.0f;
#pragma unroll
            for (int j = 0; j < NBP; ++j) acc = __builtin_fmaf(gw[(u + j) % NBP], bj[j], acc);
#pragma unroll
            for (int j = 0; j < NBP; ++j) pj[j] = __builtin_fmaf(gw[(u + j) % NBP], ai, pj[j]);
            if (i + u < m) arow[i + u] = acc;           // ga takes the place of a: this lane alone reads that entry
        }
    }
    __syncthreads();                                    // every wavefront is done with g
    float *part = lg + (wave * kRowsTile + lane) * PB;
#pragma unroll
    for (int j = 0; j < NBP; ++j) part[j] = pj[j];
    __syncthreads();
    for (int j = wave; j < nb; j += WV) {
        float tot = lg[lane * PB + j];
#pragma unroll
        for (int w = 1; w < WV; ++w) tot += lg[(w * kRowsTile + lane) * PB + j];
        lb[lane * PB + j] = tot;
    }
    __syncthreads();
    if (ga) rows_out<WG>(ga + s0 * m, la + H, pa, m, n * m, tid, accumulate & 1);
    if (gb) rows_out<WG>(gb + s0 * nb, lb, PB, nb, n * nb, tid, accumulate & 2);
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

unsigned tiles_of(int32_t batch) { return static_cast<unsigned>((static_cast<int64_t>(batch) + kRowsTile - 1) / kRowsTile); }

template <int NBP, int WV>
dol_status fwd_go(int32_t batch, int m, int nb, const RowsLayout &L, const float *a, const float *b, float *out, hipStream_t st)
{
    DOL_HIP(allow_dynamic_lds(reinterpret_cast<const void *>(damp_conv_fwd_rows_kernel<NBP, WV>), kRowsMaxLds));
    hipLaunchKernelGGL((damp_conv_fwd_rows_kernel<NBP, WV>), dim3(tiles_of(batch)), dim3(64 * WV), L.floats * sizeof(float), st,
                       batch, m, nb, L.pa, a, b, out);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

template <int NBP, int WV>
dol_status bwd_go(int32_t batch, int m, int nb, const RowsLayout &L, const float *a, const float *b, const float *g, float *ga,
                  float *gb, int32_t accumulate, hipStream_t st)
{
    DOL_HIP(allow_dynamic_lds(reinterpret_cast<const void *>(damp_conv_bwd_rows_kernel<NBP, WV>), kRowsMaxLds));
    hipLaunchKernelGGL((damp_conv_bwd_rows_kernel<NBP, WV>), dim3(tiles_of(batch)), dim3(64 * WV), L.floats * sizeof(float), st,
                       batch, m, nb, L.pa, L.pc, a, b, g, ga, gb, accumulate);
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}

// Calls GO<NBP, WV>(args...) for the padded length of the short operand and the number of wavefronts.
#define DOL_ROWS_DISPATCH(GO, nbp, waves, ...)                                                         \
    ((waves) == 4 ? ((nbp) == 4 ? GO<4, 4>(__VA_ARGS__) : (nbp) == 8 ? GO<8, 4>(__VA_ARGS__) :          \
                     (nbp) == 10 ? GO<10, 4>(__VA_ARGS__) : GO<16, 4>(__VA_ARGS__))                     \
                  : ((nbp) == 4 ? GO<4, 8>(__VA_ARGS__) : (nbp) == 8 ? GO<8, 8>(__VA_ARGS__) :          \
                     (nbp) == 10 ? GO<10, 8>(__VA_ARGS__) : GO<16, 8>(__VA_ARGS__)))

}  // namespace

bool conv_rows_ok(const dol_fn_table *f, int64_t batch, bool backward)
{
    // forward, short first operands have a kernel of their own (a thread per sample, rows in registers)
    if (!conv_path_ok(f) || batch < kRowsMinBatch || (!backward && f->na < kRowsMinM) || f->na > kRowsMaxM) return false;
    return layout_bwd(f->na, f->nb, padded_nb(f->nb)).floats * sizeof(float) <= kRowsMaxLds;
}

bool launch_damp_conv_rows_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b, int64_t ldb,
                               float *out, int64_t ldo, hipStream_t st, dol_status *status)
{
    const int m = f->na, nb = f->nb, S = m + nb - 1;
    if (!conv_rows_ok(f, batch, false) || lda != m || ldb != nb || ldo != S || !aligned16(a) || !aligned16(b) || !aligned16(out))
        return false;
    const int nbp = padded_nb(nb);
    const RowsLayout L = layout_fwd(m, nb, nbp);
    *status = DOL_ROWS_DISPATCH(fwd_go, nbp, L.waves, batch, m, nb, L, a, b, out, st);
    return true;
}

bool launch_damp_conv_rows_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b, int64_t ldb,
                               const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate, hipStream_t st,
                               dol_status *status)
{
    const int m = f->na, nb = f->nb, S = m + nb - 1;
    if (!conv_rows_ok(f, batch, true) || lda != m || ldb != nb || ldg != S || !aligned16(a) || !aligned16(b) || !aligned16(g) ||
        (ga && !aligned16(ga)) || (gb && !aligned16(gb)))
        return false;
    const int nbp = padded_nb(nb);
    const RowsLayout L = layout_bwd(m, nb, nbp);
    *status = DOL_ROWS_DISPATCH(bwd_go, nbp, L.waves, batch, m, nb, L, a, b, g, ga, gb, accumulate, st);
    return true;
}

}  // namespace dol
