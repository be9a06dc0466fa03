// DAMP apply2 for convolution-shaped function tables (f(i, j) lands in column i + j, every tuple admitted:
// the SumN program of Fig. 2) with a short second operand (nb <= 16).
//
// One wavefront owns one sample at a time.  The long operand row is staged in LDS with a zero halo, the
// short row sits in uniform registers, and lane c accumulates out[c] = sum_j a[c-j] * b[j] from LDS reads
// at immediate offsets (conflict-free: consecutive lanes, consecutive words).  Workgroups are single
// wavefronts, so the barriers that order LDS writes and reads cost nothing.  Summation runs over ascending
// i (descending j), one fma per tuple, which is the order the operator's contract fixes; halo and padding
// terms are exact no-ops.  While a sample is being computed the next one's rows are already in flight
// (register prefetch), which is what keeps HBM busy with one-wave workgroups.
#include "internal.h"

namespace dol {

constexpr int kWave = 64;
constexpr int kConvMaxNb = 16;
constexpr int kConvMaxRow = 6000;       // longest first operand (backward keeps two rows, 48 KB of LDS)
constexpr int kConvMaxP = 4;            // rows up to 64 * kConvMaxP take the register-prefetch kernels

static int padded_nb(int nb) { return nb <= 4 ? 4 : nb <= 8 ? 8 : nb <= 10 ? 10 : 16; }

bool conv_path_ok(const dol_fn_table *f)
{
    return f->conv_like && f->nb <= kConvMaxNb && f->na + 3 * kConvMaxNb <= kConvMaxRow;
}

std::string damp_kernel_name(const dol_fn_table *f, bool backward)
{
    if (!conv_path_ok(f)) return backward ? "damp_apply2_bwd_kernel" : "damp_apply2_fwd_kernel";
    const int p = (f->na + kWave - 1) / kWave;
    char buf[96];
    if (p <= kConvMaxP)
        snprintf(buf, sizeof buf, "damp_conv_%s_kernel<%d, %d>", backward ? "bwd" : "fwd", padded_nb(f->nb), p);
    else
        snprintf(buf, sizeof buf, "damp_conv_%s_loop_kernel<%d>", backward ? "bwd" : "fwd", padded_nb(f->nb));
    return buf;
}

static unsigned conv_grid(int32_t batch) { return static_cast<unsigned>(batch < 8192 ? batch : 8192); }

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x = fmaxf(x, __shfl_xor(x, d, kWave));
    return x;
}

// ---------------------------------------------------------------- forward, rows up to 64 * P

template <int NBP, int P>
__global__ void __launch_bounds__(kWave)
damp_conv_fwd_kernel(int32_t batch, int32_t m, int32_t nb, const float *__restrict__ a, int64_t lda,
                     const float *__restrict__ b, int64_t ldb, float *__restrict__ out, int64_t ldo)
{
    constexpr int H = NBP - 1, CAP = kWave * P;
    __shared__ float lds[H + CAP + H];      // [H zeros][CAP values, zero beyond m][H zeros]
    const int lane = threadIdx.x;
    const int S = m + nb - 1;
    float *row = lds + H;
    if (lane < H) { lds[lane] = 0.0f; row[CAP + lane] = 0.0f; }
    int s = blockIdx.x;                     // the grid never exceeds the batch
    float ca[P], cb[NBP];
    {
        const float *as = a + static_cast<int64_t>(s) * lda, *bs = b + static_cast<int64_t>(s) * ldb;
#pragma unroll
        for (int p = 0; p < P; ++p) { const int i = lane + kWave * p; ca[p] = i < m ? as[i] : 0.0f; }
#pragma unroll
        for (int j = 0; j < NBP; ++j) cb[j] = j < nb ? bs[j] : 0.0f;
    }
    for (;;) {
#pragma unroll
        for (int p = 0; p < P; ++p) row[lane + kWave * p] = ca[p];
        const int sn = s + gridDim.x;
        const bool more = sn < batch;
        float bj[NBP];
#pragma unroll
        for (int j = 0; j < NBP; ++j) bj[j] = cb[j];
        if (more) {                         // next sample's rows travel while this one is computed
            const float *as = a + static_cast<int64_t>(sn) * lda, *bs = b + static_cast<int64_t>(sn) * ldb;
#pragma unroll
            for (int p = 0; p < P; ++p) { const int i = lane + kWave * p; ca[p] = i < m ? as[i] : 0.0f; }
#pragma unroll
            for (int j = 0; j < NBP; ++j) cb[j] = j < nb ? bs[j] : 0.0f;
        }
        __syncthreads();
        float *os = out + static_cast<int64_t>(s) * ldo;
#pragma unroll
        for (int p = 0; p <= P; ++p) {
            const int c = lane + kWave * p;
            if (c < S) {
                float acc = 0.0f;
#pragma unroll
                for (int j = NBP - 1; j >= 0; --j) acc = __builtin_fmaf(row[c - j], bj[j], acc);
                os[c] = fminf(acc, 1.0f);
            }
        }
        __syncthreads();
        if (!more) break;
        s = sn;
    }
}

// ---------------------------------------------------------------- forward, any row length

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
    const dim3 grid(conv_grid(batch)), block(kWave);
    const int p = (f->na + kWave - 1) / kWave;
#define DOL_FWD(PP) \
    hipLaunchKernelGGL((damp_conv_fwd_kernel<NBP, PP>), grid, block, 0, st, batch, f->na, f->nb, a, lda, b, ldb, out, ldo)
    switch (p) {
    case 1: DOL_FWD(1); break;
    case 2: DOL_FWD(2); break;
    case 3: DOL_FWD(3); break;
    case 4: DOL_FWD(4); break;
    default: {
        const size_t lds = sizeof(float) * static_cast<size_t>(f->na + 2 * (NBP - 1));
        hipLaunchKernelGGL(damp_conv_fwd_loop_kernel<NBP>, grid, block, lds, st, batch, f->na, f->nb, a, lda, b, ldb,
                           out, ldo);
    }
    }
#undef DOL_FWD
}

dol_status launch_damp_conv_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                int64_t ldb, float *out, int64_t ldo, hipStream_t st)
{
    if (batch == 0) return DOL_OK;
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
// ga[i] = sum_j gh[i+j] * b[j],  gb[j] = sum_i gh[i+j] * a[i],  gh = g gated by the clamp decision [pre <= 1].
// The decision needs pre only where it can exceed 1: pre[c] <= max(a) * sum(b) for non-negative tags, so a
// sample whose bound stays below 1 passes g through; the others recompute pre in the forward kernel's order.
// gb: lane (j, q) sums chunk q of the i range for its j, the Q partial sums meet in LDS.

template <int NBP>
__device__ __forceinline__ void conv_bwd_body(int lane, int m, int nb, int S, float *row_a, float *row_g, float *part,
                                              const float (&bj)[NBP], float amax, float *gas, float *gbs,
                                              int32_t accumulate, int n_pass_a)
{
    constexpr int Q = kWave / NBP;
    float sum_b = 0.0f;
#pragma unroll
    for (int j = 0; j < NBP; ++j) sum_b += bj[j];
    if (!(amax * sum_b <= 0.9999f)) {        // uniform: some column of this sample may have been clamped
        for (int c = lane; c < S; c += kWave) {
            float pre = 0.0f;
#pragma unroll
            for (int j = NBP - 1; j >= 0; --j) pre = __builtin_fmaf(row_a[c - j], bj[j], pre);
            if (!(pre <= 1.0f)) row_g[c] = 0.0f;
        }
        __syncthreads();
    }
    if (gas) {
        for (int p = 0; p < n_pass_a; ++p) {
            const int i = lane + kWave * p;
            if (i < m) {
                float acc = 0.0f;
#pragma unroll
                for (int j = 0; j < NBP; ++j) acc = __builtin_fmaf(row_g[i + j], bj[j], acc);
                gas[i] = (accumulate & 1) ? gas[i] + acc : acc;
            }
        }
    }
    if (gbs) {
        const int jq = lane % NBP, q = lane / NBP;
        const int chunk = (m + Q - 1) / Q;
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
            gbs[lane] = (accumulate & 2) ? gbs[lane] + tot : tot;
        }
    }
}

template <int NBP, int P>
__global__ void __launch_bounds__(kWave)
damp_conv_bwd_kernel(int32_t batch, int32_t m, int32_t nb, const float *__restrict__ a, int64_t lda,
                     const float *__restrict__ b, int64_t ldb, const float *__restrict__ g, int64_t ldg,
                     float *__restrict__ ga, float *__restrict__ gb, int32_t accumulate)
{
    constexpr int H = NBP - 1, CAP = kWave * P, CAPG = kWave * (P + 1);
    __shared__ float lds[H + CAP + H + CAPG + NBP + kWave];
    const int lane = threadIdx.x;
    const int S = m + nb - 1;
    float *row_a = lds + H;                 // [H zeros][CAP, zero beyond m][H zeros]
    float *row_g = lds + H + CAP + H;       // [CAPG, zero beyond S][NBP zeros]
    float *part = row_g + CAPG + NBP;
    if (lane < H) { lds[lane] = 0.0f; row_a[CAP + lane] = 0.0f; }
    if (lane < NBP) row_g[CAPG + lane] = 0.0f;
    int s = blockIdx.x;
    float ca[P], cg[P + 1], cb[NBP];
    {
        const float *as = a + static_cast<int64_t>(s) * lda, *bs = b + static_cast<int64_t>(s) * ldb;
        const float *gs = g + static_cast<int64_t>(s) * ldg;
#pragma unroll
        for (int p = 0; p < P; ++p) { const int i = lane + kWave * p; ca[p] = i < m ? as[i] : 0.0f; }
#pragma unroll
        for (int p = 0; p <= P; ++p) { const int c = lane + kWave * p; cg[p] = c < S ? gs[c] : 0.0f; }
#pragma unroll
        for (int j = 0; j < NBP; ++j) cb[j] = j < nb ? bs[j] : 0.0f;
    }
    for (;;) {
        float amax = 0.0f;
#pragma unroll
        for (int p = 0; p < P; ++p) { row_a[lane + kWave * p] = ca[p]; amax = fmaxf(amax, ca[p]); }
#pragma unroll
        for (int p = 0; p <= P; ++p) row_g[lane + kWave * p] = cg[p];
        float bj[NBP];
#pragma unroll
        for (int j = 0; j < NBP; ++j) bj[j] = cb[j];
        const int sn = s + gridDim.x;
        const bool more = sn < batch;
        if (more) {
            const float *as = a + static_cast<int64_t>(sn) * lda, *bs = b + static_cast<int64_t>(sn) * ldb;
            const float *gs = g + static_cast<int64_t>(sn) * ldg;
#pragma unroll
            for (int p = 0; p < P; ++p) { const int i = lane + kWave * p; ca[p] = i < m ? as[i] : 0.0f; }
#pragma unroll
            for (int p = 0; p <= P; ++p) { const int c = lane + kWave * p; cg[p] = c < S ? gs[c] : 0.0f; }
#pragma unroll
            for (int j = 0; j < NBP; ++j) cb[j] = j < nb ? bs[j] : 0.0f;
        }
        amax = wave_max(amax);
        __syncthreads();
        conv_bwd_body<NBP>(lane, m, nb, S, row_a, row_g, part, bj, amax,
                           ga ? ga + static_cast<int64_t>(s) * lda : nullptr,
                           gb ? gb + static_cast<int64_t>(s) * ldb : nullptr, accumulate, P);
        __syncthreads();
        if (!more) break;
        s = sn;
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
    const int lane = threadIdx.x;
    const int S = m + nb - 1;
    float *row_a = lds + H;
    float *row_g = lds + m + 2 * H;
    float *part = row_g + S + NBP;
    if (lane < H) { lds[lane] = 0.0f; row_a[m + lane] = 0.0f; }
    if (lane < NBP) row_g[S + lane] = 0.0f;
    const int n_pass_a = (m + kWave - 1) / kWave;
    for (int s = blockIdx.x; s < batch; s += gridDim.x) {
        const float *as = a + static_cast<int64_t>(s) * lda;
        const float *bs = b + static_cast<int64_t>(s) * ldb;
        const float *gs = g + static_cast<int64_t>(s) * ldg;
        float bj[NBP];
#pragma unroll
        for (int j = 0; j < NBP; ++j) bj[j] = j < nb ? bs[j] : 0.0f;
        float amax = 0.0f;
        for (int i = lane; i < m; i += kWave) { const float v = as[i]; row_a[i] = v; amax = fmaxf(amax, v); }
        for (int c = lane; c < S; c += kWave) row_g[c] = gs[c];
        amax = wave_max(amax);
        __syncthreads();
        conv_bwd_body<NBP>(lane, m, nb, S, row_a, row_g, part, bj, amax,
                           ga ? ga + static_cast<int64_t>(s) * lda : nullptr,
                           gb ? gb + static_cast<int64_t>(s) * ldb : nullptr, accumulate, n_pass_a);
        __syncthreads();
    }
}

template <int NBP>
static void launch_bwd_nbp(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                           int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                           hipStream_t st)
{
    const dim3 grid(conv_grid(batch)), block(kWave);
    const int p = (f->na + kWave - 1) / kWave;
#define DOL_BWD(PP)                                                                                               \
    hipLaunchKernelGGL((damp_conv_bwd_kernel<NBP, PP>), grid, block, 0, st, batch, f->na, f->nb, a, lda, b, ldb, g, \
                       ldg, ga, gb, accumulate)
    switch (p) {
    case 1: DOL_BWD(1); break;
    case 2: DOL_BWD(2); break;
    case 3: DOL_BWD(3); break;
    case 4: DOL_BWD(4); break;
    default: {
        const int S = f->na + f->nb - 1;
        const size_t lds = sizeof(float) * static_cast<size_t>(f->na + 2 * (NBP - 1) + S + NBP + kWave);
        hipLaunchKernelGGL(damp_conv_bwd_loop_kernel<NBP>, grid, block, lds, st, batch, f->na, f->nb, a, lda, b, ldb,
                           g, ldg, ga, gb, accumulate);
    }
    }
#undef DOL_BWD
}

dol_status launch_damp_conv_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                                hipStream_t st)
{
    if (batch == 0 || (!ga && !gb)) return DOL_OK;
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
