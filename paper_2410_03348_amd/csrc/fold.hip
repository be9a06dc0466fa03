// Fused left fold of convolution-shaped DAMP applies (the loop of Fig. 2), forward and backward in one
// launch.  32 lanes own a sample, a wavefront two, and a workgroup is one wavefront.  Everything a sample
// needs lives in its LDS region: the running Distributions acc_0 .. acc_{n-1} back to back with shared zero
// halos (they are the operands of the backward pass), the short inputs, and two gradient rows.  HBM sees the
// inputs once, the final Distribution once and the input gradients once.
//
// Arithmetic is that of the per-operator kernels: out[c] = min(1, sum over ascending i of a[i] * b[c-i]) with
// one fma per tuple; gradients are gated by [pre <= 1], re-derived only for stages in which some lane saw
// pre > 1 during the forward sweep.
#include "internal.h"
#include "wave_util.h"

#include <cfloat>

namespace dol {

constexpr int kFoldMax = 32;            // most inputs of one fold
constexpr int kFoldTC = 32;             // lanes per sample
constexpr int kFoldMaxNb = 16;

struct FoldArgs {
    int32_t n;                          // inputs
    int32_t batch;
    int32_t m[kFoldMax];                // symbols of acc_t (m[0] = symbols of inputs[0])
    int32_t nb[kFoldMax];               // symbols of inputs[t], t >= 1
    int32_t off[kFoldMax];              // LDS offset of acc_t's first value inside a sample's region
    int32_t off_d;                      // LDS offset of the short input rows (row t at off_d + t * NBP)
    int32_t off_g0, off_g1;             // the two gradient rows
    int32_t stride;                     // floats per sample region
    const float *in[kFoldMax];
    int64_t ld[kFoldMax];
    float *gin[kFoldMax];
    float *out;
    int64_t ldo;
    const int32_t *target;
    const float *gout;
    int64_t ldg;
    int32_t backward;
};

template <int NBP>
__global__ void __launch_bounds__(kWave)
damp_fold_kernel(const FoldArgs A)
{
    extern __shared__ float lds[];
    const int lane = threadIdx.x, tc = lane & (kFoldTC - 1), half = lane / kFoldTC;
    // Workgroups are dealt round-robin to the 8 XCDs (one L2 each); give every XCD a contiguous range of
    // samples so that the 128-byte lines shared by neighbouring samples are fetched into one L2 only.
    const int wg = xcd_contiguous(blockIdx.x, gridDim.x);
    const int64_t s_raw = static_cast<int64_t>(wg) * 2 + half;
    const bool live = s_raw < A.batch;              // an odd batch leaves the last half-wavefront idle
    const int64_t s = live ? s_raw : A.batch - 1;   // it shadows the last sample and stores nothing
    float *base = lds + half * A.stride;
    for (int e = tc; e < A.stride; e += kFoldTC) base[e] = 0.0f;
    wave_lds_fence();

    // ---- inputs: acc_0 and the short rows
    {
        float v[kFoldMax];                          // every load is issued before the first LDS write waits
#pragma unroll
        for (int t = 1; t < kFoldMax; ++t)
            if (t < A.n && tc < A.nb[t]) v[t] = A.in[t][s * A.ld[t] + tc];
        const float *r0 = A.in[0] + s * A.ld[0];
        for (int i = tc; i < A.m[0]; i += kFoldTC) base[A.off[0] + i] = r0[i];
#pragma unroll
        for (int t = 1; t < kFoldMax; ++t)
            if (t < A.n && tc < A.nb[t]) base[A.off_d + t * NBP + tc] = v[t];
    }
    wave_lds_fence();

    // ---- forward sweep
    unsigned over = 0;                              // bit t: this lane saw pre > 1 in stage t
    for (int t = 1; t < A.n; ++t) {
        const float *row = base + A.off[t - 1];
        float *dst = base + A.off[t];
        float bj[NBP];
#pragma unroll
        for (int j = 0; j < NBP; ++j) bj[j] = base[A.off_d + t * NBP + j];
        const int S = A.m[t];
        for (int c = tc; c < S; c += kFoldTC) {
            float acc = 0.0f;
#pragma unroll
            for (int j = NBP - 1; j >= 0; --j) acc = __builtin_fmaf(row[c - j], bj[j], acc);
            if (!(acc <= 1.0f)) over |= 1u << t;
            dst[c] = fminf(acc, 1.0f);
        }
        wave_lds_fence();
    }
    const int n1 = A.n - 1;
    const float *last = base + A.off[n1];
    if (A.out && live) {
        float *os = A.out + s * A.ldo;
        for (int c = tc; c < A.m[n1]; c += kFoldTC) os[c] = last[c];
    }
    if (!A.backward) return;
    over = static_cast<unsigned>(reduce32_or(static_cast<int>(over)));

    // ---- upstream gradient into the first gradient row (zero tail of NBP entries)
    float *g_cur = base + A.off_g0, *g_nxt = base + A.off_g1;
    {
        const int S = A.m[n1];
        if (A.target) {
            const int tgt = A.target[s];
            for (int c = tc; c < S + NBP; c += kFoldTC)
                g_cur[c] = c == tgt && c < S ? -1.0f / fmaxf(last[c], FLT_MIN) : 0.0f;
        } else {
            const float *gs = A.gout + s * A.ldg;
            for (int c = tc; c < S + NBP; c += kFoldTC) g_cur[c] = c < S ? gs[c] : 0.0f;
        }
    }
    wave_lds_fence();

    // ---- reverse sweep
    for (int t = n1; t >= 1; --t) {
        const float *row_a = base + A.off[t - 1];
        const int m = A.m[t - 1], S = A.m[t], nb = A.nb[t];
        float bj[NBP];
#pragma unroll
        for (int j = 0; j < NBP; ++j) bj[j] = base[A.off_d + t * NBP + j];
        if ((over >> t) & 1) {                      // some column of this stage was clamped: gate its gradient
            for (int c = tc; c < S; c += kFoldTC) {
                float pre = 0.0f;
#pragma unroll
                for (int j = NBP - 1; j >= 0; --j) pre = __builtin_fmaf(row_a[c - j], bj[j], pre);
                if (!(pre <= 1.0f)) g_cur[c] = 0.0f;
            }
            wave_lds_fence();
        }
        float pj[NBP];
#pragma unroll
        for (int j = 0; j < NBP; ++j) pj[j] = 0.0f;
        for (int i = tc; i < m; i += kFoldTC) {
            float gv[NBP];
#pragma unroll
            for (int j = 0; j < NBP; ++j) gv[j] = g_cur[i + j];
            float acc = 0.0f;
#pragma unroll
            for (int j = 0; j < NBP; ++j) acc = __builtin_fmaf(gv[j], bj[j], acc);
            g_nxt[i] = acc;
            const float ai = row_a[i];
#pragma unroll
            for (int j = 0; j < NBP; ++j) pj[j] = __builtin_fmaf(gv[j], ai, pj[j]);
        }
        if (tc < NBP) g_nxt[m + tc] = 0.0f;         // the next stage reads NBP entries past its last column
        float mine = 0.0f;
#pragma unroll
        for (int j = 0; j < NBP; ++j) {
            const float tot = reduce32<AddOp>(pj[j]);
            if (tc == j) mine = tot;
        }
        if (A.gin[t] && live && tc < nb) A.gin[t][s * A.ld[t] + tc] = mine;
        wave_lds_fence();
        float *sw = g_cur; g_cur = g_nxt; g_nxt = sw;
    }
    if (A.gin[0] && live) {
        float *dst = A.gin[0] + s * A.ld[0];
        for (int i = tc; i < A.m[0]; i += kFoldTC) dst[i] = g_cur[i];
    }
}

static int fold_padded_nb(int nb) { return nb <= 4 ? 4 : nb <= 8 ? 8 : nb <= 10 ? 10 : 16; }

}  // namespace dol

using namespace dol;

extern "C" dol_status dol_fold_apply2(const dol_fold *fold, void *hip_stream)
{
    if (!fold) return fail(DOL_EINVAL, "fold is NULL");
    const int n = fold->n_inputs;
    if (n < 2 || n > kFoldMax) return fail(n < 2 ? DOL_EINVAL : DOL_EUNSUPPORTED, "n_inputs = %d outside 2..%d", n, kFoldMax);
    if (!fold->inputs || !fold->tables) return fail(DOL_EINVAL, "inputs or tables is NULL");
    FoldArgs A{};
    A.n = n;
    int max_nb = 1;
    for (int t = 0; t < n; ++t) {
        const dol_dist *d = fold->inputs[t];
        if (!d) return fail(DOL_EINVAL, "inputs[%d] is NULL", t);
        if (d->batch < 0 || d->n_sym < 1 || d->ld < d->n_sym) return fail(DOL_ESHAPE, "inputs[%d] has a bad shape", t);
        if (t == 0) A.batch = d->batch;
        if (d->batch != A.batch) return fail(DOL_ESHAPE, "inputs[%d].batch = %d, inputs[0].batch = %d", t, d->batch, A.batch);
        if (A.batch > 0 && !d->prob) return fail(DOL_EINVAL, "inputs[%d].prob is NULL", t);
        A.in[t] = d->prob;
        A.ld[t] = d->ld;
        A.gin[t] = fold->grad_inputs ? fold->grad_inputs[t] : nullptr;
        if (t == 0) { A.m[0] = d->n_sym; continue; }
        const dol_fn_table *f = fold->tables[t - 1];
        if (!f) return fail(DOL_EINVAL, "tables[%d] is NULL", t - 1);
        if (f->na != A.m[t - 1] || f->nb != d->n_sym)
            return fail(DOL_ESHAPE, "tables[%d] is %d x %d, its operands have %d and %d symbols", t - 1, f->na, f->nb, A.m[t - 1], d->n_sym);
        if (!f->conv_like || f->nb > kFoldMaxNb)
            return fail(DOL_EUNSUPPORTED, "tables[%d] is not convolution-shaped with at most %d second-operand symbols", t - 1, kFoldMaxNb);
        A.nb[t] = f->nb;
        A.m[t] = f->n_out;
        max_nb = f->nb > max_nb ? f->nb : max_nb;
    }
    const int nbp = fold_padded_nb(max_nb), H = nbp - 1;
    int off = H;
    for (int t = 0; t < n; ++t) { A.off[t] = off; off += A.m[t] + H; }
    A.off_d = off;
    off += n * nbp;
    const int g_len = A.m[n - 1] + nbp;
    A.off_g0 = off;
    A.off_g1 = off + g_len;
    off += 2 * g_len;
    A.stride = ((off + 31) / 64) * 64 + 32;         // the two samples of a wavefront use disjoint banks
    const size_t lds = sizeof(float) * 2 * static_cast<size_t>(A.stride);
    if (lds > 64 * 1024) return fail(DOL_EUNSUPPORTED, "the fold needs %zu bytes of LDS per wavefront, more than 65536", lds);
    if (fold->out) {
        const dol_dist *o = fold->out;
        if (o->batch != A.batch || o->n_sym != A.m[n - 1] || o->ld < o->n_sym)
            return fail(DOL_ESHAPE, "out has %d x %d, the fold produces %d x %d", o->batch, o->n_sym, A.batch, A.m[n - 1]);
        if (A.batch > 0 && !o->prob) return fail(DOL_EINVAL, "out.prob is NULL");
        A.out = o->prob;
        A.ldo = o->ld;
    }
    A.target = fold->target_col;
    A.gout = fold->grad_out;
    A.ldg = fold->grad_out_ld;
    A.backward = (A.target || A.gout) ? 1 : 0;
    if (A.gout && !A.target && A.ldg < A.m[n - 1]) return fail(DOL_ESHAPE, "grad_out_ld = %lld is smaller than %d", static_cast<long long>(A.ldg), A.m[n - 1]);
    if (A.batch == 0) return DOL_OK;
    const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(A.batch) + 1) / 2);
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    switch (nbp) {
    case 4: hipLaunchKernelGGL(damp_fold_kernel<4>, dim3(grid), dim3(kWave), lds, st, A); break;
    case 8: hipLaunchKernelGGL(damp_fold_kernel<8>, dim3(grid), dim3(kWave), lds, st, A); break;
    case 10: hipLaunchKernelGGL(damp_fold_kernel<10>, dim3(grid), dim3(kWave), lds, st, A); break;
    default: hipLaunchKernelGGL(damp_fold_kernel<16>, dim3(grid), dim3(kWave), lds, st, A); break;
    }
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}
