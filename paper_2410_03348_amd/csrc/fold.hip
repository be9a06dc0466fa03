// Fused left fold of convolution-shaped DAMP applies (the loop of Fig. 2), forward and backward in one
// launch.  32 lanes own a sample, a wavefront two, and a workgroup is one wavefront.  Everything a sample
// needs lives in its LDS region: the running Distributions acc_0 .. acc_{n-1} back to back with shared zero
// halos (they are the operands of the backward pass), the short inputs, and two gradient rows.  HBM sees the
// inputs once, the final Distribution once and the input gradients once.
//
// Chains whose shape fits it run the kernel that fold_chain.hip writes for the shape; the kernels of this file serve
// the others.  Two share this layout idea: damp_fold4_kernel (four consecutive columns per lane, 16-byte LDS
// accesses) and damp_fold_kernel (one column per lane, 4-byte accesses; its rows need no padding to multiples of four,
// so it still fits when the first does not).
//
// Arithmetic is that of the per-operator kernels: out[c] = min(1, sum over ascending i of a[i] * b[c-i]) with
// one fma per tuple; gradients are gated by [pre <= 1], re-derived only for stages in which some lane saw
// pre > 1 during the forward sweep.
#include "internal.h"

#include <type_traits>
#include "wave_util.h"

#include <cfloat>
#include <cstdio>

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

// ---------------------------------------------------------------- four columns per lane, 16-byte LDS accesses

constexpr int kFoldTabFloats = 6 * kFoldMax;        // LDS head: input pointers, gradient pointers, leading dimensions

// The same fold with TC = 16 or 32 lanes per sample and four consecutive columns per lane: a lane reads its
// window of the operand row with 16-byte LDS loads (NBP + 3 values feed 4 * NBP fma) instead of one 4-byte load
// per fma.  Rows start at multiples of four floats, are preceded by HB zeros and followed by zeros up to the
// next row's halo; the short rows are padded to NBR floats; gradient rows carry HB zeros past their last
// multiple of four.  Per-stage sizes and offsets sit in the lanes of three registers (lane t holds stage t) and
// are fetched with v_readlane, so that the sweeps issue no scalar memory loads; the short rows and their
// gradients move between HBM and LDS in one pass each, slot e = (t, j) = (e / NBR, e % NBR) per lane.
template <int NBP, int TC>
__global__ void __launch_bounds__(kWave)
damp_fold4_kernel(const FoldArgs A)
{
    constexpr int HB = (NBP + 2) / 4 * 4;           // zeros in front of every row, >= NBP - 1
    constexpr int NW = HB / 4 + 1;                  // 16-byte pieces of a lane's window
    constexpr int NBR = (NBP + 3) / 4 * 4;
    constexpr int kStep = 4 * TC, kPer = kWave / TC;
    constexpr int kSlots = (kFoldMax * NBR + TC - 1) / TC;
    extern __shared__ __align__(16) float lds[];
    const int lane = threadIdx.x, tc = lane & (TC - 1), q = lane / TC;
    const int wg = xcd_contiguous(blockIdx.x, gridDim.x);
    const int64_t s_raw = static_cast<int64_t>(wg) * kPer + q;
    const bool live = s_raw < A.batch;              // idle parts shadow the last sample and store nothing
    const int64_t s = live ? s_raw : A.batch - 1;

    // ---- per-stage tables: registers for the uniform ones, LDS for those a lane picks by its own slot
    const int lt = lane & (kFoldMax - 1);
    const int m_l = A.m[lt], nb_l = A.nb[lt], off_l = A.off[lt];
    uint64_t *tab_in = reinterpret_cast<uint64_t *>(lds), *tab_gin = tab_in + kFoldMax, *tab_ld = tab_gin + kFoldMax;
    int *tab_nb = reinterpret_cast<int *>(lds) + kFoldTabFloats;
    if (lane < kFoldMax) {
        tab_in[lane] = reinterpret_cast<uint64_t>(A.in[lane]);
        tab_gin[lane] = reinterpret_cast<uint64_t>(A.gin[lane]);
        tab_ld[lane] = static_cast<uint64_t>(A.ld[lane]);
        tab_nb[lane] = lane >= 1 && lane < A.n ? nb_l : 0;
    }
    auto stage = [&](int v, int t) { return __builtin_amdgcn_readlane(v, t); };

    float *base = lds + kFoldTabFloats + kFoldMax + q * A.stride;
    const float4 zero4 = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int e = 4 * tc; e < A.stride; e += kStep) *reinterpret_cast<float4 *>(base + e) = zero4;
    wave_lds_fence();

    // ---- inputs: acc_0 and the short rows.  All table reads first, then all loads, then the LDS stores.
    int64_t slot_off[kSlots];                       // element offset of the lane's slot x in its tensor, -1: none
    {
        const int n_slots = A.n * NBR;
        uint64_t src[kSlots];
#pragma unroll
        for (int x = 0; x < kSlots; ++x) {
            const int e = tc + TC * x, t = e / NBR, j = e - t * NBR, tt = t < kFoldMax ? t : 0;
            const bool ok = e < n_slots && j < tab_nb[tt];
            slot_off[x] = ok ? s * static_cast<int64_t>(tab_ld[tt]) + j : -1;
            src[x] = tab_in[tt];
        }
        float v[kSlots];
#pragma unroll
        for (int x = 0; x < kSlots; ++x)
            v[x] = slot_off[x] >= 0 ? reinterpret_cast<const float *>(src[x])[slot_off[x]] : 0.0f;
        const float *r0 = A.in[0] + s * A.ld[0];
        const int m0 = stage(m_l, 0), off0 = stage(off_l, 0);
        for (int i = tc; i < m0; i += TC) base[off0 + i] = r0[i];
#pragma unroll
        for (int x = 0; x < kSlots; ++x)
            if (tc + TC * x < n_slots) base[A.off_d + tc + TC * x] = v[x];
    }
    wave_lds_fence();

    auto load_b = [&](int t, float (&bj)[NBR]) {
#pragma unroll
        for (int p = 0; p < NBR / 4; ++p) {
            const float4 x = *reinterpret_cast<const float4 *>(base + A.off_d + t * NBR + 4 * p);
            bj[4 * p] = x.x, bj[4 * p + 1] = x.y, bj[4 * p + 2] = x.z, bj[4 * p + 3] = x.w;
        }
    };
    auto load_window = [&](const float *from, float (&w)[4 * NW]) {
#pragma unroll
        for (int p = 0; p < NW; ++p) {
            const float4 x = *reinterpret_cast<const float4 *>(from + 4 * p);
            w[4 * p] = x.x, w[4 * p + 1] = x.y, w[4 * p + 2] = x.z, w[4 * p + 3] = x.w;
        }
    };
    // pre[k] of columns c0 .. c0 + 3: ascending i = c - j, one fma per tuple
    auto columns = [&](const float *row, int c0, const float (&bj)[NBR], float (&pre)[4]) {
        float w[4 * NW];
        load_window(row + c0 - HB, w);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float acc = 0.0f;
#pragma unroll
            for (int j = NBP - 1; j >= 0; --j) acc = __builtin_fmaf(w[HB + k - j], bj[j], acc);
            pre[k] = acc;
        }
    };

    // The same for H = 1 or 2 columns per lane (stages of at most TC or 2 * TC columns): 4- or 8-byte LDS loads of
    // the H + NBP - 1 values a lane needs; the order of every column's sum is unchanged.
    auto columns_few = [&](auto hc, const float *row, int c0, const float (&bj)[NBR], float *pre) {
        constexpr int H = decltype(hc)::value;
        constexpr int FR = H == 2 ? (NBP & ~1) + ((NBP - 1) > (NBP & ~1) ? 2 : 0) : NBP - 1;   // even and >= NBP - 1 for H = 2
        constexpr int NV = FR + H;
        float w[NV + (NV & 1)];
        if (H == 2) {
#pragma unroll
            for (int p = 0; p < (NV + 1) / 2; ++p) {
                const float2 x = *reinterpret_cast<const float2 *>(row + c0 - FR + 2 * p);
                w[2 * p] = x.x, w[2 * p + 1] = x.y;
            }
        } else {
#pragma unroll
            for (int p = 0; p < NV; ++p) w[p] = row[c0 - FR + p];
        }
#pragma unroll
        for (int k = 0; k < H; ++k) {
            float acc = 0.0f;
#pragma unroll
            for (int j = NBP - 1; j >= 0; --j) acc = __builtin_fmaf(w[FR + k - j], bj[j], acc);
            pre[k] = acc;
        }
    };
    // Backward of a stage for rows i0 .. i0 + H - 1 of the first operand: their gradients (returned in o) and the
    // lane's shares of the short operand's gradient (added to pj).
    auto rows_few = [&](auto hc, const float *g_row, const float *row_a, int i0, int m, const float (&bj)[NBR],
                        float (&pj)[NBP], float *o) {
        constexpr int H = decltype(hc)::value;
        constexpr int NV = H + NBP - 1;
        float gw[NV + (NV & 1)], ak[H];
        if (H == 2) {
#pragma unroll
            for (int p = 0; p < (NV + 1) / 2; ++p) {
                const float2 x = *reinterpret_cast<const float2 *>(g_row + i0 + 2 * p);
                gw[2 * p] = x.x, gw[2 * p + 1] = x.y;
            }
            const float2 av = *reinterpret_cast<const float2 *>(row_a + i0);
            ak[0] = av.x, ak[H - 1] = av.y;
        } else {
#pragma unroll
            for (int p = 0; p < NV; ++p) gw[p] = g_row[i0 + p];
            ak[0] = row_a[i0];
        }
#pragma unroll
        for (int k = 0; k < H; ++k) {
            float acc = 0.0f;
#pragma unroll
            for (int j = 0; j < NBP; ++j) acc = __builtin_fmaf(gw[k + j], bj[j], acc);
            o[k] = i0 + k < m ? acc : 0.0f;
#pragma unroll
            for (int j = 0; j < NBP; ++j) pj[j] = __builtin_fmaf(gw[k + j], ak[k], pj[j]);
        }
    };

    // ---- forward sweep (columns past the last one come out as exact zeros: they only meet zero padding)
    unsigned over = 0;                              // bit t: this lane saw pre > 1 in stage t
    for (int t = 1; t < A.n; ++t) {
        const float *row = base + stage(off_l, t - 1);
        float *dst = base + stage(off_l, t);
        float bj[NBR];
        load_b(t, bj);
        const int S = stage(m_l, t);
        float worst = 0.0f;
        if (S <= TC) {                              // narrow stages: one or two columns per lane keep all lanes busy
            if (tc < S) {
                float pre[1];
                columns_few(std::integral_constant<int, 1>{}, row, tc, bj, pre);
                worst = pre[0];
                dst[tc] = fminf(pre[0], 1.0f);
            }
        } else if (S <= 2 * TC) {
            if (2 * tc < S) {
                float pre[2];
                columns_few(std::integral_constant<int, 2>{}, row, 2 * tc, bj, pre);
                worst = fmaxf(pre[0], pre[1]);
                *reinterpret_cast<float2 *>(dst + 2 * tc) = make_float2(fminf(pre[0], 1.0f), fminf(pre[1], 1.0f));
            }
        } else {
            for (int c0 = 4 * tc; c0 < S; c0 += kStep) {
                float pre[4];
                columns(row, c0, bj, pre);
                worst = fmaxf(worst, fmaxf(fmaxf(pre[0], pre[1]), fmaxf(pre[2], pre[3])));
                *reinterpret_cast<float4 *>(dst + c0) =
                    make_float4(fminf(pre[0], 1.0f), fminf(pre[1], 1.0f), fminf(pre[2], 1.0f), fminf(pre[3], 1.0f));
            }
        }
        if (worst > 1.0f) over |= 1u << t;
        wave_lds_fence();
    }
    const int n1 = A.n - 1;
    const int S_last = stage(m_l, n1);
    const float *last = base + stage(off_l, n1);
    if (A.out && live) {
        float *os = A.out + s * A.ldo;
        for (int c = tc; c < S_last; c += TC) os[c] = last[c];
    }
    if (!A.backward) return;
    over = static_cast<unsigned>(TC == 16 ? reduce16_or(static_cast<int>(over)) : reduce32_or(static_cast<int>(over)));

    // ---- upstream gradient into the first gradient row
    float *g_cur = base + A.off_g0, *g_nxt = base + A.off_g1;
    {
        const int S = S_last, S4 = (S + 3) & ~3;
        if (A.target) {
            const int tgt = A.target[s];
            for (int c0 = 4 * tc; c0 < S4 + HB; c0 += kStep) {
                const float4 p = *reinterpret_cast<const float4 *>(last + c0);   // past the row: other LDS, unused
                const float pk[4] = {p.x, p.y, p.z, p.w};
                float g[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) g[k] = c0 + k == tgt && tgt < S ? -1.0f / fmaxf(pk[k], FLT_MIN) : 0.0f;
                *reinterpret_cast<float4 *>(g_cur + c0) = make_float4(g[0], g[1], g[2], g[3]);
            }
        } else {
            const float *gs = A.gout + s * A.ldg;
            for (int c0 = 4 * tc; c0 < S4 + HB; c0 += kStep) {
                float g[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int c = c0 + k;
                    const float x = gs[c < S ? c : S - 1];
                    g[k] = c < S ? x : 0.0f;
                }
                *reinterpret_cast<float4 *>(g_cur + c0) = make_float4(g[0], g[1], g[2], g[3]);
            }
        }
    }
    wave_lds_fence();

    // ---- reverse sweep
    for (int t = n1; t >= 1; --t) {
        const float *row_a = base + stage(off_l, t - 1);
        const int m = stage(m_l, t - 1), S = stage(m_l, t);
        float bj[NBR];
        load_b(t, bj);
        if ((over >> t) & 1) {                      // some column of this stage was clamped: gate its gradient
            for (int c0 = 4 * tc; c0 < S; c0 += kStep) {
                float pre[4];
                columns(row_a, c0, bj, pre);
                float4 g = *reinterpret_cast<const float4 *>(g_cur + c0);
                if (!(pre[0] <= 1.0f)) g.x = 0.0f;
                if (!(pre[1] <= 1.0f)) g.y = 0.0f;
                if (!(pre[2] <= 1.0f)) g.z = 0.0f;
                if (!(pre[3] <= 1.0f)) g.w = 0.0f;
                *reinterpret_cast<float4 *>(g_cur + c0) = g;
            }
            wave_lds_fence();
        }
        float pj[NBP];
#pragma unroll
        for (int j = 0; j < NBP; ++j) pj[j] = 0.0f;
        if (m <= TC) {
            if (tc < m) {
                float o[1];
                rows_few(std::integral_constant<int, 1>{}, g_cur, row_a, tc, m, bj, pj, o);
                g_nxt[tc] = o[0];
            }
        } else if (m <= 2 * TC) {
            if (2 * tc < m) {
                float o[2];
                rows_few(std::integral_constant<int, 2>{}, g_cur, row_a, 2 * tc, m, bj, pj, o);
                *reinterpret_cast<float2 *>(g_nxt + 2 * tc) = make_float2(o[0], o[1]);
            }
        } else
        for (int i0 = 4 * tc; i0 < m; i0 += kStep) {
            float gw[4 * NW];
            load_window(g_cur + i0, gw);
            const float4 av = *reinterpret_cast<const float4 *>(row_a + i0);   // zeros past m
            const float ak[4] = {av.x, av.y, av.z, av.w};
            float o[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float acc = 0.0f;
#pragma unroll
                for (int j = 0; j < NBP; ++j) acc = __builtin_fmaf(gw[k + j], bj[j], acc);
                o[k] = i0 + k < m ? acc : 0.0f;
#pragma unroll
                for (int j = 0; j < NBP; ++j) pj[j] = __builtin_fmaf(gw[k + j], ak[k], pj[j]);
            }
            *reinterpret_cast<float4 *>(g_nxt + i0) = make_float4(o[0], o[1], o[2], o[3]);
        }
        if (m <= 2 * TC && tc < 4 && m + tc < ((m + 3) & ~3)) g_nxt[m + tc] = 0.0f;   // the narrow paths stop at m
        if (tc < HB / 4) *reinterpret_cast<float4 *>(g_nxt + ((m + 3) & ~3) + 4 * tc) = zero4;
        // Sum the NBR partial rows over the sample's lanes.  Two halving exchanges inside each quad (a lane keeps
        // half of the entries and hands the other half to its partner), then the quads of a row are added by
        // rotations of 4 and 8 lanes and the two rows by one shuffle: lane (b1, b0) ends with the totals of
        // entries H1 * b0 + H2 * b1 + [0, H2).
        {
            constexpr int H1 = NBR / 2, H2 = NBR / 4;
            const bool b0 = tc & 1, b1 = tc & 2;
            float w1[H1], w2[H2];
#pragma unroll
            for (int k = 0; k < H1; ++k) {
                const float lo = k < NBP ? pj[k < NBP ? k : 0] : 0.0f, hi = k + H1 < NBP ? pj[k + H1 < NBP ? k + H1 : 0] : 0.0f;
                w1[k] = (b0 ? hi : lo) + dpp<0xB1>(b0 ? lo : hi);            // partner: lane ^ 1
            }
#pragma unroll
            for (int k = 0; k < H2; ++k) {
                float x = (b1 ? w1[k + H2] : w1[k]) + dpp<0x4E>(b1 ? w1[k] : w1[k + H2]);   // partner: lane ^ 2
                x += dpp<0x124>(x);                                           // row_ror:4
                x += dpp<0x128>(x);                                           // row_ror:8
                if (TC == 32) x += __shfl_xor(x, 16, kWave);
                w2[k] = x;
            }
            // the stage's short row is spent: its gradient takes its place
            if (tc < 4) {
                float *dst = base + A.off_d + t * NBR + H1 * (tc & 1) + H2 * (tc >> 1);
#pragma unroll
                for (int k = 0; k < H2; ++k) dst[k] = w2[k];
            }
        }
        wave_lds_fence();
        float *sw = g_cur; g_cur = g_nxt; g_nxt = sw;
    }

    // ---- gradients out
    if (!live) return;
    {
        uint64_t dstp[kSlots];
        float v[kSlots];
#pragma unroll
        for (int x = 0; x < kSlots; ++x) {
            const int e = tc + TC * x, t = e / NBR, tt = t < kFoldMax ? t : 0;
            dstp[x] = tab_gin[tt];
            v[x] = slot_off[x] >= 0 ? base[A.off_d + e] : 0.0f;
        }
#pragma unroll
        for (int x = 0; x < kSlots; ++x)
            if (slot_off[x] >= 0 && dstp[x]) reinterpret_cast<float *>(dstp[x])[slot_off[x]] = v[x];
    }
    if (A.gin[0]) {
        float *dst = A.gin[0] + s * A.ld[0];
        const int m0 = stage(m_l, 0);
        for (int i = tc; i < m0; i += TC) dst[i] = g_cur[i];
    }
}

static int fold_padded_nb(int nb) { return nb <= 4 ? 4 : nb <= 8 ? 8 : nb <= 10 ? 10 : 16; }

}  // namespace dol

using namespace dol;

namespace {
struct FoldPlan {
    FoldArgs A;
    int nbp;
    bool wide;
    size_t lds;
    unsigned grid;
};
}  // namespace

// Checks the description and lays the sample region out in LDS.
static dol_status fold_prepare(const dol_fold *fold, FoldPlan &P)
{
    if (!fold) return fail(DOL_EINVAL, "fold is NULL");
    const int n = fold->n_inputs;
    if (n < 2 || n > kFoldMax) return fail(n < 2 ? DOL_EINVAL : DOL_EUNSUPPORTED, "n_inputs = %d outside 2..%d", n, kFoldMax);
    if (!fold->inputs || !fold->tables) return fail(DOL_EINVAL, "inputs or tables is NULL");
    FoldArgs &A = P.A;
    A = FoldArgs{};
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
    const int nbp = fold_padded_nb(max_nb);
    // Four columns per lane when its LDS layout fits, else one column per lane (both with 32 lanes per sample)
    const int lanes = 32;
    bool wide = true;
    size_t lds = 0;
    if (wide) {
        const int hb = (nbp + 2) / 4 * 4, nbr = (nbp + 3) / 4 * 4;
        int off = hb;
        for (int t = 0; t < n; ++t) { A.off[t] = off; off += ((A.m[t] + 3) & ~3) + hb; }
        A.off_d = off;
        off += n * nbr;
        const int g_len = ((A.m[n - 1] + 3) & ~3) + hb;
        A.off_g0 = off;
        A.off_g1 = off + g_len;
        off += 2 * g_len;
        A.stride = off;                              // a multiple of four floats
        const size_t head = sizeof(float) * (kFoldTabFloats + kFoldMax);
        lds = head + sizeof(float) * (kWave / lanes) * static_cast<size_t>(A.stride);
        if (lds > 64 * 1024) wide = false;
    }
    const int per_wave = wide ? kWave / lanes : 2;
    if (!wide) {
        const int H = nbp - 1;
        int off = H;
        for (int t = 0; t < n; ++t) { A.off[t] = off; off += A.m[t] + H; }
        A.off_d = off;
        off += n * nbp;
        const int g_len = A.m[n - 1] + nbp;
        A.off_g0 = off;
        A.off_g1 = off + g_len;
        off += 2 * g_len;
        A.stride = ((off + 31) / 64) * 64 + 32;     // the two samples of a wavefront use disjoint banks
        lds = sizeof(float) * 2 * static_cast<size_t>(A.stride);
    }
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
    P.nbp = nbp, P.wide = wide, P.lds = lds;
    P.grid = static_cast<unsigned>((static_cast<int64_t>(A.batch) + per_wave - 1) / per_wave);
    return DOL_OK;
}

extern "C" const char *dol_fold_kernel(const dol_fold *fold)
{
    static thread_local char name[64];
    FoldPlan P;
    if (fold_prepare(fold, P) != DOL_OK) return "";
    if (fold_chain_ok(P.A.n, P.A.m, P.A.nb, P.A.ld, P.A.ldo, P.A.ldg)) return "damp_fold_chain_kernel";
    if (P.wide) snprintf(name, sizeof name, "damp_fold4_kernel<%d, 32>", P.nbp);
    else snprintf(name, sizeof name, "damp_fold_kernel<%d>", P.nbp);
    return name;
}

extern "C" dol_status dol_fold_apply2(const dol_fold *fold, void *hip_stream)
{
    FoldPlan P;
    if (dol_status s = fold_prepare(fold, P)) return s;
    const FoldArgs &A = P.A;
    if (A.batch == 0) return DOL_OK;
    if (fold_chain_ok(A.n, A.m, A.nb, A.ld, A.ldo, A.ldg))      // the sweep written for this chain's shape
        return launch_fold_chain(A.n, A.m, A.nb, A.batch, A.in, A.ld, A.gin, A.out, A.ldo, A.target, A.gout, A.ldg, A.backward,
                                 static_cast<hipStream_t>(hip_stream));
    const unsigned grid = P.grid;
    const size_t lds = P.lds;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    if (P.wide) {
        switch (P.nbp) {
        case 4: hipLaunchKernelGGL((damp_fold4_kernel<4, 32>), dim3(grid), dim3(kWave), lds, st, A); break;
        case 8: hipLaunchKernelGGL((damp_fold4_kernel<8, 32>), dim3(grid), dim3(kWave), lds, st, A); break;
        case 10: hipLaunchKernelGGL((damp_fold4_kernel<10, 32>), dim3(grid), dim3(kWave), lds, st, A); break;
        default: hipLaunchKernelGGL((damp_fold4_kernel<16, 32>), dim3(grid), dim3(kWave), lds, st, A); break;
        }
    } else {
        switch (P.nbp) {
        case 4: hipLaunchKernelGGL(damp_fold_kernel<4>, dim3(grid), dim3(kWave), lds, st, A); break;
        case 8: hipLaunchKernelGGL(damp_fold_kernel<8>, dim3(grid), dim3(kWave), lds, st, A); break;
        case 10: hipLaunchKernelGGL(damp_fold_kernel<10>, dim3(grid), dim3(kWave), lds, st, A); break;
        default: hipLaunchKernelGGL(damp_fold_kernel<16>, dim3(grid), dim3(kWave), lds, st, A); break;
        }
    }
    DOL_HIP(hipGetLastError());
    return DOL_OK;
}
