// The fused left fold of convolution-shaped DAMP applies (the loop of Fig. 2, forward + loss gradient + reverse sweep
// in one launch) as code written for the chain's shape.
//
// The symbol side of a fold is known before any tag is touched (Sec. 3.1.2): the number of inputs and the symbol
// counts of every stage.  With those as compile-time constants the whole sweep unrolls: 16 lanes own a sample, a
// wavefront four, and in every stage a lane owns a CONTIGUOUS block of output columns (rows, in the reverse sweep)
// sized to the stage, so that
//   - the operand window of a block slides through registers: w + nb - 1 LDS reads feed w * nb multiply-adds;
//   - no lane idles in a narrow stage and no stage pays for a fixed four-column granularity;
//   - every LDS offset is an immediate, every loop is gone.
// The reverse sweep needs every running Distribution again, but a lane needs exactly the block it computed itself.  Two
// forms of the code: every Distribution keeps a row of its own in the sample's LDS region (7.8 KB per sample for Sum-15),
// or the blocks stay in their lanes' registers (63 per lane) and LDS holds two row buffers, the one a stage reads and the
// one it writes (3.4 KB per sample, a dozen wavefronts on a compute unit instead of five); the launcher picks by the size
// of the grid.  Beside the rows the region holds the short inputs and two gradient rows.
// A stage's result is kept as x = pre where pre <= 1 and -1 where the
// clamp acted: |x| is the tag (the absolute value is free in a multiply-add) and the sign is the clamp's decision, read
// by the reverse sweep with the operand it needs anyway - no stage is ever summed twice.
//
// Arithmetic is that of dol_apply2 / dol_backward: out[c] = min(1, sum over ascending i of a[i] * b[c - i]), one
// fused multiply-add per tuple from 0; gradients gated by [pre <= 1].  The gradient of a short operand is a sum over
// the sample's 16 lanes per symbol: the lanes share the symbols out while they exchange (emit_scattered_sums), every
// total ends in the lanes that store it, and the row leaves with one LDS write.
#include "internal.h"

#include <cstdarg>
#include <map>
#include <mutex>

namespace dol {

namespace {

// Lanes per sample: 16, four samples per wavefront.  (32 lanes per sample - two wavefronts per SIMD at B=4096 instead
// of one - was measured: 18.8 us against 16.4; the generator still takes the width as a parameter.)
constexpr int kLanes = 16;
constexpr int kNBR = 16;                // floats reserved per short input row
constexpr size_t kChainLdsMax = 40 * 1024;   // per wavefront: at least four wavefronts per compute unit
// From this many workgroups on, the form with the reverse sweep's operands in registers: less than half the LDS, so a
// dozen wavefronts per compute unit instead of five (Sum-15: 18.2 against 25.7 us at 2048 workgroups, 224 against 307 us
// at 32768).  Below, with one wavefront per SIMD, the form with every row in LDS is the faster one (12.6 against 13.3 us
// at 1024 workgroups).
constexpr int64_t kRegsFromWorkgroups = 1536;

struct Src {
    std::string s;
    void operator()(const char *fmt, ...) __attribute__((format(printf, 2, 3)))
    {
        char buf[1024];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        s += buf;
    }
};

struct Layout {
    int n = 0;
    int m[kFoldChainMax] = {}, nb[kFoldChainMax] = {};
    int w[kFoldChainMax] = {};          // columns of acc_t per lane
    int off[kFoldChainMax] = {};        // first value of acc_t inside a sample's region (in row buffer t & 1)
    int ext[kFoldChainMax] = {};        // entries of acc_t's row that are read (values, then zeros)
    int buf = 0;                        // floats of one of the two row buffers
    int off_d = 0, off_g0 = 0, off_g1 = 0, g_len = 0, stride = 0;
};

int ceil_div(int a, int b) { return (a + b - 1) / b; }

// regs: the reverse sweep's operands stay in the registers of the lanes that computed them and LDS holds two row buffers;
// otherwise every running Distribution keeps a row of its own in LDS.
Layout lay_out(const std::vector<int> &shape, int kL, bool regs)
{
    Layout Y;
    Y.n = shape[0];
    Y.m[0] = shape[1];
    for (int t = 1; t < Y.n; ++t) {
        Y.nb[t] = shape[1 + t];
        Y.m[t] = Y.m[t - 1] + Y.nb[t] - 1;
        Y.w[t] = ceil_div(Y.m[t], kL);
    }
    Y.w[0] = ceil_div(Y.m[0], kL);
    int pos = 0;
    if (regs) {
        // Two row buffers: acc_t lives in buffer t & 1 while the next stage reads it.  A buffer holds a zero halo in front
        // (the next stage reads nb - 1 entries before the row) and the widest extent any stage writes or reads.  Rows only
        // grow, so what a buffer holds beyond the row it carries is an earlier, shorter row's zeros.
        int halo = 0, extent = 0;
        for (int t = 0; t < Y.n; ++t) {
            if (t + 1 < Y.n) halo = std::max(halo, Y.nb[t + 1] - 1);
            int ext = std::max(Y.m[t], t >= 1 ? kL * Y.w[t] : 0);    // a stage writes whole blocks
            if (t + 1 < Y.n) ext = std::max(ext, kL * Y.w[t + 1]);   // and the next one reads whole blocks
            Y.ext[t] = ext;
            extent = std::max(extent, ext);
        }
        Y.buf = halo + extent;
        for (int t = 0; t < Y.n; ++t) Y.off[t] = (t & 1) * Y.buf + halo;
        pos = 2 * Y.buf;
    } else {
        for (int t = 0; t < Y.n; ++t) {
            const int halo = t + 1 < Y.n ? Y.nb[t + 1] - 1 : 0;       // the next stage reads nb - 1 entries before the row
            int ext = std::max(Y.m[t], t >= 1 ? kL * Y.w[t] : 0);    // a stage writes whole blocks
            if (t + 1 < Y.n) ext = std::max(ext, kL * Y.w[t + 1]);   // and the next one reads whole blocks
            Y.off[t] = pos + halo;
            Y.ext[t] = ext;
            pos = Y.off[t] + ext;
        }
    }
    Y.off_d = pos;
    pos += Y.n * kNBR;
    int g_len = Y.m[Y.n - 1];
    for (int t = 1; t < Y.n; ++t) g_len = std::max(g_len, kL * ceil_div(Y.m[t - 1], kL) + Y.nb[t] - 1);
    Y.g_len = g_len;
    Y.off_g0 = pos;
    Y.off_g1 = pos + g_len;
    pos += 2 * g_len;
    Y.stride = pos | 1;                 // odd: the samples of a wavefront start in different banks
    return Y;
}

// lanes 0 .. len-1 of every sample (in turns of kL) write zero to region[start ..]
void emit_zero(Src &o, int start, int len, int kL)
{
    for (int x = 0; x < len; x += kL) {
        if (len - x >= kL) o("  base[%d + l] = 0.0f;\n", start + x);
        else o("  if (l < %d) base[%d + l] = 0.0f;\n", len - x, start + x);
    }
}

// Sums of the n values s0 .. s<n-1> over the 16 lanes of a sample, each total ending in some lanes' s0: the four exchange
// steps pair a lane with the lane whose number differs by 15, 7, 2 and 1 (together these reach all 16), and in every step
// the two lanes of a pair share the values out - the one with the step's bit clear goes on with the first half, the other
// with the second half, an odd value out with both - so a step costs three instructions per two values instead of two
// per value.  which_sum(n) is the index of the total a lane ends up with, as an expression in l.
void emit_scattered_sums(Src &o, int n)
{
    static const int which[4] = {3, 2, 1, 0}, bit[4] = {8, 4, 2, 1};
    for (int st = 0; st < 4; ++st) {
        const int h = n / 2;
        for (int k = 0; k < h; ++k) {
            o("    { const float lo = s%d + dppx(s%d, %d), hi = s%d + dppx(s%d, %d); s%d = (l & %d) ? hi : lo; }\n", k, k, which[st], k + h, k + h,
              which[st], k, bit[st]);
        }
        if (n & 1) {
            if (h > 0) o("    s%d = s%d + dppx(s%d, %d);\n", h, n - 1, n - 1, which[st]);
            else o("    s0 += dppx(s0, %d);\n", which[st]);
        }
        n = h + (n & 1);
    }
}

std::string which_sum(int n)
{
    static const int bit[4] = {8, 4, 2, 1};
    std::vector<std::string> e(n);
    for (int j = 0; j < n; ++j) e[j] = std::to_string(j);
    for (int st = 0; st < 4; ++st) {
        const int h = n / 2;
        std::vector<std::string> f;
        for (int k = 0; k < h; ++k) f.push_back("((l & " + std::to_string(bit[st]) + ") ? " + e[k + h] + " : " + e[k] + ")");
        if (n & 1) f.push_back(e[n - 1]);
        e = f;
        n = h + (n & 1);
    }
    return e[0];
}

std::string chain_source(const std::vector<int> &shape, int kL, bool regs)
{
    const int kSP = 64 / kL;
    const Layout Y = lay_out(shape, kL, regs);
    const int n = Y.n, n1 = n - 1;
    Src o;
    o("typedef unsigned long long u64;\n");
    // (leading dimensions as 32-bit words: a row's offset is then one 32 x 32 -> 64 bit multiply-add)
    o("struct Args { int batch; int backward; const float *in[%d]; int ld[%d]; float *gin[%d]; float *out; int ldo; "
      "const int *target; const float *gout; int ldg; };\n", kFoldChainMax, kFoldChainMax, kFoldChainMax);
    o("__device__ __forceinline__ void fence() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, \"wavefront\"); __builtin_amdgcn_wave_barrier(); "
      "__builtin_amdgcn_fence(__ATOMIC_ACQUIRE, \"wavefront\"); }\n");
    o("__device__ __forceinline__ float dppx(float x, int which) {\n"
      "  switch (which) {\n"
      "  case 0: return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xF, 0xF, false));\n"
      "  case 1: return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xF, 0xF, false));\n"
      "  case 2: return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xF, 0xF, false));\n"
      "  default: return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xF, 0xF, false)); } }\n");
    // sum over the lanes of a sample: butterflies inside a row of 16 lanes; for 32 lanes the first row's total then joins
    // the second row's (row_bcast:15 into rows 1 and 3), whose lanes hold the sample's total
    o("__device__ __forceinline__ float sum_lanes(float x) { x += dppx(x, 0); x += dppx(x, 1); x += dppx(x, 2); x += dppx(x, 3);\n");
    if (kL == 32) o("  x += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x142, 0xA, 0xF, false));\n");
    o("  return x; }\n");
    o("extern \"C\" __global__ void __launch_bounds__(64) damp_fold_chain_kernel(const Args A)\n{\n");
    o("  __shared__ float lds[%d];\n", kSP * Y.stride);
    o("  const int lane = threadIdx.x, l = lane & %d, q = lane >> %d;\n", kL - 1, kL == 16 ? 4 : 5);
    // workgroups are dealt round-robin to the 8 XCDs: give every XCD a contiguous range of samples
    o("  const unsigned id = blockIdx.x, nwg = gridDim.x, xcd = id & 7u, per = nwg >> 3, rem = nwg & 7u;\n");
    o("  const long long wg = (long long)(xcd * per + (xcd < rem ? xcd : rem) + (id >> 3));\n");
    o("  const long long s_raw = wg * %d + q;\n  const bool live = s_raw < A.batch;\n  const int s = (int)(live ? s_raw : A.batch - 1);\n", kSP);
    o("  float *base = lds + q * %d;\n", Y.stride);
    // A stage's rows are addressed through an index the compiler cannot see through: every access of the stage is
    // then that register plus a small immediate (one instruction), where a folded constant beyond the reach of the
    // two-word LDS instructions' offset field would cost an address addition per access.
    o("  const int qb = q * %d;\n", 4 * Y.stride);
    {
        bool used[64] = {};
        used[0] = true;
        for (int t = 1; t < n; ++t) { used[Y.w[t]] = true; used[ceil_div(Y.m[t - 1], kL)] = true; }
        for (int x = 0; x < 64; ++x)
            if (used[x]) o("  const int lw%d = l * %d;\n", x, 4 * x);
        if (kL == 16) {     // which of a short operand's gradient sums a lane ends up with (see emit_scattered_sums)
            bool len[kNBR + 1] = {};
            for (int t = 1; t < n; ++t)
                if (!len[Y.nb[t]]) { len[Y.nb[t]] = true; o("  const int jl%d = %s;\n", Y.nb[t], which_sum(Y.nb[t]).c_str()); }
        }
    }
    o("#define DOL_ROW(name, start, step) int name##_i = qb + 4 * (start) + lw##step; asm volatile(\"\" : \"+v\"(name##_i)); "
      "float *name = reinterpret_cast<float *>(reinterpret_cast<char *>(lds) + name##_i)\n");
    if (regs) {
        // ---- both row buffers start as zeros (halos, and whatever lies beyond a row)
        emit_zero(o, 0, 2 * Y.buf, kL);
    } else {
        // ---- zeros where a window may reach beyond what is written
        int pos = 0;
        for (int t = 0; t < n; ++t) {
            emit_zero(o, pos, Y.off[t] - pos, kL);                       // the halo in front of the row
            if (t == 0) emit_zero(o, Y.off[0] + Y.m[0], Y.ext[0] - Y.m[0], kL);
            else if (Y.ext[t] > kL * Y.w[t]) emit_zero(o, Y.off[t] + kL * Y.w[t], Y.ext[t] - kL * Y.w[t], kL);
            pos = Y.off[t] + Y.ext[t];
        }
    }
    // ---- inputs: all loads first, then the LDS writes
    {
        int slot = 0;
        for (int t = 0; t < n; ++t) {
            const int cnt = t == 0 ? Y.m[0] : Y.nb[t];
            for (int x = 0; x < kSP * cnt; x += 64, ++slot) {
                o("  float in%d = 0.0f; { const int e = lane + %d; if (e < %d) { const int qq = e / %d, i = e - qq * %d; long long sr = wg * %d + qq; "
                  "const int ss = (int)(sr < A.batch ? sr : A.batch - 1); in%d = A.in[%d][(long long)ss * A.ld[%d] + i]; } }\n", slot, x, kSP * cnt, cnt, cnt, kSP, slot, t, t);
            }
        }
        slot = 0;
        for (int t = 0; t < n; ++t) {
            const int cnt = t == 0 ? Y.m[0] : Y.nb[t];
            const int dst = t == 0 ? Y.off[0] : Y.off_d + t * kNBR;
            for (int x = 0; x < kSP * cnt; x += 64, ++slot)
                o("  { const int e = lane + %d; if (e < %d) { const int qq = e / %d, i = e - qq * %d; lds[qq * %d + %d + i] = in%d; } }\n", x, kSP * cnt,
                  cnt, cnt, Y.stride, dst, slot);
        }
    }
    o("  fence();\n");
    // ---- a lane's own block of every running Distribution stays in registers for the reverse sweep (sign = clamp decision)
    if (regs) {
        for (int k = 0; k < Y.w[0]; ++k) o("  const float h0_%d = base[%d + l * %d + %d];\n", k, Y.off[0], Y.w[0], k);
        for (int t = 1; t < n; ++t)
            for (int k = 0; k < Y.w[t]; ++k) o("  float h%d_%d;\n", t, k);
    }
    // ---- forward sweep
    for (int t = 1; t < n; ++t) {
        const int nb = Y.nb[t], w = Y.w[t], win = w + nb - 1;
        o("  {\n    DOL_ROW(rp, %d, %d); DOL_ROW(dp, %d, 0);\n", Y.off[t - 1] - (nb - 1), w, Y.off_d + t * kNBR);
        for (int j = 0; j < nb; ++j) o("    const float d%d = dp[%d];\n", j, j);
        for (int k = 0; k < win; ++k) o("    const float r%d = __builtin_fabsf(rp[%d]);\n", k, k);
        for (int k = 0; k < w; ++k) {
            // column c = l * w + k: ascending i = c - j, one fma per tuple
            o("    float p%d = 0.0f;\n", k);
            for (int j = nb - 1; j >= 0; --j) o("    p%d = __builtin_fmaf(r%d, d%d, p%d);\n", k, k + (nb - 1) - j, j, k);
        }
        o("    DOL_ROW(wp, %d, %d);\n", Y.off[t], w);
        for (int k = 0; k < w; ++k) {
            if (regs) o("    h%d_%d = p%d <= 1.0f ? p%d : -1.0f; wp[%d] = h%d_%d;\n", t, k, k, k, k, t, k);
            else o("    wp[%d] = p%d <= 1.0f ? p%d : -1.0f;\n", k, k, k);
        }
        o("  }\n  fence();\n");
    }
    // ---- the result
    o("  if (A.out && live) { float *os = A.out + (long long)s * A.ldo;\n");
    for (int x = 0; x < Y.m[n1]; x += kL)
        o("    %s os[%d + l] = __builtin_fabsf(base[%d + l]);\n", Y.m[n1] - x >= kL ? "" : (std::string("if (l < ") + std::to_string(Y.m[n1] - x) + ")").c_str(),
          x, Y.off[n1] + x);
    o("  }\n  if (!A.backward) return;\n");
    // ---- upstream gradient into the first gradient row, gated by the last stage's clamp.  With a target the row is
    // zero but for one entry, which one lane works out (one division per sample instead of one per column)
    o("  if (A.target) {\n");
    for (int x = 0; x < Y.g_len; x += kL)
        o("    %sbase[%d + l] = 0.0f;\n", Y.g_len - x >= kL ? "" : (std::string("if (l < ") + std::to_string(Y.g_len - x) + ") ").c_str(), Y.off_g0 + x);
    o("    const int tgt = A.target[s];\n");
    o("    if (l == 0 && tgt >= 0 && tgt < %d) { const float xv = base[%d + tgt];\n", Y.m[n1], Y.off[n1]);
    o("      base[%d + tgt] = xv < 0.0f ? 0.0f : -1.0f / fmaxf(xv, 1.17549435e-38f); }\n", Y.off_g0);
    o("  } else { const float *gs = A.gout + (long long)s * A.ldg;\n");
    for (int x = 0; x < Y.g_len; x += kL) {
        const bool whole = Y.g_len - x >= kL;
        o("    %s{ const int c = %d + l; float gv = 0.0f;\n", whole ? "" : (std::string("if (l < ") + std::to_string(Y.g_len - x) + ") ").c_str(), x);
        if (x < Y.m[n1]) {
            o("      if (c < %d) { const float xv = base[%d + c];\n", Y.m[n1], Y.off[n1]);
            o("        gv = xv < 0.0f ? 0.0f : gs[c]; }\n");
        }
        o("      base[%d + c] = gv; }\n", Y.off_g0);
    }
    o("  }\n  fence();\n");
    // ---- reverse sweep
    for (int t = n1; t >= 1; --t) {
        const int nb = Y.nb[t], m = Y.m[t - 1], v = ceil_div(m, kL), win = v + nb - 1;
        const int g_cur = (n1 - t) & 1 ? Y.off_g1 : Y.off_g0, g_nxt = (n1 - t) & 1 ? Y.off_g0 : Y.off_g1;
        o("  {\n    DOL_ROW(gp, %d, %d); DOL_ROW(dp, %d, 0);\n", g_cur, v, Y.off_d + t * kNBR);
        if (!regs) o("    DOL_ROW(ap, %d, %d);\n", Y.off[t - 1], v);
        for (int j = 0; j < nb; ++j) o("    const float d%d = dp[%d];\n", j, j);
        for (int k = 0; k < win; ++k) o("    const float g%d = gp[%d];\n", k, k);
        for (int k = 0; k < v; ++k) {
            if (regs) o("    const float x%d = h%d_%d;\n", k, t - 1, k);
            else o("    const float x%d = ap[%d];\n", k, k);
        }
        for (int j = 0; j < nb; ++j) o("    float s%d = 0.0f;\n", j);
        o("    DOL_ROW(wp, %d, %d);\n", g_nxt, v);
        for (int k = 0; k < v; ++k) {
            o("    { float acc = 0.0f;\n");
            for (int j = 0; j < nb; ++j) o("      acc = __builtin_fmaf(g%d, d%d, acc);\n", k + j, j);
            // rows past the operand's last symbol hold 0; a row whose own sum was clamped (sign) passes no gradient on
            // (only the last lanes' last rows can lie past the end: the test is written where that can happen)
            const bool past = (kL - 1) * v + k >= m;
            if (t > 1 && past) o("      wp[%d] = (l * %d + %d < %d && !(x%d < 0.0f)) ? acc : 0.0f;\n", k, v, k, m, k);
            else if (t > 1) o("      wp[%d] = !(x%d < 0.0f) ? acc : 0.0f;\n", k, k);
            else if (past) o("      wp[%d] = l * %d + %d < %d ? acc : 0.0f;\n", k, v, k, m);
            else o("      wp[%d] = acc;\n", k);
            for (int j = 0; j < nb; ++j) o("      s%d = __builtin_fmaf(g%d, __builtin_fabsf(x%d), s%d);\n", j, k + j, k, j);
            o("    }\n");
        }
        // the next stage's windows reach past the rows just written: zeros there
        if (t > 1) {
            const int need = kL * ceil_div(Y.m[t - 2], kL) + Y.nb[t - 1] - 1, have = kL * v;
            for (int x = have; x < need; x += kL)
                o("    %s base[%d + l] = 0.0f;\n", need - x >= kL ? "" : (std::string("if (l < ") + std::to_string(need - x) + ")").c_str(), g_nxt + x);
        }
        // the short operand's gradient: sum of the lanes' shares; it takes the place of the operand's row, which is spent
        // (the empty asm keeps the last addition in front of the branch, where it takes its operand straight from the
        // other lane; inside the branch, with one lane live, it would need a separate move)
        if (kL == 32) {
            for (int j = 0; j < nb; ++j) o("    s%d = sum_lanes(s%d); asm volatile(\"\" : \"+v\"(s%d));\n", j, j, j);
            o("    if (l == 16) {\n");
            for (int j = 0; j < nb; ++j) o("      dp[%d] = s%d;\n", j, j);
            o("    }\n  }\n  fence();\n");
        } else {
            emit_scattered_sums(o, nb);
            o("    dp[jl%d] = s0;\n  }\n  fence();\n", nb);
        }
    }
    // ---- gradients out
    o("  if (!live) return;\n");
    {
        const int g_fin = (n1 & 1) ? Y.off_g1 : Y.off_g0;        // after n - 1 swaps
        o("  if (A.gin[0]) { float *dst = A.gin[0] + (long long)s * A.ld[0];\n");
        for (int x = 0; x < Y.m[0]; x += kL)
            o("    %s dst[%d + l] = base[%d + l];\n", Y.m[0] - x >= kL ? "" : (std::string("if (l < ") + std::to_string(Y.m[0] - x) + ")").c_str(), x,
              g_fin + x);
        o("  }\n");
        for (int t = 1; t < n; ++t)
            o("  if (A.gin[%d] && l < %d) A.gin[%d][(long long)s * A.ld[%d] + l] = base[%d + l];\n", t, Y.nb[t], t, t, Y.off_d + t * kNBR);
    }
    o("}\n");
    return o.s;
}

struct ChainKernel {
    hipModule_t mod = nullptr;
    hipFunction_t fn = nullptr;
    dol_status status = DOL_OK;
};

struct ChainArgs {
    int32_t batch, backward;
    const float *in[kFoldChainMax];
    int32_t ld[kFoldChainMax];
    float *gin[kFoldChainMax];
    float *out;
    int32_t ldo;
    const int32_t *target;
    const float *gout;
    int32_t ldg;
};

}  // namespace

bool fold_chain_ok(int n, const int32_t *m, const int32_t *nb, const int64_t *ld, int64_t ldo, int64_t ldg)
{
    if (n < 2 || n > kFoldChainMax) return false;
    for (int t = 0; t < n; ++t)
        if (ld[t] > INT32_MAX) return false;
    if (ldo > INT32_MAX || ldg > INT32_MAX) return false;
    std::vector<int> shape{n, m[0]};
    for (int t = 1; t < n; ++t) {
        if (nb[t] < 1 || nb[t] > kNBR) return false;
        shape.push_back(nb[t]);
    }
    if (m[0] < 1 || m[0] > 256) return false;
    const Layout Y = lay_out(shape, kLanes, false);
    return sizeof(float) * (64 / kLanes) * static_cast<size_t>(Y.stride) <= kChainLdsMax;
}

dol_status launch_fold_chain(int n, const int32_t *m, const int32_t *nb, int32_t batch, const float *const *in, const int64_t *ld,
                             float *const *gin, float *out, int64_t ldo, const int32_t *target, const float *gout, int64_t ldg,
                             int32_t backward, hipStream_t st)
{
    static std::mutex mu;
    static std::map<std::pair<int, std::vector<int>>, ChainKernel> cache;    // per device, shape and lanes per sample; lives until the process ends
    std::vector<int> shape{n, m[0]};
    for (int t = 1; t < n; ++t) shape.push_back(nb[t]);
    const int kL = kLanes, kSP = 64 / kL;
    const bool regs = (static_cast<int64_t>(batch) + kSP - 1) / kSP >= kRegsFromWorkgroups;
    int dev = 0;
    DOL_HIP(hipGetDevice(&dev));
    hipFunction_t fn = nullptr;
    {
        std::lock_guard<std::mutex> lock(mu);
        std::vector<int> keyed(shape);
        keyed.push_back(kL);
        keyed.push_back(regs ? 1 : 0);
        auto key = std::make_pair(dev, keyed);
        auto it = cache.find(key);
        if (it == cache.end()) {
            ChainKernel k;
            k.status = jit_compile(chain_source(shape, kL, regs), "damp_fold_chain_kernel", &k.mod, &k.fn);
            it = cache.emplace(key, k).first;
            if (k.status != DOL_OK) return k.status;                        // with the compiler's message
        } else if (it->second.status != DOL_OK) {
            return fail(it->second.status, "the code of this fold did not build (see the first call's message)");
        }
        fn = it->second.fn;
    }
    ChainArgs A{};
    A.batch = batch, A.backward = backward;
    for (int t = 0; t < n; ++t) { A.in[t] = in[t]; A.ld[t] = static_cast<int32_t>(ld[t]); A.gin[t] = gin ? gin[t] : nullptr; }
    A.out = out, A.ldo = static_cast<int32_t>(ldo), A.target = target, A.gout = gout, A.ldg = static_cast<int32_t>(ldg);
    void *args[] = {&A};
    const unsigned grid = static_cast<unsigned>((static_cast<int64_t>(batch) + kSP - 1) / kSP);
    DOL_HIP(hipModuleLaunchKernel(fn, grid, 1, 1, 64, 1, 1, 0, st, args, nullptr));
    return DOL_OK;
}

}  // namespace dol
