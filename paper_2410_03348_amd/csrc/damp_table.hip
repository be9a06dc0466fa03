// DAMP apply2 for small arbitrary (hashed, dense or sparse) function tables, as code written for the table.
//
//     out[s, c] = min(1, sum over the tuples (i, j) of column c, ascending (i, j), of a[s, i] * b[s, j])
//     ga[s, i]  = sum_j gh[s, col(i, j)] * b[s, j],    gb[s, j] = sum_i gh[s, col(i, j)] * a[s, i]
//
// The symbol side is batch-invariant (Sec. 3.1.2: the user function is evaluated once, before any tag is touched),
// so with one sample per lane every tuple index is the same for all 64 lanes of a wavefront.  A table whose operand
// rows fit in registers (at most 64 symbols each) is therefore compiled, once per table and on its first use, into
// straight-line code: the operand rows of a lane's sample sit in registers and every tuple is ONE fused multiply-add
// on named registers - no index loads, no operand gathers.  (A generic kernel has to fetch both operands of every
// tuple from LDS, 8 bytes per multiply-add, and stops at the rate of the LDS pipe; see damp_lds.hip, which still
// serves larger tables and padded or unaligned tensors.)  A column's tuples keep their ascending (i, j) order and
// start from 0, so the sum is bit for bit the one dol_apply2 defines and the clamp decisions agree.
//
// Layout of a launch: a workgroup of four wavefronts owns a tile of 64 samples (batches too small to give every compute
// unit two such tiles: eight wavefronts, or tiles of 32 samples; see build_for).  The tile's operand rows travel
// HBM -> LDS with flat 16-byte loads (rows padded to a pitch of n + 4 floats, which keeps a lane's 16-byte reads of
// its own row off its neighbours' banks), each lane pulls its sample's rows into registers, the wavefronts split
// the work (forward: 64 output columns at a time each; backward: half of the rows of one operand each), results go back
// through LDS and leave as flat 16-byte stores.
//
// Backward needs gh = g * [pre <= 1].  For tags in [0, 1] a column's sum is bounded by max(a) * sum(b) * M, M = the
// most tuples of one column that share a second-operand symbol (and the same with the operands' roles swapped): a
// tile whose samples all stay below 0.9999 by that bound cannot hold a clamped column and passes g through without
// ever reading the forward result; any other tile recomputes pre with the forward code and gates with it.
//
// Merged forms (dol_apply2_filter_union and its reverse): the same kernels with Filter and Union folded into their
// epilogues, so the Apply's result never leaves the chip; the forward pass leaves one word per sample saying whether
// any clamp acted, and the reverse pass re-derives decisions only for tiles that hold such a sample.  The two merged
// bodies are also emitted as device functions of one kernel (dol_apply2_filter_union_forward_backward).
#include "internal.h"

#include <hip/hiprtc.h>

#include <cstdarg>
#include <mutex>

namespace dol {

constexpr int kJitTile = 64;            // samples per tile = lanes per wavefront
constexpr int kJitWavesLarge = 4;       // wavefronts per workgroup: four, or eight in the builds for small batches
constexpr int kJitGroup = 64;           // output columns a wavefront takes at a time
constexpr int kJitMaxSym = 64;          // operand rows live in registers
constexpr int kJitMaxOut = 1024;
constexpr int kJitMaxMergeOut = 512;   // merged launches keep the Apply's whole result tile in LDS
constexpr int64_t kJitMaxTuples = 16384;

// (the last two: merged launches whose filter-union plan is `aligned`, see UnionPlan)
enum { kSlotFwd = 0, kSlotBwd = 1, kSlotMergeFwd = 2, kSlotMergeBwd = 3, kSlotMergeFwdAligned = 4, kSlotMergeBwdAligned = 5, kSlotMergeBoth = 6,
       kSlotMergeBothAligned = 7, kSlots = 8 };

struct JitState {
    std::mutex mu;
    hipModule_t mod[3 * kSlots] = {};        // (a table has up to three builds of each kernel, see build_for)
    hipFunction_t fn[3 * kSlots] = {};
    dol_status status[3 * kSlots] = {};
    bool tried[3 * kSlots] = {};
    ~JitState()
    {
        for (hipModule_t m : mod)
            if (m) (void)hipModuleUnload(m);
    }
};

void JitDeleter::operator()(JitState *p) const { delete p; }

bool table_code_ok(const dol_fn_table *f)
{
    return f->na >= 4 && f->nb >= 4 && f->n_out >= 4 && f->na <= kJitMaxSym && f->nb <= kJitMaxSym && f->n_out <= kJitMaxOut &&
           !((f->na | f->nb | f->n_out) & 3) && f->n_tuples > 0 && f->n_tuples <= kJitMaxTuples && !f->h_col_ptr.empty();
}

namespace {

struct Src {
    std::string s;
    void operator()(const char *fmt, ...) __attribute__((format(printf, 2, 3)))
    {
        char buf[768];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        s += buf;
    }
};

// Wavefronts per workgroup and samples per tile of the source being written.
thread_local int t_waves = kJitWavesLarge, t_tile_rows = kJitTile;
#define kJitWaves t_waves
#define kThreads (kJitTile * t_waves)

// Declares r0 .. r{n-1} and fills them from the lane's row of the staged tile (pitch n + 4 floats).
void emit_row_to_regs(Src &o, const char *r, const char *tile, int n)
{
    for (int i = 0; i < n; i += 4)
        o("  float %s%d, %s%d, %s%d, %s%d; { const float4 t = *reinterpret_cast<const float4 *>(%s + lane * %d + %d); %s%d = t.x; %s%d = t.y; "
          "%s%d = t.z; %s%d = t.w; }\n", r, i, r, i + 1, r, i + 2, r, i + 3, tile, n + 4, i, r, i, r, i + 1, r, i + 2, r, i + 3);
}

// Flat copy of a tile of `valid` rows of n floats from memory into LDS rows of pitch n + 4: the loads of all pieces
// of a thread first (into t<tag>_*), the LDS writes in a second step so that several tiles' loads can be in flight.
void emit_stage_load(Src &o, const char *tag, const char *src_ptr, int n)
{
    const int per_thread = (kJitTile * n / 4 + kThreads - 1) / kThreads;
    for (int x = 0; x < per_thread; ++x) o("  float4 ld%s%d;\n", tag, x);
    o("  { const float4 *g4 = reinterpret_cast<const float4 *>(%s + s0 * %d);\n", src_ptr, n);
    for (int x = 0; x < per_thread; ++x)
        o("    { const int q = tid + %d; ld%s%d = g4[q < valid * %d ? q : valid * %d - 1]; }\n", kThreads * x, tag, x, n / 4, n / 4);
    o("  }\n");
}

void emit_stage_store(Src &o, const char *tag, const char *dst, int n)
{
    const int per_thread = (kJitTile * n / 4 + kThreads - 1) / kThreads;
    for (int x = 0; x < per_thread; ++x)
        o("  { const int q = tid + %d; %s{ const int s = q / %d, k = q - s * %d; *reinterpret_cast<float4 *>(%s + s * %d + 4 * k) = ld%s%d; } }\n",
          kThreads * x, kThreads * (x + 1) <= kJitTile * n / 4 ? "" : (std::string("if (q < ") + std::to_string(kJitTile * n / 4) + ") ").c_str(), n / 4, n / 4,
          dst, n + 4, tag, x);
}

// The forward sums of the columns [c0, c1): declares p<c> and leaves the unclamped sum in it.
void emit_columns(Src &o, const dol_fn_table *f, int c0, int c1, const char *indent)
{
    for (int c = c0; c < c1; ++c) {
        o("%sfloat p%d = 0.0f;\n", indent, c);
        for (uint32_t q = f->h_col_ptr[c]; q < f->h_col_ptr[c + 1]; ++q)
            o("%sp%d = __builtin_fmaf(a%u, b%u, p%d);\n", indent, c, f->h_col_ij[q] & 0xffffu, f->h_col_ij[q] >> 16, c);
    }
}

const char *kPrologue =
    "typedef unsigned int u32;\n"
    "__device__ __forceinline__ void wave_lds_fence() {\n"
    "  __builtin_amdgcn_fence(__ATOMIC_RELEASE, \"wavefront\"); __builtin_amdgcn_wave_barrier(); __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, \"wavefront\"); }\n";

void emit_tile_head(Src &o)
{
    // (one tile per workgroup: inside a loop over tiles the compiler keeps every thread-constant offset of the body alive
    // across it, in registers the body needs)
    o("  {\n  const int tile = blockIdx.x;\n");
    o("  const long long s0 = (long long)tile * %d;\n  const int valid = batch - s0 < %d ? (int)(batch - s0) : %d;\n", t_tile_rows, t_tile_rows, t_tile_rows);
}

// Forward.  merged: the kept symbols of the result are merged with a third Distribution c in the same launch
// (out = union(filter(apply2(a, b)), c)); the Apply's own result then lives in LDS only.
// (body: a device function over an LDS array handed in, for the kernel that runs both passes; returns its LDS floats in *lds_floats)
std::string forward_source(const dol_fn_table *f, bool merged, bool aligned = false, bool body = false, int *lds_floats = nullptr)
{
    const int na = f->na, nb = f->nb, S = f->n_out;
    const int pa = na + 4, pb = nb + 4;
    const int fcols = kJitGroup * kJitWavesLarge / kJitWaves;       // columns a wavefront takes at a time: 64, or 32 of eight wavefronts
    const int po = merged ? S + 4 : fcols + 4;         // pitch of the result stage: the whole tile, or a wavefront's columns
    const int in_floats = kJitTile * (pa + pb), out_floats = merged ? kJitTile * po : kJitWaves * kJitTile * po;
    const int stage_floats = std::max(in_floats, out_floats);
    Src o;
    if (!body) o.s = kPrologue;
    if (lds_floats) *lds_floats = stage_floats + (merged ? kJitTile : 0);
    if (body)
        o("static __device__ __forceinline__ void damp_table_merge_fwd_body(float *lds, const float *__restrict__ a, const float *__restrict__ b, "
          "const float *__restrict__ c, float *__restrict__ out, const int *__restrict__ ia, const int *__restrict__ ib, int *saved, "
          "int batch, int n_tiles, int nc, int n3)\n{\n");
    else if (merged)
        o("extern \"C\" __global__ void __launch_bounds__(%d) __attribute__((amdgpu_waves_per_eu(2, 2))) damp_table_merge_fwd_kernel(const float *__restrict__ a, const float *__restrict__ b, "
          "const float *__restrict__ c, float *__restrict__ out, const int *__restrict__ ia, const int *__restrict__ ib, int *__restrict__ saved, "
          "int batch, int n_tiles, int nc, int n3)\n{\n", kThreads);
    else
        o("extern \"C\" __global__ void __launch_bounds__(%d) __attribute__((amdgpu_waves_per_eu(2, 2))) damp_table_fwd_kernel(const float *__restrict__ a, const float *__restrict__ b, "
          "float *__restrict__ out, int batch, int n_tiles)\n{\n", kThreads);
    if (!body) o("  __shared__ __align__(16) float lds[%d];\n", stage_floats + (merged ? kJitTile : 0));
    o("  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // (a scalar: branches on it are uniform)\n");
    o("  float *sa = lds, *sb = lds + %d, *so = lds + wave * %d;\n", kJitTile * pa, merged ? 0 : kJitTile * po);
    if (merged) o("  int *sflag = reinterpret_cast<int *>(lds + %d);\n", stage_floats);
    emit_tile_head(o);
    o("  __syncthreads();\n");
    if (merged) o("  if (tid < 64) sflag[tid] = 0;\n");
    emit_stage_load(o, "a", "a", na);
    emit_stage_load(o, "b", "b", nb);
    emit_stage_store(o, "a", "sa", na);
    emit_stage_store(o, "b", "sb", nb);
    o("  __syncthreads();\n");
    emit_row_to_regs(o, "a", "sa", na);
    emit_row_to_regs(o, "b", "sb", nb);
    o("  __syncthreads();\n");                  // the staged rows are spent: their LDS becomes the result stage
    for (int g = 0; g * fcols < S; ++g) {
        const int c0 = g * fcols, c1 = std::min(S, c0 + fcols);
        o("  if (wave == %d) {\n", g % kJitWaves);
        emit_columns(o, f, c0, c1, "    ");
        for (int c = c0; c < c1; c += 4)
            o("    *reinterpret_cast<float4 *>(so + lane * %d + %d) = make_float4(fminf(p%d, 1.0f), fminf(p%d, 1.0f), fminf(p%d, 1.0f), fminf(p%d, 1.0f));\n",
              po, merged ? c : c - c0, c, c + 1, c + 2, c + 3);
        if (merged) {
            o("    { bool over = false;\n");
            for (int c = c0; c < c1; ++c) o("      over |= !(p%d <= 1.0f);\n", c);
            o("      if (over) atomicOr(&sflag[lane], 1); }\n");
        } else {
            // the wavefront's own stage: program order within the wavefront is all the ordering it needs
            o("    wave_lds_fence();\n");
            const int chunks = (c1 - c0) / 4;       // 16-byte pieces per sample
            o("    for (int q = lane; q < valid * %d; q += 64) { const int s = q / %d, k = q - s * %d;\n", chunks, chunks, chunks);
            o("      *reinterpret_cast<float4 *>(out + (s0 + s) * %d + %d + 4 * k) = *reinterpret_cast<const float4 *>(so + s * %d + 4 * k); }\n", S, c0, po);
            o("    wave_lds_fence();\n");
        }
        o("  }\n");
    }
    if (merged) {
        // out[s, oc] from the Apply's column ia[oc] (in LDS) and c's column ib[oc]: 16-byte pieces of the result tile, four
        // per thread and pass with their loads in flight together; a piece whose four columns of c are neighbours comes
        // with one 16-byte load
        o("  __syncthreads();\n");
        o("  { const int chunks = n3 >> 2, total = valid * chunks;\n");
        o("    for (int qb = tid; qb < total; qb += %d) {\n", 4 * kThreads);
        for (int u = 0; u < 4; ++u) {
            o("      int pq%d = qb + %d; pq%d = pq%d < total ? pq%d : total - 1; const int ps%d = pq%d / chunks, pk%d = pq%d - ps%d * chunks;\n", u, kThreads * u, u, u, u, u,
              u, u, u, u);
            o("      const int4 ja%d = reinterpret_cast<const int4 *>(ia)[pk%d], jb%d = reinterpret_cast<const int4 *>(ib)[pk%d];\n", u, u, u, u);
        }
        for (int u = 0; u < 4; ++u) {
            o("      float4 y%d; { const float *cr = c + (s0 + ps%d) * nc;\n", u, u);
            if (aligned) {          // the result has c's symbols in c's order: one 16-byte load
                o("        y%d = *reinterpret_cast<const float4 *>(cr + 4 * pk%d); }\n", u, u);
                continue;
            }
            o("        if (jb%d.x >= 0 && !(jb%d.x & 3) && jb%d.y == jb%d.x + 1 && jb%d.z == jb%d.x + 2 && jb%d.w == jb%d.x + 3) y%d = *reinterpret_cast<const float4 *>(cr + jb%d.x);\n",
              u, u, u, u, u, u, u, u, u, u);
            o("        else y%d = make_float4(cr[jb%d.x > 0 ? jb%d.x : 0], cr[jb%d.y > 0 ? jb%d.y : 0], cr[jb%d.z > 0 ? jb%d.z : 0], cr[jb%d.w > 0 ? jb%d.w : 0]); }\n",
              u, u, u, u, u, u, u, u, u);
        }
        for (int u = 0; u < 4; ++u) {
            o("      { const float *xr = so + ps%d * %d; bool over = false; float v[4];\n", u, po);
            o("        const int ja[4] = {ja%d.x, ja%d.y, ja%d.z, ja%d.w}, jb[4] = {jb%d.x, jb%d.y, jb%d.z, jb%d.w}; const float yy[4] = {y%d.x, y%d.y, y%d.z, y%d.w};\n",
              u, u, u, u, u, u, u, u, u, u, u, u);
            if (aligned) {          // a kept column of the Apply sits at its own position in the result
                o("        const float4 x4 = 4 * pk%d < %d ? *reinterpret_cast<const float4 *>(xr + 4 * pk%d) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);\n", u, S, u);
                o("        const float xx[4] = {x4.x, x4.y, x4.z, x4.w};\n");
                o("        for (int e = 0; e < 4; ++e) { const float x = xx[e], t = x + yy[e];\n");
            } else {
                o("        for (int e = 0; e < 4; ++e) { const float x = xr[ja[e] > 0 ? ja[e] : 0], t = x + yy[e];\n");
            }
            o("          if (ja[e] >= 0 && jb[e] >= 0) { over |= !(t <= 1.0f); v[e] = fminf(t, 1.0f); } else v[e] = ja[e] >= 0 ? x : yy[e]; }\n");
            o("        if (qb + %d < total) { *reinterpret_cast<float4 *>(out + (s0 + ps%d) * n3 + 4 * pk%d) = make_float4(v[0], v[1], v[2], v[3]);\n", kThreads * u, u, u);
            o("          if (over) atomicOr(&sflag[ps%d], 1); } }\n", u);
        }
        o("    } }\n");
        o("  __syncthreads();\n  if (saved && tid < valid) saved[s0 + tid] = sflag[tid];\n");
    }
    o("  }\n}\n");
    return o.s;
}

// Most tuples of one column that share a symbol of the second (by_b) or first operand.
int max_multiplicity(const dol_fn_table *f, bool by_b)
{
    int best = 1;
    std::vector<int> cnt(static_cast<size_t>(by_b ? f->nb : f->na));
    for (int c = 0; c < f->n_out; ++c) {
        std::fill(cnt.begin(), cnt.end(), 0);
        for (uint32_t q = f->h_col_ptr[c]; q < f->h_col_ptr[c + 1]; ++q) {
            const uint32_t x = by_b ? f->h_col_ij[q] >> 16 : f->h_col_ij[q] & 0xffffu;
            best = std::max(best, ++cnt[x]);
        }
    }
    return best;
}

// Loads of one group of the gradient reaching the Apply's columns [c0, c1) into registers (th[]), and their way
// into the LDS stage.  merged: column c of the Apply is column ca[c] of the upstream gradient (or dropped).
void emit_gh_load(Src &o, int S, int c0, int c1, bool merged, bool aligned, const char *ind)
{
    const int chunks = (c1 - c0) / 4, per_thread = (kJitTile * chunks + kThreads - 1) / kThreads;
    for (int x = 0; x < per_thread; ++x) {
        // (no branches: a conditional block here would invite the compiler to sink the multiply-adds before it past it)
        o("%s{ int q = tid + %d; q = q < valid * %d ? q : valid * %d - 1; const int s = q / %d, k = q - s * %d;\n", ind, kThreads * x, chunks, chunks,
          chunks, chunks);
        if (merged) {
            o("%s  const int4 oc = reinterpret_cast<const int4 *>(ca)[%d + k]; const float *gr = g + (s0 + s) * n3;\n", ind, c0 / 4);
            if (aligned)    // a kept column of the Apply is the same column of the result: one 16-byte load
                o("%s  const float4 t = *reinterpret_cast<const float4 *>(gr + %d + 4 * k);\n", ind, c0);
            else
                o("%s  const float4 t = make_float4(gr[oc.x > 0 ? oc.x : 0], gr[oc.y > 0 ? oc.y : 0], gr[oc.z > 0 ? oc.z : 0], gr[oc.w > 0 ? oc.w : 0]);\n", ind);
            o("%s  th%d = make_float4(oc.x >= 0 ? t.x : 0.0f, oc.y >= 0 ? t.y : 0.0f, oc.z >= 0 ? t.z : 0.0f, oc.w >= 0 ? t.w : 0.0f); }\n", ind, x);
        } else {
            o("%s  th%d = reinterpret_cast<const float4 *>(g)[((s0 + s) * %d + %d) / 4 + k]; }\n", ind, x, S, c0);
        }
    }
}

// The group's way from registers into its LDS stage, gated on the way by the words of sm (all ones where no clamp acted).
void emit_gh_store(Src &o, int c0, int c1, int g, int n_groups, const char *dst, bool masked, const char *ind)
{
    const int chunks = (c1 - c0) / 4, per_thread = (kJitTile * chunks + kThreads - 1) / kThreads;
    for (int x = 0; x < per_thread; ++x) {
        const bool whole = kThreads * (x + 1) <= kJitTile * chunks;
        o("%s{ const int q = tid + %d; %s{ const int s = q / %d, k = q - s * %d;\n", ind, kThreads * x,
          whole ? "" : (std::string("if (q < ") + std::to_string(kJitTile * chunks) + ") ").c_str(), chunks, chunks);
        if (masked) {
            o("%s    const u32 mw = sm[(s * %d + %d) * 2 + (k >> 3)] >> ((4 * k) & 31);\n", ind, n_groups, g);
            o("%s    th%d = make_float4(mw & 1u ? th%d.x : 0.0f, mw & 2u ? th%d.y : 0.0f, mw & 4u ? th%d.z : 0.0f, mw & 8u ? th%d.w : 0.0f);\n", ind, x, x, x, x, x);
        }
        o("%s    *reinterpret_cast<float4 *>(%s + s * %d + 4 * k) = th%d; } }\n", ind, dst, kJitGroup + 4, x);
    }
}

std::string backward_source(const dol_fn_table *f, bool merged, bool aligned = false, bool body = false, int *lds_floats = nullptr)
{
    const int na = f->na, nb = f->nb, S = f->n_out;
    const int pa = na + 4, pb = nb + 4, pg = kJitGroup + 4;
    const int n_groups = (S + kJitGroup - 1) / kJitGroup;
    // LDS: a tile, b tile, two stages for one group of gh each (the first re-used as the result stage), gate words
    const int off_b = kJitTile * pa, off_g = off_b + kJitTile * pb;
    const int stage = std::max(kJitTile * pg, kJitTile * std::max(pa, pb));
    const int off_m = off_g + 2 * stage, off_u = off_m + kJitTile * n_groups * 2;
    const int off_x = off_u + (merged ? kJitTile * n_groups * 2 : 0), off_f = off_x + (merged ? 2 * S : 0);
    // the first half of the wavefronts share out the rows of a (they keep b), the second half those of b: two or four
    // parts each, multiples of four rows
    const int parts = kJitWaves / 2;
    const int ha = std::min(na, std::max(4, (na / parts + 3) & ~3)), hb = std::min(nb, std::max(4, (nb / parts + 3) & ~3));
    const int gh_per_thread = (kJitTile * (kJitGroup / 4) + kThreads - 1) / kThreads;
    Src o;
    if (!body) o.s = kPrologue;
    if (lds_floats) *lds_floats = off_f + 4;
    if (body)
        o("static __device__ __forceinline__ void damp_table_merge_bwd_body(float *lds, const float *__restrict__ a, const float *__restrict__ b, "
          "const float *__restrict__ c, const float *__restrict__ g, float *__restrict__ ga, float *__restrict__ gb, float *__restrict__ gc, "
          "const int *__restrict__ ia, const int *__restrict__ ib, const int *__restrict__ ca, const int *__restrict__ cb, "
          "const int *saved, int batch, int n_tiles, int nc, int n3, int accumulate)\n{\n");
    else if (merged)
        o("extern \"C\" __global__ void __launch_bounds__(%d) __attribute__((amdgpu_waves_per_eu(2, 2))) damp_table_merge_bwd_kernel(const float *__restrict__ a, const float *__restrict__ b, "
          "const float *__restrict__ c, const float *__restrict__ g, float *__restrict__ ga, float *__restrict__ gb, float *__restrict__ gc, "
          "const int *__restrict__ ia, const int *__restrict__ ib, const int *__restrict__ ca, const int *__restrict__ cb, "
          "const int *__restrict__ saved, int batch, int n_tiles, int nc, int n3, int accumulate)\n{\n", kThreads);
    else
        o("extern \"C\" __global__ void __launch_bounds__(%d) __attribute__((amdgpu_waves_per_eu(2, 2))) damp_table_bwd_kernel(const float *__restrict__ a, const float *__restrict__ b, "
          "const float *__restrict__ g, float *__restrict__ ga, float *__restrict__ gb, int batch, int n_tiles, int accumulate)\n{\n", kThreads);
    if (!body) o("  __shared__ __align__(16) float lds[%d];\n", off_f + 4);
    o("  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // (a scalar: branches on it are uniform)\n");
    o("  float *sa = lds, *sb = lds + %d, *sg0 = lds + %d, *sg1 = lds + %d;\n", off_b, off_g, off_g + stage);
    o("  u32 *sm = reinterpret_cast<u32 *>(lds + %d);\n  int *flag = reinterpret_cast<int *>(lds + %d);\n", off_m, off_f);
    if (merged) {
        // where each column of the Apply lands in the result (-1: dropped), and which column of c it meets there (-1: none)
        o("  u32 *su = reinterpret_cast<u32 *>(lds + %d);\n  int *s_oc = reinterpret_cast<int *>(lds + %d), *s_jc = s_oc + %d;\n", off_u, off_x, S);
        o("  for (int x = tid; x < %d; x += %d) { const int oc = ca[x]; s_oc[x] = oc; s_jc[x] = oc >= 0 ? ib[oc] : -1; }\n", S, kThreads);
    }
    emit_tile_head(o);
    o("  __syncthreads();\n  if (tid == 0) *flag = 0;\n");
    for (int x = 0; x < gh_per_thread; ++x) o("  float4 th%d;\n", x);
    emit_stage_load(o, "a", "a", na);
    emit_stage_load(o, "b", "b", nb);
    emit_gh_load(o, S, 0, std::min(S, kJitGroup), merged, aligned, "  ");
    if (merged) o("  int was_clamped = 1; if (saved) was_clamped = lane < valid ? saved[s0 + lane] : 0;\n");
    emit_stage_store(o, "a", "sa", na);
    emit_stage_store(o, "b", "sb", nb);
    emit_gh_store(o, 0, std::min(S, kJitGroup), 0, n_groups, "sg0", false, "  ");
    o("  __syncthreads();\n");
    emit_row_to_regs(o, "a", "sa", na);
    emit_row_to_regs(o, "b", "sb", nb);
    if (merged) {
        // the forward launch left word: did any clamp act in this sample?
        o("  if (was_clamped && lane < valid) *flag = 1;\n");
    } else {
        // can any column of this lane's sample exceed 1?
        o("  { float ma = a0, mb = b0, ta = a0, tb = b0;\n");
        for (int i = 1; i < na; ++i) o("    ma = fmaxf(ma, a%d); ta += a%d;\n", i, i);
        for (int j = 1; j < nb; ++j) o("    mb = fmaxf(mb, b%d); tb += b%d;\n", j, j);
        o("    const float bound = fminf(ma * tb * %d.0f, mb * ta * %d.0f);\n", max_multiplicity(f, true), max_multiplicity(f, false));
        o("    if (lane < valid && !(bound <= 0.9999f)) *flag = 1; }\n");
    }
    o("  __syncthreads();\n  const bool gate = *flag != 0;\n");
    // rare: recompute pre, one group of columns per wavefront, and leave one bit per (sample, column)
    o("  if (gate) {\n");
    if (merged) o("    const long long sr = s0 + (lane < valid ? lane : 0);\n");
    for (int g = 0; g < n_groups; ++g) {
        const int c0 = g * kJitGroup, c1 = std::min(S, c0 + kJitGroup);
        o("    if (wave == %d) {\n", g % kJitWaves);
        o("      u32 m0 = 0, m1 = 0;\n");
        if (merged) o("      u32 u0 = 0, u1 = 0;\n");
        for (int d0 = c0; d0 < c1; d0 += 16) {
            const int d1 = std::min(c1, d0 + 16);
            o("      {\n");
            emit_columns(o, f, d0, d1, "        ");
            for (int c = d0; c < d1; ++c) {
                if (merged) {
                    o("        { const int oc = s_oc[%d], jc = s_jc[%d];\n", c, c);
                    o("          bool open = true; if (jc >= 0) open = fminf(p%d, 1.0f) + c[sr * nc + jc] <= 1.0f;\n", c);
                    o("          if (open) u%d |= %uu; if (open && oc >= 0 && p%d <= 1.0f) m%d |= %uu; }\n", (c - c0) / 32, 1u << ((c - c0) & 31), c,
                      (c - c0) / 32, 1u << ((c - c0) & 31));
                } else {
                    o("        m%d |= p%d <= 1.0f ? %uu : 0u;\n", (c - c0) / 32, c, 1u << ((c - c0) & 31));
                }
            }
            o("      }\n      __builtin_amdgcn_sched_barrier(0);\n");
        }
        if (merged) o("      su[(lane * %d + %d) * 2] = u0; su[(lane * %d + %d) * 2 + 1] = u1;\n", n_groups, g, n_groups, g);
        o("      sm[(lane * %d + %d) * 2] = m0; sm[(lane * %d + %d) * 2 + 1] = m1;\n    }\n", n_groups, g, n_groups, g);
    }
    o("    __syncthreads();\n");
    {   // the first group is already staged: gate it in place
        const int c1 = std::min(S, kJitGroup), chunks = c1 / 4;
        o("    for (int q = tid; q < %d; q += %d) { const int s = q / %d, k = q - s * %d;\n", kJitTile * chunks, kThreads, chunks, chunks);
        o("      const u32 mw = sm[(s * %d) * 2 + (k >> 3)] >> ((4 * k) & 31); float4 *p4 = reinterpret_cast<float4 *>(sg0 + s * %d + 4 * k);\n", n_groups, pg);
        o("      const float4 t = *p4; *p4 = make_float4(mw & 1u ? t.x : 0.0f, mw & 2u ? t.y : 0.0f, mw & 4u ? t.z : 0.0f, mw & 8u ? t.w : 0.0f); }\n");
    }
    o("  } else {\n    for (int x = tid; x < %d; x += %d) sm[x] = 0xffffffffu;\n  }\n  __syncthreads();\n", kJitTile * n_groups * 2, kThreads);
    // The four roles.  Every role runs the same sequence of workgroup barriers and takes part in the same flat
    // copies; only the multiply-adds differ.  While a group's multiply-adds run, the next group's loads are in flight.
    for (int w = 0; w < kJitWaves; ++w) {
        const bool is_a = w < parts;
        const int n = is_a ? na : nb, h = is_a ? ha : hb, part = w % parts;
        const int r0 = std::min(n, part * h), r1 = part + 1 == parts ? n : std::min(n, (part + 1) * h);
        const char *acc = is_a ? "x" : "y";
        o("  %sif (wave == %d) {\n", w ? "else " : "", w);
        for (int r = r0; r < r1; ++r) o("    float %s%d = 0.0f;\n", acc, r);
        for (int g = 0; g < n_groups; ++g) {
            const int c0 = g * kJitGroup, c1 = std::min(S, c0 + kJitGroup);
            const char *cur = g & 1 ? "sg1" : "sg0", *nxt = g & 1 ? "sg0" : "sg1";
            if (g + 1 < n_groups) emit_gh_load(o, S, c1, std::min(S, c1 + kJitGroup), merged, aligned, "    ");
            // 16 columns at a time, fenced for the instruction scheduler: it would otherwise fetch the whole group first and
            // run out of registers
            o("    {\n");
            for (int d0 = c0; d0 < c1; d0 += 16) {
                const int d1 = std::min(c1, d0 + 16);
                o("    {\n");
                for (int c = d0; c < d1; c += 4)
                    o("      float h%d, h%d, h%d, h%d; { const float4 t = *reinterpret_cast<const float4 *>(%s + lane * %d + %d); h%d = t.x; h%d = t.y; h%d = t.z; h%d = t.w; }\n",
                      c, c + 1, c + 2, c + 3, cur, pg, c - c0, c, c + 1, c + 2, c + 3);
                // the tuples of these columns whose row belongs to this role
                for (int c = d0; c < d1; ++c)
                    for (uint32_t q = f->h_col_ptr[c]; q < f->h_col_ptr[c + 1]; ++q) {
                        const int i = static_cast<int>(f->h_col_ij[q] & 0xffffu), j = static_cast<int>(f->h_col_ij[q] >> 16);
                        const int r = is_a ? i : j;
                        if (r < r0 || r >= r1) continue;
                        if (is_a) o("      x%d = __builtin_fmaf(h%d, b%d, x%d);\n", i, c, j, i);
                        else o("      y%d = __builtin_fmaf(h%d, a%d, y%d);\n", j, c, i, j);
                    }
                o("    }\n    __builtin_amdgcn_sched_barrier(0);\n");
            }
            o("    }\n");
            if (g + 1 < n_groups) emit_gh_store(o, c1, std::min(S, c1 + kJitGroup), g + 1, n_groups, nxt, true, "    ");
            o("    __syncthreads();\n");
        }
        // results: through LDS (one operand's tile at a time, in the first stage), out with flat 16-byte accesses
        for (int pass = 0; pass < 2; ++pass) {
            const bool pass_a = pass == 0;
            const int pn = pass_a ? na : nb, pp = pn + 4;
            if (pass) o("    __syncthreads();\n");
            if (pass_a == is_a)
                for (int r = r0; r < r1; r += 4)
                    o("    *reinterpret_cast<float4 *>(sg0 + lane * %d + %d) = make_float4(%s%d, %s%d, %s%d, %s%d);\n", pp, r, acc, r, acc, r + 1, acc,
                      r + 2, acc, r + 3);
            o("    __syncthreads();\n");
            o("    if (%s) { float4 *d4 = reinterpret_cast<float4 *>(%s + s0 * %d);\n", pass_a ? "ga" : "gb", pass_a ? "ga" : "gb", pn);
            o("      for (int q = tid; q < valid * %d; q += %d) { const int s = q / %d, k = q - s * %d;\n", pn / 4, kThreads, pn / 4, pn / 4);
            o("        float4 v = *reinterpret_cast<const float4 *>(sg0 + s * %d + 4 * k);\n", pp);
            o("        if (accumulate & %d) { const float4 old = d4[q]; v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w; }\n", pass_a ? 1 : 2);
            o("        d4[q] = v; } }\n");
        }
        o("  }\n");
    }
    if (merged) {
        // gradient of c: column jc of c is column cb[jc] of the result; a symbol of both sides is gated by the union's clamp.
        // 16-byte pieces, four per thread and pass, one 16-byte load where the four columns are neighbours in the result.
        o("  if (gc) { const int chunks = nc >> 2, total = valid * chunks;\n");
        o("    for (int qb = tid; qb < total; qb += %d) {\n", 4 * kThreads);
        for (int u = 0; u < 4; ++u) {
            o("      int pq%d = qb + %d; pq%d = pq%d < total ? pq%d : total - 1; const int ps%d = pq%d / chunks, pk%d = pq%d - ps%d * chunks;\n", u, kThreads * u, u, u, u, u,
              u, u, u, u);
            o("      const int4 oc%d = reinterpret_cast<const int4 *>(cb)[pk%d];\n", u, u);
        }
        for (int u = 0; u < 4; ++u) {
            o("      float4 v%d; { const float *gr = g + (s0 + ps%d) * n3;\n", u, u);
            o("        if (!(oc%d.x & 3) && oc%d.y == oc%d.x + 1 && oc%d.z == oc%d.x + 2 && oc%d.w == oc%d.x + 3) v%d = *reinterpret_cast<const float4 *>(gr + oc%d.x);\n",
              u, u, u, u, u, u, u, u, u);
            o("        else v%d = make_float4(gr[oc%d.x], gr[oc%d.y], gr[oc%d.z], gr[oc%d.w]); }\n", u, u, u, u, u);
        }
        for (int u = 0; u < 4; ++u) {
            o("      if (qb + %d < total) {\n", kThreads * u);
            o("        if (gate) { const int oc[4] = {oc%d.x, oc%d.y, oc%d.z, oc%d.w}; float w[4] = {v%d.x, v%d.y, v%d.z, v%d.w};\n", u, u, u, u, u, u, u, u);
            o("          for (int e = 0; e < 4; ++e) { const int col = ia[oc[e]];\n");
            o("            if (col >= 0 && !((su[(ps%d * %d + (col >> 6)) * 2 + ((col >> 5) & 1)] >> (col & 31)) & 1u)) w[e] = 0.0f; }\n", u, n_groups);
            o("          v%d = make_float4(w[0], w[1], w[2], w[3]); }\n", u);
            o("        float4 *d4 = reinterpret_cast<float4 *>(gc + (s0 + ps%d) * nc) + pk%d;\n", u, u);
            o("        if (accumulate & 4) { const float4 old = *d4; v%d.x += old.x; v%d.y += old.y; v%d.z += old.z; v%d.w += old.w; }\n        *d4 = v%d; }\n", u, u, u, u, u);
        }
        o("    } }\n");
    }
    o("  }\n}\n");
    return o.s;
}

// Apply + Filter + Union forward and backward in one launch: the two bodies above over one LDS array.  The backward
// body reads the per-sample clamp words the forward body has just written (other threads' words: the workgroup's
// barrier between the two orders them).
std::string both_source(const dol_fn_table *f, bool aligned)
{
    int lf = 0, lb = 0;
    const std::string fwd = forward_source(f, true, aligned, true, &lf), bwd = backward_source(f, true, aligned, true, &lb);
    Src o;
    o.s = kPrologue;
    o.s += fwd;
    o.s += bwd;
    o("extern \"C\" __global__ void __launch_bounds__(%d) __attribute__((amdgpu_waves_per_eu(2, 2))) damp_table_merge_fwd_bwd_kernel("
      "const float *__restrict__ a, const float *__restrict__ b, const float *__restrict__ c, float *__restrict__ out, "
      "const float *__restrict__ g, float *__restrict__ ga, float *__restrict__ gb, float *__restrict__ gc, const int *__restrict__ ia, "
      "const int *__restrict__ ib, const int *__restrict__ ca, const int *__restrict__ cb, int *saved, int batch, int n_tiles, int nc, int n3, "
      "int accumulate)\n{\n", kThreads);
    o("  __shared__ __align__(16) float lds[%d];\n", std::max(lf, lb));
    o("  damp_table_merge_fwd_body(lds, a, b, c, out, ia, ib, saved, batch, n_tiles, nc, n3);\n");
    o("  __syncthreads();\n");
    o("  damp_table_merge_bwd_body(lds, a, b, c, g, ga, gb, gc, ia, ib, ca, cb, saved, batch, n_tiles, nc, n3, accumulate);\n}\n");
    return o.s;
}

}  // namespace

dol_status jit_compile(const std::string &src, const char *name, hipModule_t *mod, hipFunction_t *fn)
{
    // DOL_JIT_DUMP_DIR names a folder that receives the source of every kernel generated in this process, so that
    // the code written for a table or a chain can be read and compiled by hand.
    if (const char *dump = getenv("DOL_JIT_DUMP_DIR")) {
        const std::string path = std::string(dump) + "/" + name + ".hip";
        if (FILE *fh = fopen(path.c_str(), "w")) { fputs(src.c_str(), fh); fclose(fh); }
    }
    hiprtcProgram prog = nullptr;
    if (hiprtcCreateProgram(&prog, src.c_str(), "dol_table.hip", 0, nullptr, nullptr) != HIPRTC_SUCCESS)
        return fail(DOL_EHIP, "hiprtcCreateProgram failed");
    const char *opts[] = {"--offload-arch=gfx950", "-O3", "-ffp-contract=off", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"};
    const hiprtcResult rc = hiprtcCompileProgram(prog, static_cast<int>(sizeof opts / sizeof *opts), opts);
    if (rc != HIPRTC_SUCCESS) {
        size_t n = 0;
        std::string log;
        if (hiprtcGetProgramLogSize(prog, &n) == HIPRTC_SUCCESS && n > 1) {
            log.resize(n);
            (void)hiprtcGetProgramLog(prog, &log[0]);
        }
        (void)hiprtcDestroyProgram(&prog);
        return fail(DOL_EHIP, "compiling the table's code failed (%s): %.300s", hiprtcGetErrorString(rc), log.c_str());
    }
    size_t size = 0;
    std::vector<char> code;
    if (hiprtcGetCodeSize(prog, &size) != HIPRTC_SUCCESS || size == 0) {
        (void)hiprtcDestroyProgram(&prog);
        return fail(DOL_EHIP, "hiprtcGetCodeSize failed");
    }
    code.resize(size);
    const hiprtcResult rc2 = hiprtcGetCode(prog, code.data());
    (void)hiprtcDestroyProgram(&prog);
    if (rc2 != HIPRTC_SUCCESS) return fail(DOL_EHIP, "hiprtcGetCode failed");
    DOL_HIP(hipModuleLoadData(mod, code.data()));
    DOL_HIP(hipModuleGetFunction(fn, *mod, name));
    return DOL_OK;
}

namespace {

unsigned tile_grid(int n_tiles) { return static_cast<unsigned>(n_tiles); }

// How a batch is cut up.  The registers of these kernels allow two wavefronts on a SIMD, and the chip has 256 compute
// units.  With tiles of 64 samples and four wavefronts to a tile, a batch of up to 256 tiles leaves every unit with one
// wavefront per SIMD and the tile's loads, arithmetic and stores one after the other.  Such a batch gets a build of its
// own: up to 128 tiles' worth of samples are cut into tiles of 32 (half of the lanes idle, twice the workgroups), more
// keep tiles of 64 and give each to eight wavefronts, which share its columns (rows, in the reverse pass) out finer.
// Config 3 in one launch: 22.7 us at B = 8192 (tiles of 32; 23.2 with eight wavefronts), 27.3 us at B = 16384 (eight
// wavefronts; 28.9 in tiles of 32, 32.2 in the build for large batches).
struct JitBuild {
    int rows, waves;        // samples per tile, wavefronts per workgroup
    int variant;            // which of the table's builds
};
JitBuild build_for(int32_t batch)
{
    if (batch > 256 * kJitTile) return {kJitTile, kJitWavesLarge, 0};
    if (batch > 128 * kJitTile) return {kJitTile, 2 * kJitWavesLarge, 1};
    return {kJitTile / 2, kJitWavesLarge, 2};
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

JitState *state_of(const dol_fn_table *f)
{
    static std::mutex mu;
    std::lock_guard<std::mutex> lock(mu);
    if (!f->jit) f->jit.reset(new JitState);
    return f->jit.get();
}

}  // namespace

// The kernel of `slot` for this table, built on first use.
static dol_status kernel_of(const dol_fn_table *f, int kind, const JitBuild &bd, hipFunction_t *fn)
{
    const int slot = kind + bd.variant * kSlots;
    static const char *const names[kSlots] = {"damp_table_fwd_kernel", "damp_table_bwd_kernel", "damp_table_merge_fwd_kernel",
                                              "damp_table_merge_bwd_kernel", "damp_table_merge_fwd_kernel", "damp_table_merge_bwd_kernel",
                                              "damp_table_merge_fwd_bwd_kernel", "damp_table_merge_fwd_bwd_kernel"};
    JitState *js = state_of(f);
    std::lock_guard<std::mutex> lock(js->mu);
    if (!js->tried[slot]) {
        js->tried[slot] = true;
        t_tile_rows = bd.rows, t_waves = bd.waves;
        const std::string src = kind == kSlotFwd ? forward_source(f, false) : kind == kSlotBwd ? backward_source(f, false) :
                                kind == kSlotMergeFwd ? forward_source(f, true) : kind == kSlotMergeBwd ? backward_source(f, true) :
                                kind == kSlotMergeFwdAligned ? forward_source(f, true, true) :
                                kind == kSlotMergeBwdAligned ? backward_source(f, true, true) : both_source(f, kind == kSlotMergeBothAligned);
        t_tile_rows = kJitTile, t_waves = kJitWavesLarge;
        js->status[slot] = jit_compile(src, names[kind], &js->mod[slot], &js->fn[slot]);
        if (js->status[slot] != DOL_OK) return js->status[slot];      // with the compiler's message
    } else if (js->status[slot] != DOL_OK) {
        return fail(js->status[slot], "the code of this function table did not build (see the first call's message)");
    }
    *fn = js->fn[slot];
    return DOL_OK;
}

// *done = the call was taken (otherwise the caller uses the generic kernels).
dol_status launch_damp_table_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, float *out, int64_t ldo, hipStream_t st, bool *done)
{
    *done = false;
    if (!table_code_ok(f) || batch < 1) return DOL_OK;
    if (lda != f->na || ldb != f->nb || ldo != f->n_out || !aligned16(a) || !aligned16(b) || !aligned16(out)) return DOL_OK;
    hipFunction_t fn = nullptr;
    if (dol_status s = kernel_of(f, kSlotFwd, build_for(batch), &fn)) return s;
    const JitBuild bd = build_for(batch);
    int n_tiles = (batch + bd.rows - 1) / bd.rows;
    void *args[] = {&a, &b, &out, &batch, &n_tiles};
    DOL_HIP(hipModuleLaunchKernel(fn, tile_grid(n_tiles), 1, 1, kJitTile * bd.waves, 1, 1, 0, st, args, nullptr));
    *done = true;
    return DOL_OK;
}

dol_status launch_damp_table_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                                 hipStream_t st, bool *done)
{
    *done = false;
    if (!table_code_ok(f) || batch < 1 || (ga && ga == gb)) return DOL_OK;
    if (lda != f->na || ldb != f->nb || ldg != f->n_out || !aligned16(a) || !aligned16(b) || !aligned16(g) || !aligned16(ga) ||
        !aligned16(gb))
        return DOL_OK;
    hipFunction_t fn = nullptr;
    if (dol_status s = kernel_of(f, kSlotBwd, build_for(batch), &fn)) return s;
    const JitBuild bd = build_for(batch);
    int n_tiles = (batch + bd.rows - 1) / bd.rows;
    void *args[] = {&a, &b, &g, &ga, &gb, &batch, &n_tiles, &accumulate};
    DOL_HIP(hipModuleLaunchKernel(fn, tile_grid(n_tiles), 1, 1, kJitTile * bd.waves, 1, 1, 0, st, args, nullptr));
    *done = true;
    return DOL_OK;
}

bool table_merge_ok(const dol_fn_table *f) { return table_code_ok(f) && f->n_out <= kJitMaxMergeOut; }

dol_status launch_damp_table_merge_fwd(const dol_fn_table *f, const UnionPlan *p, int32_t batch, const float *a, const float *b,
                                       const float *c, float *out, int32_t *saved, hipStream_t st)
{
    hipFunction_t fn = nullptr;
    if (dol_status s = kernel_of(f, p->aligned ? kSlotMergeFwdAligned : kSlotMergeFwd, build_for(batch), &fn)) return s;
    const JitBuild bd = build_for(batch);
    int n_tiles = (batch + bd.rows - 1) / bd.rows, nc = p->nb, n3 = p->n_out;
    const int32_t *ia = p->d_ia.ptr, *ib = p->d_ib.ptr;
    void *args[] = {&a, &b, &c, &out, &ia, &ib, &saved, &batch, &n_tiles, &nc, &n3};
    DOL_HIP(hipModuleLaunchKernel(fn, tile_grid(n_tiles), 1, 1, kJitTile * bd.waves, 1, 1, 0, st, args, nullptr));
    return DOL_OK;
}

dol_status launch_damp_table_merge_bwd(const dol_fn_table *f, const UnionPlan *p, int32_t batch, const float *a, const float *b,
                                       const float *c, const float *g, float *ga, float *gb, float *gc, const int32_t *saved,
                                       int32_t accumulate, hipStream_t st)
{
    hipFunction_t fn = nullptr;
    if (dol_status s = kernel_of(f, p->aligned ? kSlotMergeBwdAligned : kSlotMergeBwd, build_for(batch), &fn)) return s;
    const JitBuild bd = build_for(batch);
    int n_tiles = (batch + bd.rows - 1) / bd.rows, nc = p->nb, n3 = p->n_out;
    const int32_t *ia = p->d_ia.ptr, *ib = p->d_ib.ptr, *ca = p->d_ca.ptr, *cb = p->d_cb.ptr;
    void *args[] = {&a, &b, &c, &g, &ga, &gb, &gc, &ia, &ib, &ca, &cb, &saved, &batch, &n_tiles, &nc, &n3, &accumulate};
    DOL_HIP(hipModuleLaunchKernel(fn, tile_grid(n_tiles), 1, 1, kJitTile * bd.waves, 1, 1, 0, st, args, nullptr));
    return DOL_OK;
}

dol_status launch_damp_table_merge_both(const dol_fn_table *f, const UnionPlan *p, int32_t batch, const float *a, const float *b,
                                        const float *c, float *out, int32_t *saved, const float *g, float *ga, float *gb, float *gc,
                                        int32_t accumulate, hipStream_t st)
{
    hipFunction_t fn = nullptr;
    if (dol_status s = kernel_of(f, p->aligned ? kSlotMergeBothAligned : kSlotMergeBoth, build_for(batch), &fn)) return s;
    const JitBuild bd = build_for(batch);
    int n_tiles = (batch + bd.rows - 1) / bd.rows, nc = p->nb, n3 = p->n_out;
    const int32_t *ia = p->d_ia.ptr, *ib = p->d_ib.ptr, *ca = p->d_ca.ptr, *cb = p->d_cb.ptr;
    void *args[] = {&a, &b, &c, &out, &g, &ga, &gb, &gc, &ia, &ib, &ca, &cb, &saved, &batch, &n_tiles, &nc, &n3, &accumulate};
    DOL_HIP(hipModuleLaunchKernel(fn, tile_grid(n_tiles), 1, 1, kJitTile * bd.waves, 1, 1, 0, st, args, nullptr));
    return DOL_OK;
}

}  // namespace dol
