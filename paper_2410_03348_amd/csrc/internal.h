// Internal declarations shared by the translation units of libdolphin_hip.so.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <memory>
#include <string>
#include <algorithm>
#include <numeric>
#include <vector>

#include "dolphin_hip.h"

namespace dol {

// ---------------------------------------------------------------- errors

void set_error(const char *fmt, ...) __attribute__((format(printf, 1, 2)));
dol_status fail(dol_status st, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
dol_status hip_fail(hipError_t e, const char *what);

#define DOL_HIP(call)                                        \
    do {                                                     \
        hipError_t e_ = (call);                              \
        if (e_ != hipSuccess) return ::dol::hip_fail(e_, #call); \
    } while (0)

// A kernel that asks for more than 64 KB of dynamic LDS has to be told so, once per device: this does it the first time
// a (device, kernel) pair is seen (thread-safe) and is a table lookup afterwards.
hipError_t allow_dynamic_lds(const void *kernel, size_t bytes);

// ---------------------------------------------------------------- device arrays owned by plans

template <typename T>
struct DevArray {
    T *ptr = nullptr;
    size_t n = 0;
    DevArray() = default;
    DevArray(const DevArray &) = delete;
    DevArray &operator=(const DevArray &) = delete;
    ~DevArray() { release(); }
    void release()
    {
        if (ptr) (void)hipFree(ptr);   // hipFree waits for work that may still read the array
        ptr = nullptr;
        n = 0;
    }
    // Synchronous upload; an empty vector leaves ptr == nullptr.
    hipError_t upload(const std::vector<T> &h)
    {
        release();
        if (h.empty()) return hipSuccess;
        hipError_t e = hipMalloc(reinterpret_cast<void **>(&ptr), h.size() * sizeof(T));
        if (e != hipSuccess) { ptr = nullptr; return e; }
        n = h.size();
        e = hipMemcpy(ptr, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice);
        if (e != hipSuccess) release();
        return e;
    }
};

// ---------------------------------------------------------------- symbol-side plans

constexpr int kLongTableRow = 64;   // backward: table rows with more tuples are reduced by a whole wavefront
constexpr int kLongTableCol = 64;   // forward: output columns with more tuples are summed by a whole wavefront
constexpr int kLongDtkpCol = 16;    // the same under DTKP, where a tuple costs a few hundred instructions
constexpr int kHugeTableCol = 4096; // columns with more tuples get a workgroup of 16 wavefronts instead of one wavefront
constexpr int kHugeDtkpCol = 1024;  // the same under DTKP
constexpr int kWaveDtkpCol = 64;    // DTKP columns of kLongDtkpCol+1 .. this many tuples share a wavefront four at a time
constexpr int32_t kStageMinRow = 2048;       // operand rows of at least this many tags are staged in LDS before gathers;
constexpr size_t kStageMaxBytes = 158 * 1024;   // narrower ones stay with the cached gathers; of the 160 KB of a compute unit
constexpr int kByJMax = 16;         // tables whose second operand has at most this many symbols get dense per-j maps
constexpr int kByJMaxNa = 65000;    // ... and whose first operand leaves room for the three marks below
constexpr uint16_t kByJNone = 0xFFFF, kByJWave = 0xFFFE, kByJList = 0xFFFD;

// Code compiled for one function table on its first use (damp_table.hip)
struct JitState;
struct JitDeleter {
    void operator()(JitState *p) const;
};

// A tuple of the function table packed for the kernels: low 16 bits = first index, high 16 = second.
__host__ __device__ static inline uint32_t pack16(uint32_t lo, uint32_t hi) { return lo | (hi << 16); }

}  // namespace dol

// Eq. 1-2: admitted tuples grouped by the output column they land in (the "shuffle" stage),
// plus the two transposed groupings the vector-Jacobian products walk.
struct dol_fn_table {
    int32_t na = 0, nb = 0, n_out = 0;
    int64_t n_tuples = 0;
    int32_t max_col_len = 0;             // most tuples landing in one column
    int32_t max_rowa_len = 0;            // most tuples of one symbol of the first operand
    int32_t n_long_rowa = 0;               // first-operand rows among long_rows
    bool sum_like = false;               // every column's tuples have i ascending by 1 and j descending by 1
    bool conv_like = false;              // all na*nb tuples admitted and tuple (i, j) lands in column i + j:
                                         // the operator is a discrete convolution of the two tag rows
    std::vector<int32_t> out_syms;       // [n_out] ascending ids
    std::string kernel_fwd, kernel_bwd;  // names of the DAMP kernels chosen for this table
    // host copies (kept for the chain planner)
    std::vector<uint32_t> h_col_ptr, h_col_ij;
    // forward: column c owns entries col_ptr[c] .. col_ptr[c+1] of col_ij = pack16(i, j), ascending (i, j)
    dol::DevArray<uint32_t> col_ptr, col_ij;
    // the first four tuples of every column again, 16 bytes per column (0xFFFFFFFF = no tuple): the forward kernel
    // for irregular tables gets a short column with one load
    dol::DevArray<uint32_t> col_head;
    dol::DevArray<uint32_t> col_head_ord;   // the same, entry r being that of column col_order[r] (read coalesced there)
    // backward w.r.t. a: row i owns rowa_ptr[i] .. rowa_ptr[i+1] of rowa_jc = pack16(j, column), ascending j
    dol::DevArray<uint32_t> rowa_ptr, rowa_jc;
    // backward w.r.t. b: row j owns rowb_ptr[j] .. rowb_ptr[j+1] of rowb_ic = pack16(i, column), ascending i
    dol::DevArray<uint32_t> rowb_ptr, rowb_ic;
    // square tables (n_out == na) only: rowb_pos[q] = position in rowa_jc of the tuple at position q of rowb_ic
    dol::DevArray<uint32_t> rowb_pos;
    // rows with more than dol::kLongTableRow tuples (x < na: row x of a, else row x - na of b)
    dol::DevArray<uint32_t> long_rows;
    // output columns with more than dol::kLongTableCol / dol::kLongDtkpCol tuples
    dol::DevArray<uint32_t> long_cols, dtkp_long_cols;
    // all columns in the order the thread-per-column kernels over long operand rows take them
    // (dol::columns_by_length, with the DTKP kernel's limit on the length of a column)
    dol::DevArray<uint32_t> col_order;
    // the tuple lists of the columns of at most dol::kLongDtkpCol tuples, interleaved in that order: tuple k of column
    // col_order[r] is ord_tuples[k * n_out + r] and its list has ord_len[r] entries (0: a longer column), so that lanes on
    // neighbouring r read neighbouring words
    dol::DevArray<uint32_t> ord_tuples, ord_len;
    // each list starts with its huge columns (more than dol::kHugeTableCol / dol::kHugeDtkpCol tuples)
    int32_t n_huge_cols = 0, n_huge_dtkp_cols = 0, n_huge_byj_cols = 0;
    int32_t n_wave_dtkp_cols = 0;        // dtkp_long_cols: huge, then this many one-wavefront columns, then the shorter ones
    // LDS gather kernels (damp_lds.hip): per output column (forward), row of a, row of b (backward) a list of
    // 16-byte packets of four tuples; *_ptr[x] .. *_ptr[x+1] are the packets of x
    bool lds_fwd_ok = false, lds_bwd_ok = false;
    size_t lds_fwd_bytes = 0, lds_bwd_bytes = 0;
    dol::DevArray<uint32_t> lds_pk, lds_pk_ptr, lds_pka, lds_pka_ptr, lds_pkb, lds_pkb_ptr;
    // Tables with a short second operand (nb <= dol::kByJMax, na <= dol::kByJMaxNa) that take neither path above:
    // dense 16-bit maps walked one j at a time, so that lane-adjacent elements read the operand through one map each
    // (adjacent addresses for monotone functions).  byj_src[j * n_out + c] = the i with f(i, j) = column c, or
    // dol::kByJNone; a long column has dol::kByJWave at j = 0 and is listed in byj_wave_cols (summed by a wavefront); a
    // short column where some j occurs twice has dol::kByJList there and is summed from its tuple list.
    // byj_col[j * na + i] = column of (i, j) or dol::kByJNone.
    bool byj_ok = false;
    int32_t byj_nbp = 0;               // rows of the two maps: nb padded to 4, 8, 10 or 16 (the extra rows hold kByJNone)
    bool byj_fwd = false;              // forward uses the map only where it is at least half full (else the tuple lists)
    dol::DevArray<uint16_t> byj_src, byj_col;
    dol::DevArray<uint32_t> byj_wave_cols;
    // tables whose operand rows fit in registers: straight-line kernels written for the table (built on first use)
    mutable std::unique_ptr<dol::JitState, dol::JitDeleter> jit;
    int device = 0;
};

namespace dol {

// The order in which a thread-per-column kernel takes the columns of a table: inside every block of kOrderBlock
// consecutive columns, longest tuple list first (columns above `skip_above` tuples, which such a kernel leaves to
// another one, last), equal lengths in ascending column order.  The 64 lanes of a wavefront then walk lists of (nearly)
// one length instead of waiting for the longest of 64 arbitrary ones, while a block's results still land in one
// contiguous stretch of the output.
constexpr int32_t kOrderBlock = 4096;

inline std::vector<uint32_t> columns_by_length(const std::vector<uint32_t> &col_ptr, int32_t n_cols, uint32_t skip_above)
{
    std::vector<uint32_t> order(static_cast<size_t>(n_cols));
    std::iota(order.begin(), order.end(), 0u);
    auto work = [&](uint32_t c) {
        const uint32_t len = col_ptr[c + 1] - col_ptr[c];
        return len > skip_above ? 0u : len;
    };
    for (int32_t b = 0; b < n_cols; b += kOrderBlock)
        std::stable_sort(order.begin() + b, order.begin() + std::min(n_cols, b + kOrderBlock),
                         [&](uint32_t x, uint32_t y) { return work(x) > work(y); });
    return order;
}

struct FilterPlan {
    int32_t n_in = 0, n_out = 0;
    std::vector<int32_t> keep_idx;        // [n_out] position in the input
    DevArray<int32_t> d_keep_idx;         // same, device
    DevArray<int32_t> d_pos;              // [n_in] position in the output or -1
};

struct UnionPlan {
    int32_t na = 0, nb = 0, n_out = 0;
    std::vector<int32_t> out_syms;
    DevArray<int32_t> d_ia, d_ib;         // [n_out] position in a / b or -1
    DevArray<int32_t> d_ca, d_cb;         // [na] / [nb] output column of each input position (-1: none, filter-union only)
    // filter-union plans: the result has exactly b's symbols in b's order and every kept symbol of a sits at its own
    // position (ia[c] is c or -1, ib[c] = c): true when a's symbols are 0 .. na-1 of b's id list, as in a program
    // that merges an Apply's result into a Distribution over all its possible symbols
    bool aligned = false;
};

// Content-addressed caches: the same predicate / symbol lists give the same plan object.  A cache holds at most 4096
// plans and then releases the one unused longest, so a returned pointer is for the call that asked for it.
dol_status get_filter_plan(int32_t n, const uint8_t *pred, const FilterPlan **plan);
dol_status get_union_plan(int32_t na, const int32_t *sa, int32_t nb, const int32_t *sb, const UnionPlan **plan);
// union(filter(d, pred), c) as one merge plan: na = symbols of d, ia points into d, ca is -1 for dropped symbols.
dol_status get_filter_union_plan(int32_t n, const int32_t *sd, const uint8_t *pred, int32_t nc, const int32_t *sc,
                                 const UnionPlan **plan);

// Masks of the exclusion groups that hold at least two facts (kernel argument, by value).
struct GroupMasks {
    int32_t n;
    uint64_t m[32];
};
dol_status make_group_masks(const dol_prov *prov, GroupMasks *gm);
// Device copy of a small host int32 array, cached by content.
dol_status get_i32_array(int32_t n, const int32_t *data, const int32_t **dptr);

// ---------------------------------------------------------------- argument checks (api.hip)

bool is_dtkp(const dol_prov *prov);
dol_status check_prov(const dol_prov *prov, int32_t batch);
// Shape and pointer checks of one Distribution.  need_ids: the call reads sym_ids.
dol_status check_dist(const dol_dist *d, const char *name, bool dtkp, bool need_ids, bool need_prob);
dol_status check_work(int64_t batch, int64_t per_sample);

// ---------------------------------------------------------------- launchers (damp.hip / dtkp.hip)

dol_status launch_damp_apply2_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                  int64_t ldb, float *out, int64_t ldo, hipStream_t st);
dol_status launch_damp_apply2_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                  int64_t ldb, const float *out, int64_t ldo, const float *g, int64_t ldg, float *ga,
                                  float *gb, int32_t accumulate, hipStream_t st);
dol_status launch_nll_grad(int32_t batch, int32_t n, const float *p, int64_t ld, const int32_t *target, float *grad,
                           hipStream_t st);
// Convolution-shaped tables with a short second operand (damp_conv.hip)
bool conv_path_ok(const dol_fn_table *f);
bool byj_fwd_staged_ok(const dol_fn_table *f);   // forward through the per-j map with the first operand's row in LDS
bool staged_fwd_ok(const dol_fn_table *f);   // forward through the kernel that stages both operand rows in LDS
std::string damp_kernel_name(const dol_fn_table *f, bool backward, int64_t batch = 0);
// Large batches of contiguous, 16-byte aligned tensors (damp_conv_rows.hip); false: the call was not taken.
bool conv_rows_ok(const dol_fn_table *f, int64_t batch, bool backward);
bool apply2_bwd_staged(const dol_fn_table *f);       // the tuple-list backward stages the gated gradient row in LDS
bool launch_damp_conv_rows_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b, int64_t ldb,
                               float *out, int64_t ldo, hipStream_t st, dol_status *status);
bool launch_damp_conv_rows_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b, int64_t ldb,
                               const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate, hipStream_t st,
                               dol_status *status);
dol_status launch_damp_conv_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                int64_t ldb, float *out, int64_t ldo, hipStream_t st);
dol_status launch_damp_conv_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                                hipStream_t st);
// Arbitrary tables whose operand rows fit in LDS (damp_lds.hip); *done = false: the call was not taken.
dol_status lds_plan_build(dol_fn_table *tb, const std::vector<uint32_t> &col_ptr, const std::vector<uint32_t> &col_ij,
                          const std::vector<uint32_t> &rowa_ptr, const std::vector<uint32_t> &rowa_jc,
                          const std::vector<uint32_t> &rowb_ptr, const std::vector<uint32_t> &rowb_ic);
dol_status launch_damp_lds_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                               int64_t ldb, float *out, int64_t ldo, hipStream_t st, bool *done);
dol_status launch_damp_lds_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                               int64_t ldb, const float *out, int64_t ldo, const float *g, int64_t ldg, float *ga,
                               float *gb, int32_t accumulate, hipStream_t st, bool *done);
// Compiles `src` (HIP C++) for gfx950 at run time and returns the kernel `name` of it (damp_table.hip).
dol_status jit_compile(const std::string &src, const char *name, hipModule_t *mod, hipFunction_t *fn);
// A fold of convolution-shaped applies as code written for the chain's shape (fold_chain.hip): m[t] = symbols of the t-th
// running Distribution, nb[t] = symbols of input t >= 1.
constexpr int kFoldChainMax = 32;
bool fold_chain_ok(int n, const int32_t *m, const int32_t *nb, const int64_t *ld, int64_t ldo, int64_t ldg);
dol_status launch_fold_chain(int n, const int32_t *m, const int32_t *nb, int32_t batch, const float *const *in, const int64_t *ld,
                             float *const *gin, float *out, int64_t ldo, const int32_t *target, const float *gout, int64_t ldg,
                             int32_t backward, hipStream_t st);
// Small arbitrary tables as code written for the table (damp_table.hip); *done = false: the call was not taken
bool table_code_ok(const dol_fn_table *f);
dol_status launch_damp_table_fwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, float *out, int64_t ldo, hipStream_t st, bool *done);
dol_status launch_damp_table_bwd(const dol_fn_table *f, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                                 hipStream_t st, bool *done);
// out = union(filter(apply2(a, b, f)), c) and its reverse in one launch each; p = the filter-union plan over f's symbols
// and c's.  Contiguous 16-byte aligned tensors only (the callers check).
bool table_merge_ok(const dol_fn_table *f);
dol_status launch_damp_table_merge_fwd(const dol_fn_table *f, const UnionPlan *p, int32_t batch, const float *a, const float *b,
                                       const float *c, float *out, int32_t *saved, hipStream_t st);
dol_status launch_damp_table_merge_bwd(const dol_fn_table *f, const UnionPlan *p, int32_t batch, const float *a, const float *b,
                                       const float *c, const float *g, float *ga, float *gb, float *gc, const int32_t *saved,
                                       int32_t accumulate, hipStream_t st);
dol_status launch_damp_table_merge_both(const dol_fn_table *f, const UnionPlan *p, int32_t batch, const float *a, const float *b,
                                        const float *c, float *out, int32_t *saved, const float *g, float *ga, float *gb, float *gc,
                                        int32_t accumulate, hipStream_t st);
// Filter / Union on contiguous 16-byte aligned tensors (damp_rows.hip); *done = false: not taken
dol_status launch_rows_gather(int32_t batch, int32_t n_in, int32_t n_out, const int32_t *src_col, const float *in,
                              int64_t ldi, float *out, int64_t ldo, int32_t accumulate, hipStream_t st, bool *done);
dol_status launch_rows_union_fwd(const UnionPlan *p, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, float *out, int64_t ldo, hipStream_t st, bool *done);
dol_status launch_rows_union_bwd(const UnionPlan *p, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                                 hipStream_t st, bool *done);
dol_status launch_zero_rows(int32_t batch, int32_t n, float *x, int64_t ld, hipStream_t st);
dol_status launch_damp_filter_fwd(const FilterPlan *p, int32_t batch, const float *in, int64_t ldi, float *out,
                                  int64_t ldo, hipStream_t st);
dol_status launch_damp_filter_bwd(const FilterPlan *p, int32_t batch, const float *g, int64_t ldg, float *gin,
                                  int64_t ldgi, int32_t accumulate, hipStream_t st);
dol_status launch_damp_union_fwd(const UnionPlan *p, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, float *out, int64_t ldo, hipStream_t st);
dol_status launch_damp_union_bwd(const UnionPlan *p, int32_t batch, const float *a, int64_t lda, const float *b,
                                 int64_t ldb, const float *g, int64_t ldg, float *ga, float *gb, int32_t accumulate,
                                 hipStream_t st);

// Repeated Apply with feedback (iterate.hip).  Forward: any of hist / ckpt / out may be nullptr.  Backward: reads either
// the full history (hist) or r0 and the checkpoints written every `every` rounds.
dol_status check_iterate(const dol_dist *e, const dol_fn_table *f, int32_t rounds);
dol_status check_r0(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f);
dol_status launch_iterate_fwd(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds,
                              float *hist, float *ckpt, int32_t every, float *out, int64_t ldo, hipStream_t st);
dol_status launch_iterate_bwd(const dol_dist *e, const dol_fn_table *f, int32_t rounds, const float *hist,
                              const float *r0, int64_t ldr, const float *ckpt, int32_t every, const float *grad_out,
                              int64_t ldg, float *grad_r0, float *grad_e, hipStream_t st);

dol_status launch_dtkp_init(int32_t batch, int32_t n_sym, int32_t k, int32_t n_facts, const int32_t *d_fact_of_sym,
                            const float *fact_prob, uint64_t *mask, float *pprob, float *prob, int64_t ld,
                            hipStream_t st);
// fact_b != nullptr: the second operand is an input Distribution under natural initialisation, symbol j = fact
// fact_b[j] (device array); bm / bp are not read
dol_status launch_dtkp_apply2(const dol_fn_table *f, int32_t batch, int32_t k, int32_t n_facts, const GroupMasks &gm,
                              const float *fact_prob, const uint64_t *am, const float *ap, const uint64_t *bm,
                              const float *bp, const int32_t *fact_b, uint64_t *om, float *op, float *oprob, int64_t ldo,
                              hipStream_t st);
dol_status launch_dtkp_union(const UnionPlan *p, int32_t batch, int32_t k, const uint64_t *am, const float *ap,
                             const uint64_t *bm, const float *bp, uint64_t *om, float *op, float *oprob, int64_t ldo,
                             hipStream_t st);
dol_status launch_dtkp_prob_bwd(int32_t batch, int32_t n_sym, int32_t k, int32_t n_facts, const uint64_t *mask,
                                const float *pprob, const float *fact_prob, const float *g, int64_t ldg, float *gfact,
                                hipStream_t st);
dol_status launch_dtkp_filter(const FilterPlan *p, int32_t batch, int32_t k, const uint64_t *im, const float *ip,
                              const float *iprob, int64_t ldi, uint64_t *om, float *op, float *oprob, int64_t ldo,
                              hipStream_t st);

}  // namespace dol
