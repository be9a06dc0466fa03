// Repeated DAMP Apply with feedback (the fixed-round form of the recursion of App. B, Fig. 9):
//     r_{t+1}[c] = min(1, sum over the tuples (i, j) of column c of r_t[i] * e[j]),
// every round in one launch.  One workgroup owns a sample: r_t, r_{t+1} and the second operand sit in LDS; the
// function table never changes between rounds, so every thread keeps the first tuples of its own columns (rows, for
// the reverse sweep) in registers together with the tags of e they name, and a round is one burst of LDS reads,
// a short fma chain and a barrier.  Tuples beyond the first few of a column are read through the caches.
// Summation order and clamp decisions are those of dol_apply2 / dol_backward.
//
// What the reverse sweep needs of the rounds in between comes from one of two places: the full history r_0 ..
// r_rounds that the forward launch wrote when asked to (dol_iterate_apply2), or checkpoints r_R, r_2R, ... written
// every R rounds (dol_iterate_apply2_ckpt), from which the sweep replays a segment of R rounds forward in LDS before
// walking it backwards.  Inside LDS a round's result is kept as x = pre where pre <= 1 and -1 where the clamp acted:
// |x| is the clamped tag and the sign is the clamp's decision, so the reverse sweep never re-derives a sum.
//
// dol_iterate_apply2_backward runs both sweeps in one launch (damp_iterate_fwd_bwd_kernel) while the batch leaves units
// idle: the tables are fetched once, and the forward sweep writes the rounds of its last segment where the reverse sweep
// starts, so that segment is not replayed.  Larger batches get the two kernels back to back.  Every kernel is built for
// tables with columns or rows longer than the tuples a thread keeps in registers (TAILS) and for tables without, whose
// rounds then carry no tail loops and no workgroup-wide rows; and with five or six register slots per symbol.
//
// Rows in LDS lie a constant number of floats apart (the shape's threads times symbols per thread, plus one) and the
// reverse sweep's rounds run in unrolled stretches of eight: every LDS access of a round is then an address the thread
// computed once plus a constant carried by the instruction.
//
// The gradient w.r.t. e has one share per tuple and round.  A share belongs to the thread that owns the tuple's row
// and is summed over the rounds in a register (or in the tuple's own LDS word); at the end the shares of every symbol
// of e are added in ascending order of the first operand's symbol by one thread (rows of more than 64 tuples: by one
// wavefront, strided, then a fixed exchange tree).  No atomics: the result is the same bit for bit on every run.
#include "internal.h"
#include "wave_util.h"

#include <mutex>

namespace dol {

constexpr int kItMaxRow = 4096;         // most symbols of either operand
constexpr size_t kItLdsMax = 160 * 1024;

// The tuples [q0, q1) of one column or row: the first N in registers (with the tag of e each names), the rest
// behind `list`.  Register slots past the end of a short list point at the zero entry kept behind the operand
// row and carry the tag 0: their product is an exact +0 added after the real tuples, so no slot needs a branch.
template <int N>
struct Cached {
    uint32_t t[N];
    float e[N];
    uint32_t q0, q1;
};

// lo16 of a column tuple = symbol of r, hi16 = symbol of e; of a row tuple: lo16 = symbol of e, hi16 = column.
template <int N>
__device__ __forceinline__ void load_cached(Cached<N> &c, const uint32_t *__restrict__ ptr,
                                            const uint32_t *__restrict__ list, int r, int n, uint32_t dummy)
{
    c.q0 = c.q1 = 0;
    if (r < n) { c.q0 = ptr[r]; c.q1 = ptr[r + 1]; }
#pragma unroll
    for (int x = 0; x < N; ++x) c.t[x] = c.q0 + x < c.q1 ? list[c.q0 + x] : dummy;
}

// The tags of e the cached tuples name, from the staged row (whose entry nb is 0: the dummy tuples point there).
template <int N, bool E_IN_LO>
__device__ __forceinline__ void load_cached_tags(Cached<N> &c, const float *le)
{
#pragma unroll
    for (int x = 0; x < N; ++x) c.e[x] = le[E_IN_LO ? c.t[x] & 0xffffu : c.t[x] >> 16];
}

// pre of one column: sum over its tuples of |x[i]| * e[j], in list order, one fma each, starting from 0
// (TAILS = false: the table has no column or row of more than N tuples, so nothing lies behind the registers)
template <int N, bool TAILS>
__device__ __forceinline__ float col_pre(const Cached<N> &c, const uint32_t *__restrict__ list, const float *x,
                                         const float *le)
{
    float acc = 0.0f;
#pragma unroll
    for (int k = 0; k < N; ++k) acc = __builtin_fmaf(fabsf(x[c.t[k] & 0xffffu]), c.e[k], acc);
    if constexpr (TAILS) {
        for (uint32_t q = c.q0 + N; q < c.q1; ++q) {
            const uint32_t t = list[q];
            acc = __builtin_fmaf(fabsf(x[t & 0xffffu]), le[t >> 16], acc);
        }
    }
    return acc;
}

__device__ __forceinline__ float signed_tag(float pre) { return pre <= 1.0f ? pre : -1.0f; }

struct ItFwdArgs {
    int32_t batch, na, nb, rounds;
    const uint32_t *col_ptr, *col_ij;
    const float *r0;
    int64_t ldr;
    const float *e;
    int64_t lde;
    float *hist;                        // [rounds + 1, batch, na] or nullptr
    float *ckpt;                        // [n_ckpt, batch, na] or nullptr: r_every, r_2*every, ... (those before r_rounds)
    int32_t every;
    float *out;                         // [batch, ldo] or nullptr: r_rounds
    int64_t ldo;
};

// ---------------------------------------------------------------- rows in LDS

// Rows of tags lie T * K + 1 floats apart whatever the width of the operand: the shape's threads cover T * K symbols, so
// an element's address is a byte offset its thread keeps in a register plus a constant that the LDS instruction
// carries.  The entries from na on are zero in every row (the register slots of short tuple lists point at entry na,
// and threads past na own empty columns and rows: what they write there is zero again).
template <int T>
__device__ __forceinline__ void zero_row_ends(float *rows, int n_rows, int rs, int na)
{
    const int w = rs - na;
    for (int q = threadIdx.x; q < n_rows * w; q += T) rows[(q / w) * rs + na + q % w] = 0.0f;
}

// LDS addresses as 32-bit numbers: what a thread keeps in a register is the address of its element in the first row.
typedef __attribute__((address_space(3))) float lds_float;

__device__ __forceinline__ uint32_t lds_address(const float *p)
{
    return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((const lds_float *)p));
}

__device__ __forceinline__ float lds_at(uint32_t address) { return *reinterpret_cast<const lds_float *>(static_cast<uintptr_t>(address)); }

__device__ __forceinline__ void lds_put(uint32_t address, float v) { *reinterpret_cast<lds_float *>(static_cast<uintptr_t>(address)) = v; }

// (an address the compiler must take as it is: what is added to it afterwards stays a constant on the instruction)
__device__ __forceinline__ uint32_t fixed_offset(uint32_t x)
{
    asm volatile("" : "+v"(x));
    return x;
}

// `len` rounds inside LDS: row x + 1 (of `rows`, whose LDS address is rows_at) from row x, for x = 0 .. len - 1, a barrier
// after each; pre[k] = the unclamped sums of the last round.  Eight rounds per trip: the row is then a constant on the
// LDS instruction and the addresses of a thread's operands stay in registers.
template <int T, int K, int CA, bool TAILS>
__device__ __forceinline__ void rounds_in_rows(const float *rows, uint32_t rows_at, int len, const Cached<CA> (&col)[K],
                                               const uint32_t *__restrict__ list, const float *le, float (&pre)[K])
{
    constexpr int RS = T * K + 1, U = 8;
    constexpr uint32_t RB = RS * sizeof(float);
    const int tid = threadIdx.x;
    for (int xb = 0; xb < len; xb += U) {
        const uint32_t base = rows_at + xb * RB;
        uint32_t src[K][CA], dst[K];
#pragma unroll
        for (int k = 0; k < K; ++k) {
            dst[k] = fixed_offset(base + static_cast<uint32_t>(tid + T * k) * 4u);
#pragma unroll
            for (int y = 0; y < CA; ++y) src[k][y] = fixed_offset(base + (col[k].t[y] & 0xffffu) * 4u);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            if (xb + u < len) {
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    float acc = 0.0f;
#pragma unroll
                    for (int y = 0; y < CA; ++y) acc = __builtin_fmaf(fabsf(lds_at(src[k][y] + u * RB)), col[k].e[y], acc);
                    if constexpr (TAILS) {
                        const float *x_cur = rows + (xb + u) * RS;
                        for (uint32_t q = col[k].q0 + CA; q < col[k].q1; ++q) {
                            const uint32_t tu = list[q];
                            acc = __builtin_fmaf(fabsf(x_cur[tu & 0xffffu]), le[tu >> 16], acc);
                        }
                    }
                    pre[k] = acc;
                    lds_put(dst[k] + (u + 1) * RB, signed_tag(acc));
                }
                lds_barrier();
            }
        }
    }
}

// ---------------------------------------------------------------- forward

// One round from the row at `xc` into the row at `xn` (this thread's columns), then the workgroup's barrier.
// pre[k] = the column's unclamped sum.
template <int T, int K, int CA, bool TAILS>
__device__ __forceinline__ void iterate_round(const Cached<CA> (&col)[K], const uint32_t *__restrict__ list, const float *xc,
                                              float *xn, const float *le, float (&pre)[K])
{
    const int tid = threadIdx.x;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        pre[k] = col_pre<CA, TAILS>(col[k], list, xc, le);
        xn[tid + T * k] = signed_tag(pre[k]);
    }
    lds_barrier();
}

// (PRE: the caller has already fetched the columns' tuples into `col`)
template <int T, int K, int CA, bool TAILS, bool PRE = false>
__device__ __forceinline__ void iterate_forward(const ItFwdArgs &A, float *lds, Cached<CA> (&col)[K])
{
    // lds: x (two rows), e (nb + 1, ending with a zero).  PRE (both sweeps in one launch): the layout of the reverse
    // sweep instead, whose first two segment rows serve as x; the rounds of the last segment are then written row
    // after row into that segment, where the reverse sweep finds them without replaying them.
    constexpr int RS = T * K + 1;
    const int na = A.na, nb = A.nb;
    float *seg = lds + (PRE ? 2 * RS : 0);
    float *x0 = seg, *x1 = seg + RS;
    float *le = lds + (PRE ? A.every + 3 : 2) * RS;
    const int tid = threadIdx.x;
    const int64_t s = blockIdx.x;
    const int64_t plane = static_cast<int64_t>(A.batch) * na;
    const float *e_row = A.e + s * A.lde;
    for (int c = tid; c < na; c += T) {
        const float v = A.r0[s * A.ldr + c];
        x0[c] = v;
        if (A.hist) A.hist[s * na + c] = v;
        if (A.rounds == 0 && A.out) A.out[s * A.ldo + c] = v;
    }
    for (int j = tid; j <= nb; j += T) le[j] = j < nb ? e_row[j] : 0.0f;
    zero_row_ends<T>(lds, PRE ? A.every + 3 : 2, RS, na);
    if constexpr (!PRE) {
#pragma unroll
        for (int k = 0; k < K; ++k) load_cached(col[k], A.col_ptr, A.col_ij, tid + T * k, na, pack16(na, nb));
    }
    lds_barrier();
#pragma unroll
    for (int k = 0; k < K; ++k) load_cached_tags<CA, false>(col[k], le);
    // Rounds run in stretches that end where something leaves the chip: every round with a history, every
    // `every`-th with checkpoints, the last one always.  Inside a stretch a round is LDS reads, the fma chain, one
    // LDS write and the barrier; the two rows swap roles from round to round.
    const int stride = A.hist ? 1 : A.every;
    const int t_keep = PRE && A.rounds > 0 ? (A.rounds - 1) / A.every * A.every : A.rounds;    // first round of the kept segment
    float pre[K];
    int t = 0, n_ckpt = 0;
    while (t < t_keep) {
        const int stop = min(A.rounds, (t / stride + 1) * stride);
        for (; t + 1 < stop; t += 2) {
            iterate_round<T, K, CA, TAILS>(col, A.col_ij, x0, x1, le, pre);
            iterate_round<T, K, CA, TAILS>(col, A.col_ij, x1, x0, le, pre);
        }
        if (t < stop) {                     // an odd stretch: one more round, and the rows change names
            iterate_round<T, K, CA, TAILS>(col, A.col_ij, x0, x1, le, pre);
            float *sw = x0; x0 = x1; x1 = sw;
            ++t;
        }
        float *dst = nullptr;
        if (A.hist) dst = A.hist + t * plane + s * na;
        else if (t < A.rounds && A.ckpt) dst = A.ckpt + (n_ckpt++) * plane + s * na;
#pragma unroll
        for (int k = 0; k < K; ++k) {
            const int c = tid + T * k;
            const float v = fminf(pre[k], 1.0f);
            if (c < na) {
                if (dst) dst[c] = v;
                if (t == A.rounds && A.out) A.out[s * A.ldo + c] = v;
            }
        }
    }
    if constexpr (PRE) {
        if (A.rounds > 0) {
            if (x0 != seg) {                // r_t sits in the second row: every thread moves its own columns to the first
#pragma unroll
                for (int k = 0; k < K; ++k) seg[tid + T * k] = x0[tid + T * k];
                lds_barrier();
            }
            rounds_in_rows<T, K, CA, TAILS>(seg, lds_address(seg), A.rounds - t, col, A.col_ij, le, pre);
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int c = tid + T * k;
                if (c < na && A.out) A.out[s * A.ldo + c] = fminf(pre[k], 1.0f);
            }
        }
    }
}

template <int T, int K, int CA, bool TAILS>
__global__ void __launch_bounds__(T)
damp_iterate_fwd_kernel(const ItFwdArgs A)
{
    extern __shared__ float lds[];
    Cached<CA> col[K];
    iterate_forward<T, K, CA, TAILS>(A, lds, col);
}

// ---------------------------------------------------------------- backward

struct ItBwdArgs {
    int32_t batch, na, nb, rounds, every;   // every: rounds per segment (the checkpoint interval)
    int32_t n_tuples, n_long;
    int32_t shares_in_seg;                  // every tuple's share lives in a register during the sweep: the LDS words they
                                            // are gathered through at the end take the place of the (then spent) segment
    const uint32_t *col_ptr, *col_ij, *rowa_ptr, *rowa_jc, *rowb_ptr, *rowb_pos, *long_rows;
    const float *e;
    int64_t lde;
    const float *hist;                      // full history, or nullptr: then r0 and ckpt
    const float *r0;
    int64_t ldr;
    const float *ckpt;
    const float *gout;                      // upstream gradient w.r.t. r_rounds, or
    int64_t ldg;
    const int32_t *target;                  // [batch]: the loss is -log r_rounds[target], read from `out`
    const float *out;
    int64_t ldo;
    float *grad_r0;                         // [batch, na] or nullptr
    float *grad_e;                          // [batch, ldge] or nullptr
    int64_t ldge;
};

// Sum of x over the workgroup (every thread gets the total); `red` holds one float per wavefront.  Successive
// calls must alternate between two such arrays: a wavefront may still be reading the last call's partial sums.
template <int T>
__device__ __forceinline__ float block_sum(float x, float *red)
{
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) x += __shfl_xor(x, d, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) red[threadIdx.x / kWave] = x;
    lds_barrier();
    float tot = 0.0f;
#pragma unroll
    for (int w = 0; w < T / kWave; ++w) tot += red[w];
    return tot;
}

// Reverse sweep.  LDS: two gradient rows G[0], G[1], then seg[0 .. every] = the rounds of the segment being walked
// (seg[x] = signed r_{t0 + x}), e, one word per tuple for its share of d loss / d e, partial sums.  A thread owns the
// same symbols i of the first operand in every round.  The round at place x of its segment finds gh = the gradient
// reaching the unclamped sums of that round in G[(x + 1) & 1]; for each tuple (i, j, c) of its rows the thread reads
// gh[c] once: e[j] * gh[c] goes into g[i] = d loss / d r_t[i], and r_t[i] * gh[c] into the tuple's share.  g[i] gated
// with the sign of seg[x][i] (the decision of the round that produced r_t) is the next gh and goes to G[x & 1]; the
// first row of a segment comes from a checkpoint and carries no decision, so its gradient is handed over ungated, in
// G[0], and gated after the next segment has been replayed.  Rounds run in unrolled stretches of eight, so the row a
// read or write goes to is a constant on the instruction and a thread's byte offsets stay in registers.
template <int T, int K, int CA, bool TAILS, bool PRE = false>
__device__ __forceinline__ void iterate_backward(const ItBwdArgs &A, float *lds, Cached<CA> (&col)[K], Cached<CA> (&rowa)[K])
{
    constexpr int RS = T * K + 1;
    constexpr uint32_t RB = RS * sizeof(float);     // a row in bytes
    constexpr int U = 8;                            // rounds per unrolled stretch
    const int na = A.na, nb = A.nb;
    float *G = lds;
    float *seg = lds + 2 * RS;
    float *le = seg + static_cast<size_t>(A.every + 1) * RS;
    float *share_buf = A.shares_in_seg ? seg : le + nb + 1;
    float *red = A.shares_in_seg ? le + nb + 1 : share_buf + A.n_tuples;    // two arrays of T / 64
    const int tid = threadIdx.x;
    const int64_t s = blockIdx.x;
    const int64_t plane = static_cast<int64_t>(A.batch) * na;
    const float *e_row = A.e + s * A.lde;
    const float *gs = A.gout + s * A.ldg;
    if (A.rounds == 0) {
        if (A.grad_r0)
            for (int c = tid; c < na; c += T)
                A.grad_r0[s * na + c] = !A.target ? gs[c] : c == A.target[s] ? -1.0f / fmaxf(A.out[s * A.ldo + c], 1.17549435e-38f) : 0.0f;
        if (A.grad_e)
            for (int j = tid; j < nb; j += T) A.grad_e[s * A.ldge + j] = 0.0f;
        return;
    }
    for (int j = tid; j <= nb; j += T) le[j] = j < nb ? e_row[j] : 0.0f;
    if (!A.shares_in_seg)
        for (int q = tid; q < A.n_tuples; q += T) share_buf[q] = 0.0f;
    if (A.target) {
        const int tgt = A.target[s];
        for (int c = tid; c < na; c += T) G[c] = c == tgt ? -1.0f / fmaxf(A.out[s * A.ldo + c], 1.17549435e-38f) : 0.0f;
    } else {
        for (int c = tid; c < na; c += T) G[c] = gs[c];
    }
    if constexpr (!PRE) zero_row_ends<T>(lds, A.every + 3, RS, na);
    bool wide[K];                           // this row is summed by the whole workgroup
    float share[K][CA];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        if constexpr (!PRE) {
            load_cached(col[k], A.col_ptr, A.col_ij, tid + T * k, na, pack16(na, nb));
            load_cached(rowa[k], A.rowa_ptr, A.rowa_jc, tid + T * k, na, pack16(nb, na));
        }
        wide[k] = rowa[k].q1 - rowa[k].q0 > static_cast<uint32_t>(kLongTableRow);
#pragma unroll
        for (int x = 0; x < CA; ++x) share[k][x] = 0.0f;
    }
    int n_long_a = 0;                       // the long rows of the first operand come first in the list
    for (int l = 0; l < A.n_long; ++l) n_long_a += static_cast<int>(A.long_rows[l]) < na;
    int red_sel = 0;
    lds_barrier();                          // e is staged
    // addresses in the first row of LDS: of the columns a row's tuples read, of the thread's own symbols
    const uint32_t lds0 = lds_address(lds);
    uint32_t row_at[K][CA], own_at[K];
#pragma unroll
    for (int k = 0; k < K; ++k) {
        load_cached_tags<CA, false>(col[k], le);
        load_cached_tags<CA, true>(rowa[k], le);
        own_at[k] = fixed_offset(lds0 + static_cast<uint32_t>(tid + T * k) * 4u);
#pragma unroll
        for (int y = 0; y < CA; ++y) {
            row_at[k][y] = fixed_offset(lds0 + (rowa[k].t[y] >> 16) * 4u);
        }
    }

    const int n_seg = (A.rounds + A.every - 1) / A.every;
    for (int sg = n_seg - 1; sg >= 0; --sg) {
        const int t0 = sg * A.every, len = min(A.every, A.rounds - t0);
        // ---- the rounds of this segment into seg[0 .. len] (PRE: the forward sweep has left the last segment there)
        if (PRE && sg == n_seg - 1) {
        } else if (A.hist) {
            for (int x = 0; x <= len; ++x) {
                const float *h = A.hist + (t0 + x) * plane + s * na;
                for (int c = tid; c < na; c += T) seg[x * RS + c] = h[c];
            }
            lds_barrier();
            // a stored 1 may be a clamped sum: give it the sign of the decision (the magnitudes others read stay 1)
            for (int x = 1; x <= len; ++x) {
#pragma unroll
                for (int k = 0; k < K; ++k) {
                    const int c = tid + T * k;
                    if (c < na && seg[x * RS + c] >= 1.0f)
                        seg[x * RS + c] = signed_tag(col_pre<CA, TAILS>(col[k], A.col_ij, seg + (x - 1) * RS, le)) < 0.0f ? -1.0f : 1.0f;
                }
            }
            lds_barrier();
        } else {
            const float *first = sg == 0 ? A.r0 + s * A.ldr : A.ckpt + (sg - 1) * plane + s * na;
            for (int c = tid; c < na; c += T) seg[c] = first[c];
            lds_barrier();
            float pre[K];
            rounds_in_rows<T, K, CA, TAILS>(seg, lds_address(seg), len, col, A.col_ij, le, pre);
        }
        // ---- the gradient handed over by the later segment (or the upstream gradient), in G[0], meets the decision of
        // this segment's last round and goes where that round looks for it
        {
            float *g_top = G + (len & 1) * RS;
#pragma unroll
            for (int k = 0; k < K; ++k) {
                const int c = tid + T * k;
                if (c < na) g_top[c] = seg[len * RS + c] < 0.0f ? 0.0f : G[c];
            }
        }
        lds_barrier();
        // ---- walk the segment backwards
        for (int xb = (len - 1) / U * U; xb >= 0; xb -= U) {
            const uint32_t base = (2 + xb) * RB;
            uint32_t own_x[K];
#pragma unroll
            for (int k = 0; k < K; ++k) own_x[k] = fixed_offset(own_at[k] + base);
#pragma unroll
            for (int u = U - 1; u >= 0; --u) {
                if (xb + u < len) {
                    const int x = xb + u;
                    const uint32_t g_in = ((u + 1) & 1) * RB, g_nx = (u & 1) * RB;
                    float g_wide[K];
#pragma unroll
                    for (int k = 0; k < K; ++k) g_wide[k] = 0.0f;
                    if constexpr (TAILS) {
                        // rows with many tuples: the whole workgroup takes strided shares of the row
                        const float *gin = G + ((u + 1) & 1) * RS, *xr = seg + x * RS;
                        for (int l = 0; l < n_long_a; ++l) {
                            const int i = static_cast<int>(A.long_rows[l]);
                            const float ri = fabsf(xr[i]);
                            float acc = 0.0f;
                            for (uint32_t q = A.rowa_ptr[i] + tid, q1 = A.rowa_ptr[i + 1]; q < q1; q += T) {
                                const uint32_t tu = A.rowa_jc[q];
                                const float ghc = gin[tu >> 16];
                                acc = __builtin_fmaf(le[tu & 0xffffu], ghc, acc);
                                share_buf[q] = __builtin_fmaf(ri, ghc, share_buf[q]);
                            }
                            const float tot = block_sum<T>(acc, red + red_sel * (T / kWave));
                            red_sel ^= 1;
#pragma unroll
                            for (int k = 0; k < K; ++k)
                                if (i == tid + T * k) g_wide[k] = tot;
                        }
                    }
#pragma unroll
                    for (int k = 0; k < K; ++k) {
                        const float xi = lds_at(own_x[k] + u * RB);
                        const float ri = fabsf(xi);
                        float g = g_wide[k];
                        if (!TAILS || !wide[k]) {
                            float g_odd = 0.0f;             // two chains of half the length
#pragma unroll
                            for (int y = 0; y < CA; ++y) {
                                const float ghc = lds_at(row_at[k][y] + g_in);
                                if (y & 1) g_odd = __builtin_fmaf(rowa[k].e[y], ghc, g_odd);
                                else g = __builtin_fmaf(rowa[k].e[y], ghc, g);
                                share[k][y] = __builtin_fmaf(ri, ghc, share[k][y]);
                            }
                            g += g_odd;
                            if constexpr (TAILS) {
                                const float *gin = G + ((u + 1) & 1) * RS;
                                for (uint32_t q = rowa[k].q0 + CA; q < rowa[k].q1; ++q) {   // tuples past the registers
                                    const uint32_t tu = A.rowa_jc[q];
                                    const float ghc = gin[tu >> 16];
                                    g = __builtin_fmaf(le[tu & 0xffffu], ghc, g);
                                    share_buf[q] = __builtin_fmaf(ri, ghc, share_buf[q]);
                                }
                            }
                        }
                        lds_put(own_at[k] + g_nx, (x > 0 && xi < 0.0f) ? 0.0f : g);
                    }
                    lds_barrier();
                }
            }
        }
    }
    if (A.grad_r0)
        for (int c = tid; c < na; c += T) A.grad_r0[s * na + c] = G[c];
    if (!A.grad_e) return;
    // ---- the tuples' shares meet per symbol of e, in the order of the symbol's row (ascending first operand)
#pragma unroll
    for (int k = 0; k < K; ++k)
        if (!wide[k])
#pragma unroll
            for (int y = 0; y < CA; ++y)
                if (rowa[k].q0 + y < rowa[k].q1) share_buf[rowa[k].q0 + y] = share[k][y];
    lds_barrier();
    for (int j = tid; j < nb; j += T) {
        const uint32_t q0 = A.rowb_ptr[j], q1 = A.rowb_ptr[j + 1];
        if (q1 - q0 > static_cast<uint32_t>(kLongTableRow)) continue;
        float tot = 0.0f;
        for (uint32_t q = q0; q < q1; ++q) tot += share_buf[A.rowb_pos[q]];
        A.grad_e[s * A.ldge + j] = tot;
    }
    const int wave = tid / kWave, lane = tid & (kWave - 1);
    for (int l = n_long_a + wave; l < A.n_long; l += T / kWave) {
        const int j = static_cast<int>(A.long_rows[l]) - na;
        float tot = 0.0f;
        for (uint32_t q = A.rowb_ptr[j] + lane, q1 = A.rowb_ptr[j + 1]; q < q1; q += kWave) tot += share_buf[A.rowb_pos[q]];
#pragma unroll
        for (int d = 32; d >= 1; d >>= 1) tot += __shfl_xor(tot, d, kWave);
        if (lane == 0) A.grad_e[s * A.ldge + j] = tot;
    }
}

// (at least four wavefronts per SIMD, 128 registers per lane; eight, 64 registers, for the shape that large batches of a
// five-tuple table run in, so that two of its workgroups share a unit)
template <int T, int K, int CA, bool TAILS>
__global__ void __launch_bounds__(T, (T == 1024 && K == 1 && CA == 5 ? 8 : 4))
damp_iterate_bwd_kernel(const ItBwdArgs A)
{
    extern __shared__ float lds[];
    Cached<CA> col[K], rowa[K];
    iterate_backward<T, K, CA, TAILS>(A, lds, col, rowa);
}

// Forward and reverse sweep in one launch: the tables are found in cache the second time, nothing waits for a second
// launch, and a thread reads back only checkpoint and result entries that it wrote itself.
template <int T, int K, int CA, bool TAILS>
__global__ void __launch_bounds__(T, 4)
damp_iterate_fwd_bwd_kernel(const ItFwdArgs F, const ItBwdArgs B)
{
    extern __shared__ float lds[];
    // both sweeps' tuples are fetched once, up front: the reverse sweep then starts without waiting for its tables
    Cached<CA> col[K], rowa[K];
    const int tid = threadIdx.x;
#pragma unroll
    for (int k = 0; k < K; ++k) {
        load_cached(col[k], F.col_ptr, F.col_ij, tid + T * k, F.na, pack16(F.na, F.nb));
        load_cached(rowa[k], B.rowa_ptr, B.rowa_jc, tid + T * k, F.na, pack16(F.nb, F.na));
    }
    iterate_forward<T, K, CA, TAILS, true>(F, lds, col);
    __syncthreads();
    iterate_backward<T, K, CA, TAILS, true>(B, lds, col, rowa);
}

// ---------------------------------------------------------------- host side

dol_status check_iterate(const dol_dist *e, const dol_fn_table *f, int32_t rounds)
{
    if (!e || !f) return fail(DOL_EINVAL, "NULL argument");
    if (rounds < 0) return fail(DOL_EINVAL, "rounds is negative");
    if (e->batch < 0 || e->n_sym != f->nb || e->ld < e->n_sym) return fail(DOL_ESHAPE, "e has %d symbols, the table needs %d", e->n_sym, f->nb);
    if (f->n_out != f->na) return fail(DOL_EUNSUPPORTED, "the table maps %d symbols to %d: not square", f->na, f->n_out);
    if (f->na > kItMaxRow || f->nb > kItMaxRow) return fail(DOL_EUNSUPPORTED, "operands of more than %d symbols", kItMaxRow);
    if (e->batch > 0 && e->n_sym > 0 && !e->prob) return fail(DOL_EINVAL, "e.prob is NULL");
    return DOL_OK;
}

dol_status check_r0(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f)
{
    if (!r0) return fail(DOL_EINVAL, "r0 is NULL");
    if (r0->batch != e->batch || r0->n_sym != f->na || r0->ld < r0->n_sym)
        return fail(DOL_ESHAPE, "r0 has %d x %d, the table needs %d x %d", r0->batch, r0->n_sym, e->batch, f->na);
    if (r0->sym_ids)
        for (int32_t c = 0; c < f->na; ++c)
            if (r0->sym_ids[c] != f->out_syms[c])
                return fail(DOL_EUNSUPPORTED, "the table produces symbol %d where r0 has %d: a round's result cannot feed the next", f->out_syms[c], r0->sym_ids[c]);
    if (r0->batch > 0 && f->na > 0 && !r0->prob) return fail(DOL_EINVAL, "r0.prob is NULL");
    return DOL_OK;
}

// Launch shape: threads per workgroup, symbols of the first operand per thread, tuples of a column or row in registers;
// tails: some column or row of the table has more tuples than that.
// (a batch that leaves units idle gets the widest workgroup: a round is then bound by the latency of its LDS reads
// and barrier, which more wavefronts hide; a batch of several workgroups per unit gets two columns per thread; a
// table of at most five tuples per column and row - a grid's four neighbours and the node itself - gets five slots)
struct ItShape {
    int T, K, CA;
    bool tails;
    size_t row() const { return static_cast<size_t>(T) * K + 1; }     // floats between two rows in LDS
};

static ItShape pick_shape(const dol_fn_table *f, int32_t batch, bool reverse)
{
    const int longest = static_cast<int>(std::max(f->max_col_len, f->max_rowa_len));
    ItShape s;
    if (f->na <= 512) s = {512, 1, 6, false};
    // (the reverse sweep of a table of five tuples fits 64 registers with one symbol per thread: two workgroups of
    // sixteen wavefronts then fill a unit, and that is its fastest shape at any batch)
    else if (f->na <= 1024 && (batch <= 512 || (reverse && longest <= 5))) s = {1024, 1, 6, false};
    else if (f->na <= 1024) s = {512, 2, 6, false};
    else if (f->na <= 2048) s = {512, 4, 3, false};
    else s = {1024, 4, 3, false};
    if (s.CA == 6 && longest <= 5) s.CA = 5;
    s.tails = longest > s.CA;
    return s;
}

#define DOL_IT_ALL(X)                                                                                                  \
    X(512, 1, 5, false) X(512, 1, 6, false) X(512, 1, 6, true)                                                         \
    X(1024, 1, 5, false) X(1024, 1, 6, false) X(1024, 1, 6, true)                                                      \
    X(512, 2, 5, false) X(512, 2, 6, false) X(512, 2, 6, true)                                                         \
    X(512, 4, 3, false) X(512, 4, 3, true) X(1024, 4, 3, false) X(1024, 4, 3, true)

struct FwdKernels {
    template <int T, int K, int CA, bool TL> static const void *get() { return reinterpret_cast<const void *>(&damp_iterate_fwd_kernel<T, K, CA, TL>); }
};
struct BwdKernels {
    template <int T, int K, int CA, bool TL> static const void *get() { return reinterpret_cast<const void *>(&damp_iterate_bwd_kernel<T, K, CA, TL>); }
};
struct FwdBwdKernels {
    template <int T, int K, int CA, bool TL> static const void *get() { return reinterpret_cast<const void *>(&damp_iterate_fwd_bwd_kernel<T, K, CA, TL>); }
};

// One workgroup per sample; `args` are the kernel's arguments in order.  (The reverse sweep may ask for more than
// 64 KB of LDS.)
template <class Kernels, class... Args>
static dol_status launch_shape(const ItShape &sh, int32_t batch, size_t lds, hipStream_t st, const Args &...args)
{
    const void *kern = nullptr;
#define DOL_IT_ONE(T_, K_, CA_, TL_)                                                                                   \
    if (sh.T == T_ && sh.K == K_ && sh.CA == CA_ && sh.tails == TL_) kern = Kernels::template get<T_, K_, CA_, TL_>();
    DOL_IT_ALL(DOL_IT_ONE)
#undef DOL_IT_ONE
    if (!kern) return fail(DOL_EUNSUPPORTED, "no iteration kernel of %d threads x %d symbols with %d tuples", sh.T, sh.K, sh.CA);
    if (lds > 64 * 1024) DOL_HIP(allow_dynamic_lds(kern, kItLdsMax));
    void *argv[] = {const_cast<void *>(static_cast<const void *>(&args))...};
    DOL_HIP(hipLaunchKernel(kern, dim3(static_cast<unsigned>(batch)), dim3(static_cast<unsigned>(sh.T)), argv, lds, st));
    return DOL_OK;
}

static size_t fwd_lds(const dol_fn_table *f, const ItShape &sh) { return sizeof(float) * (2 * sh.row() + f->nb + 1); }

// The shares of d loss / d e can wait in registers alone when no row of the first operand has more tuples than the
// registers hold (a long row of e only matters when the shares are gathered); the words they are gathered through at
// the end then fit where the segment was.
static bool shares_in_seg(const dol_fn_table *f, const ItShape &sh, int32_t every)
{
    return static_cast<int>(f->max_rowa_len) <= sh.CA && f->n_long_rowa == 0 &&
           static_cast<size_t>(f->n_tuples) <= (static_cast<size_t>(every) + 1) * sh.row();
}

static size_t bwd_lds(const dol_fn_table *f, const ItShape &sh, int32_t every)
{
    const size_t shares = shares_in_seg(f, sh, every) ? 0 : static_cast<size_t>(f->n_tuples);
    return sizeof(float) * ((static_cast<size_t>(every) + 3) * sh.row() + f->nb + 1 + shares + 2 * 16);
}

static ItFwdArgs fwd_args(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds, float *hist, float *ckpt,
                          int32_t every, float *out, int64_t ldo)
{
    ItFwdArgs A{};
    A.batch = r0->batch, A.na = f->na, A.nb = f->nb, A.rounds = rounds;
    A.col_ptr = f->col_ptr.ptr, A.col_ij = f->col_ij.ptr;
    A.r0 = r0->prob, A.ldr = r0->ld, A.e = e->prob, A.lde = e->ld;
    A.hist = hist, A.ckpt = ckpt, A.every = every > 0 ? every : rounds + 1, A.out = out, A.ldo = ldo;
    return A;
}

static ItBwdArgs bwd_args(const dol_dist *e, const dol_fn_table *f, const ItShape &sh, int32_t rounds, const float *hist, const float *r0,
                          int64_t ldr, const float *ckpt, int32_t every, const float *grad_out, int64_t ldg, float *grad_r0, float *grad_e)
{
    ItBwdArgs A{};
    A.batch = e->batch, A.na = f->na, A.nb = f->nb, A.rounds = rounds, A.every = every;
    A.n_tuples = static_cast<int32_t>(f->n_tuples), A.n_long = static_cast<int32_t>(f->long_rows.n);
    A.shares_in_seg = shares_in_seg(f, sh, every) ? 1 : 0;
    A.col_ptr = f->col_ptr.ptr, A.col_ij = f->col_ij.ptr, A.rowa_ptr = f->rowa_ptr.ptr, A.rowa_jc = f->rowa_jc.ptr;
    A.rowb_ptr = f->rowb_ptr.ptr, A.rowb_pos = f->rowb_pos.ptr, A.long_rows = f->long_rows.ptr;
    A.e = e->prob, A.lde = e->ld, A.hist = hist, A.r0 = r0, A.ldr = ldr, A.ckpt = ckpt;
    A.gout = grad_out, A.ldg = ldg, A.grad_r0 = grad_r0, A.grad_e = grad_e, A.ldge = e->ld;
    return A;
}

dol_status launch_iterate_fwd(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds,
                                     float *hist, float *ckpt, int32_t every, float *out, int64_t ldo, hipStream_t st)
{
    const ItShape sh = pick_shape(f, r0->batch, false);
    const size_t lds = fwd_lds(f, sh);
    if (lds > 64 * 1024) return fail(DOL_EUNSUPPORTED, "the rows need %zu bytes of LDS, more than 65536", lds);
    const ItFwdArgs A = fwd_args(r0, e, f, rounds, hist, ckpt, every, out, ldo);
    return launch_shape<FwdKernels>(sh, r0->batch, lds, st, A);
}

// (target: the loss is -log r_rounds[target], read from `out`; else grad_out is the upstream gradient)
static dol_status launch_reverse(const dol_dist *e, const dol_fn_table *f, int32_t rounds, const float *hist, const float *r0,
                                 int64_t ldr, const float *ckpt, int32_t every, const int32_t *target, const float *out, int64_t ldo,
                                 const float *grad_out, int64_t ldg, float *grad_r0, float *grad_e, hipStream_t st)
{
    if (!f->rowb_pos.ptr && f->n_tuples > 0) return fail(DOL_EINVAL, "the table lacks the row cross-index of square tables");
    const ItShape sh = pick_shape(f, e->batch, true);
    const size_t lds = bwd_lds(f, sh, every);
    if (lds > kItLdsMax)
        return fail(DOL_EUNSUPPORTED, "segments of %d rounds need %zu bytes of LDS, more than %zu", every, lds, kItLdsMax);
    ItBwdArgs A = bwd_args(e, f, sh, rounds, hist, r0, ldr, ckpt, every, grad_out, ldg, grad_r0, grad_e);
    A.target = target, A.out = out, A.ldo = ldo;
    return launch_shape<BwdKernels>(sh, e->batch, lds, st, A);
}

dol_status launch_iterate_bwd(const dol_dist *e, const dol_fn_table *f, int32_t rounds, const float *hist,
                                     const float *r0, int64_t ldr, const float *ckpt, int32_t every,
                                     const float *grad_out, int64_t ldg, float *grad_r0, float *grad_e, hipStream_t st)
{
    return launch_reverse(e, f, rounds, hist, r0, ldr, ckpt, every, nullptr, nullptr, 0, grad_out, ldg, grad_r0, grad_e, st);
}

// Both sweeps of one call.  A batch that leaves units idle runs them in one launch (nothing waits for a second launch,
// the tables are fetched once, the last segment is not replayed); a larger batch in two launches back to back, each in
// the shape and with the LDS of its own sweep: the forward sweep then runs four workgroups to a unit instead of the
// reverse sweep's two, which is worth more than the replayed segment (B = 8192, 32 x 32 grid: 0.26 + 0.77 ms against 1.09).
constexpr int32_t kOneLaunchBatch = 512;

static dol_status launch_iterate_fwd_bwd(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds, int32_t every,
                                         float *out, int64_t ldo, float *ckpt, const int32_t *target, const float *grad_out,
                                         int64_t ldg, float *grad_r0, float *grad_e, hipStream_t st)
{
    if (!f->rowb_pos.ptr && f->n_tuples > 0) return fail(DOL_EINVAL, "the table lacks the row cross-index of square tables");
    if (e->batch > kOneLaunchBatch) {
        if (dol_status s = launch_iterate_fwd(r0, e, f, rounds, nullptr, ckpt, every, out, ldo, st)) return s;
        return launch_reverse(e, f, rounds, nullptr, r0->prob, r0->ld, ckpt, every, target, out, ldo, grad_out, ldg, grad_r0, grad_e, st);
    }
    const ItShape sh = pick_shape(f, e->batch, true);
    const size_t lds = bwd_lds(f, sh, every);           // (holds the forward sweep's rows as well)
    if (lds > kItLdsMax)
        return fail(DOL_EUNSUPPORTED, "segments of %d rounds need %zu bytes of LDS, more than %zu", every, lds, kItLdsMax);
    const ItFwdArgs F = fwd_args(r0, e, f, rounds, nullptr, ckpt, every, out, ldo);
    ItBwdArgs B = bwd_args(e, f, sh, rounds, nullptr, r0->prob, r0->ld, ckpt, every, grad_out, ldg, grad_r0, grad_e);
    B.target = target, B.out = out, B.ldo = ldo;
    return launch_shape<FwdBwdKernels>(sh, e->batch, lds, st, F, B);
}

// Rounds per segment when the sweep reads a full history: as many as fit beside one more workgroup on the unit.
static int32_t hist_segment(const dol_fn_table *f, int32_t batch, int32_t rounds)
{
    const ItShape sh = pick_shape(f, batch, true);
    int32_t every = 8;
    while (every > 1 && bwd_lds(f, sh, every) > kItLdsMax / 2) every >>= 1;
    return std::max(1, std::min(every, std::max(rounds, 1)));
}

}  // namespace dol

using namespace dol;

extern "C" {

dol_status dol_iterate_apply2(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds, float *hist,
                              void *hip_stream)
{
    if (dol_status st = check_iterate(e, f, rounds)) return st;
    if (dol_status st = check_r0(r0, e, f)) return st;
    if (r0->batch == 0 || f->na == 0) return DOL_OK;
    if (!hist) return fail(DOL_EINVAL, "hist is NULL");
    return launch_iterate_fwd(r0, e, f, rounds, hist, nullptr, 0, nullptr, 0, static_cast<hipStream_t>(hip_stream));
}

dol_status dol_iterate_backward(const dol_dist *e, const dol_fn_table *f, int32_t rounds, const float *hist,
                                const float *grad_out, int64_t grad_out_ld, float *grad_r0, float *grad_e,
                                void *hip_stream)
{
    if (dol_status st = check_iterate(e, f, rounds)) return st;
    if (e->batch == 0 || f->na == 0 || (!grad_r0 && !grad_e)) return DOL_OK;
    if (!hist || !grad_out) return fail(DOL_EINVAL, "hist or grad_out is NULL");
    if (grad_out_ld < f->na) return fail(DOL_ESHAPE, "grad_out_ld = %lld is smaller than %d", static_cast<long long>(grad_out_ld), f->na);
    return launch_iterate_bwd(e, f, rounds, hist, nullptr, 0, nullptr, hist_segment(f, e->batch, rounds), grad_out, grad_out_ld,
                              grad_r0, grad_e, static_cast<hipStream_t>(hip_stream));
}

int32_t dol_iterate_ckpt_every(const dol_fn_table *f, int32_t batch, int32_t rounds)
{
    if (!f || rounds <= 1 || f->na <= 0) return 1;
    const ItShape sh = pick_shape(f, batch, true);
    // a batch that leaves units idle: one workgroup has a unit's LDS to itself; else as many workgroups as fill a
    // unit's 32 wavefronts share it
    const size_t sharers = batch <= kOneLaunchBatch ? 1 : std::max(1, 32 / (sh.T / kWave));
    const size_t budget = batch <= kOneLaunchBatch ? kItLdsMax - 4096 : kItLdsMax / sharers - 1024;
    for (int32_t n_seg = 1; n_seg <= rounds; ++n_seg) {
        const int32_t every = (rounds + n_seg - 1) / n_seg;
        if (bwd_lds(f, sh, every) <= budget) return every;
    }
    return 1;
}

int32_t dol_iterate_ckpt_count(int32_t rounds, int32_t ckpt_every)
{
    if (rounds <= 0 || ckpt_every <= 0) return 0;
    return (rounds + ckpt_every - 1) / ckpt_every - 1;
}

dol_status dol_iterate_apply2_ckpt(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds,
                                   int32_t ckpt_every, dol_dist *out, float *ckpt, void *hip_stream)
{
    if (dol_status st = check_iterate(e, f, rounds)) return st;
    if (dol_status st = check_r0(r0, e, f)) return st;
    if (ckpt_every < 1) return fail(DOL_EINVAL, "ckpt_every = %d, must be at least 1", ckpt_every);
    if (!out) return fail(DOL_EINVAL, "out is NULL");
    if (out->batch != r0->batch || out->n_sym != f->na || out->ld < out->n_sym)
        return fail(DOL_ESHAPE, "out has %d x %d, the rounds produce %d x %d", out->batch, out->n_sym, r0->batch, f->na);
    if (r0->batch == 0 || f->na == 0) return DOL_OK;
    if (!out->prob) return fail(DOL_EINVAL, "out.prob is NULL");
    if (dol_iterate_ckpt_count(rounds, ckpt_every) > 0 && !ckpt) return fail(DOL_EINVAL, "ckpt is NULL");
    return launch_iterate_fwd(r0, e, f, rounds, nullptr, ckpt, ckpt_every, out->prob, out->ld, static_cast<hipStream_t>(hip_stream));
}

dol_status dol_iterate_backward_ckpt(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds,
                                     int32_t ckpt_every, const float *ckpt, const float *grad_out, int64_t grad_out_ld,
                                     float *grad_r0, float *grad_e, void *hip_stream)
{
    if (dol_status st = check_iterate(e, f, rounds)) return st;
    if (dol_status st = check_r0(r0, e, f)) return st;
    if (ckpt_every < 1) return fail(DOL_EINVAL, "ckpt_every = %d, must be at least 1", ckpt_every);
    if (e->batch == 0 || f->na == 0 || (!grad_r0 && !grad_e)) return DOL_OK;
    if (!grad_out) return fail(DOL_EINVAL, "grad_out is NULL");
    if (grad_out_ld < f->na) return fail(DOL_ESHAPE, "grad_out_ld = %lld is smaller than %d", static_cast<long long>(grad_out_ld), f->na);
    if (dol_iterate_ckpt_count(rounds, ckpt_every) > 0 && !ckpt) return fail(DOL_EINVAL, "ckpt is NULL");
    const int32_t every = std::max(1, std::min(ckpt_every, std::max(rounds, 1)));
    return launch_iterate_bwd(e, f, rounds, nullptr, r0->prob, r0->ld, ckpt, every, grad_out, grad_out_ld, grad_r0,
                              grad_e, static_cast<hipStream_t>(hip_stream));
}

dol_status dol_iterate_apply2_backward(const dol_dist *r0, const dol_dist *e, const dol_fn_table *f, int32_t rounds,
                                       int32_t ckpt_every, dol_dist *out, float *ckpt, const int32_t *target_col,
                                       const float *grad_out, int64_t grad_out_ld, float *grad_r0, float *grad_e,
                                       void *hip_stream)
{
    if (dol_status st = check_iterate(e, f, rounds)) return st;
    if (dol_status st = check_r0(r0, e, f)) return st;
    if (ckpt_every < 1) return fail(DOL_EINVAL, "ckpt_every = %d, must be at least 1", ckpt_every);
    if (!out) return fail(DOL_EINVAL, "out is NULL");
    if (out->batch != r0->batch || out->n_sym != f->na || out->ld < out->n_sym)
        return fail(DOL_ESHAPE, "out has %d x %d, the rounds produce %d x %d", out->batch, out->n_sym, r0->batch, f->na);
    if (!target_col && !grad_out) return fail(DOL_EINVAL, "target_col and grad_out are both NULL");
    if (target_col && grad_out) return fail(DOL_EINVAL, "target_col and grad_out are both given");
    if (grad_out && grad_out_ld < f->na) return fail(DOL_ESHAPE, "grad_out_ld = %lld is smaller than %d", static_cast<long long>(grad_out_ld), f->na);
    if (!grad_r0 && !grad_e) return fail(DOL_EINVAL, "grad_r0 and grad_e are both NULL");
    if (r0->batch == 0 || f->na == 0) return DOL_OK;
    if (!out->prob) return fail(DOL_EINVAL, "out.prob is NULL");
    if (dol_iterate_ckpt_count(rounds, ckpt_every) > 0 && !ckpt) return fail(DOL_EINVAL, "ckpt is NULL");
    const int32_t every = std::max(1, std::min(ckpt_every, std::max(rounds, 1)));
    return launch_iterate_fwd_bwd(r0, e, f, rounds, every, out->prob, out->ld, ckpt, target_col, grad_out, grad_out_ld, grad_r0,
                                  grad_e, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"
