// One thread per (sample, element) of a [batch, n] space, consecutive lanes on consecutive elements of one row:
// a workgroup owns a chunk of whole rows (about 2048 elements) and splits its flat element index into
// (row, column) with a float reciprocal, which is exact for such small indices.  A row wider than a chunk is cut
// into chunks of its own, one workgroup each, so that a small batch of wide rows still fills the chip.
#pragma once

#include "internal.h"

namespace dol {

constexpr int kThreads = 256;
constexpr int kChunk = 2048;            // elements per workgroup (whole rows)

struct Rows {                           // how a [batch, n] element space is cut into workgroup chunks
    int32_t batch, n, rpb;
    int32_t cpr;                        // rpb == 1: chunks (workgroups) per row
    float inv_n;
    unsigned grid;
};

static inline Rows rows_of(int32_t batch, int32_t n)
{
    Rows r;
    r.batch = batch;
    r.n = n;
    r.rpb = n >= kChunk ? 1 : kChunk / n;
    r.cpr = r.rpb == 1 ? (n + kChunk - 1) / kChunk : 1;
    r.inv_n = 1.0f / static_cast<float>(n);
    r.grid = static_cast<unsigned>((static_cast<int64_t>(batch) + r.rpb - 1) / r.rpb * r.cpr);
    return r;
}

// Calls f(sample, column) for every element of this workgroup's chunk.
template <typename F>
__device__ __forceinline__ void for_each_element(const Rows &R, F f)
{
    if (R.rpb == 1) {
        const int64_t s = blockIdx.x / static_cast<unsigned>(R.cpr);
        const int c0 = static_cast<int>(blockIdx.x - s * R.cpr) * kChunk, c1 = min(R.n, c0 + kChunk);
        for (int c = c0 + threadIdx.x; c < c1; c += kThreads) f(s, c);
        return;
    }
    const int64_t s0 = static_cast<int64_t>(blockIdx.x) * R.rpb;
    const int rows = static_cast<int>(min(static_cast<int64_t>(R.rpb), R.batch - s0));
    const int total = rows * R.n;
#pragma unroll 4
    for (int e = threadIdx.x; e < total; e += kThreads) {
        int r = static_cast<int>(static_cast<float>(e) * R.inv_n);
        int c = e - r * R.n;
        if (c < 0) { c += R.n; --r; } else if (c >= R.n) { c -= R.n; ++r; }
        f(s0 + r, c);
    }
}

}  // namespace dol
