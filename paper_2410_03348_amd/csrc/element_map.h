// One thread per (sample, element) of a [batch, n] space, consecutive lanes on consecutive elements of one row:
// a workgroup owns a chunk of whole rows (about 2048 elements) and splits its flat element index into
// (row, column) with a float reciprocal, which is exact for such small indices.  A row wider than a chunk is cut
// into chunks of its own, one workgroup each, so that a small batch of wide rows still fills the chip.
#pragma once

#include "internal.h"

#include <algorithm>

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

// ---- operand rows staged whole in LDS: one workgroup of kStageThreads per (sample, part of the output row)
//
// A gather from a row of thousands of tags misses the first-level cache on nearly every lane; from LDS it costs a
// bank conflict or two.  So for wide operand rows a workgroup first copies the sample's row(s) into LDS with
// coalesced loads and then gathers there.  Small batches are cut into several parts per sample (each stages the row
// again) so that the chip still fills.
constexpr int kStageThreads = 1024;
constexpr int kStageUnroll = 4;                       // outputs a thread works on at a time (their loads in flight together)

static inline bool stage_fits(int64_t row_floats) { return row_floats >= kStageMinRow && row_floats * 4 <= static_cast<int64_t>(kStageMaxBytes); }

// Parts per sample: enough workgroups for about two per compute unit, at most one per kStageThreads outputs.
static inline int32_t stage_parts(int32_t batch, int32_t n_out)
{
    const int32_t most = (n_out + kStageThreads - 1) / kStageThreads;
    const int32_t want = (512 + batch - 1) / batch;
    return std::max(1, std::min(most, want));
}

// Copies n floats into LDS with every thread of the workgroup; 16-byte pieces when the source row allows.
__device__ __forceinline__ void stage_row(float *__restrict__ dst, const float *__restrict__ src, int n)
{
    if ((reinterpret_cast<uintptr_t>(src) & 15u) == 0) {
        const int n4 = n >> 2;
#pragma unroll 4
        for (int e = threadIdx.x; e < n4; e += kStageThreads)
            reinterpret_cast<float4 *>(dst)[e] = reinterpret_cast<const float4 *>(src)[e];
        for (int e = (n4 << 2) + threadIdx.x; e < n; e += kStageThreads) dst[e] = src[e];
    } else {
#pragma unroll 4
        for (int e = threadIdx.x; e < n; e += kStageThreads) dst[e] = src[e];
    }
}

// The columns [c0, c1) of part `part` of `parts` of a row of n.
__device__ __forceinline__ void stage_part(int n, int parts, int part, int &c0, int &c1)
{
    const int per = (n + parts - 1) / parts;
    c0 = part * per;
    c1 = min(n, c0 + per);
}

}  // namespace dol
