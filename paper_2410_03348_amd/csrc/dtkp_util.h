// Device helpers shared by the DTKP kernels: the bitmask encoding of proofs, their probabilities, the exclusion
// test and the k-entry sorted list (Sec. 3.2, Table 1, App. A).
#pragma once

#include "internal.h"

namespace dol {

constexpr uint64_t kAbsent = ~uint64_t(0);

// A symbol's k proof masks and k proof probabilities are 8k and 4k contiguous bytes, aligned to 8 and 4: they move
// with 16-byte accesses of that declared alignment (the target allows global accesses that are not naturally
// aligned), so that a gathered list costs two or three memory instructions instead of 2k.
typedef uint32_t __attribute__((ext_vector_type(4), aligned(8))) u32x4_a8;
typedef float __attribute__((ext_vector_type(4), aligned(4))) f32x4_a4;
typedef float __attribute__((ext_vector_type(3), aligned(4))) f32x3_a4;
typedef float __attribute__((ext_vector_type(2), aligned(4))) f32x2_a4;

template <int K>
__device__ __forceinline__ void load_masks(const uint64_t *__restrict__ src, uint64_t (&m)[K])
{
#pragma unroll
    for (int x = 0; x + 1 < K; x += 2) {
        const u32x4_a8 v = *reinterpret_cast<const u32x4_a8 *>(src + x);
        m[x] = (static_cast<uint64_t>(v.y) << 32) | v.x;
        m[x + 1] = (static_cast<uint64_t>(v.w) << 32) | v.z;
    }
    if constexpr ((K & 1) != 0) m[K - 1] = src[K - 1];
}

template <int K>
__device__ __forceinline__ void load_probs(const float *__restrict__ src, float (&p)[K])
{
#pragma unroll
    for (int x = 0; x + 3 < K; x += 4) {
        const f32x4_a4 v = *reinterpret_cast<const f32x4_a4 *>(src + x);
        p[x] = v.x, p[x + 1] = v.y, p[x + 2] = v.z, p[x + 3] = v.w;
    }
    constexpr int R = K & 3, B = K - R;
    if constexpr (R == 3) {
        const f32x3_a4 v = *reinterpret_cast<const f32x3_a4 *>(src + B);
        p[B] = v.x, p[B + 1] = v.y, p[B + 2] = v.z;
    } else if constexpr (R == 2) {
        const f32x2_a4 v = *reinterpret_cast<const f32x2_a4 *>(src + B);
        p[B] = v.x, p[B + 1] = v.y;
    } else if constexpr (R == 1) {
        p[B] = src[B];
    }
}

template <int K>
__device__ __forceinline__ void store_masks(uint64_t *__restrict__ dst, const uint64_t (&m)[K])
{
#pragma unroll
    for (int x = 0; x + 1 < K; x += 2) {
        u32x4_a8 v;
        v.x = static_cast<uint32_t>(m[x]), v.y = static_cast<uint32_t>(m[x] >> 32);
        v.z = static_cast<uint32_t>(m[x + 1]), v.w = static_cast<uint32_t>(m[x + 1] >> 32);
        *reinterpret_cast<u32x4_a8 *>(dst + x) = v;
    }
    if constexpr ((K & 1) != 0) dst[K - 1] = m[K - 1];
}

template <int K>
__device__ __forceinline__ void store_probs(float *__restrict__ dst, const float (&p)[K])
{
#pragma unroll
    for (int x = 0; x + 3 < K; x += 4) {
        f32x4_a4 v;
        v.x = p[x], v.y = p[x + 1], v.z = p[x + 2], v.w = p[x + 3];
        *reinterpret_cast<f32x4_a4 *>(dst + x) = v;
    }
    constexpr int R = K & 3, B = K - R;
    if constexpr (R == 3) {
        f32x3_a4 v;
        v.x = p[B], v.y = p[B + 1], v.z = p[B + 2];
        *reinterpret_cast<f32x3_a4 *>(dst + B) = v;
    } else if constexpr (R == 2) {
        f32x2_a4 v;
        v.x = p[B], v.y = p[B + 1];
        *reinterpret_cast<f32x2_a4 *>(dst + B) = v;
    } else if constexpr (R == 1) {
        dst[B] = p[B];
    }
}

template <int K>
struct TopK {
    uint64_t m[K];
    float p[K];   // absent slots carry -1 so that every real proof (probability >= 0) ranks before them

    __device__ __forceinline__ void clear()
    {
#pragma unroll
        for (int x = 0; x < K; ++x) { m[x] = kAbsent; p[x] = -1.0f; }
    }

    static __device__ __forceinline__ bool before(uint64_t ma, float pa, uint64_t mb, float pb)
    {
        return pa > pb || (pa == pb && ma < mb);
    }

    // (a proof's probability is a function of its mask, so a candidate whose probability equals none of the kept ones is
    // none of the kept proofs and ranks among them by probability alone: the kept list, sorted, takes it in through one
    // max and K - 1 medians, and no mask is compared)
    __device__ __forceinline__ void insert(uint64_t mask, float prob)
    {
        bool tie = false;
#pragma unroll
        for (int x = 0; x < K; ++x) tie |= (prob == p[x]);
        if (!tie) {
            bool gt[K];
#pragma unroll
            for (int x = 0; x < K; ++x) gt[x] = prob > p[x];
#pragma unroll
            for (int x = K - 1; x >= 0; --x) {
                const bool above = x > 0 ? gt[x - 1] : false;
                m[x] = above ? m[x - 1] : gt[x] ? mask : m[x];
                p[x] = x > 0 ? __builtin_amdgcn_fmed3f(p[x - 1], p[x], prob) : fmaxf(p[0], prob);
            }
            return;
        }
        bool dup = false;
#pragma unroll
        for (int x = 0; x < K; ++x) dup |= (m[x] == mask);
        if (dup) return;
        if (!before(mask, prob, m[K - 1], p[K - 1])) return;
#pragma unroll
        for (int x = K - 1; x >= 0; --x) {
            const bool here = before(mask, prob, m[x], p[x]);
            const bool above = x > 0 ? before(mask, prob, m[x - 1], p[x - 1]) : false;
            if (above) { m[x] = m[x - 1]; p[x] = p[x - 1]; }
            else if (here) { m[x] = mask; p[x] = prob; }
        }
    }

    // Writes the k slots and returns the tag probability min(1, sum in rank order) (App. A.1).
    __device__ __forceinline__ float store(uint64_t *__restrict__ om, float *__restrict__ op) const
    {
        float sum = 0.0f, q[K];
#pragma unroll
        for (int x = 0; x < K; ++x) {
            const bool present = m[x] != kAbsent;
            q[x] = present ? p[x] : 0.0f;
            if (present) sum = sum + p[x];
        }
        store_masks<K>(om, m);
        store_probs<K>(op, q);
        return fminf(sum, 1.0f);
    }
};

__device__ __forceinline__ float proof_prob(uint64_t mask, const float *__restrict__ fp)
{
    float pr = 1.0f;
    while (mask) {
        const int j = __builtin_ctzll(mask);
        pr = pr * fp[j];
        mask &= mask - 1;
    }
    return pr;
}

__device__ __forceinline__ bool proof_conflict(uint64_t mask, const GroupMasks &gm)
{
    bool bad = false;
    for (int g = 0; g < gm.n; ++g) bad |= __builtin_popcountll(mask & gm.m[g]) > 1;
    return bad;
}

// pr * (probabilities of the facts in `bits`, ascending)
__device__ __forceinline__ float extend_prob(float pr, uint64_t bits, const float *__restrict__ fp)
{
    while (bits) {
        pr = pr * fp[__builtin_ctzll(bits)];
        bits &= bits - 1;
    }
    return pr;
}

// Probability of the union of two proofs.  The product runs over the facts in ascending index; when every fact
// that one side adds lies above the other side's highest fact, that side's stored probability is exactly the
// product's prefix and only the added facts remain to be multiplied (the case of a fold whose new operand brings
// new input slots).  pa / pb < 0: that side's probabilities are not available.
__device__ __forceinline__ float union_prob(uint64_t ma, float pa, uint64_t mb, float pb, const float *__restrict__ fp)
{
    const uint64_t add_b = mb & ~ma, add_a = ma & ~mb;
    const int hi_a = ma ? 63 - __builtin_clzll(ma) : -1, hi_b = mb ? 63 - __builtin_clzll(mb) : -1;
    if (pa >= 0.0f && (add_b == 0 || __builtin_ctzll(add_b) > hi_a)) return extend_prob(pa, add_b, fp);
    if (pb >= 0.0f && (add_a == 0 || __builtin_ctzll(add_a) > hi_b)) return extend_prob(pb, add_a, fp);
    return proof_prob(ma | mb, fp);
}

// All lanes of every aligned group of LANES lanes end with the merge of the group's lists.
template <int K, int LANES = 64>
__device__ __forceinline__ void merge_lists(TopK<K> &top)
{
#pragma unroll
    for (int d = LANES / 2; d >= 1; d >>= 1) {
        uint64_t pm[K];
        float pp[K];
#pragma unroll
        for (int x = 0; x < K; ++x) {
            const uint32_t lo = __shfl_xor(static_cast<uint32_t>(top.m[x]), d, 64);
            const uint32_t hi = __shfl_xor(static_cast<uint32_t>(top.m[x] >> 32), d, 64);
            pm[x] = (static_cast<uint64_t>(hi) << 32) | lo;
            pp[x] = __shfl_xor(top.p[x], d, 64);
        }
#pragma unroll
        for (int x = 0; x < K; ++x)
            if (pm[x] != kAbsent) top.insert(pm[x], pp[x]);
    }
}

}  // namespace dol
