// Per-channel statistics in groups of 64 rows, in one fixed order.
//
// BatchNorm's forward statistics (mean, sum of squared deviations) over the rows of an [rows x C] tensor are
// built from partial results of 64 consecutive rows each.  Both producers of those partial results, the
// stand-alone statistics kernel and the epilogue of the forward convolution that writes the tensor, go through
// the functions below with the same assignment of elements to lanes, so the bits do not depend on which of the
// two ran.  Within a group of 64 rows a wave handles 64 columns: lane l owns the four columns 4*(l & 15) ..
// +3 of rows (l >> 4) + 4*i + 16*q, visited in the order q = 0..3, i = 0..3; the four lanes that share the
// columns are then merged pairwise (lanes l and l ^ 16, then l ^ 32).
#pragma once
#include <hip/hip_runtime.h>

namespace monet {

constexpr int STAT_ROWS = 64;

struct LaneStats {
    float pv[4], s1[4], s2[4];
    float n;
    __device__ inline void init() {
        n = 0.0f;
#pragma unroll
        for (int j = 0; j < 4; ++j) pv[j] = s1[j] = s2[j] = 0.0f;
    }
    // sums are taken relative to the lane's first element (no cancellation when |mean| >> deviation)
    __device__ inline void add(float v0, float v1, float v2, float v3) {
#pragma clang fp contract(off)   // the same roundings wherever this is inlined
        const float v[4] = {v0, v1, v2, v3};
        if (n == 0.0f) {
#pragma unroll
            for (int j = 0; j < 4; ++j) pv[j] = v[j];
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float d = v[j] - pv[j];
            s1[j] += d;
            s2[j] = __builtin_fmaf(d, d, s2[j]);
        }
        n += 1.0f;
    }
    // The same for a lane whose sixteen elements all exist, the first one and the later ones: what add() does on its
    // first call (the element becomes the reference, its own deviation is zero) and on the following ones, without
    // the test of n.  Same bits as add() for finite values.
    __device__ inline void add_first(float v0, float v1, float v2, float v3) {
        pv[0] = v0; pv[1] = v1; pv[2] = v2; pv[3] = v3;
        n = 1.0f;
    }
    __device__ inline void add_next(float v0, float v1, float v2, float v3) {
#pragma clang fp contract(off)
        const float v[4] = {v0, v1, v2, v3};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float d = v[j] - pv[j];
            s1[j] += d;
            s2[j] = __builtin_fmaf(d, d, s2[j]);
        }
        n += 1.0f;
    }
};

// Merges the four lanes that share their columns; afterwards each of them holds the group's row count,
// means and sums of squared deviations of its four columns.  Every lane of the wave must call this.
__device__ inline void merge_lane_stats(const LaneStats &ls, int lane, float &n, float (&mean)[4], float (&m2)[4]) {
#pragma clang fp contract(off)
    n = ls.n;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        mean[j] = n > 0.0f ? ls.pv[j] + ls.s1[j] / n : 0.0f;
        const float q = n > 0.0f ? ls.s2[j] - ls.s1[j] * ls.s1[j] / n : 0.0f;
        m2[j] = q < 0.0f ? 0.0f : q;
    }
#pragma unroll
    for (int mask = 16; mask <= 32; mask <<= 1) {
        const bool low = (lane & mask) == 0;
        const float n_o = __shfl_xor(n, mask);
        const float na = low ? n : n_o, nb = low ? n_o : n, nt = na + nb;   // a = the lane with the bit clear
        // whole groups (every lane of the wave holds the same non-zero count): nb / nt is one half and na * nb / nt is
        // na / 2, both exact, so the general formula below gives these bits without its divisions
        const bool whole = __all(n == n_o && n > 0.0f) != 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float mean_o = __shfl_xor(mean[j], mask), m2_o = __shfl_xor(m2[j], mask);
            const float ma = low ? mean[j] : mean_o, mb = low ? mean_o : mean[j];
            const float qa = low ? m2[j] : m2_o, qb = low ? m2_o : m2[j];
            if (whole) {
                const float d = mb - ma;
                mean[j] = ma + d * 0.5f;
                m2[j] = qa + qb + d * d * (na * 0.5f);
            } else if (nb > 0.0f) {
                const float d = mb - ma;
                mean[j] = na > 0.0f ? ma + d * (nb / nt) : mb;
                m2[j] = qa + qb + (na > 0.0f ? d * d * (na * nb / nt) : 0.0f);
            } else {
                mean[j] = ma;
                m2[j] = qa;
            }
        }
        n = nt;
    }
}

// lane l < 16 writes {mean, M2} of its four columns of row group `grp`: part[(grp * C + c) * 2 + {0, 1}]
__device__ inline void store_group_stats(float *part, int64_t grp, int C, int col, int lane, const float (&mean)[4], const float (&m2)[4]) {
    if ((lane >> 4) != 0 || col >= C) return;
    float4 *dst = (float4 *)(part + (grp * C + col) * 2);
    dst[0] = make_float4(mean[0], m2[0], mean[1], m2[1]);
    dst[1] = make_float4(mean[2], m2[2], mean[3], m2[3]);
}

}  // namespace monet
