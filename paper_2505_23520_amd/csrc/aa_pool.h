// Block mean of the queries, qbar_i (arXiv 2505.23520 Sec. 3.2; Algorithm 2, avgpool(Q)), from query
// fragments held in registers in the layout of the bf16 tile engines: lane (n, hf) of a wave holds,
// for one query row, the eight 16-byte pieces Q[row][16 ks + 8 hf .. + 8), ks = 0..7.
// The stage-1 engines pool the block they have just attended (its Q fragments are still in
// registers); stripe_select's own pooling kernel loads the same fragments and runs the same code, so
// both produce the same bits: the order of every floating-point addition is fixed here.
#pragma once
#include "aa_common.h"

namespace aa {

typedef __bf16 pool_bf16x8 __attribute__((ext_vector_type(8)));

// Column sums over the 32 rows of a wave's half (lanes with the same hf): a reduce-scatter over
// the lane bits 16, 8, 4, 2, 1 -- at every level a lane keeps one half of its values and receives
// its partner's partial sums for that half.  On return lane (n, hf) holds the sums of columns
// 16 (n / 4) + 8 hf + 2 (n % 4) and that + 1.  Rows that do not exist must hold zeros.
__device__ __forceinline__ void pool_wave_columns(const pool_bf16x8 (&qf)[8], int n, float& s0, float& s1) {
    float f[64];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) f[8 * ks + e] = (float)qf[ks][e];
#define AA_POOL_LEVEL(width, dist)                                   \
    {                                                                \
        const bool upper = (n & (dist)) != 0;                        \
        _Pragma("unroll") for (int i = 0; i < (width); ++i) {        \
            const float keep = upper ? f[(width) + i] : f[i];        \
            const float send = upper ? f[i] : f[(width) + i];        \
            f[i] = keep + __shfl_xor(send, (dist), 64);              \
        }                                                            \
    }
    AA_POOL_LEVEL(32, 16)
    AA_POOL_LEVEL(16, 8)
    AA_POOL_LEVEL(8, 4)
    AA_POOL_LEVEL(4, 2)
    AA_POOL_LEVEL(2, 1)
#undef AA_POOL_LEVEL
    s0 = f[0];
    s1 = f[1];
}

// Work-group part: part[tile][column] receives every wave's column sums (tile = the wave's 32-row
// tile inside its query block, 0..3), then threads 0..63 of the block's `team` of 256 threads add
// the four tiles in the order (0 + 1) + (2 + 3), scale by 1 / nrows, split the mean into bf16 hi +
// lo parts and write rows `bi` of qp_hi / qp_lo (128 entries each) and the Euclidean norm of the
// lo row.  All threads of the work-group must call this (it holds barriers); `tteam` is the
// thread's index inside its team, part points at the team's float[4][128].
__device__ __forceinline__ void pool_block_finish(float (*part)[128], int tile, int n, int hf, float s0, float s1,
                                                  int tteam, int nrows, long long bi, bool block_exists,
                                                  void* qp_hi, void* qp_lo, float* qlo_norm) {
    const int c0 = 16 * (n >> 2) + 8 * hf + 2 * (n & 3);
    part[tile][c0] = s0;
    part[tile][c0 + 1] = s1;
    __syncthreads();
    if (tteam < 64 && block_exists) {
        const float inv = 1.f / (float)nrows;
        const float m0 = ((part[0][2 * tteam] + part[1][2 * tteam]) + (part[2][2 * tteam] + part[3][2 * tteam])) * inv;
        const float m1 = ((part[0][2 * tteam + 1] + part[1][2 * tteam + 1]) +
                          (part[2][2 * tteam + 1] + part[3][2 * tteam + 1])) * inv;
        auto to_bf16 = [](float x) -> unsigned short {          // round to nearest even
            unsigned u = __float_as_uint(x);
            u += 0x7fffu + ((u >> 16) & 1u);
            return (unsigned short)(u >> 16);
        };
        auto from_bf16 = [](unsigned short b) -> float { return __uint_as_float((unsigned)b << 16); };
        const unsigned short h0 = to_bf16(m0), h1 = to_bf16(m1);
        const unsigned short l0 = to_bf16(m0 - from_bf16(h0)), l1 = to_bf16(m1 - from_bf16(h1));
        ((unsigned*)qp_hi)[bi * 64 + tteam] = (unsigned)h0 | ((unsigned)h1 << 16);
        ((unsigned*)qp_lo)[bi * 64 + tteam] = (unsigned)l0 | ((unsigned)l1 << 16);
        // what hi + lo leave out (below 2^-16 of an entry) is far inside the tolerance of the
        // decision; the norm of lo bounds what leaving out the lo products would change
        float ln = from_bf16(l0) * from_bf16(l0) + from_bf16(l1) * from_bf16(l1);
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) ln += __shfl_xor(ln, off, 64);
        if (tteam == 0) qlo_norm[bi] = sqrtf(ln);
    }
}

}  // namespace aa
