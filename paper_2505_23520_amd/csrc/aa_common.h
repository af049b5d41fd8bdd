// Shared device-side plumbing of the AnchorAttention kernels (gfx950).
// Index conventions (rows, blocks, groups, packed batches) are those of
// include/anchor_attention.h; regions follow Algorithm 1-3 of arXiv 2505.23520.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aa {

constexpr int kLane = 64;          // wavefront width on CDNA4
constexpr int kIdxPad = 64;        // list chunks are 64 entries (one K/V tile)

// Launch with the launch's own status as return value (hipGetLastError() after a <<<>>> launch
// would also report, and clear, an error some earlier and unrelated call left behind).
template <class T> struct arg_of { using type = T; };
template <class... KArgs>
inline hipError_t launch_kernel(void (*kern)(KArgs...), dim3 grid, dim3 block, size_t lds, hipStream_t st,
                                typename arg_of<KArgs>::type... args) {
    void* ptrs[] = {(void*)&args...};
    return hipLaunchKernel((const void*)kern, grid, block, ptrs, lds, st);
}

// Kernel-side copy of the call's parameters (plain data, passed by value).
struct KParams {
    int B, Hq, Hkv, N, d;
    int bq, n_init, w, step;
    int grp;                // Hq / Hkv
    int packed;             // cu != nullptr
    int use_anchor;
    float theta, sigma;
    long long qs[3], ks[3], vs[3], os[3];
    const int* cu;
    long long total;        // packed: total tokens
    long long blk_cap, grp_cap;
    int nblk_max, ngrp_max; // blocks / groups of the longest sequence
};

// Where sequence b lives.
struct Seq {
    int len;                // tokens
    long long tok0;         // first token on the packed axis (0 when fixed length)
    long long blk0, grp0;   // blocks / groups of earlier sequences (packed only)
};

__device__ __forceinline__ Seq seq_of(const KParams& p, int b) {
    Seq s;
    if (!p.packed) {
        s.len = p.N; s.tok0 = 0; s.blk0 = 0; s.grp0 = 0;
        return s;
    }
    long long blk = 0, grp = 0;
    const int span = p.bq * p.step;
    for (int i = 0; i < b; ++i) {
        int len = p.cu[i + 1] - p.cu[i];
        blk += (len + p.bq - 1) / p.bq;
        grp += (len + span - 1) / span;
    }
    s.len = p.cu[b + 1] - p.cu[b];
    s.tok0 = p.cu[b];
    s.blk0 = blk; s.grp0 = grp;
    return s;
}

__device__ __forceinline__ long long row_index(const KParams& p, const Seq& s, int b, int h, int r) {
    return p.packed ? (long long)h * p.total + s.tok0 + r : ((long long)b * p.Hq + h) * p.N + r;
}
__device__ __forceinline__ long long blk_index(const KParams& p, const Seq& s, int b, int h, int i) {
    return p.packed ? (long long)h * p.blk_cap + s.blk0 + i : ((long long)b * p.Hq + h) * p.blk_cap + i;
}
__device__ __forceinline__ long long grp_index(const KParams& p, const Seq& s, int b, int h, int g) {
    return p.packed ? (long long)h * p.grp_cap + s.grp0 + g : ((long long)b * p.Hq + h) * p.grp_cap + g;
}
// bf16 path (d = 128, b_q = 128): the cached accumulator Acc is kept per query block as four tiles
// of 32 rows x 128 columns, each tile in the register order of the MFMA accumulators, so that a
// wave stores and reloads its 64 accumulator registers with 1 KB of consecutive addresses per
// instruction.  Float offset of tile `tile` of block i; inside the tile, element (row n, column c)
// sits at ((c / 32) * 4 + (c % 32) / 8) * 256 + (n + 32 * ((c % 8) / 4)) * 4 + c % 4.
__device__ __forceinline__ long long acc_tile(const KParams& p, const Seq& s, int b, int h, int i, int tile) {
    return (blk_index(p, s, b, h, i) * 4 + tile) * 4096;
}
// Element offset of token r of head h (d contiguous); batch stride unused when packed.
__device__ __forceinline__ long long tok_offset(const KParams& p, const long long* st, const Seq& s,
                                                int b, int h, int r) {
    return (p.packed ? 0 : (long long)b * st[0]) + (long long)h * st[1] + (s.tok0 + r) * st[2];
}
// First key of group g's local window (Algorithm 1, window range, in tokens).
__device__ __forceinline__ int window_start(const KParams& p, int g) {
    long long W = (long long)g * p.step * p.bq - p.w;
    return W > p.n_init ? (int)W : p.n_init;
}

// Work-group id -> (batch, query head, query block).  The hardware deals
// consecutive work-groups round-robin to the 8 XCDs; this map keeps all query
// heads of one KV head on one XCD (its K/V stay in that XCD's L2) and hands out
// the longest query blocks first (causal work grows with the block index).
struct Work { int b, h, i; };
__device__ __forceinline__ Work decode_work(const KParams& p, int nblk, unsigned id) {
    Work wk;
    const unsigned pairs = (unsigned)p.B * p.Hkv;
    const unsigned per_pair = (unsigned)nblk * p.grp;
    unsigned pr, within;
    if (pairs % 8 == 0) {
        unsigned xcd = id & 7, slot = id >> 3;
        pr = xcd + 8 * (slot / per_pair);
        within = slot % per_pair;
    } else {
        pr = id / per_pair;
        within = id % per_pair;
    }
    wk.b = pr / p.Hkv;
    int hk = pr % p.Hkv;
    wk.h = hk * p.grp + (within % p.grp);
    wk.i = nblk - 1 - (int)(within / p.grp);
    return wk;
}

}  // namespace aa
