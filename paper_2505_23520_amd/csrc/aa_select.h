// Arguments of the stage-2 (stripe identification) kernels.
#pragma once
#include "aa_common.h"

namespace aa {

constexpr int kMaskChunkKeys = 1024;   // keys per chunk of the bf16 mask kernel (its LDS holds one chunk's compare words)
constexpr int kMaskChunksPerWG = 2;    // consecutive chunks walked by one work-group (2: -3 %, 4: no further gain)

// bf16 mask kernel: pooled rows per row tile, and the number of key chunks a row tile has
// candidates in (all groups of the tile end their candidates before the last group's window).
// Host and device use the same arithmetic: the host sizes the grid with it, the kernel decodes
// its work-group index with it.
__host__ __device__ inline int mask_row_tile(int step) { return 128 - 128 % step; }
__host__ __device__ inline int mask_tile_chunks(int nblk, int rt, int step, int bq, int w, int n_init) {
    const int RT = mask_row_tile(step);
    if (rt < 0 || rt * RT >= nblk) return 0;
    const int rows = nblk - rt * RT < RT ? nblk - rt * RT : RT;
    const int g_last = (rt * RT + rows - 1) / step;
    const long long W = (long long)g_last * step * bq - w;
    const int Wmax = W > n_init ? (int)W : n_init;
    const int key_lo = (n_init / 64) * 64;
    const int span = kMaskChunkKeys * kMaskChunksPerWG;
    return Wmax > key_lo ? (Wmax - key_lo + span - 1) / span : 0;
}
// Work items of one (sequence, KV head) pair in the bf16 mask kernel: one per (row tile, key chunk
// that holds candidates of the tile).  The count for the longest sequence sizes the grid; a
// shorter sequence has fewer and its surplus work-groups return.
__host__ __device__ inline int mask_pair_items(int nblk, int step, int bq, int w, int n_init) {
    const int RT = mask_row_tile(step);
    const int ny = (nblk + RT - 1) / RT;
    int n = 0;
    for (int y = 0; y < ny; ++y) n += mask_tile_chunks(nblk, y, step, bq, w, n_init);
    return n;
}

struct SelectArgs {
    KParams p;
    const void *q, *k;
    const float* xa;          // pooled anchors, per block
    void *qp_hi, *qp_lo;      // bf16 path: pooled queries, hi / lo parts, rows of 128
    float* qp_f32;            // fp32 path: pooled queries, rows of d
    float* kp_f32;            // block granularity: pooled keys per (KV head, key block), rows of d
    float* qlo_norm;          // bf16 path: Euclidean norm of the lo part of each pooled query row
    float* kmax_blk;          // bf16 stripe path: largest key norm per (KV head, key block)
    int is_bf16;              // element type of q, k
    int pool_skip_q;          // bf16: the pooled queries are there already (stage 1 wrote them)
    unsigned* bits;           // [groups][nwords] selection bit words, bit (j % 32) of word j / 32
    int nwords;               // ceil(N / 32)
    int* segcount;            // [groups][nseg] selected columns per segment of 64 bit words (2048 keys)
    int nseg;                 // ceil(nwords / 64)
    int* counts;
    long long* offsets;
    int* idx;
    long long idx_capacity;
    int* overflow;
    long long groups_total;
    long long* stats;         // nullable, int64[4]: { attended pairs, selected entries, 0, 0 }
    // bf16 mask kernel: work items per (sequence, KV head) pair for the longest sequence (sizes the grid)
    int mask_items;
};

__global__ void pool_q_bf16_kernel(SelectArgs a);
__global__ void pool_q_fp32_kernel(SelectArgs a);
__global__ void mask_bf16_kernel(SelectArgs a);
__global__ void mask_fp32_kernel(SelectArgs a);
__global__ void pool_k_kernel(SelectArgs a);
__global__ void mask_block_kernel(SelectArgs a);
size_t mask_block_lds_bytes(int N, int d, int bq, int step);
constexpr size_t kMaskBlockLdsMax = 128 * 1024;   // dynamic LDS limit set for mask_block_kernel
__global__ void zero_i32_kernel(int* x, long long nelem);
__global__ void count_kernel(SelectArgs a);
__global__ void scan_kernel(SelectArgs a);
__global__ void fill_kernel(SelectArgs a);

}  // namespace aa
