// Arguments of the stage-2 (stripe identification) kernels.
#pragma once
#include "aa_common.h"

namespace aa {

constexpr int kMaskChunkKeys = 1024;   // keys per chunk of the bf16 mask kernel (its LDS holds one chunk's compare words)
constexpr int kMaskChunksPerWG = 1;    // consecutive chunks walked by one work-group (more was slower)

struct SelectArgs {
    KParams p;
    const void *q, *k;
    const float* xa;          // pooled anchors, per block
    void *qp_hi, *qp_lo;      // bf16 path: pooled queries, hi / lo parts, rows of 128
    float* qp_f32;            // fp32 path: pooled queries, rows of d
    float* kp_f32;            // block granularity: pooled keys per (KV head, key block), rows of d
    int is_bf16;              // element type of q, k
    unsigned* bits;           // [groups][nwords] selection bit words, bit (j % 32) of word j / 32
    int nwords;               // ceil(N / 32)
    int keys_per_chunk;       // bf16 mask kernel: keys per work-group, kMaskChunkKeys * kMaskChunksPerWG
    int* counts;
    long long* offsets;
    int* idx;
    long long idx_capacity;
    int* overflow;
    long long groups_total;
};

__global__ void pool_q_bf16_kernel(SelectArgs a);
__global__ void pool_q_fp32_kernel(SelectArgs a);
__global__ void mask_bf16_kernel(SelectArgs a);
__global__ void mask_fp32_kernel(SelectArgs a);
__global__ void pool_k_kernel(SelectArgs a);
__global__ void mask_block_kernel(SelectArgs a);
size_t mask_block_lds_bytes(int N, int d, int bq, int step);
__global__ void zero_i32_kernel(int* x, long long nelem);
__global__ void count_kernel(SelectArgs a);
__global__ void scan_kernel(SelectArgs a);
__global__ void fill_kernel(SelectArgs a);

}  // namespace aa
