// Stage 2 of AnchorAttention, difference-aware stripe identification
// (arXiv 2505.23520 Sec. 3.2 mask, Algorithm 2, and the step rule of Sec. 3.4):
//   pool_q   : qbar_i = mean of query block i's rows               (Alg. 2, avgpool(Q))
//   mask     : bit (g, j) = OR_{i in g} [ xbar_i - sigma <qbar_i, k_j> <= theta ],  j in C_g
//   count    : |I_g| = popcount of the group's bits
//   scan     : offsets = exclusive prefix sum of the counts rounded up to 64
//   fill     : ballot / prefix-popcount stream compaction of the bits into ascending lists
// The bf16 mask kernel is a skinny MFMA GEMM (pooled rows x keys); the pooled
// query, an fp32 mean, is split into bf16 hi + lo parts so that the products with
// the (exactly bf16) keys carry ~16 mantissa bits and the threshold decision does
// not depend on bf16 rounding of the mean.
#include "aa_common.h"
#include "aa_pool.h"
#include "aa_select.h"

namespace aa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
constexpr floatx16 kZero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

namespace {
__device__ __forceinline__ float bf16_to_f(unsigned short b) { return __uint_as_float((unsigned)b << 16); }
__device__ __forceinline__ unsigned short f_to_bf16_rne(float f) {
    unsigned u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}
}  // namespace

// ------------------------------------------------------------------ pool_q
// grid (nblk_max, Hq [+ Hkv], B).  bf16: 256 threads = the four waves of the tile engines; writes
// hi/lo bf16 rows of 128 and the norm of the lo row (aa_pool.h).  With kmax_blk set the grid has Hkv
// more rows in y: those work-groups write the largest key norm of their key block (the mask kernel
// bounds |<lo, k>| by |lo| |k| to decide whether the lo products are needed).  pool_skip_q: the
// queries were pooled by stage 1 already, the grid holds the Hkv key rows only.
// fp32: 128 threads, float rows of d.
__global__ __launch_bounds__(256) void pool_q_bf16_kernel(SelectArgs a) {
    const KParams& p = a.p;
    const int i = blockIdx.x, b = blockIdx.z;
    const Seq sq = seq_of(p, b);
    const int r0 = i * p.bq;
    if (r0 >= sq.len) return;
    const int r1 = min(r0 + p.bq, sq.len);
    const int tid = threadIdx.x, c = tid & 15, rs = tid >> 4;
    __shared__ float red[16][128];
    const int y = blockIdx.y + (a.pool_skip_q ? p.Hq : 0);
    if (y >= p.Hq) {
        // key block i of KV head hk: squared norm of every row (16 threads per row), largest
        const int hk = y - p.Hq;
        const unsigned short* src = (const unsigned short*)a.k + tok_offset(p, p.ks, sq, b, hk, 0) + 8 * c;
        float big = 0.f;
        for (int r = r0 + rs; r < r1; r += 16) {
            const uintx4 x = *(const uintx4*)(src + (long long)r * p.ks[2]);
            float ss = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = __uint_as_float(x[e] << 16), hi = __uint_as_float(x[e] & 0xffff0000u);
                ss = fmaf(lo, lo, ss);
                ss = fmaf(hi, hi, ss);
            }
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) ss += __shfl_xor(ss, off, 64);
            big = fmaxf(big, ss);
        }
#pragma unroll
        for (int off = 32; off >= 16; off >>= 1) big = fmaxf(big, __shfl_xor(big, off, 64));
        if ((tid & 63) == 0) red[0][tid >> 6] = big;
        __syncthreads();
        if (tid == 0) {
            const long long kb = (p.packed ? (long long)hk * p.blk_cap + sq.blk0
                                           : ((long long)b * p.Hkv + hk) * p.blk_cap) + i;
            a.kmax_blk[kb] = sqrtf(fmaxf(fmaxf(red[0][0], red[0][1]), fmaxf(red[0][2], red[0][3])));
        }
        return;
    }
    // query block i of head h: the fragments of the tile engines (wave w: rows 32 w .. 32 w + 31, lane
    // (n, hf): the 16-byte pieces 16 ks + 8 hf of row n), pooled by the code the engines use
    const int h = y;
    const int lane = tid & 63, wave = tid >> 6, n = lane & 31, hf = lane >> 5;
    const int r = r0 + 32 * wave + n;
    bf16x8 qf[8];
    {
        const __bf16* src = (const __bf16*)a.q + tok_offset(p, p.qs, sq, b, h, r < r1 ? r : r0);
        const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 x = *(const bf16x8*)(src + 16 * ks + 8 * hf);
            qf[ks] = r < r1 ? x : zero8;
        }
    }
    float s0, s1;
    pool_wave_columns(qf, n, s0, s1);
    pool_block_finish((float(*)[128])red, wave, n, hf, s0, s1, tid, r1 - r0, blk_index(p, sq, b, h, i), true,
                      a.qp_hi, a.qp_lo, a.qlo_norm);
}

__global__ __launch_bounds__(128) void pool_q_fp32_kernel(SelectArgs a) {
    const KParams& p = a.p;
    const int i = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const Seq sq = seq_of(p, b);
    const int r0 = i * p.bq;
    if (r0 >= sq.len) return;
    const int r1 = min(r0 + p.bq, sq.len);
    const float* src = (const float*)a.q + tok_offset(p, p.qs, sq, b, h, 0);
    const long long bi = blk_index(p, sq, b, h, i);
    for (int c = threadIdx.x; c < p.d; c += blockDim.x) {
        float s = 0.f;
        for (int r = r0; r < r1; ++r) s += src[(long long)r * p.qs[2] + c];
        a.qp_f32[bi * p.d + c] = s / (float)(r1 - r0);
    }
}

// ------------------------------------------------------------------ mask, bf16 MFMA
// One work-group = one (query head, row tile, key chunk): 256 threads = 4 waves, three work-groups
// per CU.  A row tile holds RT = 128 - 128 % step pooled rows, so no group straddles two tiles; wave
// w owns its rows 32 w .. 32 w + 31.  The chunk's keys pass through LDS in 64-key tiles (16-byte
// direct-to-LDS loads, two stages, same padded group layout as the attention engine).
// C[key][row] = K qbar^T: keys are the M dimension, pooled rows the N dimension, so one lane owns
// one pooled row and collects the compare bits of its row in registers.
//
// Grid: one dimension.  Every launched work-group has exactly one chunk of work (row tiles only
// count the chunks below their last group's window).  A key chunk (256 KB of K) is needed by the
// query heads of its KV head times the row tiles at or above it -- up to 32 work-groups at 128k
// tokens -- and is read from HBM once if those run at the same time on one XCD (each XCD has its
// own L2).  The hardware deals consecutive work-group ids round-robin to the 8 XCDs, so id
// -> logical index L = (id % 8) * per_xcd + id / 8 gives each XCD a contiguous range of L, walked
// in order; L enumerates sequences, inside a sequence the KV heads, inside a (sequence, KV head)
// pair the key chunks in ascending order, inside a chunk the row tiles that need it, and the
// query heads of the KV head fastest.
constexpr int kMaskTileKeys = 64;
constexpr int kMaskChunkTiles = kMaskChunkKeys / kMaskTileKeys;   // tiles per work-group
constexpr int kKGrp = 1024 + 16;                         // bytes per group of four K rows + pad
constexpr int kKTile = 16 * kKGrp;
typedef __attribute__((address_space(3))) void lds_void;

namespace {
// Work-group barrier that makes LDS writes visible but leaves vector-memory operations in flight
// (__syncthreads() also waits for every outstanding load, the prefetched tiles included).
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_s_waitcnt(0xC07F);                  // lgkmcnt(0)
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}
}  // namespace

__global__ __launch_bounds__(256, 3) void mask_bf16_kernel(SelectArgs a) {
    const KParams& p = a.p;
    // Work items that exist: per sequence, items(len) x Hq (a packed batch's shorter sequences have
    // fewer than the longest one, for which the host sized the grid).  Every XCD gets an equal,
    // contiguous share of them, so the load is balanced whatever the mix of lengths.
    const int span_blk = p.bq;
    long long real = 0;
    if (p.packed) {
        for (int s = 0; s < p.B; ++s)
            real += mask_pair_items((p.cu[s + 1] - p.cu[s] + span_blk - 1) / span_blk, p.step, p.bq, p.w, p.n_init);
        real *= p.Hq;
    } else {
        real = (long long)a.mask_items * p.Hq * p.B;
    }
    const long long per_xcd = (real + 7) / 8;
    const long long slot = blockIdx.x >> 3;
    long long L = (long long)(blockIdx.x & 7u) * per_xcd + slot;
    if (slot >= per_xcd || L >= real) return;
    // L -> sequence b, then inside the sequence KV head, item, query head of the KV head
    int b = 0, items_b = a.mask_items;
    if (p.packed) {
        for (;; ++b) {
            items_b = mask_pair_items((p.cu[b + 1] - p.cu[b] + span_blk - 1) / span_blk, p.step, p.bq, p.w, p.n_init);
            const long long n = (long long)items_b * p.Hq;
            if (L < n) break;
            L -= n;
        }
    } else {
        b = (int)(L / ((long long)items_b * p.Hq));
        L -= (long long)b * items_b * p.Hq;
    }
    const int per_pair = items_b * p.grp;
    const int hk = (int)(L / per_pair), e = (int)(L % per_pair);
    const int h = hk * p.grp + e % p.grp;
    const Seq sq = seq_of(p, b);
    const int nblk = (sq.len + p.bq - 1) / p.bq;
    const int RT = mask_row_tile(p.step);
    const int ny = (nblk + RT - 1) / RT;
    // item e / grp of this sequence -> (chunk, row tile).  Row tile y has candidates in its first
    // n(y) chunks and n is non-decreasing in y, so chunks n(y-1) .. n(y)-1 are needed by the
    // ny - y row tiles y .. ny-1: walk these levels.
    int rt = -1, chunk = 0;
    {
        int item = e / p.grp, prev = 0;
        for (int y = 0; y < ny; ++y) {
            const int n = mask_tile_chunks(nblk, y, p.step, p.bq, p.w, p.n_init);
            const int width = ny - y, items = (n - prev) * width;
            if (item < items) {
                chunk = prev + item / width;
                rt = y + item % width;
                break;
            }
            item -= items;
            prev = n;
        }
    }
    if (rt < 0) return;                                  // a shorter sequence of a packed batch
    const int row_t0 = rt * RT;                          // first pooled row (query block) of the tile
    if (row_t0 >= nblk) return;
    const int rows_here = min(RT, nblk - row_t0);
    const int g_first = row_t0 / p.step;
    const int g_last = (row_t0 + rows_here - 1) / p.step;
    const int Wmax = window_start(p, g_last);            // candidates of the tile end before Wmax
    const int key_lo = (p.n_init / kMaskTileKeys) * kMaskTileKeys;
    if (key_lo + chunk * kMaskChunksPerWG * kMaskChunkKeys >= Wmax) return;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = lane & 31, hf = lane >> 5;
    // one LDS object per stage: the compiler can then tell that the asynchronous loads into one stage
    // do not alias the operand reads from another (with a single array it waits for the loads it
    // has just issued before every tile's first read)
    __shared__ __attribute__((aligned(16))) char kt0[kKTile], kt1[kKTile];
    // compare words of the whole chunk: [tile][pooled row][word]
    __shared__ unsigned rowword[kMaskChunkTiles][128][2];

    // B operand: this lane's pooled query row, hi and lo parts, columns 16 ks + 8 hf .. +8
    bf16x8 bhi[8], blo[8];
    const int lr = 32 * wave + n;                        // row inside the tile
    const bool rok = lr < rows_here;
    const long long bi = blk_index(p, sq, b, h, row_t0 + (rok ? lr : 0));
    {
        const unsigned short* hi = (const unsigned short*)a.qp_hi + bi * 128;
        const unsigned short* lo = (const unsigned short*)a.qp_lo + bi * 128;
        const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 x = *(const bf16x8*)(hi + 16 * ks + 8 * hf);
            const bf16x8 y = *(const bf16x8*)(lo + 16 * ks + 8 * hf);
            bhi[ks] = rok ? x : zero8;
            blo[ks] = rok ? y : zero8;
        }
    }
    // The threshold test xbar - sigma s <= theta is the sign of s + (theta - xbar) / sigma: that
    // constant of the lane's row is the initial accumulator of the score MFMAs, so the accumulators
    // come out as margins (in raw dot-product units) and their sign bits are the decisions.
    // -inf = no such row (never selects).
    const float toff = rok ? (p.theta - (p.use_anchor ? a.xa[bi] : 0.f)) / p.sigma : -INFINITY;
    floatx16 cinit;
#pragma unroll
    for (int v = 0; v < 16; ++v) cinit[v] = toff;
    const float lo_norm = rok ? a.qlo_norm[bi] : 0.f;

    const unsigned short* kbase = (const unsigned short*)a.k + tok_offset(p, p.ks, sq, b, hk, 0);
    const unsigned kstb = (unsigned)p.ks[2] * 2u;
    const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc(
        (void*)kbase, 0, (int)((unsigned)(sq.len - 1) * kstb + 256u), 0x00020000);
    // loader: in the load of group gi lane l fetches the 16-byte chunk l % 16 of key 16 (l / 16) + gi
    auto load_tile = [&](int t0, char* buf) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int gi = 4 * wave + j;
            const int key = min(t0 + 16 * (lane >> 4) + gi, sq.len - 1);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(krs, (lds_void*)(buf + gi * kKGrp), 16,
                                                     (int)((unsigned)key * kstb + 16u * (lane & 15)), 0, 0, 0);
        }
    };
    const int nwords = a.nwords;
    const int ngrp = (nblk + p.step - 1) / p.step;
    const int ngt = g_last - g_first + 1;
    // OR the rows of each group, clip to the group's candidate range, write the bit words of a tile
    // a work-group walks kMaskChunksPerWG chunks of kMaskChunkKeys keys: the pooled rows stay in
    // registers, the compare words of a chunk are combined and written before the next one starts
    const int koff = (n & 15) * kKGrp + (n >> 4) * 256 + 16 * hf;   // K row of key 32 kb + n
    for (int cc = 0; cc < kMaskChunksPerWG; ++cc) {
    const int chunk0 = key_lo + (chunk * kMaskChunksPerWG + cc) * kMaskChunkKeys;
    if (chunk0 >= Wmax) break;
    const int chunk1 = min(chunk0 + kMaskChunkKeys, ((Wmax + kMaskTileKeys - 1) / kMaskTileKeys) * kMaskTileKeys);
    const int ntiles = (chunk1 - chunk0) / kMaskTileKeys;
    // |sigma <lo, k>| <= sigma |lo| max|k| over the chunk's keys: a score whose margin from the hi
    // products alone is farther from zero than that keeps its sign whatever the lo products add
    float kbig = 0.f;
    {
        const long long kb0 = p.packed ? (long long)hk * p.blk_cap + sq.blk0 : ((long long)b * p.Hkv + hk) * p.blk_cap;
        const int J1 = min(chunk1 - 1, sq.len - 1) / p.bq;
        for (int J = chunk0 / p.bq; J <= J1; ++J) kbig = fmaxf(kbig, a.kmax_blk[kb0 + J]);
    }
    const float lo_bound = 1.001f * lo_norm * kbig;
    // After the tile loop: OR the rows of each group, clip to the group's candidate range, write the
    // bit words of the chunk.  (This stays outside the tile loop: before an inner loop that reads
    // LDS, and before an LDS atomic, the compiler waits for every outstanding asynchronous load
    // into LDS, which would serialise the tile loads with the arithmetic.)
    auto combine_all = [&]() {
        // consecutive threads take consecutive words of one group (coalesced stores); each starts
        // its walk over the group's rows at a different row, which spreads a wave's LDS reads over
        // the banks (from the same row they would be 16 reads to one bank)
        for (int e = tid; e < ngt * 2 * ntiles; e += 256) {
            const int wi = e & 1, tl = (e >> 1) % ntiles, gi = (e >> 1) / ntiles;
            const int g = g_first + gi;
            const int lr0 = g * p.step - row_t0;
            const int nr = min(p.step, rows_here - lr0);
            unsigned wd = 0;
            int s = tl % nr;
            for (int c = 0; c < nr; ++c) {
                wd |= rowword[tl][lr0 + s][wi];
                s = s + 1 == nr ? 0 : s + 1;
            }
            const int j0 = chunk0 + tl * kMaskTileKeys + 32 * wi;
            const int Wg = window_start(p, g);
            const int lo = max(p.n_init - j0, 0), hi = min(Wg - j0, 32);   // keep n_init <= j0 + bit < Wg
            unsigned keep = 0;
            if (hi > lo) keep = (hi - lo >= 32) ? 0xffffffffu : (((1u << (hi - lo)) - 1u) << lo);
            if (g < ngrp && j0 / 32 < nwords)
                a.bits[grp_index(p, sq, b, h, g) * nwords + j0 / 32] = wd & keep;
        }
    };

    // two stages: the loads of tile t + 1 are issued at the start of tile t and awaited at its end.
    // (Three stages with a two-tile lead were 12 % slower: 50 KB of LDS per work-group leave room for
    // three work-groups per CU, 66 KB only for two, and the third hides both the load latency and
    // the 4 us a CU needs to replace a finished work-group.)  Every tile issues its four loads
    // unconditionally (past the chunk's end the last tile is fetched again into the stage nobody
    // reads any more), so no statically possible path reads a stage whose loads might be pending.
    load_tile(chunk0, kt0);
    __builtin_amdgcn_s_waitcnt(0x0F70);              // tile 0 is there
    lds_barrier();
    auto tile_step = [&](int t, const char* Kcur, char* Kld) {
        load_tile(chunk0 + min(t + 1, ntiles - 1) * kMaskTileKeys, Kld);
        // higher issue priority for the MFMA block than for the bit packing: a wave with matrix work
        // wins over the SIMD's other waves that are in their vector-ALU part (-3 %)
        __builtin_amdgcn_s_setprio(2);
        const char* Kb = Kcur + koff;
        floatx16 c[2];
        // hi products first.  The two accumulators alternate, so no MFMA waits for the one issued
        // just before it
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 kf0 = *(const bf16x8*)(Kb + 32 * ks);
            const bf16x8 kf1 = *(const bf16x8*)(Kb + 512 + 32 * ks);
            c[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf0, bhi[ks], ks == 0 ? cinit : c[0], 0, 0, 0);
            c[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf1, bhi[ks], ks == 0 ? cinit : c[1], 0, 0, 0);
        }
        // operand reads run ahead of their MFMAs
        __builtin_amdgcn_sched_group_barrier(0x100, 4, 0);
#pragma unroll
        for (int i = 0; i < 6; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
        __builtin_amdgcn_s_setprio(0);
        float nearest = INFINITY;                    // smallest |margin| of the lane's 32 scores
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int v = 0; v < 16; v += 2)
                nearest = fminf(fminf(nearest, fabsf(c[kb][v])), fabsf(c[kb][v + 1]));       // v_min3_f32
        if (__any(nearest <= lo_bound)) {
            // some decision of this wave's tile hangs on the lo products: add them (rare: only
            // margins within ~1e-2 of zero get here)
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const bf16x8 kf0 = *(const bf16x8*)(Kb + 32 * ks);
                const bf16x8 kf1 = *(const bf16x8*)(Kb + 512 + 32 * ks);
                c[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf0, blo[ks], c[0], 0, 0, 0);
                c[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf1, blo[ks], c[1], 0, 0, 0);
            }
            __builtin_amdgcn_s_setprio(0);
        }
        // Sign bits shifted into a word (one instruction per score, no compare / select chains).
        // The lane gathers the bits of its 16 keys per 32-key block (accumulator register v holds
        // key 8 (v / 4) + 4 hf + v % 4, i.e. its nibbles alternate with those of the lane 32 away,
        // which holds the other 16 keys of the same row).
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
            unsigned neg = 0;                        // bit v = sign of score v's margin
#pragma unroll
            for (int v = 15; v >= 0; --v)
                neg = __builtin_amdgcn_alignbit(neg, __float_as_uint(c[kb][v]), 31);
            unsigned wd = ~neg & 0xffffu;
            wd = (wd | (wd << 8)) & 0x00ff00ffu;     // nibble i of the 16 bits -> nibble 2 i of the word
            wd = (wd | (wd << 4)) & 0x0f0f0f0fu;
            wd <<= 4 * hf;
            const auto both = __builtin_amdgcn_permlane32_swap(wd, wd, false, false);
            if (hf == 0) rowword[t][lr][kb] = both[0] | both[1];
        }
        // tile t + 1 has landed
        __builtin_amdgcn_s_waitcnt(0x0F70);
        lds_barrier();
    };
    static_assert(kMaskChunkTiles % 2 == 0, "the tile loop below alternates two stages");
#pragma unroll 1
    for (int t2 = 0; t2 < ntiles; t2 += 2) {
        tile_step(t2, kt0, kt1);
        if (t2 + 1 >= ntiles) break;
        tile_step(t2 + 1, kt1, kt0);
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);              // the trailing loads have landed before LDS is reused
    combine_all();
    __syncthreads();                                 // rowword is reused by the next chunk
    }
}

// ------------------------------------------------------------------ mask, fp32 vector FMA
// grid (key chunks of 256, ngrp_max, B*Hq), 256 threads: one key per thread.
__global__ __launch_bounds__(256) void mask_fp32_kernel(SelectArgs a) {
    const KParams& p = a.p;
    const int b = blockIdx.z / p.Hq, h = blockIdx.z % p.Hq, hk = h / p.grp;
    const int g = blockIdx.y;
    const Seq sq = seq_of(p, b);
    const int nblk = (sq.len + p.bq - 1) / p.bq;
    const int i0 = g * p.step;
    if (i0 >= nblk) return;
    const int nb = min(p.step, nblk - i0);
    const int Wg = window_start(p, g);
    const int j = blockIdx.x * 256 + threadIdx.x;
    if ((int)(blockIdx.x * 256) >= Wg) return;
    extern __shared__ float qs[];                      // nb pooled rows of d floats
    for (int e = threadIdx.x; e < nb * p.d; e += 256)
        qs[e] = a.qp_f32[blk_index(p, sq, b, h, i0 + e / p.d) * p.d + e % p.d];
    __syncthreads();
    bool pred = false;
    if (j >= p.n_init && j < Wg) {
        const float* kr = (const float*)a.k + tok_offset(p, p.ks, sq, b, hk, j);
        for (int s = 0; s < nb; ++s) {
            float dot = 0.f;
            for (int c = 0; c < p.d; ++c) dot = fmaf(qs[s * p.d + c], kr[c], dot);
            const float xbar = p.use_anchor ? a.xa[blk_index(p, sq, b, h, i0 + s)] : 0.f;
            pred = pred || ((xbar - p.sigma * dot) <= p.theta);
        }
    }
    const unsigned long long bal = __ballot(pred);
    const int lane = threadIdx.x & 63;
    const long long t = grp_index(p, sq, b, h, g);
    const int w0 = (blockIdx.x * 256 + (threadIdx.x & ~63)) / 32;
    if (lane == 0 && w0 < a.nwords) a.bits[t * a.nwords + w0] = (unsigned)bal;
    if (lane == 32 && w0 + 1 < a.nwords) a.bits[t * a.nwords + w0 + 1] = (unsigned)(bal >> 32);
}

// ------------------------------------------------------------------ block granularity
// One decision per key block (Sec. 2.1.2 / Table 1's block granularity) instead of one per column:
// the difference test of Sec. 3.2 on the block's average key.  Tiny next to the stripe mask
// (pooled rows x pooled keys), so plain fp32 FMAs.

// kbar_J = mean of key block J.  grid (nblk_max, Hkv, B), 256 threads.  bf16 (d = 128): thread
// (c, rs) sums the 16-byte chunk c of rows rs, rs + 16, ...; fp32: one column per thread.
__global__ __launch_bounds__(256) void pool_k_kernel(SelectArgs a) {
    const KParams& p = a.p;
    const int J = blockIdx.x, hk = blockIdx.y, b = blockIdx.z;
    const Seq sq = seq_of(p, b);
    const int r0 = J * p.bq;
    if (r0 >= sq.len) return;
    const int r1 = min(r0 + p.bq, sq.len);
    const long long kb = (p.packed ? (long long)hk * p.blk_cap + sq.blk0 : ((long long)b * p.Hkv + hk) * p.blk_cap) + J;
    const long long base = tok_offset(p, p.ks, sq, b, hk, 0);
    const int tid = threadIdx.x;
    if (a.is_bf16) {
        const int c = tid & 15, rs = tid >> 4;
        const unsigned short* src = (const unsigned short*)a.k + base + 8 * c;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int r = r0 + rs; r < r1; r += 16) {
            const uintx4 x = *(const uintx4*)(src + (long long)r * p.ks[2]);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[2 * e] += __uint_as_float(x[e] << 16);
                acc[2 * e + 1] += __uint_as_float(x[e] & 0xffff0000u);
            }
        }
        __shared__ float red[16][128];
#pragma unroll
        for (int e = 0; e < 8; ++e) red[rs][8 * c + e] = acc[e];
        __syncthreads();
        if (tid < 128) {
            float s0 = 0.f;
#pragma unroll
            for (int k = 0; k < 16; ++k) s0 += red[k][tid];
            a.kp_f32[kb * 128 + tid] = s0 / (float)(r1 - r0);
        }
    } else {
        const float* src = (const float*)a.k + base;
        for (int c = tid; c < p.d; c += 256) {
            float s0 = 0.f;
            for (int r = r0; r < r1; ++r) s0 += src[(long long)r * p.ks[2] + c];
            a.kp_f32[kb * p.d + c] = s0 / (float)(r1 - r0);
        }
    }
}

// dynamic LDS of mask_block_kernel: step pooled query rows, step anchors, a tile of 64 pooled keys
// (rows padded by 4 floats), one flag per key block
constexpr int kBlkTile = 64;
size_t mask_block_lds_bytes(int N, int d, int bq, int step) {
    return (size_t)step * d * 4 + (size_t)step * 4 + (size_t)kBlkTile * (d + 4) * 4 + (size_t)((N / bq + 15) / 16) * 16;
}

// grid (ngrp_max, Hq, B), 256 threads.  Per pass a tile of 64 pooled keys sits in LDS; lane l of
// every wave owns key block l of the tile, wave w the pooled rows w, w + 4, ... of the group (so
// the query operand is a broadcast read), four rows at a time.
// Needs n_init and the window start to be multiples of bq, so every half word (16 keys) of the
// bit map lies inside one key block and inside or outside C_g as a whole.
__global__ __launch_bounds__(256) void mask_block_kernel(SelectArgs a) {
    const KParams& p = a.p;
    const int g = p.ngrp_max - 1 - (int)blockIdx.x;    // long candidate ranges first
    const int h = blockIdx.y, b = blockIdx.z, hk = h / p.grp;
    const Seq sq = seq_of(p, b);
    const int nblk = (sq.len + p.bq - 1) / p.bq;
    const int i0 = g * p.step;
    if (i0 >= nblk) return;
    const int nb = min(p.step, nblk - i0);
    const int Wg = window_start(p, g);
    if (Wg <= p.n_init) return;
    const int d = p.d, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kst = d + 4;                             // floats per row of the key tile
    extern __shared__ __attribute__((aligned(16))) float bsm[];
    float* qs = bsm;                                   // [step][d]
    float* xs = qs + p.step * d;                       // [step]
    float* kt = xs + p.step;                           // [64][d + 4]
    unsigned char* flag = (unsigned char*)(kt + kBlkTile * kst);   // [key blocks of C_g]
    for (int e = tid; e < nb * d; e += 256) {
        const long long bi = blk_index(p, sq, b, h, i0 + e / d);
        const int c = e % d;
        qs[e] = a.is_bf16 ? bf16_to_f(((const unsigned short*)a.qp_hi)[bi * 128 + c]) +
                                bf16_to_f(((const unsigned short*)a.qp_lo)[bi * 128 + c])
                          : a.qp_f32[bi * d + c];
    }
    for (int s = tid; s < nb; s += 256) xs[s] = p.use_anchor ? a.xa[blk_index(p, sq, b, h, i0 + s)] : 0.f;
    const int J_lo = p.n_init / p.bq, J_hi = Wg / p.bq;
    const long long kb0 = p.packed ? (long long)hk * p.blk_cap + sq.blk0 : ((long long)b * p.Hkv + hk) * p.blk_cap;
    const int d4 = d / 4;
    for (int J0 = J_lo; J0 < J_hi; J0 += kBlkTile) {
        const int nJ = min(kBlkTile, J_hi - J0);
        __syncthreads();                               // previous tile consumed (first pass: qs, xs written)
        for (int e = tid; e < nJ * d4; e += 256) {
            const int r = e / d4, c = e % d4;
            *(float4*)(kt + r * kst + 4 * c) = *(const float4*)(a.kp_f32 + (kb0 + J0 + r) * d + 4 * c);
        }
        __syncthreads();
        int pred = 0;
        if (lane < nJ) {
            const float4* kr = (const float4*)(kt + lane * kst);
            for (int s0 = wave; s0 < nb; s0 += 16) {   // rows s0, s0 + 4, s0 + 8, s0 + 12
                float dot[4] = {0.f, 0.f, 0.f, 0.f};
                for (int c = 0; c < d4; ++c) {
                    const float4 y = kr[c];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int s = min(s0 + 4 * e, nb - 1);
                        const float4 x = *(const float4*)(qs + s * d + 4 * c);
                        dot[e] = fmaf(x.x, y.x, dot[e]); dot[e] = fmaf(x.y, y.y, dot[e]);
                        dot[e] = fmaf(x.z, y.z, dot[e]); dot[e] = fmaf(x.w, y.w, dot[e]);
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int s = min(s0 + 4 * e, nb - 1);    // a clamped row repeats a real one: same OR
                    pred |= ((xs[s] - p.sigma * dot[e]) <= p.theta) ? 1 : 0;
                }
            }
        }
        // OR over the four waves: each wave ORs its bit into the block's flag byte
        if (wave == 0 && lane < nJ) flag[J0 - J_lo + lane] = (unsigned char)pred;
        __syncthreads();
        if (wave != 0 && lane < nJ && pred) flag[J0 - J_lo + lane] = 1;   // same value from every writer
    }
    __syncthreads();
    unsigned* bits = a.bits + grp_index(p, sq, b, h, g) * a.nwords;
    for (int w = p.n_init / 32 + tid; w < (Wg + 31) / 32; w += 256) {
        unsigned wd = 0;
#pragma unroll
        for (int hw = 0; hw < 2; ++hw) {
            const int j = 32 * w + 16 * hw;
            if (j >= p.n_init && j < Wg && flag[j / p.bq - J_lo]) wd |= 0xffffu << (16 * hw);
        }
        bits[w] = wd;
    }
}

// ------------------------------------------------------------------ count / scan / fill
__global__ void zero_i32_kernel(int* x, long long nelem) {
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nelem) x[i] = 0;
}

// grid (ngrp_max, Hq, B), 256 threads: selected columns of the group, in total and per segment of
// 64 bit words (the segment counts let fill_kernel expand the segments independently)
__global__ __launch_bounds__(256) void count_kernel(SelectArgs a) {
    const KParams& p = a.p;
    const int g = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const Seq sq = seq_of(p, b);
    const int ngrp = (sq.len + p.bq * p.step - 1) / (p.bq * p.step);
    if (g >= ngrp) return;
    const int Wg = window_start(p, g);
    const long long t = grp_index(p, sq, b, h, g);
    const unsigned* bits = a.bits + t * a.nwords;
    int* segc = a.segcount + t * a.nseg;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int w_lo = p.n_init / 32, w_hi = Wg > p.n_init ? (Wg + 31) / 32 : w_lo;
    int total = 0;
    for (int seg = wave; seg * 64 < w_hi; seg += 4) {
        const int w = seg * 64 + lane;
        int c = (w >= w_lo && w < w_hi) ? __popc(bits[w]) : 0;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) c += __shfl_xor(c, off, 64);
        if (lane == 0) segc[seg] = c;
        total += c;
    }
    __shared__ int wsum[4];
    if (lane == 0) wsum[wave] = total;
    __syncthreads();
    if (threadIdx.x == 0) a.counts[t] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

// one work-group of 1024 threads: offsets[t] = sum_{t' < t} roundup64(counts[t']).  With a.stats set
// it also adds up what the prefill reports: attended (row, key) pairs = every row's anchor region
// (closed form per group) plus its group's list, and the selected entries.
namespace {
__device__ __forceinline__ long long tri(long long m) { return m > 0 ? m * (m + 1) / 2 : 0; }
// pairs of the anchor regions of the rows r0 .. r1-1 of a group with window start W:
// sum over r of min(n_init, r + 1) + max(0, r - W + 1)
__device__ __forceinline__ long long anchor_pairs(long long n_init, long long W, long long r0, long long r1) {
    const long long e = min(r1, n_init);
    long long s = e > r0 ? tri(e) - tri(r0) : 0;            // rows inside the initial tokens see r + 1 of them
    s += n_init * max(0ll, r1 - max(r0, n_init));           // later rows see all of them
    s += tri(r1 - W) - tri(r0 - W);                         // window: W .. r
    return s;
}
}  // namespace

__global__ __launch_bounds__(1024) void scan_kernel(SelectArgs a) {
    const KParams& p = a.p;
    const long long T = a.groups_total;
    const int tid = threadIdx.x;
    const long long per = (T + 1023) / 1024;
    const long long lo = min(T, per * tid), hi = min(T, lo + per);
    long long s = 0, pairs = 0, entries = 0;
    for (long long t = lo; t < hi; ++t) {
        const int cnt = a.counts[t];
        s += (cnt + kIdxPad - 1) / kIdxPad * (long long)kIdxPad;
        if (a.stats) {
            // group t -> (sequence, group in the sequence); slots past a packed batch's groups hold 0
            const long long slot = t % p.grp_cap;
            const long long span = (long long)p.bq * p.step;
            long long len = p.N, g = slot;
            if (p.packed) {
                len = 0;
                for (int b = 0; b < p.B; ++b) {
                    const long long n = p.cu[b + 1] - p.cu[b], ng = (n + span - 1) / span;
                    if (g < ng) { len = n; break; }
                    g -= ng;
                }
            }
            if (g * span < len) {
                const long long r0 = g * span, r1 = min(r0 + span, len);
                pairs += anchor_pairs(p.n_init, window_start(p, (int)g), r0, r1) + (r1 - r0) * cnt;
                entries += cnt;
            }
        }
    }
    __shared__ long long part[1024];
    part[tid] = s;
    __syncthreads();
    for (int off = 1; off < 1024; off <<= 1) {
        long long x = tid >= off ? part[tid - off] : 0;
        __syncthreads();
        part[tid] += x;
        __syncthreads();
    }
    long long run = part[tid] - s;
    for (long long t = lo; t < hi; ++t) {
        a.offsets[t] = run;
        run += (a.counts[t] + kIdxPad - 1) / kIdxPad * (long long)kIdxPad;
    }
    if (tid == 1023) {
        a.offsets[T] = part[1023];
        if (a.overflow) *a.overflow = part[1023] > a.idx_capacity ? 1 : 0;
    }
    if (a.stats) {                                           // block sums of pairs and entries
        __syncthreads();
        for (int pass = 0; pass < 2; ++pass) {
            long long x = pass ? entries : pairs;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
            if ((tid & 63) == 0) part[pass * 16 + (tid >> 6)] = x;
        }
        __syncthreads();
        if (tid < 4) {
            long long x = 0;
            if (tid < 2)
                for (int w = 0; w < 16; ++w) x += part[tid * 16 + w];
            a.stats[tid] = x;
        }
    }
}

// grid (ngrp_max, ceil(nseg / 4), B*Hq), 256 threads: each wave expands one segment (64 bit words =
// 2048 keys) of the group's bit words into its part of the ascending list; the segment counts give
// its position.  No barriers: a wave without work returns.
__global__ __launch_bounds__(256) void fill_kernel(SelectArgs a) {
    const KParams& p = a.p;
    const int g = blockIdx.x, h = blockIdx.z % p.Hq, b = blockIdx.z / p.Hq;
    const Seq sq = seq_of(p, b);
    const int ngrp = (sq.len + p.bq * p.step - 1) / (p.bq * p.step);
    if (g >= ngrp) return;
    const int Wg = window_start(p, g);
    if (Wg <= p.n_init) return;
    const int lane = threadIdx.x & 63;
    const int seg = __builtin_amdgcn_readfirstlane(4 * blockIdx.y + (threadIdx.x >> 6));
    const int w_lo = p.n_init / 32, w_hi = (Wg + 31) / 32;
    if (seg * 64 >= w_hi) return;
    const long long t = grp_index(p, sq, b, h, g);
    // every load is issued before the first decision, so the wave pays one memory round trip
    const int* segc = a.segcount + t * a.nseg;
    const int cnt = a.counts[t];
    const int own = segc[seg];
    const long long base = a.offsets[t];
    int pre = 0;                                         // selected columns in earlier segments
    for (int s = lane; s < seg; s += 64) pre += segc[s];
    const int w = seg * 64 + lane;                       // this lane's word
    const unsigned wd = (w >= w_lo && w < w_hi) ? a.bits[t * a.nwords + w] : 0u;
    if (own == 0) return;                                // the group's last entry is never in such a segment
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) pre += __shfl_xor(pre, off, 64);
    // two words per step: lanes 0..31 test word 2 i, lanes 32..63 word 2 i + 1 (coalesced stores)
    long long pos = base + pre;
    const int bit = lane & 31, half = lane >> 5;
    // only the word pairs that hold a selected column are visited (scalar loop over a bit mask)
    const unsigned long long nzw = __ballot(wd != 0u);
    unsigned long long pairs = (nzw | (nzw >> 1)) & 0x5555555555555555ull;
    while (pairs) {
        const int i = __builtin_ctzll(pairs) >> 1;
        pairs &= pairs - 1;
        const unsigned first = __builtin_amdgcn_readlane(wd, 2 * i), second = __builtin_amdgcn_readlane(wd, 2 * i + 1);
        const unsigned mine = half ? second : first;
        const bool on = (mine >> bit) & 1u;
        const long long dst = pos + __popc(mine & ((1u << bit) - 1u)) + (half ? __popc(first) : 0);
        if (on && dst < a.idx_capacity) a.idx[dst] = (seg * 64 + 2 * i + half) * 32 + bit;
        pos += __popc(first) + __popc(second);
    }
    // the wave that wrote the group's last entry pads the list to the next multiple of 64 with it
    if (pre + own == cnt) {
        const unsigned long long nz = __ballot(wd != 0u);
        const int top = 63 - __builtin_clzll(nz);        // own > 0: some word is non-zero
        const unsigned lastw = __shfl(wd, top, 64);
        const int last_key = (seg * 64 + top) * 32 + 31 - __clz(lastw);
        const int padded = (cnt + kIdxPad - 1) / kIdxPad * kIdxPad;
        for (int e = cnt + lane; e < padded; e += 64)
            if (base + e < a.idx_capacity) a.idx[base + e] = last_key;
    }
}

}  // namespace aa
