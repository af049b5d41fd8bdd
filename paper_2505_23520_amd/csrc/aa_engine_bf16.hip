// bf16 tile engine: one online-softmax (flash-style) kernel that serves
//   * stage 1, anchor computation          (Sec. 3.1 Eq. 1, Algorithm 1),
//   * stage 3, gathered sparse attention   (Sec. 3.3 Eq. 3-5, Algorithm 3),
//   * the dense causal comparator
// of arXiv 2505.23520 on gfx950.  The three differ only in which K/V rows feed
// the tiles (a contiguous masked range or the rows a selected-column list names)
// and in what is read before / written after the loop.
//
// Shape of the computation (d = 128, b_q = 128, bf16 in, fp32 accumulate):
//   work-group = one query block = 4 waves x 32 query rows, two work-groups per CU
//   (two waves per SIMD, so one wave's softmax overlaps the other's MFMAs);
//   K/V tile   = 64 keys, double-buffered in LDS, filled by 16-byte direct-to-LDS buffer
//   loads (no staging registers; a gathered row and a contiguous row cost the same);
//   S^T = K Q^T  with v_mfma_f32_32x32x16_bf16 (keys are the M dimension, query
//   rows the N dimension, so one lane owns one query row and the row max / sum
//   are in-lane reductions plus one exchange between the wave's halves);
//   O^T = V^T P^T with the same instruction; V stays row-major in LDS and its operand
//   is read with the transposing LDS load ds_read_b64_tr_b16.
// LDS layout of a tile: a direct-to-LDS load writes the 64 lanes' 16 bytes to consecutive
// addresses, i.e. 1 KB = four 256-byte rows per instruction ("group").  Key kk of the tile
// sits in group kk % 16, row kk / 16; groups are padded (K: 16 B, V: 64 B) so that the 16
// lanes of an operand read fall into different banks.
// The running reference m of exp(s - m) is only raised when a row's maximum
// exceeds it by more than 2^8; the accumulators (which live in AGPRs) are then
// rescaled, otherwise they are left alone.  The true row maximum, which is the
// anchor that stage 1 exports, is tracked separately.
#include "aa_engine_bf16_common.h"
#include "aa_pool.h"

namespace aa {

using namespace eng;

// FLAGS (a combination of kEng*) is a compile-time parameter: every mode gets its own code without
// the other modes' branches, registers and, above all, merged control-flow paths (where paths with
// different numbers of outstanding loads meet, the compiler's waits assume the shortest).
template <int FLAGS>
__global__ __launch_bounds__(256, 2) void engine_bf16_kernel(EngineArgs a) {
    constexpr int flags = FLAGS;
    constexpr int NW = 4;                            // waves per work-group
    static_assert(NW == 4, "the loader deals four groups of a tile to every wave");
    // one LDS object per stage, so that the compiler can tell that the asynchronous loads into
    // one stage do not alias the operand reads from the other
    __shared__ __attribute__((aligned(16))) char Ks0[KBYTES], Ks1[KBYTES], Vs0[VBYTES], Vs1[VBYTES];
    __shared__ float red[NW];
    __shared__ float qpart[(FLAGS & kEngStoreState) ? 4 : 1][128];   // pooled-query partial sums (stage 1)
    const KParams& p = a.p;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it scalar
    const int n = lane & 31, hf = lane >> 5;

    if (!engine_selected(a)) return;
    const Work wk = decode_work(p, p.nblk_max, blockIdx.x);
    const Seq sq = seq_of(p, wk.b);
    const int row0 = wk.i * BQ;
    if (row0 >= sq.len) return;
    // Two waves share a SIMD (one from each resident work-group).  A wave raises its issue priority
    // for its MFMA blocks and drops it for its softmax, so a wave with matrix work wins over a
    // sibling that is in its vector-ALU part, and the pair does not settle into lockstep.
    __builtin_amdgcn_s_setprio(2);
    const int hk = wk.h / p.grp;
    const int g = wk.i / p.step;
    const int rw = row0 + 32 * wave;                 // first row of this wave
    const int r = rw + n;                            // this lane's query row
    const bool rok = r < sq.len;
    const int rlast = min(row0 + BQ, sq.len) - 1;    // last row of the block

    // ---- tile sequence: [range 1: initial tokens][range 2: window .. diagonal][list chunks]
    int W = 0, ninit = 0, T1 = 0, t2s = 0, nA = 0;
    if (flags & kEngAnchorRegion) {
        if (!(flags & kEngDense)) { W = window_start(p, g); ninit = p.n_init; }
        const int e1 = min(ninit, rlast + 1);
        T1 = (e1 + TK - 1) / TK;
        t2s = max(T1, W / TK);
        const int T2 = rlast / TK + 1;
        nA = T1 + max(0, T2 - t2s);
    }
    int cnt = 0;
    long long lbase = 0;
    if (flags & kEngList) {
        const long long t = grp_index(p, sq, wk.b, wk.h, g);
        cnt = a.counts[t];
        lbase = a.offsets[t];
    }
    const int nL = (cnt + TK - 1) / TK;
    const int nT = nA + nL;

    // K / V rows of this KV head are fetched with raw buffer loads: scalar base, 32-bit byte offsets
    const unsigned short* kb_ = (const unsigned short*)a.k + tok_offset(p, p.ks, sq, wk.b, hk, 0);
    const unsigned short* vb_ = (const unsigned short*)a.v + tok_offset(p, p.vs, sq, wk.b, hk, 0);
    const unsigned kstb = (unsigned)p.ks[2] * 2u, vstb = (unsigned)p.vs[2] * 2u;   // token strides in bytes
    const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc(
        (void*)kb_, 0, (int)((unsigned)(sq.len - 1) * kstb + 2u * D), 0x00020000);
    const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc(
        (void*)vb_, 0, (int)((unsigned)(sq.len - 1) * vstb + 2u * D), 0x00020000);

    // ---- loader role of this wave: GPW = 16 / NW groups of every tile.  In the load of group gi
    // lane l fetches the 16-byte chunk l % 16 of key 16 (l / 16) + gi of the tile, so each lane deals
    // with the GPW consecutive keys 16 (l / 16) + GPW wave + j.
    constexpr int GPW = 16 / NW;
    const int lch = lane & 15;
    const int kq0 = 16 * (lane >> 4) + GPW * wave;   // first of this lane's keys inside the tile

    auto tile_start = [&](int t) -> int {            // first key of contiguous tile t (t < nA)
        return TK * (t < T1 ? t : t2s + (t - T1));
    };
    // Keys of a list tile come from the index list: they are fetched one step ahead into kidx.
    // Nothing else ever writes kidx's registers: a vector-ALU write to registers that may still
    // be the target of an outstanding load makes the compiler wait for every outstanding load,
    // the asynchronous tile loads included.  Keys of a contiguous tile are plain arithmetic.
    intx4 kidx = {0, 0, 0, 0};
    auto idx_prefetch = [&](int t) {
        if (t >= nA && t < nT) kidx = *(const intx4*)(a.idx + lbase + (long long)(t - nA) * TK + kq0);
    };
    // asynchronous: completion is awaited by wait_vmem()
    auto tile_load = [&](int t, char* Kb, char* Vb) {
        char* kd = Kb + GPW * wave * KGRP;
        char* vd = Vb + GPW * wave * VGRP;
        if (t < nA) {
            const int t0 = tile_start(t) + kq0;
#pragma unroll
            for (int j = 0; j < GPW; ++j) {
                const unsigned key = (unsigned)min(t0 + j, sq.len - 1);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(krs, (lds_void*)(kd + j * KGRP), 16,
                                                         (int)(key * kstb + 16u * lch), 0, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(vrs, (lds_void*)(vd + j * VGRP), 16,
                                                         (int)(key * vstb + 16u * lch), 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int j = 0; j < GPW; ++j) {
                __builtin_amdgcn_raw_ptr_buffer_load_lds(krs, (lds_void*)(kd + j * KGRP), 16,
                                                         (int)((unsigned)kidx[j] * kstb + 16u * lch), 0, 0, 0);
                __builtin_amdgcn_raw_ptr_buffer_load_lds(vrs, (lds_void*)(vd + j * VGRP), 16,
                                                         (int)((unsigned)kidx[j] * vstb + 16u * lch), 0, 0, 0);
            }
        }
    };

    // The first list indices are requested before everything else: the first tile's loads need them,
    // and only them, so they go out while the Q fragments and the cached state are still on their way
    // (waits are in issue order: behind those loads the indices would arrive last).
    if (nT > 0) idx_prefetch(0);

    // ---- Q fragments (B operand of S^T = K Q^T): lane (n, hf) holds Q[row][16 ks + 8 hf .. +8)
    bf16x8 qf[8];
    load_q_fragments(qf, a, sq, wk.b, wk.h, r, rok, 0, hf);

    // ---- running state (see load_state)
    const float c2 = p.sigma * 1.4426950408889634f;  // exp(sigma*x) = exp2(c2*x)
    const float rescale_gap = kRescaleLog2 / c2;
    const long long ri = row_index(p, sq, wk.b, wk.h, rok ? r : row0);
    const long long tile = acc_tile(p, sq, wk.b, wk.h, wk.i, wave);
    float mref, mtrue, l;
    floatx16 o[4];
    if (flags & kEngLoadState) load_state(a, ri, tile, lane, hf, mref, mtrue, l, o);
    else init_state(mref, mtrue, l, o);

    // ---- pipeline prologue
    if (nT > 0) {
        tile_load(0, Ks0, Vs0);
        idx_prefetch(1);
    }
    wait_vmem();
    __syncthreads();

    // operand addresses inside a stage (bytes): K row of key 32 kb + n; V chunk read by this lane
    // in the transposing load (lane 16 G + s: key offset s / 4, 8-byte piece s % 4 of d-half G % 2)
    const int koff = (n & 15) * KGRP + (n >> 4) * 256 + 16 * hf;
    const int ls = lane & 15, lg = lane >> 4;
    const int voff = (4 * hf + (ls >> 2)) * VGRP + 32 * (lg & 1) + 8 * (ls & 3);

    auto tile_step = [&](int t, const char* Kcur, const char* Vcur, char* Knext, char* Vnext) {
        if (t + 1 < nT) {
            tile_load(t + 1, Knext, Vnext);
            idx_prefetch(t + 2);
        }
        const char* Kb = Kcur + koff;
        const char* Vb = Vcur + voff;

        // S^T = K Q^T : s[kb], 32 keys x 32 rows each.  Masks (tiles that touch a region
        // boundary, the diagonal or a list tail) enter as the initial accumulator: 0 for a
        // visible (key, row) pair, -inf otherwise; the common unmasked tile starts from literal 0.
        int mode = 0, t0 = 0;
        if (t < nA) {
            t0 = tile_start(t);
            const bool interior = (t0 + TK - 1 <= rw) && (t0 + TK <= ninit || t0 >= W);
            mode = interior ? 0 : 1;
        } else if (t == nT - 1 && (cnt & (TK - 1))) {
            mode = 2;
        }
        // a contiguous tile that starts beyond this wave's last row is hidden from all its rows
        // (the work-group still needs it for its later rows): nothing to compute
        if (!(t < nA && t0 > rw + 31)) {
        floatx16 s[2];
        if (__builtin_expect(mode == 0, 1)) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const bf16x8 kf = *(const bf16x8*)(Kb + 512 * kb);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[0], kZero16, 0, 0, 0);
            }
        } else {
            // key j = t0 + jl is visible to row r iff j <= r and (j < ninit or j >= W);
            // entry jl of the last list chunk is real iff jl < rem
            const int jr = mode == 1 ? r - t0 : cnt - (t - nA) * TK - 1;
            const int jn = mode == 1 ? ninit - t0 : TK;
            const int jw = W - t0;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                floatx16 bias;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int jl = 32 * kb + 8 * (v >> 2) + 4 * hf + (v & 3);
                    const bool ok = (jl <= jr) & ((jl < jn) | (jl >= jw));
                    bias[v] = ok ? 0.f : -INFINITY;
                }
                const bf16x8 kf = *(const bf16x8*)(Kb + 512 * kb);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[0], bias, 0, 0, 0);
            }
        }
#pragma unroll
        for (int ks = 1; ks < 8; ++ks)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const bf16x8 kf = *(const bf16x8*)(Kb + 512 * kb + 32 * ks);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kb], 0, 0, 0);
            }
        __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 6, 0);

        __builtin_amdgcn_s_setprio(0);
        bf16x8 pf[2][2];  // [kb][s16]
        if constexpr ((FLAGS & kEngStoreState) != 0) softmax_tile(s, pf, c2, rescale_gap, mref, mtrue, l, o);
        else softmax_tile_lazy(s, pf, c2, mref, l, o);

        __builtin_amdgcn_s_setprio(2);
        // O^T += V^T P^T
#pragma unroll
        for (int sg = 0; sg < 4; ++sg)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                // keys 16 sg + 8 rd + 4 hf + (0..3) live in groups 8 rd + 4 hf + (0..3), row sg
                const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) shortx4*)(Vb + sg * 256 + 64 * db));
                const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                    (__attribute__((address_space(3))) shortx4*)(Vb + 8 * VGRP + sg * 256 + 64 * db));
                const shortx8 vv = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), pf[sg >> 1][sg & 1],
                                                                 o[db], 0, 0, 0);
            }

        }
        wait_vmem();                                 // next tile has landed in LDS
        __syncthreads();
    };
    for (int t = 0; t < nT; t += 2) {
        tile_step(t, Ks0, Vs0, Ks1, Vs1);
        if (t + 1 < nT) tile_step(t + 1, Ks1, Vs1, Ks0, Vs0);
    }

    // ---- epilogue
    // The tile stages are free now (every wave has passed the barrier that ends the last tile):
    // each wave takes one of them as a private staging area for coalesced stores.  LDS operations
    // of one wave execute in order, so no barrier separates its writes from its reads.
    char* const stg = wave == 0 ? Ks0 : wave == 1 ? Ks1 : wave == 2 ? Vs0 : Vs1;
    const int wave_rows = min(32, sq.len - rw);      // rows of this wave inside the sequence (<= 0: none)
    const float lt = row_sum(l);                     // row sum relative to mref
    if (flags & kEngStoreState) {
        const float ms = store_state(a, ri, tile, rok, wave_rows > 0, lane, hf, c2, mref, mtrue, lt, o);
        if (a.qp_hi) {
            // pooled query of the block (Algorithm 2, avgpool of Q) from the fragments in registers
            float s0, s1;
            pool_wave_columns(qf, n, s0, s1);
            pool_block_finish(qpart, wave, n, hf, s0, s1, tid, rlast - row0 + 1,
                              blk_index(p, sq, wk.b, wk.h, wk.i), true, a.qp_hi, a.qp_lo, a.qlo_norm);
        }
        if (a.xa) {
            // pooled anchor of the block: mean of M over its rows (Algorithm 2, avgpool of the anchor)
            float red_m = (rok && hf == 0) ? ms : 0.f;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) red_m += __shfl_xor(red_m, off, 64);
            if (lane == 0) red[wave] = red_m;
            __syncthreads();
            if (tid == 0) {
                const int nrows = rlast - row0 + 1;
                a.xa[blk_index(p, sq, wk.b, wk.h, wk.i)] = (red[0] + red[1] + red[2] + red[3]) / (float)nrows;
            }
        }
    }
    if ((flags & kEngStoreOut) && wave_rows > 0) {
        store_out(a, stg, tok_offset(p, p.os, sq, wk.b, wk.h, rw), wave_rows, lane, n, hf, lt, o);
        if (rok && a.lse && hf == 0) a.lse[ri] = mref * p.sigma + __logf(lt);
    }
}


int launch_engine_bf16(const EngineArgs& ea, unsigned grid, hipStream_t st) {
    switch (ea.flags) {
#define AA_ENGINE_CASE(F) \
    case (F): return (int)launch_kernel(engine_bf16_kernel<(F)>, dim3(grid), dim3(256), 0, st, ea);
    AA_ENGINE_CASE(kEngAnchorRegion | kEngStoreState)                 // stage 1
    AA_ENGINE_CASE(kEngList | kEngLoadState | kEngStoreOut)           // stage 3 from the cached state
    AA_ENGINE_CASE(kEngList | kEngAnchorRegion | kEngStoreOut)        // stage 3 recomputing the anchor region
    AA_ENGINE_CASE(kEngAnchorRegion | kEngDense | kEngStoreOut)       // dense causal attention
#undef AA_ENGINE_CASE
    default: return -1;
    }
}

}  // namespace aa
