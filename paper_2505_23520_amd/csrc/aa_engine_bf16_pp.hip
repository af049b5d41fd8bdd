// bf16 tile engine, ping-pong variant: the same computation as engine_bf16_kernel (stage 1,
// stage 3 and the dense comparator of arXiv 2505.23520; see that file for the fragment and LDS
// layouts, which are identical), organised so that the matrix pipe and the vector ALU of a SIMD
// are busy at the same time by construction instead of by chance:
//   work-group = two consecutive query blocks of one head = 8 waves x 32 query rows, one
//   work-group per CU.  Waves w and w + 4 share a SIMD; waves 0-3 form group A, waves 4-7
//   group B.  Time is cut into slots by work-group barriers.  In every slot one group runs its
//   MFMA phase (this wave's share of the tile loads, S^T = K Q^T of tile t + 1, then
//   O^T += V^T P^T of tile t: 32 MFMAs interleaved with their LDS operand reads) while the other
//   runs its softmax phase (masks, row max, exp2, row sum, bf16 conversion of tile t: vector ALU
//   only); then they swap.  Group B runs one slot behind group A.
//   K/V tiles are triple-buffered in LDS and shared by the 256 rows.  Group A's waves issue the
//   direct-to-LDS loads of the K tiles (three tiles ahead), group B's those of the V tiles (two
//   tiles ahead), from inside their MFMA phase, and wait for them at the start of their next
//   MFMA phase (two slots later).  Masks are applied to the scores in the softmax phase.
// The two query blocks must share their window start and their selected-column list: the host
// launches this kernel for dense attention and for even `step`, the 128-row kernel otherwise.
#include "aa_engine_bf16_common.h"
#include "aa_pool.h"

namespace aa {

using namespace eng;

namespace {

constexpr int PAIR = 2 * BQ;         // query rows per work-group

// Slot boundary.  LDS operand reads of the ending phase have been consumed by its MFMAs and the
// asynchronous loads a wave publishes here were awaited with wait_vmem(), so the bare barrier
// is enough; the fences around it only keep the compiler from moving work across the boundary.
__device__ __forceinline__ void slot_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);
}

}  // namespace

// FLAGS >= 0: compile-time mode, as in engine_bf16_kernel (the two modes that matter: stage 3
// from the cached state and dense attention); FLAGS < 0: the mode is read from the arguments.
template <int FLAGS>
__global__ __launch_bounds__(512, 1) void engine_bf16_pp_kernel(EngineArgs a) {
    const int flags = FLAGS >= 0 ? FLAGS : a.flags;
    __shared__ __attribute__((aligned(16))) char Ks0[KBYTES], Ks1[KBYTES], Ks2[KBYTES];
    __shared__ __attribute__((aligned(16))) char Vs0[VBYTES], Vs1[VBYTES], Vs2[VBYTES];
    __shared__ float red[8];
    __shared__ float qpart[(FLAGS < 0) ? 2 : 1][(FLAGS < 0) ? 4 : 1][128];   // pooled-query partial sums (stage 1)
    const KParams& p = a.p;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it scalar
    const int n = lane & 31, hf = lane >> 5;
    const int grpB = wave >> 2;                      // 0: group A, 1: group B
    const int simd = wave & 3;
    const int chunk = 2 * simd + grpB;               // the wave's 32 rows inside the pair

    if (!engine_selected(a)) return;
    const int npair = (p.nblk_max + 1) >> 1;
    const Work wk = decode_work(p, npair, blockIdx.x);   // wk.i = pair index
    const Seq sq = seq_of(p, wk.b);
    const int row0 = wk.i * PAIR;
    if (row0 >= sq.len) return;
    const int hk = wk.h / p.grp;
    const int g = (2 * wk.i) / p.step;
    const int rw = row0 + 32 * chunk;                // first row of this wave
    const int r = rw + n;                            // this lane's query row
    const bool rok = r < sq.len;
    const bool wave_on = rw < sq.len;
    const int rlast = min(row0 + PAIR, sq.len) - 1;  // last row of the pair

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

    const unsigned short* kb_ = (const unsigned short*)a.k + tok_offset(p, p.ks, sq, wk.b, hk, 0);
    const unsigned short* vb_ = (const unsigned short*)a.v + tok_offset(p, p.vs, sq, wk.b, hk, 0);
    // this wave loads rows of one tensor only: K (group A) or V (group B)
    const unsigned short* lb_ = grpB ? vb_ : kb_;
    const unsigned lstb = (unsigned)(grpB ? p.vs[2] : p.ks[2]) * 2u;              // token stride in bytes
    const __amdgpu_buffer_rsrc_t lrs = __builtin_amdgcn_make_buffer_rsrc(
        (void*)lb_, 0, (int)((unsigned)(sq.len - 1) * lstb + 2u * D), 0x00020000);
    const int lgrp = grpB ? VGRP : KGRP;

    // ---- loader role: groups 4 simd .. 4 simd + 3 of every tile.  In the load of group gi lane l
    // fetches the 16-byte chunk l % 16 of key 16 (l / 16) + gi of the tile.
    const int lch = lane & 15;
    const int kq0 = 16 * (lane >> 4) + 4 * simd;     // first of this lane's keys inside the tile

    auto tile_start = [&](int t) -> int {            // first key of contiguous tile t (t < nA)
        return TK * (t < T1 ? t : t2s + (t - T1));
    };
    // Keys of a list tile come from the index list.  The MFMA phase of round position i (tile
    // number mod 3) takes the keys of the tile it loads from kidx[i]; they are fetched there two
    // phases earlier.  Nothing else ever writes these registers: a vector-ALU write to registers
    // that may still be the target of an outstanding load makes the compiler wait for every
    // outstanding load, the asynchronous tile loads included.  With a list the fetch is issued
    // for every tile (clamped into the list), so that exactly one load is younger than the tile
    // loads an MFMA phase awaits.  Keys of a contiguous tile are plain arithmetic.
    const bool has_list = nL > 0;
    intx4 kidx[3] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}};
    auto idx_fetch = [&](int t) -> intx4 {
        const int c = min(max(t - nA, 0), nL - 1);
        return *(const intx4*)(a.idx + lbase + (long long)c * TK + kq0);
    };
    // asynchronous: completion is awaited by wait_vmem()
    auto tile_load = [&](int t, char* Kb, char* Vb) {
        char* dst = (grpB ? Vb : Kb) + 4 * simd * lgrp;
        if (t < nA) {
            const int t0 = tile_start(t) + kq0;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(lrs, (lds_void*)(dst + j * lgrp), 16,
                                                         (int)((unsigned)min(t0 + j, sq.len - 1) * lstb + 16u * lch),
                                                         0, 0, 0);
        } else {
            const intx4 key = idx_fetch(t);
#pragma unroll
            for (int j = 0; j < 4; ++j)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(lrs, (lds_void*)(dst + j * lgrp), 16,
                                                         (int)((unsigned)key[j] * lstb + 16u * lch), 0, 0, 0);
        }
    };

    // In the main loop the loads are issued from inside the MFMA phase, which must stay one basic
    // block: byte offsets of the wave's four rows without a branch (contiguous tile: scalar tile
    // base + per-lane constants, clamped to the last row; list tile: index * stride).
    unsigned lpre[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) lpre[j] = (unsigned)(kq0 + j) * lstb + 16u * lch;
    const unsigned lmax = (unsigned)(sq.len - 1) * lstb + 16u * lch;

    // ---- Q fragments (B operand of S^T = K Q^T): lane (n, hf) holds Q[row][16 ks + 8 hf .. +8)
    bf16x8 qf[8];
    load_q_fragments(qf, a, sq, wk.b, wk.h, r, rok, 0, hf);

    // ---- running state (see load_state).  The wave's 32 rows are tile chunk % 4 of block
    // 2 i + chunk / 4; a wave whose rows lie past the end of the sequence reads the pair's first
    // block (in bounds, unused).
    const float c2 = p.sigma * 1.4426950408889634f;  // exp(sigma*x) = exp2(c2*x)
    const float rescale_gap = kRescaleLog2 / c2;
    const long long ri = row_index(p, sq, wk.b, wk.h, rok ? r : row0);
    const long long tile = acc_tile(p, sq, wk.b, wk.h, 2 * wk.i + (wave_on ? chunk >> 2 : 0), chunk & 3);
    float mref, mtrue, l;
    floatx16 o[4];
    if (flags & kEngLoadState) load_state(a, ri, tile, lane, hf, mref, mtrue, l, o);
    else init_state(mref, mtrue, l, o);

    // operand addresses inside a stage (bytes): K row of key 32 kb + n; V chunk read by this lane
    // in the transposing load (lane 16 G + s: key offset s / 4, 8-byte piece s % 4 of d-half G % 2)
    const int koff = (n & 15) * KGRP + (n >> 4) * 256 + 16 * hf;
    const int ls = lane & 15, lg = lane >> 4;
    const int voff = (4 * hf + (ls >> 2)) * VGRP + 32 * (lg & 1) + 8 * (ls & 3);

    // a contiguous tile that starts beyond this wave's last row is hidden from all its rows (the
    // work-group still needs it for later rows): the wave computes nothing for it
    auto tile_on = [&](int t) -> bool { return wave_on && t < nT && !(t < nA && tile_start(t) > rw + 31); };
    // 0: every (key, row) pair of the tile is visible; 1: contiguous tile that touches a region
    // boundary or the diagonal; 2: last chunk of a list with padding entries
    auto tile_mode = [&](int t) -> int {
        if (t < nA) {
            const int t0 = tile_start(t);
            return ((t0 + TK - 1 <= rw) && (t0 + TK <= ninit || t0 >= W)) ? 0 : 1;
        }
        return (t == nT - 1 && (cnt & (TK - 1))) ? 2 : 0;
    };

    floatx16 s[2];      // scores of the tile between its QK and its softmax phase
    bf16x8 pf[2][2];    // probabilities of the tile between its softmax and its PV phase

    // MFMA phase, one basic block: S^T = K Q^T of the next tile (s[kb]: 32 keys x 32 rows each),
    // then O^T += V^T P^T of the current one, 32 MFMAs with their 48 LDS operand reads spread
    // between them.  A wave gets a transposing read through only every ~24 cycles and a 16-byte
    // read every ~14, so the reads of a tile take about as long as its MFMAs: the order below
    // keeps both going (left alone, the compiler issues each read right before its MFMA and the
    // phase waits out every LDS latency).  A tile this wave skips enters with pf = 0; scores of a
    // skipped next tile are computed and ignored.
    auto mfma_phase = [&](const char* Knext, const char* Vcur, char* Kld, char* Vld, int u, const intx4& keys) {
        const char* Kb = Knext + koff;
        const char* Vb = Vcur + voff;
        // this wave's share of the loads of tile u (asynchronous; awaited by wait_vmem())
        {
            char* dst = (grpB ? Vld : Kld) + 4 * simd * lgrp;
            const bool is_list = u >= nA;
            const unsigned sbase = (unsigned)tile_start(u) * lstb;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const unsigned oc = min(sbase + lpre[j], lmax);
                const unsigned ol = (unsigned)keys[j] * lstb + 16u * lch;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(lrs, (lds_void*)(dst + j * lgrp), 16,
                                                         (int)(is_list ? ol : oc), 0, 0, 0);
            }
        }
        // Issue order written out and pinned with scheduling fences (a sched_group_barrier
        // pipeline for the same order is honoured in some instantiations of this kernel and not in
        // others): K operands run four MFMAs ahead; the V operands (two transposing reads each) of
        // the first four P V MFMAs are read under the last four score MFMAs, then four ahead.
        __builtin_amdgcn_sched_barrier(0);
        bf16x8 kf[16];
        shortx4 vlo[16], vhi[16];
        auto read_k = [&](int i) { kf[i] = *(const bf16x8*)(Kb + 512 * (i & 1) + 32 * (i >> 1)); };
        auto read_v = [&](int i) {                 // operand of P V MFMA i: sg = i / 4, db = i % 4
            // keys 16 sg + 8 rd + 4 hf + (0..3) live in groups 8 rd + 4 hf + (0..3), row sg
            vlo[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) shortx4*)(Vb + (i >> 2) * 256 + 64 * (i & 3)));
            vhi[i] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (__attribute__((address_space(3))) shortx4*)(Vb + 8 * VGRP + (i >> 2) * 256 + 64 * (i & 3)));
        };
#pragma unroll
        for (int i = 0; i < 4; ++i) read_k(i);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < 16; ++i) {             // score MFMA i: ks = i / 2, kb = i % 2
            s[i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], qf[i >> 1], i < 2 ? kZero16 : s[i & 1], 0, 0, 0);
            if (i + 4 < 16) read_k(i + 4); else read_v(i - 12);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {             // P V MFMA i
            const shortx8 vv = __builtin_shufflevector(vlo[i], vhi[i], 0, 1, 2, 3, 4, 5, 6, 7);
            const int sg = i >> 2, db = i & 3;
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), pf[sg >> 1][sg & 1],
                                                             o[db], 0, 0, 0);
            if (i + 4 < 16) read_v(i + 4);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // online softmax of this lane's query row (the other half of the row is 32 lanes away).
    // In a masked tile key j = t0 + jl is visible to row r iff j <= r and (j < ninit or j >= W);
    // entry jl of the last list chunk is real iff jl < rem; hidden scores count as -inf.  The
    // hidden scores are overwritten in place before the common code.
    auto softmax_phase = [&](int t) {
        if (__builtin_expect(!tile_on(t), 0)) {
            const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
            pf[0][0] = zero8; pf[0][1] = zero8; pf[1][0] = zero8; pf[1][1] = zero8;
            return;
        }
        const int mode = tile_mode(t);
        if (__builtin_expect(mode != 0, 0)) {
            const int t0 = mode == 1 ? tile_start(t) : 0;
            const int jr = mode == 1 ? r - t0 : cnt - (t - nA) * TK - 1;
            const int jn = mode == 1 ? ninit - t0 : TK;
            const int jw = mode == 1 ? W - t0 : 0;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int jl = 32 * kb + 8 * (v >> 2) + 4 * hf + (v & 3);
                    const bool ok = (jl <= jr) & ((jl < jn) | (jl >= jw));
                    s[kb][v] = ok ? s[kb][v] : -INFINITY;
                }
        }
        // The lazy variant (row maximum only when needed) wherever the true maximum is not exported.
        // Its rare branch, like the other rare branches of the tile loop, is marked unlikely: the
        // compiler then lays the loop body out compactly, and that decides more than instruction
        // count here.  With the rescue code inside the loop body the launch with lists (128k, every
        // column selected) fetched 240 GiB from HBM instead of 19 GiB and ran slower than the eager
        // form: the work-groups that share one KV head's stream through an XCD's L2 no longer kept
        // within its 4 MB of each other.
        if constexpr (FLAGS >= 0 && (FLAGS & kEngStoreState) == 0) softmax_tile_lazy(s, pf, c2, mref, l, o);
        else softmax_tile(s, pf, c2, rescale_gap, mref, mtrue, l, o);
    };

    // ---- The MFMA phase always runs, also for a tile this wave skips (P = 0) and for the padding
    // tiles of the last round, and 0 x V must then be 0: no V stage may hold leftovers of another
    // kernel that decode as Inf or NaN.  Clear them before the first loads.
    {
        const intx4 z = {0, 0, 0, 0};
        for (int e = tid; e < VBYTES / 16; e += 512) {
            *(intx4*)(Vs0 + 16 * e) = z; *(intx4*)(Vs1 + 16 * e) = z; *(intx4*)(Vs2 + 16 * e) = z;
        }
        __syncthreads();
    }
    // ---- prologue: K tiles 0..2 (group A) / V tiles 0..1 (group B), then the slot offset of group B
    const int la = grpB ? 2 : 3;                     // how many tiles ahead this wave loads
    if (nT > 0) {
        tile_load(0, Ks0, Vs0);
        if (nT > 1) tile_load(1, Ks1, Vs1);
        if (nT > 2 && !grpB) tile_load(2, Ks2, Vs2);
        if (has_list) {
            kidx[2] = idx_fetch(min(la - 1, nT - 1));    // for the first MFMA phase below
            kidx[0] = idx_fetch(min(la, nT - 1));        // for the MFMA phase of tile 0
        }
    }
    {
        const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
        pf[0][0] = zero8; pf[0][1] = zero8; pf[1][0] = zero8; pf[1][1] = zero8;
    }
    wait_vmem();
    slot_barrier();
    // scores of tile 0 (P = 0: O unchanged); its loads repeat tile la - 1 into its own stage
    if (!grpB && nT > 0) mfma_phase(Ks0, Vs0, Ks2, Vs1, min(la - 1, nT - 1), kidx[2]);
    slot_barrier();
    if (grpB) {
        if (nT > 0) mfma_phase(Ks0, Vs0, Ks2, Vs1, min(la - 1, nT - 1), kidx[2]);
        slot_barrier();
    }

    // one tile: softmax phase, then MFMA phase.  The MFMA phase starts by awaiting the loads this wave
    // issued during its previous MFMA phase (the barrier that ends this phase publishes them); it
    // issues those of tile t + 3 (K, group A: the stage tile t has left a slot ago) or t + 2 (V,
    // group B: the stage tile t - 1 has left).  Past the end the last tile is loaded again into
    // a stage nobody reads any more, which keeps the phase free of branches.
    auto tile_iter = [&](int t, char* Kld, char* Vld, const char* Vcur, const char* Knext, intx4& keys,
                         intx4& keys_next) {
        softmax_phase(t);
        if (has_list) keys_next = idx_fetch(min(t + 1 + la, nT - 1));   // for the MFMA phase after this one
        slot_barrier();
        // everything but the index fetch just issued, which is the youngest load
        if (has_list) __builtin_amdgcn_s_waitcnt(0x0F71); else wait_vmem();
        // the wave in its MFMA phase wins issue arbitration against its SIMD sibling's vector ALU work (+1 %)
        __builtin_amdgcn_s_setprio(2);
        mfma_phase(Knext, Vcur, Kld, Vld, min(t + la, nT - 1), keys);
        __builtin_amdgcn_s_setprio(0);
        slot_barrier();
    };
    // whole rounds of three tiles (one per LDS stage); tiles past the end only keep the barriers
    for (int t = 0; t < nT; t += 3) {
        tile_iter(t, Ks0, Vs2, Vs0, Ks1, kidx[0], kidx[1]);
        tile_iter(t + 1, Ks1, Vs0, Vs1, Ks2, kidx[1], kidx[2]);
        tile_iter(t + 2, Ks2, Vs1, Vs2, Ks0, kidx[2], kidx[0]);
    }
    if (!grpB) slot_barrier();

    // ---- epilogue
    const float lt = row_sum(l);                     // row sum relative to mref
    if (flags & kEngStoreState) {
        const float ms = store_state(a, ri, tile, rok, wave_on, lane, hf, c2, mref, mtrue, lt, o);
        if (FLAGS < 0 && a.qp_hi) {
            // pooled query of each block (Algorithm 2, avgpool of Q) from the fragments in registers;
            // the four waves of a block are a team
            const int blk = (FLAGS < 0) ? chunk >> 2 : 0, b0 = row0 + BQ * blk;
            float s0, s1;
            pool_wave_columns(qf, n, s0, s1);
            pool_block_finish(qpart[blk], chunk & 3, n, hf, s0, s1, 64 * (chunk & 3) + lane, min(b0 + BQ, sq.len) - b0,
                              blk_index(p, sq, wk.b, wk.h, 2 * wk.i + blk), b0 < sq.len, a.qp_hi, a.qp_lo, a.qlo_norm);
        }
        if (a.xa) {
            // pooled anchor of each block: mean of M over its rows (Algorithm 2, avgpool of the anchor)
            float red_m = (rok && hf == 0) ? ms : 0.f;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) red_m += __shfl_xor(red_m, off, 64);
            if (lane == 0) red[chunk] = red_m;
            __syncthreads();
            if (tid < 2) {
                const int b0 = row0 + BQ * tid;      // first row of block 2 i + tid
                if (b0 < sq.len) {
                    const int nrows = min(b0 + BQ, sq.len) - b0;
                    a.xa[blk_index(p, sq, wk.b, wk.h, 2 * wk.i + tid)] =
                        (red[4 * tid] + red[4 * tid + 1] + red[4 * tid + 2] + red[4 * tid + 3]) / (float)nrows;
                }
            }
        }
    }
    if (flags & kEngStoreOut) {
        // The MFMA phases issue tile loads to the end (past the last tile into stages nobody reads):
        // once every wave's loads have landed the stages are free, and each wave takes a piece of
        // one as private staging area for coalesced stores.
        wait_vmem();
        __syncthreads();
        char* const stg = wave == 0 ? Ks0 : wave == 1 ? Ks1 : wave == 2 ? Ks2
                        : (wave < 5 ? Vs0 : wave < 7 ? Vs1 : Vs2) + ((wave - 3) & 1) * kOutStageBytes;
        static_assert(KBYTES >= kOutStageBytes && VBYTES >= 2 * kOutStageBytes, "staging areas of the output rows");
        const int wave_rows = min(32, sq.len - rw);
        if (wave_rows > 0) {
            store_out(a, stg, tok_offset(p, p.os, sq, wk.b, wk.h, rw), wave_rows, lane, n, hf, lt, o);
            if (rok && a.lse && hf == 0) a.lse[ri] = mref * p.sigma + __logf(lt);
        }
    }
}

int launch_engine_bf16_pp(const EngineArgs& ea, unsigned grid, hipStream_t st) {
    switch (ea.flags) {
#define AA_ENGINE_CASE(F) \
    case (F): return (int)launch_kernel(engine_bf16_pp_kernel<(F)>, dim3(grid), dim3(512), 0, st, ea);
    AA_ENGINE_CASE(kEngList | kEngLoadState | kEngStoreOut)           // stage 3 from the cached state
    AA_ENGINE_CASE(kEngAnchorRegion | kEngDense | kEngStoreOut)       // dense causal attention
#undef AA_ENGINE_CASE
    default:                                                          // any other mode: flags read at run time
        return (int)launch_kernel(engine_bf16_pp_kernel<-1>, dim3(grid), dim3(512), 0, st, ea);
    }
}

}  // namespace aa
