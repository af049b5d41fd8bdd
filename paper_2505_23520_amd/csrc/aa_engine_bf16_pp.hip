// bf16 tile engine, ping-pong variant: the same computation as engine_bf16_kernel (stage 1,
// stage 3 and the dense comparator of arXiv 2505.23520; see that file for the fragment and LDS
// layouts, which are identical), organised so that the matrix pipe and the vector ALU of a SIMD
// are busy at the same time by construction instead of by chance:
//   work-group = two consecutive query blocks of one head = 8 waves x 32 query rows, one
//   work-group per CU.  Waves w and w + 4 share a SIMD; waves 0-3 form group A, waves 4-7
//   group B.  Time is cut into slots by work-group barriers.  In every slot one group runs its
//   MFMA phase (O^T += V^T P^T of tile t, then S^T = K Q^T of tile t + 1: 32 MFMAs) while the
//   other runs its softmax phase (row max, exp2, row sum, bf16 conversion of tile t on the
//   vector ALU, and the 32 transposing LDS reads that fetch the tile's V^T operands into
//   registers); then they swap.  Group B runs one slot behind group A.
//   K/V tiles are triple-buffered in LDS and shared by the 256 rows.  Group A's waves issue the
//   direct-to-LDS loads of the K tiles, group B's those of the V tiles, three tiles ahead, at the
//   start of an MFMA phase, and wait for them at the start of their next MFMA phase (two slots
//   later).
// The two query blocks must share their window start and their selected-column list: the host
// launches this kernel for dense attention and for even `step`, the 128-row kernel otherwise.
#include "aa_common.h"
#include "aa_engine.h"

namespace aa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void lds_void;

namespace {

constexpr int D = 128;
constexpr int BQ = 128;
constexpr int PAIR = 2 * BQ;         // query rows per work-group
constexpr int TK = 64;               // keys per tile
constexpr int KGRP = 1024 + 16;      // bytes per K group: 4 rows + pad
constexpr int VGRP = 1024 + 64;      // bytes per V group
constexpr int KBYTES = 16 * KGRP;
constexpr int VBYTES = 16 * VGRP;
constexpr float kRescaleLog2 = 8.f;  // raise the reference only for jumps above 2^8
constexpr floatx16 kZero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

// s_waitcnt vmcnt(0) only (gfx9 encoding: expcnt and lgkmcnt fields left at their maxima)
__device__ __forceinline__ void wait_vmem() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// x of this lane and x of the lane 32 away, in an order that depends on the half (fine for
// max and sum); v_permlane32_swap is a plain VALU operation, no trip through the LDS crossbar
__device__ __forceinline__ void both_halves(float x, float& u, float& v) {
    const unsigned b = __float_as_uint(x);
    const auto r = __builtin_amdgcn_permlane32_swap(b, b, false, false);
    u = __uint_as_float(r[0]);
    v = __uint_as_float(r[1]);
}

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

__global__ __launch_bounds__(512, 1) void engine_bf16_pp_kernel(EngineArgs a) {
    __shared__ __attribute__((aligned(16))) char Ks0[KBYTES], Ks1[KBYTES], Ks2[KBYTES];
    __shared__ __attribute__((aligned(16))) char Vs0[VBYTES], Vs1[VBYTES], Vs2[VBYTES];
    __shared__ float red[8];
    const KParams& p = a.p;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: keep it scalar
    const int n = lane & 31, hf = lane >> 5;
    const int grpB = wave >> 2;                      // 0: group A, 1: group B
    const int simd = wave & 3;
    const int chunk = 2 * simd + grpB;               // the wave's 32 rows inside the pair

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
    if (a.flags & kEngAnchorRegion) {
        if (!(a.flags & kEngDense)) { W = window_start(p, g); ninit = p.n_init; }
        const int e1 = min(ninit, rlast + 1);
        T1 = (e1 + TK - 1) / TK;
        t2s = max(T1, W / TK);
        const int T2 = rlast / TK + 1;
        nA = T1 + max(0, T2 - t2s);
    }
    int cnt = 0;
    long long lbase = 0;
    if (a.flags & kEngList) {
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
        char* dst = (grpB ? Vb : Kb) + 4 * simd * lgrp;
        if (t < nA) {
            const int t0 = tile_start(t) + kq0;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(lrs, (lds_void*)(dst + j * lgrp), 16,
                                                         (int)((unsigned)min(t0 + j, sq.len - 1) * lstb + 16u * lch),
                                                         0, 0, 0);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(lrs, (lds_void*)(dst + j * lgrp), 16,
                                                         (int)((unsigned)kidx[j] * lstb + 16u * lch), 0, 0, 0);
        }
    };

    // ---- Q fragments (B operand of S^T = K Q^T): lane (n, hf) holds Q[row][16 ks + 8 hf .. +8)
    bf16x8 qf[8];
    {
        const __bf16* src = (const __bf16*)a.q + tok_offset(p, p.qs, sq, wk.b, wk.h, rok ? r : 0);
        const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 x = *(const bf16x8*)(src + 16 * ks + 8 * hf);
            qf[ks] = rok ? x : zero8;
        }
    }

    // ---- running state, raw dot-product units (see engine_bf16_kernel)
    const float c2 = p.sigma * 1.4426950408889634f;  // exp(sigma*x) = exp2(c2*x)
    const float rescale_gap = kRescaleLog2 / c2;
    const long long ri = row_index(p, sq, wk.b, wk.h, rok ? r : row0);
    float mref, mtrue, l;
    floatx16 o[4];
    if (a.flags & kEngLoadState) {
        mref = a.Min[ri] / p.sigma;
        mtrue = mref;
        l = hf == 0 ? a.Lin[ri] : 0.f;
        const float* acc = a.Accin + ri * D;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const floatx4 x = *(const floatx4*)(acc + 32 * db + 8 * v4 + 4 * hf);
                o[db][4 * v4 + 0] = x.x; o[db][4 * v4 + 1] = x.y;
                o[db][4 * v4 + 2] = x.z; o[db][4 * v4 + 3] = x.w;
            }
    } else {
        mref = -INFINITY; mtrue = -INFINITY; l = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
    }

    // operand addresses inside a stage (bytes): K row of key 32 kb + n; V chunk read by this lane
    // in the transposing load (lane 16 G + s: key offset s / 4, 8-byte piece s % 4 of d-half G % 2)
    const int koff = (n & 15) * KGRP + (n >> 4) * 256 + 16 * hf;
    const int ls = lane & 15, lg = lane >> 4;
    const int voff = (4 * hf + (ls >> 2)) * VGRP + 32 * (lg & 1) + 8 * (ls & 3);

    // a contiguous tile that starts beyond this wave's last row is hidden from all its rows (the
    // work-group still needs it for later rows): the wave computes nothing for it
    auto tile_on = [&](int t) -> bool { return wave_on && t < nT && !(t < nA && tile_start(t) > rw + 31); };

    floatx16 s[2];      // scores of the tile between its QK and its softmax phase
    bf16x8 pf[2][2];    // probabilities of the tile between its softmax and its PV phase
    shortx8 vf[16];     // V^T operands of the tile, fetched during its softmax phase
    bf16x8 kpre[2];     // first K operands of the next tile, fetched ahead of the PV MFMAs

    // S^T = K Q^T : s[kb], 32 keys x 32 rows each.  Masks (tiles that touch a region boundary, the
    // diagonal or a list tail) enter as the initial accumulator: 0 for a visible (key, row) pair,
    // -inf otherwise; the common unmasked tile starts from literal 0.
    auto qk_prefetch = [&](int t, const char* Kcur) {
        if (!tile_on(t)) return;
        const char* Kb = Kcur + koff;
#pragma unroll
        for (int i = 0; i < 2; ++i) kpre[i] = *(const bf16x8*)(Kb + 512 * i);
    };
    auto qk = [&](int t, const char* Kcur) {
        if (!tile_on(t)) return;
        const char* Kb = Kcur + koff;
        int mode = 0, t0 = 0;
        if (t < nA) {
            t0 = tile_start(t);
            const bool interior = (t0 + TK - 1 <= rw) && (t0 + TK <= ninit || t0 >= W);
            mode = interior ? 0 : 1;
        } else if (t == nT - 1 && (cnt & (TK - 1))) {
            mode = 2;
        }
        if (mode == 0) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kpre[kb], qf[0], kZero16, 0, 0, 0);
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
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kpre[kb], qf[0], bias, 0, 0, 0);
            }
        }
#pragma unroll
        for (int ks = 1; ks < 8; ++ks)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const bf16x8 kf = *(const bf16x8*)(Kb + 512 * kb + 32 * ks);
                s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[kb], 0, 0, 0);
            }
        // the remaining LDS operand reads run ahead of their MFMAs: six are issued up front (the
        // two MFMAs on the prefetched operands cover part of their latency), then one per MFMA
        // (left alone, the compiler issues each read right before its MFMA)
        __builtin_amdgcn_sched_group_barrier(0x100, 6, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 6, 0);
    };

    // online softmax of this lane's query row (the other half of the row is 32 lanes away)
    auto softmax = [&](int t, const char* Vcur) {
        if (!tile_on(t)) return;
        float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(fmaxf(mx, s[0][v]), s[1][v]);     // v_max3_f32
        {
            float u, w;
            both_halves(mx, u, w);
            mx = fmaxf(u, w);
        }
        mtrue = fmaxf(mtrue, mx);
        if (__any(mx > mref + rescale_gap)) {                 // rare after the first tiles
            const float mnew = fmaxf(mref, mx);
            const float alpha = (mnew == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f((mref - mnew) * c2);
            mref = mnew;
            l *= alpha;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
        }
        const float mc = (mref == -INFINITY) ? 0.f : mref * c2;
        // V^T operands of this tile for the coming MFMA phase.  A wave gets one transposing LDS read
        // through about every 24 cycles, so the 32 reads of a tile cost more than its 16 PV MFMAs;
        // issued here, spread between the exponentials, they cost nothing.
        // keys 16 sg + 8 rd + 4 hf + (0..3) live in groups 8 rd + 4 hf + (0..3), row sg
        {
            const char* Vb = Vcur + voff;
#pragma unroll
            for (int sg = 0; sg < 4; ++sg)
#pragma unroll
                for (int db = 0; db < 4; ++db) {
                    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) shortx4*)(Vb + sg * 256 + 64 * db));
                    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                        (__attribute__((address_space(3))) shortx4*)(Vb + 8 * VGRP + sg * 256 + 64 * db));
                    vf[4 * sg + db] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                }
        }
        float rs = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int h8 = 0; h8 < 2; ++h8) {
                floatx8 pv;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    pv[e] = __builtin_amdgcn_exp2f(fmaf(s[kb][8 * h8 + e], c2, -mc));
                    rs += pv[e];
                }
                pf[kb][h8] = __builtin_convertvector(pv, bf16x8);
            }
#pragma unroll
        for (int i = 0; i < 32; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x002, 3, 0);
        }
        l += rs;
    };

    // O^T += V^T P^T
    auto pv = [&](int t) {
        if (!tile_on(t)) return;
#pragma unroll
        for (int sg = 0; sg < 4; ++sg)
#pragma unroll
            for (int db = 0; db < 4; ++db)
                o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf[4 * sg + db]),
                                                                 pf[sg >> 1][sg & 1], o[db], 0, 0, 0);
    };

    // ---- prologue: tiles 0..2 (K by group A, V by group B), then the slot offset of group B
    if (nT > 0) {
        idx_prefetch(0);
        tile_load(0, Ks0, Vs0);
        if (nT > 1) {
            idx_prefetch(1);
            tile_load(1, Ks1, Vs1);
        }
        if (nT > 2) {
            idx_prefetch(2);
            tile_load(2, Ks2, Vs2);
        }
        idx_prefetch(3);
    }
    wait_vmem();
    slot_barrier();
    if (!grpB) { qk_prefetch(0, Ks0); qk(0, Ks0); }
    slot_barrier();
    if (grpB) {
        qk_prefetch(0, Ks0);
        qk(0, Ks0);
        slot_barrier();
    }

    // one tile: softmax phase (which also fetches the tile's V operands), then MFMA phase.  The MFMA
    // phase starts by awaiting the loads this wave issued at the start of its previous MFMA phase
    // (they are published by the barrier that ends this phase) and issuing those of tile t + 3 into
    // the stage tile t has left: its K was last read a slot ago, its V in the softmax phases.
    auto tile_iter = [&](int t, char* Kcur, char* Vcur, const char* Knext) {
        softmax(t, Vcur);
        slot_barrier();
        wait_vmem();
        if (t + 3 < nT) {
            tile_load(t + 3, Kcur, Vcur);
            idx_prefetch(t + 4);
        }
        qk_prefetch(t + 1, Knext);
        pv(t);
        qk(t + 1, Knext);
        slot_barrier();
    };
    // whole rounds of three tiles (one per LDS stage); tiles past the end only keep the barriers
    for (int t = 0; t < nT; t += 3) {
        tile_iter(t, Ks0, Vs0, Ks1);
        tile_iter(t + 1, Ks1, Vs1, Ks2);
        tile_iter(t + 2, Ks2, Vs2, Ks0);
    }
    if (!grpB) slot_barrier();

    // ---- epilogue
    float lt;                                        // row sum relative to mref
    {
        float u, w;
        both_halves(l, u, w);
        lt = u + w;
    }
    if (a.flags & kEngStoreState) {
        // exported state is relative to the true maximum (Algorithm 1's m, l, acc)
        const float down = (mref == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f((mref - mtrue) * c2);
        const float ms = mtrue * p.sigma;
        if (rok && hf == 0) { a.Mout[ri] = ms; a.Lout[ri] = lt * down; }
        if (rok && a.Accout) {
            float* acc = a.Accout + ri * D;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4)
                    *(floatx4*)(acc + 32 * db + 8 * v4 + 4 * hf) =
                        floatx4{o[db][4 * v4] * down, o[db][4 * v4 + 1] * down, o[db][4 * v4 + 2] * down,
                                o[db][4 * v4 + 3] * down};
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
    if ((a.flags & kEngStoreOut) && rok) {
        const float inv = 1.f / lt;
        unsigned short* dst = (unsigned short*)a.out + tok_offset(p, p.os, sq, wk.b, wk.h, r);
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                const floatx4 x = {o[db][4 * v4] * inv, o[db][4 * v4 + 1] * inv, o[db][4 * v4 + 2] * inv,
                                   o[db][4 * v4 + 3] * inv};
                *(bf16x4*)(dst + 32 * db + 8 * v4 + 4 * hf) = __builtin_convertvector(x, bf16x4);
            }
        if (a.lse && hf == 0) a.lse[ri] = mref * p.sigma + __logf(lt);
    }
}

}  // namespace aa
