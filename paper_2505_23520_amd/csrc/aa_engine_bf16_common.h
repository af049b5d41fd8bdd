// Pieces shared by the two bf16 tile engines (engine_bf16_kernel: 128 query rows per work-group,
// engine_bf16_pp_kernel: 256): types, tile geometry in LDS, and everything a wave does to its own
// 32 query rows outside the tile loop -- Q fragment load, state load / store, the online-softmax
// update of one tile's scores (Algorithm 1 / 3 of arXiv 2505.23520: m' = max(m, max(qk)), p = exp,
// l' = l e^(m - m') + sum p), output store.  Fragment layout, both engines:
//   S^T = K Q^T with v_mfma_f32_32x32x16_bf16, keys = M dimension, query rows = N dimension: lane
//   (n, hf) = (lane % 32, lane / 32) owns query row n of the wave; score register v of a 32-key block
//   holds key 8 (v / 4) + 4 hf + v % 4; accumulator o[db][4 v4 + e] holds column 32 db + 8 v4 + 4 hf + e.
#pragma once
#include "aa_common.h"
#include "aa_engine.h"

namespace aa {
namespace eng {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef int intx4 __attribute__((ext_vector_type(4)));
typedef short shortx4 __attribute__((ext_vector_type(4)));
typedef short shortx8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr int D = 128;               // head dimension
constexpr int BQ = 128;              // query block
constexpr int TK = 64;               // keys per tile
// A direct-to-LDS load writes the 64 lanes' 16 bytes to consecutive addresses: 1 KB = four 256-byte
// rows per instruction ("group").  Key kk of a tile sits in group kk % 16, row kk / 16; groups are
// padded (K: 16 B, V: 64 B) so that the 16 lanes of an operand read fall into different banks.
constexpr int KGRP = 1024 + 16;
constexpr int VGRP = 1024 + 64;
constexpr int KBYTES = 16 * KGRP;
constexpr int VBYTES = 16 * VGRP;
constexpr float kRescaleLog2 = 8.f;  // raise the reference only for jumps above 2^8
constexpr floatx16 kZero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
constexpr int kOutPitch = 136;       // bf16 per row of the output staging area in LDS
constexpr int kOutStageBytes = 32 * kOutPitch * 2;   // one wave's 32 rows

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

// Q fragments (B operand of S^T = K Q^T): lane (n, hf) holds Q[row][16 ks + 8 hf .. +8); a row past
// the end of the sequence reads row `safe_row` and holds zeros.
__device__ __forceinline__ void load_q_fragments(bf16x8 (&qf)[8], const EngineArgs& a, const Seq& sq, int b, int h,
                                                 int r, bool rok, int safe_row, int hf) {
    const KParams& p = a.p;
    const __bf16* src = (const __bf16*)a.q + tok_offset(p, p.qs, sq, b, h, rok ? r : safe_row);
    const bf16x8 zero8 = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
        const bf16x8 x = *(const bf16x8*)(src + 16 * ks + 8 * hf);
        qf[ks] = rok ? x : zero8;
    }
}

// Running state of a lane's query row, raw dot-product units: reference mref of the exponentials,
// true maximum mtrue (the anchor that stage 1 exports), per-lane partial row sum l (the two halves
// of a row are added at the end), O^T accumulators.
// Start from the cached (M, L, Acc) of stage 1: ri = the row's index in M / L, tile = float offset
// of the wave's 32-row tile in Acc (fragment order, see acc_tile).
__device__ __forceinline__ void load_state(const EngineArgs& a, long long ri, long long tile, int lane, int hf,
                                           float& mref, float& mtrue, float& l, floatx16 (&o)[4]) {
    mref = a.Min[ri] / a.p.sigma;
    mtrue = mref;
    l = hf == 0 ? a.Lin[ri] : 0.f;
    const float* acc = a.Accin + tile;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            const floatx4 x = *(const floatx4*)(acc + (4 * db + v4) * 256 + 4 * lane);
            o[db][4 * v4 + 0] = x.x; o[db][4 * v4 + 1] = x.y;
            o[db][4 * v4 + 2] = x.z; o[db][4 * v4 + 3] = x.w;
        }
}
__device__ __forceinline__ void init_state(float& mref, float& mtrue, float& l, floatx16 (&o)[4]) {
    mref = -INFINITY; mtrue = -INFINITY; l = 0.f;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v = 0; v < 16; ++v) o[db][v] = 0.f;
}

// Online softmax of one tile for this lane's query row (the other half of the row's keys is 32
// lanes away).  s: the tile's scores, hidden pairs already at -inf.  The reference is raised only
// when some row's maximum exceeds it by more than 2^8 (wave-uniform branch, rare after the first
// tiles); the accumulators are then rescaled, otherwise untouched.  pf: probabilities as bf16, the
// B operand of O^T += V^T P^T.
__device__ __forceinline__ void softmax_tile(const floatx16 (&s)[2], bf16x8 (&pf)[2][2], float c2, float rescale_gap,
                                             float& mref, float& mtrue, float& l, floatx16 (&o)[4]) {
    float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
    for (int v = 1; v < 16; ++v) mx = fmaxf(fmaxf(mx, s[0][v]), s[1][v]);     // v_max3_f32
    {
        float u, w;
        both_halves(mx, u, w);
        mx = fmaxf(u, w);
    }
    mtrue = fmaxf(mtrue, mx);
    if (__builtin_expect(__any(mx > mref + rescale_gap), 0)) {
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
    l += rs;
}

// The same for the modes that do not export the true row maximum (stage 3, dense attention): the
// maximum is only looked for when it is needed.  The probabilities are computed against the
// current reference straight away; only if some lane's partial row sum shows a probability above
// 2^8 (or infinite), or some row has no reference yet (the first tiles), the wave
// finds the row maxima, raises the references, rescales the accumulators and computes the tile's
// probabilities again (wave-uniform branch, rare after the first tiles).
__device__ __forceinline__ void softmax_tile_lazy(const floatx16 (&s)[2], bf16x8 (&pf)[2][2], float c2, float& mref,
                                                  float& l, floatx16 (&o)[4]) {
    float mc = (mref == -INFINITY) ? 0.f : mref * c2;
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
    if (__builtin_expect(__any(rs > 256.f || mref == -INFINITY), 0)) {
        float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(fmaxf(mx, s[0][v]), s[1][v]);
        {
            float u, w;
            both_halves(mx, u, w);
            mx = fmaxf(u, w);
        }
        const float mnew = fmaxf(mref, mx);
        const float alpha = (mnew == -INFINITY || mref == mnew) ? 1.f : __builtin_amdgcn_exp2f((mref - mnew) * c2);
        mref = mnew;
        l *= alpha;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) o[db][v] *= alpha;
        mc = (mref == -INFINITY) ? 0.f : mref * c2;
        rs = 0.f;
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
    }
    l += rs;
}

// Row sum of the whole row (both halves), relative to mref.
__device__ __forceinline__ float row_sum(float l) {
    float u, w;
    both_halves(l, u, w);
    return u + w;
}

// Stage 1's exports for this lane's row, relative to the true maximum (Algorithm 1's m, l, acc):
// M and L at ri, the wave's Acc tile in fragment order (every store instruction writes 1 KB of
// consecutive addresses; stage 3 reads the tile back the same way).  Returns M in scaled-logit units.
__device__ __forceinline__ float store_state(const EngineArgs& a, long long ri, long long tile, bool rok,
                                             bool wave_has_rows, int lane, int hf, float c2, float mref, float mtrue,
                                             float lt, const floatx16 (&o)[4]) {
    const float down = (mref == -INFINITY) ? 1.f : __builtin_amdgcn_exp2f((mref - mtrue) * c2);
    const float ms = mtrue * a.p.sigma;
    if (rok && hf == 0) { a.Mout[ri] = ms; a.Lout[ri] = lt * down; }
    if (a.Accout && wave_has_rows) {
        float* acc = a.Accout + tile;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4)
                *(floatx4*)(acc + (4 * db + v4) * 256 + 4 * lane) =
                    floatx4{o[db][4 * v4] * down, o[db][4 * v4 + 1] * down, o[db][4 * v4 + 2] * down,
                            o[db][4 * v4 + 3] * down};
    }
    return ms;
}

// out = acc / l for the wave's 32 rows (wave_rows of them exist), through a private staging area of
// kOutStageBytes in LDS so that 16 lanes write one 256-byte row together instead of every lane
// writing 8-byte pieces of its own row.  LDS operations of one wave execute in order, so no barrier
// separates its writes from its reads; out_row0 = element offset of the wave's first row.
__device__ __forceinline__ void store_out(const EngineArgs& a, char* stg, long long out_row0, int wave_rows, int lane,
                                          int n, int hf, float lt, const floatx16 (&o)[4]) {
    const float inv = 1.f / lt;
    unsigned short* sb = (unsigned short*)stg;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            const floatx4 x = {o[db][4 * v4] * inv, o[db][4 * v4 + 1] * inv, o[db][4 * v4 + 2] * inv,
                               o[db][4 * v4 + 3] * inv};
            *(bf16x4*)(sb + n * kOutPitch + 32 * db + 8 * v4 + 4 * hf) = __builtin_convertvector(x, bf16x4);
        }
    const long long ostride = a.p.os[2];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int f = 64 * i + lane, row = f >> 4, c = f & 15;
        const intx4 x = *(const intx4*)(sb + row * kOutPitch + 8 * c);
        if (row < wave_rows) *(intx4*)((unsigned short*)a.out + out_row0 + row * ostride + 8 * c) = x;
    }
}

}  // namespace eng
}  // namespace aa
