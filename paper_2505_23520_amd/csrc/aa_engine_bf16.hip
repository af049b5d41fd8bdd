// bf16 tile engine: one online-softmax (flash-style) kernel that serves
//   * stage 1, anchor computation          (Sec. 3.1 Eq. 1, Algorithm 1),
//   * stage 3, gathered sparse attention   (Sec. 3.3 Eq. 3-5, Algorithm 3),
//   * the dense causal comparator
// of arXiv 2505.23520 on gfx950.  The three differ only in which K/V rows feed
// the tiles (a contiguous masked range or the rows a selected-column list names)
// and in what is read before / written after the loop.
//
// Shape of the computation (d = 128, b_q = 128, bf16 in, fp32 accumulate):
//   work-group = one query block = 2 waves x 64 query rows;
//   K/V tile   = 64 keys, double-buffered in LDS;
//   S^T = K Q^T  with v_mfma_f32_32x32x16_bf16 (keys are the M dimension, query
//   rows the N dimension, so one lane owns one query row and the row max / sum
//   are in-lane reductions plus one exchange between the wave's halves);
//   O^T = V^T P^T with the same instruction; V is transposed on its way into LDS
//   so that both operands are read with 16-byte LDS loads.
#include "aa_common.h"
#include "aa_engine.h"

namespace aa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

namespace {

constexpr int D = 128;
constexpr int BQ = 128;
constexpr int TK = 64;               // keys per tile
constexpr int KSTR = D + 8;          // K tile row stride (elements): 272 B, conflict-free 16 B reads
constexpr int VSTR = TK + 8;         // V^T tile row stride (elements): 144 B
constexpr int KELEMS = TK * KSTR;
constexpr int VELEMS = D * VSTR;
constexpr int BUF = KELEMS + VELEMS; // one stage, in 2-byte elements

union Frag8 {
    bf16x8 v;
    bf16x2 h[4];
    uint4 u;
};

__device__ __forceinline__ float xhalf(float x) {  // value held by the lane 32 away
    return __shfl_xor(x, 32, 64);
}

}  // namespace

__global__ __launch_bounds__(128) void engine_bf16_kernel(EngineArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned short smem[];
    const KParams& p = a.p;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n = lane & 31, hf = lane >> 5;

    const Work wk = decode_work(p, p.nblk_max, blockIdx.x);
    const Seq sq = seq_of(p, wk.b);
    const int row0 = wk.i * BQ;
    if (row0 >= sq.len) return;
    const int hk = wk.h / p.grp;
    const int g = wk.i / p.step;
    const int rw = row0 + 64 * wave;                 // first row of this wave
    const int rlast = min(row0 + BQ, sq.len) - 1;    // last row of the block

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

    const __bf16* qb = (const __bf16*)a.q;
    const unsigned short* kb_ = (const unsigned short*)a.k + tok_offset(p, p.ks, sq, wk.b, hk, 0);
    const unsigned short* vb_ = (const unsigned short*)a.v + tok_offset(p, p.vs, sq, wk.b, hk, 0);
    const long long kst = p.ks[2], vst = p.vs[2];

    // ---- loader role of this thread: 16-byte column chunk c of 8 keys
    const int lc = tid & 15, ksid = tid >> 4;        // ksid = 2*sg + hh
    int koff[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) koff[e] = 16 * (ksid >> 1) + 4 * (ksid & 1) + (e & 3) + 8 * (e >> 2);

    auto tile_start = [&](int t) -> int {            // first key of contiguous tile t (t < nA)
        return TK * (t < T1 ? t : t2s + (t - T1));
    };
    auto tile_keys = [&](int t, int* key) {
        if (t < nA) {
            const int t0 = tile_start(t);
#pragma unroll
            for (int e = 0; e < 8; ++e) key[e] = min(t0 + koff[e], sq.len - 1);
        } else {
            const int* src = a.idx + lbase + (long long)(t - nA) * TK + koff[0];
            const int4 x = *(const int4*)src;
            const int4 y = *(const int4*)(src + 8);
            key[0] = x.x; key[1] = x.y; key[2] = x.z; key[3] = x.w;
            key[4] = y.x; key[5] = y.y; key[6] = y.z; key[7] = y.w;
        }
    };
    uint4 kreg[8], vreg[8];
    auto tile_load = [&](const int* key) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            kreg[e] = *(const uint4*)(kb_ + (long long)key[e] * kst + 8 * lc);
            vreg[e] = *(const uint4*)(vb_ + (long long)key[e] * vst + 8 * lc);
        }
    };
    auto tile_store = [&](int buf) {
        unsigned short* Ks = smem + buf * BUF;
        unsigned short* Vt = Ks + KELEMS;
#pragma unroll
        for (int e = 0; e < 8; ++e) *(uint4*)(Ks + koff[e] * KSTR + 8 * lc) = kreg[e];
        // transpose the 8 keys x 8 columns held by this thread: one 16 B row of V^T per column
        const unsigned* vr = (const unsigned*)vreg;  // vr[4*e + a] = columns (2a, 2a+1) of key e
#pragma unroll
        for (int a2 = 0; a2 < 4; ++a2) {
            uint4 lo, hi;
            unsigned* plo = (unsigned*)&lo;
            unsigned* phi = (unsigned*)&hi;
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                const unsigned x = vr[4 * (2 * e2) + a2], y = vr[4 * (2 * e2 + 1) + a2];
                plo[e2] = (x & 0xffffu) | (y << 16);
                phi[e2] = (x >> 16) | (y & 0xffff0000u);
            }
            *(uint4*)(Vt + (8 * lc + 2 * a2) * VSTR + 8 * ksid) = lo;
            *(uint4*)(Vt + (8 * lc + 2 * a2 + 1) * VSTR + 8 * ksid) = hi;
        }
    };

    // ---- Q fragments (B operand of S^T = K Q^T): lane (n, hf) holds Q[row][16 ks + 8 hf .. +8)
    Frag8 qf[2][8];
#pragma unroll
    for (int qa = 0; qa < 2; ++qa) {
        const int r = rw + 32 * qa + n;
        const bool ok = r < sq.len;
        const __bf16* src = qb + tok_offset(p, p.qs, sq, wk.b, wk.h, ok ? r : 0);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            uint4 x = *(const uint4*)(src + 16 * ks + 8 * hf);
            if (!ok) x = make_uint4(0, 0, 0, 0);
            qf[qa][ks].u = x;
        }
    }

    // ---- running state: m in raw dot-product units, l per lane (the two halves of a
    // row are added at the end), O^T accumulators
    const float c2 = p.sigma * 1.4426950408889634f;  // exp(sigma*x) = exp2(c2*x)
    float m[2], l[2];
    floatx16 o[4][2];
    if (a.flags & kEngLoadState) {
#pragma unroll
        for (int qa = 0; qa < 2; ++qa) {
            const int r = rw + 32 * qa + n;
            const bool ok = r < sq.len;
            const long long ri = row_index(p, sq, wk.b, wk.h, ok ? r : row0);
            m[qa] = a.Min[ri] / p.sigma;
            l[qa] = hf == 0 ? a.Lin[ri] : 0.f;
            const float* acc = a.Accin + ri * D;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    const float4 x = *(const float4*)(acc + 32 * db + 8 * v4 + 4 * hf);
                    o[db][qa][4 * v4 + 0] = x.x; o[db][qa][4 * v4 + 1] = x.y;
                    o[db][qa][4 * v4 + 2] = x.z; o[db][qa][4 * v4 + 3] = x.w;
                }
        }
    } else {
#pragma unroll
        for (int qa = 0; qa < 2; ++qa) {
            m[qa] = -INFINITY; l[qa] = 0.f;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][qa][v] = 0.f;
        }
    }

    // ---- pipeline prologue
    int keys[8];
    if (nT > 0) {
        tile_keys(0, keys);
        tile_load(keys);
        if (nT > 1) tile_keys(1, keys);
        tile_store(0);
    }
    __syncthreads();

    for (int t = 0; t < nT; ++t) {
        if (t + 1 < nT) {
            tile_load(keys);
            if (t + 2 < nT) tile_keys(t + 2, keys);
        }
        const unsigned short* Ks = smem + (t & 1) * BUF;
        const unsigned short* Vt = Ks + KELEMS;

        // S^T = K Q^T : s[kb][qa], 32 keys x 32 rows each
        floatx16 s[2][2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int qa = 0; qa < 2; ++qa)
#pragma unroll
                for (int v = 0; v < 16; ++v) s[kb][qa][v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const bf16x8 kf = *(const bf16x8*)(Ks + (32 * kb + n) * KSTR + 16 * ks + 8 * hf);
#pragma unroll
                for (int qa = 0; qa < 2; ++qa)
                    s[kb][qa] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qa][ks].v, s[kb][qa], 0, 0, 0);
            }

        // masks: only tiles that touch a region boundary, the diagonal or a list tail
        if (t < nA) {
            const int t0 = tile_start(t);
            const bool interior = (t0 + TK - 1 <= rw) && (t0 + TK <= ninit || t0 >= W);
            if (!interior) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int qa = 0; qa < 2; ++qa) {
                        const int r = rw + 32 * qa + n;
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int j = t0 + 32 * kb + 8 * (v >> 2) + 4 * hf + (v & 3);
                            const bool ok = (j <= r) && (j < ninit || j >= W);
                            if (!ok) s[kb][qa][v] = -INFINITY;
                        }
                    }
            }
        } else if (t == nT - 1 && (cnt & (TK - 1))) {
            const int rem = cnt - (t - nA) * TK;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qa = 0; qa < 2; ++qa)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int pos = 32 * kb + 8 * (v >> 2) + 4 * hf + (v & 3);
                        if (pos >= rem) s[kb][qa][v] = -INFINITY;
                    }
        }

        // online softmax per query row (one lane pair per row)
        Frag8 pf[2][2][2];  // [kb][s16][qa]
#pragma unroll
        for (int qa = 0; qa < 2; ++qa) {
            float mx = s[0][qa][0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[0][qa][v]);
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[1][qa][v]);
            mx = fmaxf(mx, xhalf(mx));
            const float mnew = fmaxf(m[qa], mx);
            const float muse = (mnew == -INFINITY) ? 0.f : mnew;
            const float alpha = __builtin_amdgcn_exp2f((m[qa] - muse) * c2);
            const float mc = muse * c2;
            m[qa] = mnew;
            float rs = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int v = 0; v < 16; v += 2) {
                    const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kb][qa][v], c2, -mc));
                    const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kb][qa][v + 1], c2, -mc));
                    rs += p0 + p1;
                    floatx2 pp = {p0, p1};
                    pf[kb][v >> 3][qa].h[(v & 7) >> 1] = __builtin_convertvector(pp, bf16x2);
                }
            l[qa] = l[qa] * alpha + rs;
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) o[db][qa][v] *= alpha;
        }

        // O^T += V^T P^T
#pragma unroll
        for (int sg = 0; sg < 4; ++sg)
#pragma unroll
            for (int db = 0; db < 4; ++db) {
                const bf16x8 vf = *(const bf16x8*)(Vt + (32 * db + n) * VSTR + 16 * sg + 8 * hf);
#pragma unroll
                for (int qa = 0; qa < 2; ++qa)
                    o[db][qa] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[sg >> 1][sg & 1][qa].v,
                                                                         o[db][qa], 0, 0, 0);
            }

        if (t + 1 < nT) tile_store((t + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue
    float red_m = 0.f;  // sum of this wave's anchors over valid rows (for the pooled anchor)
#pragma unroll
    for (int qa = 0; qa < 2; ++qa) {
        const int r = rw + 32 * qa + n;
        const bool ok = r < sq.len;
        const float lt = l[qa] + xhalf(l[qa]);
        const float ms = m[qa] * p.sigma;
        const long long ri = row_index(p, sq, wk.b, wk.h, ok ? r : row0);
        if (a.flags & kEngStoreState) {
            if (ok && hf == 0) { a.Mout[ri] = ms; a.Lout[ri] = lt; red_m += ms; }
            if (ok && a.Accout) {
                float* acc = a.Accout + ri * D;
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int v4 = 0; v4 < 4; ++v4)
                        *(float4*)(acc + 32 * db + 8 * v4 + 4 * hf) =
                            make_float4(o[db][qa][4 * v4], o[db][qa][4 * v4 + 1], o[db][qa][4 * v4 + 2],
                                        o[db][qa][4 * v4 + 3]);
            }
        }
        if (a.flags & kEngStoreOut) {
            const float inv = 1.f / lt;
            if (ok) {
                unsigned short* dst = (unsigned short*)a.out + tok_offset(p, p.os, sq, wk.b, wk.h, r);
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int v4 = 0; v4 < 4; ++v4) {
                        floatx2 x0 = {o[db][qa][4 * v4] * inv, o[db][qa][4 * v4 + 1] * inv};
                        floatx2 x1 = {o[db][qa][4 * v4 + 2] * inv, o[db][qa][4 * v4 + 3] * inv};
                        union { bf16x2 h[2]; uint2 u; } pk;
                        pk.h[0] = __builtin_convertvector(x0, bf16x2);
                        pk.h[1] = __builtin_convertvector(x1, bf16x2);
                        *(uint2*)(dst + 32 * db + 8 * v4 + 4 * hf) = pk.u;
                    }
                if (a.lse && hf == 0) a.lse[ri] = ms + __logf(lt);
            }
        }
    }
    if ((a.flags & kEngStoreState) && a.xa) {
        // pooled anchor of the block: mean of M over its rows (Algorithm 2, avgpool of the anchor)
        float* red = (float*)smem;                   // all tile reads are behind the last barrier
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) red_m += __shfl_xor(red_m, off, 64);
        if (lane == 0) red[wave] = red_m;
        __syncthreads();
        if (tid == 0) {
            const int nrows = rlast - row0 + 1;
            a.xa[blk_index(p, sq, wk.b, wk.h, wk.i)] = (red[0] + red[1]) / (float)nrows;
        }
    }
}

size_t engine_bf16_lds_bytes() { return 2 * BUF * sizeof(unsigned short); }

}  // namespace aa
