// fp32 tile engine: the same online-softmax walk as the bf16 engine (stage 1
// anchor computation, Algorithm 1; stage 3 gathered sparse attention, Algorithm 3;
// dense causal comparator -- arXiv 2505.23520) with fp32 inputs, fp32 products and
// fp32 probabilities.  On gfx950 the fp32 matrix and vector pipes have the same
// peak rate, so this instantiation uses plain vector FMAs over LDS tiles: two
// lanes share one query row, each owning half of the head dimension.
#include "aa_common.h"
#include "aa_engine.h"

namespace aa {

namespace {
constexpr int TK = 64;  // keys per tile (one list chunk)

template <int DH>  // DH = d / 2
__device__ __forceinline__ void engine_fp32_body(const EngineArgs& a, float* smem) {
    constexpr int Dd = 2 * DH;
    constexpr int STR = Dd + 4;                      // padded row stride of the K and V tiles
    const KParams& p = a.p;
    const int tid = threadIdx.x;
    const int lr = tid >> 1, hh = tid & 1;
    const int BQ = p.bq;

    if (!engine_selected(a)) return;
    const Work wk = decode_work(p, p.nblk_max, blockIdx.x);
    const Seq sq = seq_of(p, wk.b);
    const int row0 = wk.i * BQ;
    if (row0 >= sq.len) return;
    const int hk = wk.h / p.grp;
    const int g = wk.i / p.step;
    const int rlast = min(row0 + BQ, sq.len) - 1;
    const int r = row0 + lr;
    const bool rok = r < sq.len;

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

    const float* kb_ = (const float*)a.k + tok_offset(p, p.ks, sq, wk.b, hk, 0);
    const float* vb_ = (const float*)a.v + tok_offset(p, p.vs, sq, wk.b, hk, 0);
    float* Ks = smem;
    float* Vs = smem + TK * STR;

    float q[DH], acc[DH];
    {
        const float* src = (const float*)a.q + tok_offset(p, p.qs, sq, wk.b, wk.h, rok ? r : row0) + hh * DH;
#pragma unroll
        for (int c = 0; c < DH; c += 4) {
            const float4 x = *(const float4*)(src + c);
            q[c] = x.x; q[c + 1] = x.y; q[c + 2] = x.z; q[c + 3] = x.w;
        }
    }
    const float c2 = p.sigma * 1.4426950408889634f;
    float m, l;
    const long long ri = row_index(p, sq, wk.b, wk.h, rok ? r : row0);
    if (a.flags & kEngLoadState) {
        m = a.Min[ri] / p.sigma;
        l = a.Lin[ri];
        const float* src = a.Accin + ri * Dd + hh * DH;
#pragma unroll
        for (int c = 0; c < DH; c += 4) {
            const float4 x = *(const float4*)(src + c);
            acc[c] = x.x; acc[c + 1] = x.y; acc[c + 2] = x.z; acc[c + 3] = x.w;
        }
    } else {
        m = -INFINITY; l = 0.f;
#pragma unroll
        for (int c = 0; c < DH; ++c) acc[c] = 0.f;
    }

    for (int t = 0; t < nT; ++t) {
        const bool contiguous = t < nA;
        const int t0 = contiguous ? TK * (t < T1 ? t : t2s + (t - T1)) : 0;
        __syncthreads();                             // previous tile fully consumed
        for (int e = tid; e < TK * (Dd / 4); e += blockDim.x) {
            const int kk = e / (Dd / 4), c4 = e % (Dd / 4);
            const int key = contiguous ? min(t0 + kk, sq.len - 1) : a.idx[lbase + (long long)(t - nA) * TK + kk];
            *(float4*)(Ks + kk * STR + 4 * c4) = *(const float4*)(kb_ + (long long)key * p.ks[2] + 4 * c4);
            *(float4*)(Vs + kk * STR + 4 * c4) = *(const float4*)(vb_ + (long long)key * p.vs[2] + 4 * c4);
        }
        __syncthreads();

        float s[TK];
#pragma unroll
        for (int jj = 0; jj < TK; ++jj) {
            const float* kr = Ks + jj * STR + hh * DH;
            float d0 = 0.f;
#pragma unroll
            for (int c = 0; c < DH; c += 4) {
                const float4 x = *(const float4*)(kr + c);
                d0 = fmaf(q[c], x.x, d0); d0 = fmaf(q[c + 1], x.y, d0);
                d0 = fmaf(q[c + 2], x.z, d0); d0 = fmaf(q[c + 3], x.w, d0);
            }
            s[jj] = d0 + __shfl_xor(d0, 1, 64);
        }
        if (contiguous) {
#pragma unroll
            for (int jj = 0; jj < TK; ++jj) {
                const int j = t0 + jj;
                if (!((j <= r) && (j < ninit || j >= W))) s[jj] = -INFINITY;
            }
        } else {
            const int rem = cnt - (t - nA) * TK;
#pragma unroll
            for (int jj = 0; jj < TK; ++jj)
                if (jj >= rem) s[jj] = -INFINITY;
        }
        float mx = s[0];
#pragma unroll
        for (int jj = 1; jj < TK; ++jj) mx = fmaxf(mx, s[jj]);
        const float mnew = fmaxf(m, mx);
        const float muse = (mnew == -INFINITY) ? 0.f : mnew;
        const float alpha = __builtin_amdgcn_exp2f((m - muse) * c2);
        const float mc = muse * c2;
        m = mnew;
        float rs = 0.f;
#pragma unroll
        for (int jj = 0; jj < TK; ++jj) {
            s[jj] = __builtin_amdgcn_exp2f(fmaf(s[jj], c2, -mc));
            rs += s[jj];
        }
        l = l * alpha + rs;
#pragma unroll
        for (int c = 0; c < DH; ++c) acc[c] *= alpha;
#pragma unroll
        for (int jj = 0; jj < TK; ++jj) {
            const float* vr = Vs + jj * STR + hh * DH;
#pragma unroll
            for (int c = 0; c < DH; c += 4) {
                const float4 x = *(const float4*)(vr + c);
                acc[c] = fmaf(s[jj], x.x, acc[c]); acc[c + 1] = fmaf(s[jj], x.y, acc[c + 1]);
                acc[c + 2] = fmaf(s[jj], x.z, acc[c + 2]); acc[c + 3] = fmaf(s[jj], x.w, acc[c + 3]);
            }
        }
    }

    const float ms = m * p.sigma;
    if (a.flags & kEngStoreState) {
        if (rok) {
            if (hh == 0) { a.Mout[ri] = ms; a.Lout[ri] = l; }
            if (a.Accout) {
                float* dst = a.Accout + ri * Dd + hh * DH;
#pragma unroll
                for (int c = 0; c < DH; c += 4) *(float4*)(dst + c) = make_float4(acc[c], acc[c + 1], acc[c + 2], acc[c + 3]);
            }
        }
        if (a.xa) {
            __syncthreads();
            if (hh == 0) smem[lr] = rok ? ms : 0.f;
            __syncthreads();
            if (tid == 0) {
                const int nrows = rlast - row0 + 1;
                float sum = 0.f;
                for (int e = 0; e < nrows; ++e) sum += smem[e];
                a.xa[blk_index(p, sq, wk.b, wk.h, wk.i)] = sum / (float)nrows;
            }
        }
    }
    if ((a.flags & kEngStoreOut) && rok) {
        const float inv = 1.f / l;
        float* dst = (float*)a.out + tok_offset(p, p.os, sq, wk.b, wk.h, r) + hh * DH;
#pragma unroll
        for (int c = 0; c < DH; c += 4)
            *(float4*)(dst + c) = make_float4(acc[c] * inv, acc[c + 1] * inv, acc[c + 2] * inv, acc[c + 3] * inv);
        if (a.lse && hh == 0) a.lse[ri] = ms + logf(l);
    }
}
}  // namespace

__global__ __launch_bounds__(256) void engine_fp32_kernel(EngineArgs a) {
    extern __shared__ __attribute__((aligned(16))) float smem_f[];
    switch (a.p.d) {
        case 32: engine_fp32_body<16>(a, smem_f); break;
        case 64: engine_fp32_body<32>(a, smem_f); break;
        case 128: engine_fp32_body<64>(a, smem_f); break;
        default: break;
    }
}

size_t engine_fp32_lds_bytes(int d, int bq) {
    size_t tiles = 2 * (size_t)TK * (d + 4) * sizeof(float);
    size_t red = (size_t)bq * sizeof(float);
    return tiles > red ? tiles : red;
}

}  // namespace aa
