// Host side of the C ABI (include/anchor_attention.h): argument checks, buffer
// arithmetic and kernel launches.  Nothing here allocates device memory or waits
// for the stream.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>

#include "../../include/anchor_attention.h"
#include "aa_common.h"
#include "aa_engine.h"
#include "aa_select.h"

namespace aa {
namespace {

thread_local char g_hip_err[256] = "";

int hip_fail(hipError_t e, const char* what) {
    snprintf(g_hip_err, sizeof(g_hip_err), "%s: %s", what, hipGetErrorString(e));
    return AA_EHIP;
}
#define AA_HIP(call)                                         \
    do {                                                     \
        hipError_t e_ = (call);                              \
        if (e_ != hipSuccess) return hip_fail(e_, #call);    \
    } while (0)
// AA_LAUNCH(kernel, grid, block, lds bytes, stream, args...): the launch's own status
#define AA_LAUNCH(kern, ...)                                 \
    do {                                                     \
        hipError_t e_ = launch_kernel(kern, __VA_ARGS__);    \
        if (e_ != hipSuccess) return hip_fail(e_, #kern);    \
    } while (0)

inline long long cdiv(long long a, long long b) { return (a + b - 1) / b; }
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Plan {
    KParams kp;
    aa_sizes sz;
    int nwords;
    // byte offsets inside the workspaces
    size_t sel_qhi, sel_qlo, sel_qln, sel_kmax, sel_bits, sel_segc, sel_kp;   // stripe_select workspace
    size_t pf_M, pf_L, pf_Acc, pf_xa, pf_counts, pf_offsets, pf_flag, pf_idx, pf_sel;  // prefill workspace
};

// candidates of the first `ngroups` groups of a sequence, each group's count rounded up to a list
// chunk (a group's candidate range depends on its index alone, not on the sequence's length)
long long padded_candidates(const aa_params* p, long long ngroups) {
    const long long span = (long long)p->block_q * p->step;
    long long tot = 0;
    for (long long g = 0; g < ngroups; ++g) {
        long long W = g * span - p->window;
        if (W < p->n_init) W = p->n_init;
        tot += cdiv(W - p->n_init, kIdxPad) * kIdxPad;
    }
    return tot;
}

int make_plan(const aa_params* p, Plan* pl) {
    if (!p || !pl) return AA_EINVAL;
    if (p->B <= 0 || p->Hq <= 0 || p->Hkv <= 0 || p->N <= 0 || p->d <= 0) return AA_EINVAL;
    if (p->Hq % p->Hkv != 0) return AA_EINVAL;
    if (p->block_q <= 0 || p->block_kv != p->block_q) return AA_EINVAL;
    if (p->n_init < 0 || p->window < 0 || p->step < 1) return AA_EINVAL;
    if (std::isnan(p->theta) || std::isnan(p->softmax_scale) || p->softmax_scale < 0.f) return AA_EINVAL;
    if (p->dtype != AA_FP32 && p->dtype != AA_BF16) return AA_EINVAL;
    if (p->granularity != AA_STRIPE && p->granularity != AA_BLOCK) return AA_EINVAL;
    if (p->granularity == AA_BLOCK && (p->n_init % p->block_kv || p->window % p->block_kv)) return AA_EINVAL;
    if (p->engine != AA_ENGINE_AUTO && p->engine != AA_ENGINE_128 && p->engine != AA_ENGINE_256) return AA_EINVAL;
    if (p->cu_seqlens && (p->total_tokens <= 0 || p->N > p->total_tokens)) return AA_EINVAL;
    if (p->causal != 1) return AA_EUNSUPPORTED;
    if (p->step > 128) return AA_EUNSUPPORTED;
    // the block-granularity mask kernel keeps a group's pooled rows and one flag per key block in LDS
    if (p->granularity == AA_BLOCK && mask_block_lds_bytes(p->N, p->d, p->block_q, p->step) > kMaskBlockLdsMax)
        return AA_EUNSUPPORTED;
    const int vec = p->dtype == AA_BF16 ? 8 : 4;             // elements per 16-byte access
    if (p->dtype == AA_BF16) {
        if (p->d != 128 || p->block_q != 128) return AA_EUNSUPPORTED;
        // K / V rows are addressed with 32-bit byte offsets from the head's first row
        if ((int64_t)p->N * p->k_stride[2] * 2 >= (1ll << 31) || (int64_t)p->N * p->v_stride[2] * 2 >= (1ll << 31))
            return AA_EUNSUPPORTED;
    } else {
        if (p->d != 32 && p->d != 64 && p->d != 128) return AA_EUNSUPPORTED;
        if (p->block_q < 16 || p->block_q > 128 || p->block_q % 16) return AA_EUNSUPPORTED;
    }
    const int64_t* st[4] = {p->q_stride, p->k_stride, p->v_stride, p->o_stride};
    for (int t = 0; t < 4; ++t) {
        if (st[t][2] < p->d || st[t][1] <= 0) return AA_EINVAL;
        for (int e = 0; e < 3; ++e)
            if (st[t][e] < 0 || st[t][e] % vec) return AA_EINVAL;
    }

    KParams& k = pl->kp;
    memset(&k, 0, sizeof(k));
    k.B = p->B; k.Hq = p->Hq; k.Hkv = p->Hkv; k.N = p->N; k.d = p->d;
    k.bq = p->block_q; k.n_init = p->n_init; k.w = p->window; k.step = p->step;
    k.grp = p->Hq / p->Hkv;
    k.packed = p->cu_seqlens != nullptr;
    k.use_anchor = p->use_anchor != 0;
    k.theta = p->theta;
    k.sigma = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->d);
    for (int e = 0; e < 3; ++e) {
        k.qs[e] = p->q_stride[e]; k.ks[e] = p->k_stride[e];
        k.vs[e] = p->v_stride[e]; k.os[e] = p->o_stride[e];
    }
    k.cu = p->cu_seqlens;
    k.total = k.packed ? p->total_tokens : (long long)p->B * p->N;
    const long long span = (long long)p->block_q * p->step;
    k.nblk_max = (int)cdiv(p->N, p->block_q);
    k.ngrp_max = (int)cdiv(p->N, span);
    // launch grids put heads (times sequences) on y / z, and the fp32 mask kernel puts groups on y
    if ((long long)p->Hq * p->B > 65535 || p->Hq + p->Hkv > 65535) return AA_EUNSUPPORTED;
    if (p->dtype == AA_FP32 && k.ngrp_max > 65535) return AA_EUNSUPPORTED;

    aa_sizes& s = pl->sz;
    memset(&s, 0, sizeof(s));
    if (k.packed) {
        s.rows = (int64_t)p->Hq * p->total_tokens;
        s.blk_cap = p->total_tokens / p->block_q + p->B;
        s.grp_cap = p->total_tokens / span + p->B;
        s.blocks = (int64_t)p->Hq * s.blk_cap;
        s.groups = (int64_t)p->Hq * s.grp_cap;
        // Worst split of total_tokens into B sequences of at most N tokens.  A group counts in full
        // as soon as it has one row, so the bound goes over group counts: the sequences have at most
        // gtot groups together and at most ngrp_max each, and the candidates of a sequence with n
        // groups, F(n), are convex in n (later groups have longer candidate ranges): the maximum of
        // sum F(n_b) puts as many sequences as possible at ngrp_max and the remainder into one more.
        long long gtot = p->total_tokens / span + p->B;
        if (gtot > (long long)p->B * k.ngrp_max) gtot = (long long)p->B * k.ngrp_max;
        s.idx_capacity_max = (int64_t)p->Hq * ((gtot / k.ngrp_max) * padded_candidates(p, k.ngrp_max) +
                                               padded_candidates(p, gtot % k.ngrp_max));
    } else {
        s.rows = (int64_t)p->B * p->Hq * p->N;
        s.blk_cap = k.nblk_max;
        s.grp_cap = k.ngrp_max;
        s.blocks = (int64_t)p->B * p->Hq * s.blk_cap;
        s.groups = (int64_t)p->B * p->Hq * s.grp_cap;
        s.idx_capacity_max = (int64_t)p->B * p->Hq * padded_candidates(p, k.ngrp_max);
    }
    if (s.idx_capacity_max < kIdxPad) s.idx_capacity_max = kIdxPad;
    // fp32: row-major, d floats per row; bf16: per query block, four 32-row tiles in fragment order
    s.acc_elems = p->dtype == AA_BF16 ? s.blocks * (int64_t)p->block_q * p->d : s.rows * p->d;
    k.blk_cap = s.blk_cap;
    k.grp_cap = s.grp_cap;
    pl->nwords = (int)cdiv(p->N, 32);

    size_t off = 0;
    if (p->dtype == AA_BF16) {
        pl->sel_qhi = off; off += align256((size_t)s.blocks * 128 * 2);
        pl->sel_qlo = off; off += align256((size_t)s.blocks * 128 * 2);
        pl->sel_qln = off; off += align256((size_t)s.blocks * 4);
        pl->sel_kmax = off; off += align256((size_t)(s.blocks / k.grp) * 4);
    } else {
        pl->sel_qhi = off; off += align256((size_t)s.blocks * p->d * 4);
        pl->sel_qlo = off; pl->sel_qln = off; pl->sel_kmax = off;
    }
    pl->sel_bits = off; off += align256((size_t)s.groups * pl->nwords * 4);
    pl->sel_segc = off; off += align256((size_t)s.groups * cdiv(pl->nwords, 64) * 4);
    pl->sel_kp = off;
    if (p->granularity == AA_BLOCK) off += align256((size_t)(s.blocks / k.grp) * p->d * 4);
    s.select_ws_bytes = off;

    off = 0;
    pl->pf_M = off; off += align256((size_t)s.rows * 4);
    pl->pf_L = off; off += align256((size_t)s.rows * 4);
    pl->pf_Acc = off; off += align256((size_t)s.acc_elems * 4);
    pl->pf_xa = off; off += align256((size_t)s.blocks * 4);
    pl->pf_counts = off; off += align256((size_t)s.groups * 4);
    pl->pf_offsets = off; off += align256((size_t)(s.groups + 1) * 8);
    pl->pf_flag = off; off += 256;
    pl->pf_idx = off; off += align256((size_t)s.idx_capacity_max * 4);
    pl->pf_sel = off; off += s.select_ws_bytes;
    s.prefill_ws_bytes = off;
    return AA_OK;
}

bool misaligned(const void* ptr) { return ((uintptr_t)ptr & 15) != 0; }

// ---- workspace of stripe_select_noalloc: a device array that is part of the loaded library, one
// copy per GPU, held until the process ends.  Its name is a host-side handle, not a device
// address: host code uses the address hipGetSymbolAddress reports for the current device.
constexpr size_t kScratchBytes = (size_t)AA_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
__device__ __align__(256) static unsigned char scratch[kScratchBytes];
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int scratch_of_current_device(void** out) {
    int dev = -1;
    AA_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return AA_EUNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        AA_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return AA_EHIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return AA_OK;
}

// kernels that ask for more dynamic LDS than the default limit: raised once per process
std::once_flag g_attr_once;
hipError_t g_attr_status = hipSuccess;
hipError_t raise_lds_limits() {
    std::call_once(g_attr_once, [] {
        g_attr_status = hipFuncSetAttribute((const void*)engine_fp32_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                            (int)engine_fp32_lds_bytes(128, 128));
        if (g_attr_status == hipSuccess)
            g_attr_status = hipFuncSetAttribute((const void*)mask_block_kernel,
                                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaskBlockLdsMax);
    });
    return g_attr_status;
}

int engine_status(int rc, const char* name) {
    if (rc < 0) return AA_EUNSUPPORTED;
    return rc == (int)hipSuccess ? AA_OK : hip_fail((hipError_t)rc, name);
}

int launch_engine(const Plan& pl, const aa_params* prm, EngineArgs& ea, hipStream_t st) {
    const KParams& k = pl.kp;
    const unsigned grid = (unsigned)((long long)k.nblk_max * k.Hq * k.B);
    ea.groups_total = pl.sz.groups;
    ea.sel = 0;
    if (prm->dtype == AA_BF16) {
        // Two bf16 engines: 128 query rows per work-group (two work-groups per CU) and 256 rows
        // per work-group with the MFMA / softmax phases of the two waves of a SIMD alternating.
        // The second is faster on long tile loops and slower on short ones (its prologue and
        // epilogue overlap with nothing); it needs both blocks of a pair to share window and list.
        const bool pair_ok = (ea.flags & kEngDense) || k.step % 2 == 0;
        int choice = prm->engine;                   // 0 auto, 1: 128 rows, 2: 256 rows
        if (!pair_ok) choice = AA_ENGINE_128;
        if (choice == AA_ENGINE_AUTO) {
            if (ea.flags & kEngList) choice = 3;    // decided on the device from the list lengths
            else if (ea.flags & kEngDense) choice = k.N >= 8192 ? AA_ENGINE_256 : AA_ENGINE_128;
            else choice = AA_ENGINE_128;            // anchor region alone: at most step + 3 blocks of keys
        }
        const unsigned gridp = (unsigned)((long long)((k.nblk_max + 1) / 2) * k.Hq * k.B);
        int rc = AA_OK;
        if (choice == 3) {
            ea.sel_entries = 48ll * 64 * pl.sz.groups;   // mean list of 48 tiles
            ea.sel = 1;
            rc = engine_status(launch_engine_bf16(ea, grid, st), "engine_bf16_kernel");
            if (rc != AA_OK) return rc;
            ea.sel = 2;
            rc = engine_status(launch_engine_bf16_pp(ea, gridp, st), "engine_bf16_pp_kernel");
        } else if (choice == AA_ENGINE_256) {
            rc = engine_status(launch_engine_bf16_pp(ea, gridp, st), "engine_bf16_pp_kernel");
        } else {
            rc = engine_status(launch_engine_bf16(ea, grid, st), "engine_bf16_kernel");
        }
        return rc;
    }
    AA_HIP(raise_lds_limits());
    AA_LAUNCH(engine_fp32_kernel, dim3(grid), dim3(2 * k.bq), engine_fp32_lds_bytes(k.d, k.bq), st, ea);
    return AA_OK;
}

// sel_ws (nullable): a stripe_select workspace; the bf16 engines then also leave the pooled queries of
// stage 2 there (run_select is told so)
int run_anchor(const Plan& pl, const aa_params* p, const void* q, const void* k, const void* v, float* M, float* L,
               float* Acc, float* xa, char* sel_ws, hipStream_t st) {
    EngineArgs ea;
    memset(&ea, 0, sizeof(ea));
    ea.p = pl.kp;
    ea.flags = kEngAnchorRegion | kEngStoreState;
    ea.q = q; ea.k = k; ea.v = v;
    ea.Mout = M; ea.Lout = L; ea.Accout = Acc; ea.xa = xa;
    if (sel_ws && p->dtype == AA_BF16) {
        ea.qp_hi = sel_ws + pl.sel_qhi; ea.qp_lo = sel_ws + pl.sel_qlo; ea.qlo_norm = (float*)(sel_ws + pl.sel_qln);
    }
    return launch_engine(pl, p, ea, st);
}

// q_pooled: stage 1 has written the pooled queries into ws already (bf16 only)
// stats (nullable): the scan kernel also reports attended pairs and selected entries there
int run_select(const Plan& pl, const aa_params* p, const void* q, const void* k, const float* xa, int32_t* counts,
               int64_t* offsets, int32_t* idx, int64_t cap, int32_t* flag, char* ws, bool q_pooled, int64_t* stats,
               hipStream_t st) {
    const KParams& kp = pl.kp;
    SelectArgs sa;
    memset(&sa, 0, sizeof(sa));
    sa.p = kp;
    sa.q = q; sa.k = k; sa.xa = xa;
    sa.qp_hi = ws + pl.sel_qhi; sa.qp_lo = ws + pl.sel_qlo; sa.qp_f32 = (float*)(ws + pl.sel_qhi);
    sa.bits = (unsigned*)(ws + pl.sel_bits);
    sa.kp_f32 = (float*)(ws + pl.sel_kp);
    sa.qlo_norm = (float*)(ws + pl.sel_qln);
    sa.kmax_blk = nullptr;
    sa.segcount = (int*)(ws + pl.sel_segc);
    sa.nseg = (int)cdiv(pl.nwords, 64);
    sa.is_bf16 = p->dtype == AA_BF16;
    sa.nwords = pl.nwords;
    sa.counts = counts; sa.offsets = (long long*)offsets; sa.idx = idx;
    sa.idx_capacity = cap; sa.overflow = flag;
    sa.groups_total = pl.sz.groups;
    sa.stats = (long long*)stats;

    const dim3 gblk(kp.nblk_max, kp.Hq, kp.B), ggrp(kp.ngrp_max, kp.Hq, kp.B);
    if (p->granularity == AA_BLOCK) AA_HIP(raise_lds_limits());   // before anything is enqueued
    if (kp.packed)
        AA_LAUNCH(zero_i32_kernel, dim3((unsigned)cdiv(pl.sz.groups, 256)), dim3(256), 0, st, counts,
                  (long long)pl.sz.groups);
    q_pooled = q_pooled && p->dtype == AA_BF16;
    sa.pool_skip_q = q_pooled;
    if (p->granularity == AA_BLOCK) {
        if (p->dtype != AA_BF16)
            AA_LAUNCH(pool_q_fp32_kernel, gblk, dim3(128), 0, st, sa);
        else if (!q_pooled)
            AA_LAUNCH(pool_q_bf16_kernel, gblk, dim3(256), 0, st, sa);
        AA_LAUNCH(pool_k_kernel, dim3(kp.nblk_max, kp.Hkv, kp.B), dim3(256), 0, st, sa);
        AA_LAUNCH(mask_block_kernel, ggrp, dim3(256), mask_block_lds_bytes(kp.N, kp.d, kp.bq, kp.step), st, sa);
    } else if (p->dtype == AA_BF16) {
        sa.kmax_blk = (float*)(ws + pl.sel_kmax);
        AA_LAUNCH(pool_q_bf16_kernel, dim3(kp.nblk_max, (q_pooled ? 0 : kp.Hq) + kp.Hkv, kp.B), dim3(256), 0, st, sa);
        // one work-group per (query head, row tile, key chunk with candidates); the longest
        // sequence bounds every other
        sa.mask_items = mask_pair_items(kp.nblk_max, kp.step, kp.bq, kp.w, kp.n_init);
        const long long mask_per_xcd = cdiv((long long)sa.mask_items * kp.Hq * kp.B, 8);
        if (mask_per_xcd * 8 > 0x7fffffffll) return AA_EUNSUPPORTED;
        const dim3 gm((unsigned)(mask_per_xcd > 0 ? mask_per_xcd * 8 : 8));
        AA_LAUNCH(mask_bf16_kernel, gm, dim3(256), 0, st, sa);
    } else {
        AA_LAUNCH(pool_q_fp32_kernel, gblk, dim3(128), 0, st, sa);
        const dim3 gm((unsigned)cdiv(kp.N, 256), (unsigned)kp.ngrp_max, (unsigned)(kp.B * kp.Hq));
        AA_LAUNCH(mask_fp32_kernel, gm, dim3(256), (size_t)kp.step * kp.d * 4, st, sa);
    }
    AA_LAUNCH(count_kernel, ggrp, dim3(256), 0, st, sa);
    AA_LAUNCH(scan_kernel, dim3(1), dim3(1024), 0, st, sa);
    AA_LAUNCH(fill_kernel, dim3(kp.ngrp_max, (unsigned)cdiv(sa.nseg, 4), kp.Hq * kp.B), dim3(256), 0, st, sa);
    return AA_OK;
}

int run_sparse(const Plan& pl, const aa_params* p, const void* q, const void* k, const void* v, const float* M,
               const float* L, const float* Acc, const int32_t* counts, const int64_t* offsets, const int32_t* idx,
               int64_t idx_capacity, void* out, float* lse, hipStream_t st) {
    EngineArgs ea;
    memset(&ea, 0, sizeof(ea));
    ea.p = pl.kp;
    ea.flags = kEngList | kEngStoreOut | (M ? kEngLoadState : kEngAnchorRegion);
    ea.q = q; ea.k = k; ea.v = v;
    ea.Min = M; ea.Lin = L; ea.Accin = Acc;
    ea.counts = counts; ea.offsets = (const long long*)offsets; ea.idx = idx;
    ea.idx_capacity = idx_capacity;
    ea.out = out; ea.lse = lse;
    return launch_engine(pl, p, ea, st);
}

}  // namespace
}  // namespace aa

using namespace aa;

extern "C" {

int anchor_sizes(const aa_params* params, aa_sizes* out) {
    Plan pl;
    int rc = make_plan(params, &pl);
    if (rc != AA_OK) return rc;
    if (!out) return AA_EINVAL;
    *out = pl.sz;
    return AA_OK;
}

int anchor_workspace_bytes(const aa_params* params, size_t* bytes_out) {
    Plan pl;
    int rc = make_plan(params, &pl);
    if (rc != AA_OK) return rc;
    if (!bytes_out) return AA_EINVAL;
    *bytes_out = pl.sz.prefill_ws_bytes;
    return AA_OK;
}

int anchor_compute(const aa_params* params, const void* q, const void* k, const void* v, float* M, float* L,
                   float* Acc, float* xa_pooled, void* stream) {
    Plan pl;
    int rc = make_plan(params, &pl);
    if (rc != AA_OK) return rc;
    if (!q || !k || !v || !M || !L || !xa_pooled) return AA_EINVAL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(Acc)) return AA_EINVAL;
    return run_anchor(pl, params, q, k, v, M, L, Acc, xa_pooled, nullptr, (hipStream_t)stream);
}

int stripe_select(const aa_params* params, const void* q, const void* k, const float* xa_pooled, int32_t* counts,
                  int64_t* offsets, int32_t* idx, int64_t idx_capacity, int32_t* overflow_flag, void* ws,
                  size_t ws_bytes, void* stream) {
    Plan pl;
    int rc = make_plan(params, &pl);
    if (rc != AA_OK) return rc;
    if (!q || !k || !xa_pooled || !counts || !offsets || !idx || !overflow_flag || !ws) return AA_EINVAL;
    if (idx_capacity < 0 || misaligned(q) || misaligned(k) || misaligned(idx) || misaligned(ws)) return AA_EINVAL;
    if (ws_bytes < pl.sz.select_ws_bytes) return AA_EWORKSPACE;
    return run_select(pl, params, q, k, xa_pooled, counts, offsets, idx, idx_capacity, overflow_flag, (char*)ws,
                      false, nullptr, (hipStream_t)stream);
}

int stripe_select_noalloc(const aa_params* params, const void* q, const void* k, const float* xa_pooled,
                          int32_t* counts, int64_t* offsets, int32_t* idx, int64_t idx_capacity,
                          int32_t* overflow_flag, void* stream) {
    Plan pl;
    int rc = make_plan(params, &pl);
    if (rc != AA_OK) return rc;
    if (!q || !k || !xa_pooled || !counts || !offsets || !idx || !overflow_flag) return AA_EINVAL;
    if (idx_capacity < 0 || misaligned(q) || misaligned(k) || misaligned(idx)) return AA_EINVAL;
    if (pl.sz.select_ws_bytes > kScratchBytes) return AA_EWORKSPACE;
    void* ws = nullptr;
    rc = scratch_of_current_device(&ws);
    if (rc != AA_OK) return rc;
    return run_select(pl, params, q, k, xa_pooled, counts, offsets, idx, idx_capacity, overflow_flag, (char*)ws,
                      false, nullptr, (hipStream_t)stream);
}

int sparse_attn(const aa_params* params, const void* q, const void* k, const void* v, const float* M, const float* L,
                const float* Acc, const int32_t* counts, const int64_t* offsets, const int32_t* idx,
                int64_t idx_capacity, void* out, float* lse, void* stream) {
    Plan pl;
    int rc = make_plan(params, &pl);
    if (rc != AA_OK) return rc;
    if (!q || !k || !v || !counts || !offsets || !idx || !out || idx_capacity < 0) return AA_EINVAL;
    const int nstate = (M != nullptr) + (L != nullptr) + (Acc != nullptr);
    if (nstate != 0 && nstate != 3) return AA_EINVAL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(idx) || misaligned(Acc))
        return AA_EINVAL;
    return run_sparse(pl, params, q, k, v, M, L, Acc, counts, offsets, idx, idx_capacity, out, lse,
                      (hipStream_t)stream);
}

int anchor_attention_prefill(const aa_params* params, const void* q, const void* k, const void* v, void* out,
                             float* lse, int64_t* stats, void* ws, size_t ws_bytes, void* stream) {
    Plan pl;
    int rc = make_plan(params, &pl);
    if (rc != AA_OK) return rc;
    if (!q || !k || !v || !out || !ws) return AA_EINVAL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out) || misaligned(ws)) return AA_EINVAL;
    if (ws_bytes < pl.sz.prefill_ws_bytes) return AA_EWORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    char* w = (char*)ws;
    float* M = (float*)(w + pl.pf_M);
    float* L = (float*)(w + pl.pf_L);
    float* Acc = (float*)(w + pl.pf_Acc);
    float* xa = (float*)(w + pl.pf_xa);
    int32_t* counts = (int32_t*)(w + pl.pf_counts);
    int64_t* offsets = (int64_t*)(w + pl.pf_offsets);
    int32_t* flag = (int32_t*)(w + pl.pf_flag);
    int32_t* idx = (int32_t*)(w + pl.pf_idx);
    // the block means of Q (first step of stage 2) come out of stage 1, which holds the block's
    // queries in registers; the stage-wise entry points compute the same bits in a kernel of their own
    rc = run_anchor(pl, params, q, k, v, M, L, Acc, xa, w + pl.pf_sel, st);
    if (rc != AA_OK) return rc;
    rc = run_select(pl, params, q, k, xa, counts, offsets, idx, pl.sz.idx_capacity_max, flag, w + pl.pf_sel, true, stats, st);
    if (rc != AA_OK) return rc;
    rc = run_sparse(pl, params, q, k, v, M, L, Acc, counts, offsets, idx, pl.sz.idx_capacity_max, out, lse, st);
    if (rc != AA_OK) return rc;
    return AA_OK;
}

int dense_causal_flash(const aa_params* params, const void* q, const void* k, const void* v, void* out, float* lse,
                       void* stream) {
    Plan pl;
    int rc = make_plan(params, &pl);
    if (rc != AA_OK) return rc;
    if (!q || !k || !v || !out) return AA_EINVAL;
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(out)) return AA_EINVAL;
    EngineArgs ea;
    memset(&ea, 0, sizeof(ea));
    ea.p = pl.kp;
    ea.flags = kEngAnchorRegion | kEngDense | kEngStoreOut;
    ea.q = q; ea.k = k; ea.v = v;
    ea.out = out; ea.lse = lse;
    return launch_engine(pl, params, ea, (hipStream_t)stream);
}

const char* anchor_strerror(int code) {
    switch (code) {
        case AA_OK: return "ok";
        case AA_EINVAL: return "invalid argument";
        case AA_EUNSUPPORTED: return "unsupported configuration";
        case AA_EWORKSPACE: return "workspace too small";
        case AA_EHIP: return "HIP error";
        default: return "unknown error code";
    }
}

const char* anchor_last_hip_error(void) { return g_hip_err; }

}  // extern "C"
