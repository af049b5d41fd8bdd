// Arguments of the online-softmax tile engines (bf16 MFMA and fp32 vector-FMA).
#pragma once
#include "aa_common.h"

namespace aa {

enum : int {
    kEngAnchorRegion = 1,   // walk the tiles of A(r): initial tokens + window .. diagonal
    kEngDense = 2,          // with kEngAnchorRegion: A(r) := [0, r] (dense causal attention)
    kEngList = 4,           // walk the chunks of the group's selected-column list
    kEngLoadState = 8,      // start from (M, L, Acc) instead of (-inf, 0, 0)
    kEngStoreState = 16,    // write M, L, (Acc), pooled anchor
    kEngStoreOut = 32       // write out = acc / l and lse
};

struct EngineArgs {
    KParams p;
    int flags;
    const void *q, *k, *v;
    const float *Min, *Lin, *Accin;
    const int* counts;
    const long long* offsets;
    const int* idx;
    float *Mout, *Lout, *Accout, *xa;
    // stage 1 only, nullable: pooled queries of stage 2 (bf16 hi / lo rows of 128, norm of lo),
    // written from the Q fragments the block's work-group holds anyway (see aa_pool.h)
    void *qp_hi, *qp_lo;
    float* qlo_norm;
    void* out;
    float* lse;
    // List-driven calls: offsets[groups_total] is the total (padded) list length.  Lists that do not
    // fit the caller's idx buffer (idx_capacity entries) are incomplete: the launch then does nothing.
    // Two engines can be launched for the same list-driven call; each decides on the device from that
    // total whether it is the one to run: sel = 0 runs always, sel = 1 runs iff the total is below
    // sel_entries, sel = 2 iff not.
    long long groups_total, idx_capacity;
    int sel;
    long long sel_entries;
};

// true iff this launch has work to do (uniform over the grid)
__device__ __forceinline__ bool engine_selected(const EngineArgs& a) {
    if (!(a.flags & kEngList)) return true;
    const long long total = a.offsets[a.groups_total];
    if (total > a.idx_capacity) return false;
    if (a.sel == 0) return true;
    return (a.sel == 2) == (total >= a.sel_entries);
}

// Launchers: the launch's hipError_t, or -1 if there is no instantiation for ea.flags.
// 128 query rows per work-group, one instantiation per mode
int launch_engine_bf16(const EngineArgs& ea, unsigned grid, hipStream_t st);
// 256 query rows (two consecutive blocks) per work-group; needs dense mode or an even step
int launch_engine_bf16_pp(const EngineArgs& ea, unsigned grid, hipStream_t st);

__global__ void engine_fp32_kernel(EngineArgs a);
size_t engine_fp32_lds_bytes(int d, int bq);

}  // namespace aa
