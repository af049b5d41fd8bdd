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
    void* out;
    float* lse;
    // Two engines can be launched for the same list-driven call; each decides on the device from
    // the total (padded) list length offsets[sel_groups] whether it is the one to run:
    // sel = 0 runs always, sel = 1 runs iff the total is below sel_entries, sel = 2 iff not.
    int sel;
    long long sel_groups, sel_entries;
};

// true iff this launch is the one that was chosen (uniform over the grid)
__device__ __forceinline__ bool engine_selected(const EngineArgs& a) {
    if (a.sel == 0) return true;
    const bool big = a.offsets[a.sel_groups] >= a.sel_entries;
    return (a.sel == 2) == big;
}

// 128 query rows per work-group, one instantiation per mode; false: no instantiation for ea.flags
bool launch_engine_bf16(const EngineArgs& ea, unsigned grid, hipStream_t st);
// 256 query rows (two consecutive blocks) per work-group; needs dense mode or an even step
bool launch_engine_bf16_pp(const EngineArgs& ea, unsigned grid, hipStream_t st);

__global__ void engine_fp32_kernel(EngineArgs a);
size_t engine_fp32_lds_bytes(int d, int bq);

}  // namespace aa
