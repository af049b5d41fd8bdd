// Measurement aid of bench.py, built into its own shared object (libanchor_probe.so), not into the
// attention library: a register-only loop of v_mfma_f32_32x32x16_bf16.  Timed with events on the
// stream it is enqueued on, it gives the bf16 matrix rate this GPU sustains at its actual clock,
// next to which bench.py quotes the attention kernels' rates.
#include <hip/hip_runtime.h>

typedef __bf16 probe_bf16x8 __attribute__((ext_vector_type(8)));
typedef float probe_floatx16 __attribute__((ext_vector_type(16)));

namespace {
constexpr int kProbeGroups = 1024, kProbeThreads = 256, kProbeMfmaPerIter = 16;

__global__ __launch_bounds__(256) void probe_mfma_kernel(int iters, float* sink) {
    probe_floatx16 c[4];
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) c[i][v] = threadIdx.x * 1e-3f;
    probe_bf16x8 x, y;
    for (int i = 0; i < 8; ++i) { x[i] = (__bf16)(threadIdx.x * 0.001f); y[i] = (__bf16)(i * 0.01f); }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < kProbeMfmaPerIter; ++i)
            c[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(x, y, c[i & 3], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 4; ++i)
        for (int v = 0; v < 16; ++v) s += c[i][v];
    sink[blockIdx.x * kProbeThreads + threadIdx.x] = s;
}
}  // namespace

extern "C" {

// Enqueues the loop on `stream` (a hipStream_t): 1024 work-groups of 4 waves, `iters` x 16 MFMAs per
// wave.  scratch: device buffer of at least 1 MiB (receives one float per thread).  Returns 0, -1 for
// bad arguments, -2 if the launch failed.
int anchor_probe_mfma(int iters, void* scratch, void* stream) {
    if (iters <= 0 || !scratch) return -1;
    float* sink = (float*)scratch;
    void* args[] = {(void*)&iters, (void*)&sink};
    return hipLaunchKernel((const void*)probe_mfma_kernel, dim3(kProbeGroups), dim3(kProbeThreads), args, 0,
                           (hipStream_t)stream) == hipSuccess ? 0 : -2;
}

// FLOP of one call with `iters` iterations (2 x 32 x 32 x 16 per MFMA).
double anchor_probe_mfma_flop(int iters) {
    return (double)kProbeGroups * (kProbeThreads / 64) * (double)iters * kProbeMfmaPerIter * 32768.0;
}

}  // extern "C"
