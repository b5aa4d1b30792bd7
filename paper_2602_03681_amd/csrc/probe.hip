// Measurement helper: the rate at which this chip issues the fp16 MFMA the forward kernels use,
// with nothing else in the way (no loads, no LDS, independent accumulators).  Benchmarks report
// kernel rates against this measured ceiling beside the published peak.
#include "mfma_util.h"
#include "nats_common.h"
#include "nats_measure.h"

namespace nats {

constexpr int PROBE_THREADS = 256;
constexpr int PROBE_BLOCKS = 256 * 8;
constexpr int PROBE_ACC = 8;   // independent accumulators per wavefront: hides the MFMA latency

__global__ __launch_bounds__(PROBE_THREADS) void mfma_probe_kernel(int iters, float* __restrict__ out) {
    const int lane = threadIdx.x & 63;
    half8 a, b;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        a[j] = (half_t)(0.001f * (float)((lane + j) & 7));
        b[j] = (half_t)(0.002f * (float)((lane * 3 + j) & 7));
    }
    f32x4 acc[PROBE_ACC];
#pragma unroll
    for (int i = 0; i < PROBE_ACC; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < PROBE_ACC; ++i) acc[i] = mfma16(a, b, acc[i]);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < PROBE_ACC; ++i) s += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
    // one store per block keeps the loop alive; the value is not meaningful
    if (threadIdx.x == 0) out[blockIdx.x] = s;
}

}  // namespace nats

extern "C" double nats_probe_mfma(int iters, float* out, size_t out_floats, void* hip_stream) {
    using namespace nats;
    if (iters < 1 || out == nullptr || out_floats < (size_t)PROBE_BLOCKS) {
        set_error("nats_probe_mfma: iters >= 1 and a device buffer of %d floats are required", PROBE_BLOCKS);
        return -1.0;
    }
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(PROBE_BLOCKS), dim3(PROBE_THREADS), 0,
                       reinterpret_cast<hipStream_t>(hip_stream), iters, out);
    if (check_launch("mfma_probe") != NATS_OK) return -1.0;
    // wavefronts x iterations x accumulators x (16 x 16 x 32 multiply-adds, 2 FLOP each)
    return (double)PROBE_BLOCKS * (PROBE_THREADS / 64) * (double)iters * PROBE_ACC * (16.0 * 16.0 * 32.0 * 2.0);
}
