// Mask scan + K/V compaction (paper Section 4.1: the softmax branch loads only the
// tokens routed to it; Eq. 12 gives the column set).  For every (batch, head):
//   cnt[t] = #softmax tokens among 0..t,  idx[c] = position of the c-th one,
//   n_s = cnt[L-1],  Kc[c] = K[idx[c]],  Vc[c] = V[idx[c]].
// Integer work, exactly one correct answer.  HBM-bound.
//
// Grid (ceil(L / SEG), B*H).  A block owns SEG consecutive tokens.  Its base
// count is recomputed from the mask bytes in front of the segment (at most L
// bytes, read 16 at a time and served by L2), so blocks need no ordering and
// no inter-block communication.
#include "scan_compact_block.h"

namespace nats {

template <typename T>
__global__ __launch_bounds__(SCAN_THREADS) void scan_compact_kernel(const ScanArgs<T> a) {
    __shared__ int lds[SCAN_LDS_INTS];
    scan_compact_block<T>(a, blockIdx.x, blockIdx.y, lds);
}

nats_status launch_scan_compact(const FwdPlan& pl, const uint8_t* mask, const void* K, const void* V,
                                int32_t* cnt, int32_t* idx, int32_t* n_s, void* Kc, void* Vc,
                                void* Kc_user, void* Vc_user, int cap_user, void* VhT, hipStream_t st) {
    dim3 grid((pl.L + SCAN_SEG - 1) / SCAN_SEG, pl.BHG);
    if (pl.dtype == NATS_BF16) {
        const ScanArgs<bf16_t> a{mask, (const bf16_t*)K, (const bf16_t*)V, pl.L, pl.d, cnt, idx, n_s, (bf16_t*)Kc,
                                 (bf16_t*)Vc, (bf16_t*)Kc_user, (bf16_t*)Vc_user, cap_user, (half_t*)VhT,
                                 pl.routing == NATS_ROUTE_CHUNK ? (pl.RC == 128 ? 7 : 6) : 0, pl.G, pl.qk_per_out_head};
        hipLaunchKernelGGL(scan_compact_kernel<bf16_t>, grid, dim3(SCAN_THREADS), 0, st, a);
    } else {
        const ScanArgs<float> a{mask, (const float*)K, (const float*)V, pl.L, pl.d, cnt, idx, n_s, (float*)Kc,
                                (float*)Vc, (float*)Kc_user, (float*)Vc_user, cap_user, (half_t*)VhT,
                                pl.routing == NATS_ROUTE_CHUNK ? (pl.RC == 128 ? 7 : 6) : 0, pl.G, pl.qk_per_out_head};
        hipLaunchKernelGGL(scan_compact_kernel<float>, grid, dim3(SCAN_THREADS), 0, st, a);
    }
    return check_launch("scan_compact");
}

}  // namespace nats
