// Weights of the merge (Eq. 22): for every token and head, the two output weights of Eq. 21 are a
// softmax over two logits, each a linear map of the token's query,
//     [w_nla, w_la] = softmax([W_nla q_t, W_la q_t]),
// with one pair of weight vectors per head.  The ablation "(iv)" of Section 5 replaces the softmax by a
// sigmoid of each logit, or by nothing (act = 1, 2).  HBM-bound: Q is read once (2 d FLOP per logit).
//
// A row of Q is spread over d / EPL lanes (16 bytes each); partial dot products are reduced with xor
// shuffles inside that lane group.
#include <math.h>

#include "nats_common.h"

namespace nats {

constexpr int MW_THREADS = 256;

template <typename T, int D>
__global__ __launch_bounds__(MW_THREADS) void merge_weights_kernel(
    const T* __restrict__ Q, const float* __restrict__ W_out, float* __restrict__ w_nla,
    float* __restrict__ w_la, int H, int L, size_t n_rows, int act, int G) {
    constexpr int EPL = Vec16<T>::N;
    constexpr int LPR = D / EPL;                  // lanes per row: 8 (bf16, d=64) .. 32 (f32, d=128)
    constexpr int ROWS = MW_THREADS / LPR;        // rows per block pass
    const int part = threadIdx.x % LPR;
    for (size_t row = (size_t)blockIdx.x * ROWS + threadIdx.x / LPR; row < n_rows; row += (size_t)gridDim.x * ROWS) {
        // rows count (batch, output head, token); with head grouping (H = output heads per batch element) the G
        // heads of a group weigh their outputs by their own W_out applied to the linear head's query
        const size_t bo = row / L;
        const int h = (int)(bo % H);
        float q[EPL];
        Vec16<T>::load(Q + ((bo / G) * L + row % L) * D + part * EPL, q);
        const float* w0 = W_out + ((size_t)h * 2) * D + part * EPL;   // W_nla of this head
        const float* w1 = w0 + D;                                      // W_la
        float a = 0.f, b = 0.f;
#pragma unroll
        for (int j = 0; j < EPL; ++j) { a += q[j] * w0[j]; b += q[j] * w1[j]; }
#pragma unroll
        for (int off = 1; off < LPR; off <<= 1) { a += __shfl_xor(a, off); b += __shfl_xor(b, off); }
        if (part == 0) {
            if (act == 0) {          // Eq. 22
                const float m = fmaxf(a, b);
                const float ea = expf(a - m), eb = expf(b - m);
                const float inv = 1.f / (ea + eb);
                w_nla[row] = ea * inv;
                w_la[row] = eb * inv;
            } else if (act == 1) {   // sigmoid weights
                w_nla[row] = 1.f / (1.f + expf(-a));
                w_la[row] = 1.f / (1.f + expf(-b));
            } else {                 // linear weights
                w_nla[row] = a;
                w_la[row] = b;
            }
        }
    }
}

template <typename T>
static void launch_mw(int B, int H, int L, int d, const void* Q, const float* W_out, float* w_nla, float* w_la,
                      int act, int G, hipStream_t st) {
    const size_t n_rows = (size_t)B * H * L;
    const int rows_per_block = MW_THREADS / (d / Vec16<T>::N);
    size_t blocks = (n_rows + rows_per_block - 1) / rows_per_block;
    if (blocks > 256 * 16) blocks = 256 * 16;     // grid-stride beyond a few blocks per CU
    if (d == 64)
        hipLaunchKernelGGL((merge_weights_kernel<T, 64>), dim3((unsigned)blocks), dim3(MW_THREADS), 0, st, (const T*)Q,
                           W_out, w_nla, w_la, H, L, n_rows, act, G);
    else
        hipLaunchKernelGGL((merge_weights_kernel<T, 128>), dim3((unsigned)blocks), dim3(MW_THREADS), 0, st, (const T*)Q,
                           W_out, w_nla, w_la, H, L, n_rows, act, G);
}

// Q [B,H/G,L,d] (dtype), W_out [H,2,d] f32 -> w_nla, w_la [B,H,L] f32 (H output heads, G per linear head)
nats_status launch_merge_weights(int B, int H, int L, int d, int dtype, const void* Q, const float* W_out,
                                 float* w_nla, float* w_la, int act, int G, hipStream_t st) {
    if (dtype == NATS_BF16) launch_mw<bf16_t>(B, H, L, d, Q, W_out, w_nla, w_la, act, G, st);
    else launch_mw<float>(B, H, L, d, Q, W_out, w_nla, w_la, act, G, st);
    return check_launch("merge_weights");
}

}  // namespace nats
