// Routing decision per chunk (Section 4.1, Eq. 8-9): the score layer mean-pools the layer's input
// features over the chunk's C tokens, maps the mean with one linear layer to a score per head and
// operation, and the operation with the highest score gets the chunk:
//     score[b, c, h, :] = W_s[h, :, :] . mean_{t in chunk c} X[b, t, :]        (Eq. 8)
//     mask_c[b, h, c]   = 1 (softmax chunk) iff score[.., 0] >= score[.., 1]   (Eq. 9; softmax over the two
//                          scores is monotone, so the argmax is taken on the scores themselves)
// Operation 0 is softmax attention, operation 1 the linear one (the order of W_out in Eq. 22).
//
// HBM-bound: X is read once.  One block per (batch, chunk), RC_GROUPS groups of RC_COLS threads: a group
// takes every RC_GROUPS-th token of the chunk, a thread owns 8 (bf16) or 4 (f32) consecutive features
// (one 16-byte load per token, all of a thread's loads in flight together) and sums them in fp32.  The
// groups' column sums meet in LDS; there each wavefront takes up to four of the 2 H outputs, its lanes
// striding over the columns (coalesced 16-byte reads of W_s, independent of one another), and one
// reduction over the wavefront per output finishes the dot product.  Wider inputs than one pass covers
// (RC_COLS * 8 or 4 features) repeat the two phases per slice of columns and accumulate.  Every sum has
// a fixed order: a launch gives the same bits on every run.  Scores are fp32; the mask is decided from
// those fp32 scores, which are also returned so that a caller can see the margin.
// The token split is there for the short grids of small batches (one block per CU or fewer): the life of
// one block is a chain of two memory latencies, not of sixty-four.  Dealing whole chunks to the groups
// instead (W_s read once per four chunks) measured no faster on long grids and is not kept.
#include "nats_common.h"

namespace nats {

constexpr int RC_COLS = 256;     // threads across the features
constexpr int RC_GROUPS = 4;     // groups of RC_COLS threads across the chunk's tokens
constexpr int RC_THREADS = RC_COLS * RC_GROUPS;
constexpr int RC_WAVES = RC_THREADS / 64;
constexpr int RC_MAX_OUT = 64;   // 2 * H at most
constexpr int RC_OPW = RC_MAX_OUT / RC_WAVES;   // outputs per wavefront

template <typename T>
__global__ __launch_bounds__(RC_THREADS) void route_chunks_kernel(
    const T* __restrict__ X, const float* __restrict__ W_s, float* __restrict__ scores,
    uint8_t* __restrict__ mask_c, int L, int C, int d_model, int H, float* __restrict__ w_nla,
    float* __restrict__ w_la, int act) {
    constexpr int EPL = Vec16<T>::N;
    constexpr int SLICE = RC_COLS * EPL;           // columns per pass
    __shared__ float s_sum[RC_GROUPS][SLICE];
    __shared__ float s_out[RC_MAX_OUT];
    const int n_chunks = L / C;
    const int b = blockIdx.x / n_chunks, c = blockIdx.x % n_chunks;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ct = tid % RC_COLS, grp = tid / RC_COLS;
    const int n_out = 2 * H;
    const T* Xc = X + ((size_t)b * L + (size_t)c * C) * d_model;
    float acc[RC_OPW];
#pragma unroll
    for (int k = 0; k < RC_OPW; ++k) acc[k] = 0.f;

    for (int col0 = 0; col0 < d_model; col0 += SLICE) {
        // ---- column sums of this group's tokens ----
        const int col = col0 + ct * EPL;
        float sum[EPL];
#pragma unroll
        for (int j = 0; j < EPL; ++j) sum[j] = 0.f;
        if (col < d_model) {
#pragma unroll 16
            for (int t = grp; t < C; t += RC_GROUPS) {
                float x[EPL];
                Vec16<T>::load(Xc + (size_t)t * d_model + col, x);
#pragma unroll
                for (int j = 0; j < EPL; ++j) sum[j] += x[j];
            }
        }
        if (col0 > 0) __syncthreads();   // the previous slice's sums have been consumed
#pragma unroll
        for (int j = 0; j < EPL; ++j) s_sum[grp][ct * EPL + j] = sum[j];
        __syncthreads();
        // ---- this slice's share of the dot products: wavefront `wave` owns outputs wave + RC_WAVES * k;
        //      four columns per lane and step ----
        const int width = min(SLICE, d_model - col0);
#pragma unroll
        for (int it = 0; it < SLICE / 256; ++it) {
            const int cl = (it * 64 + lane) * 4;
            if (cl < width) {
                float4 x = *reinterpret_cast<const float4*>(&s_sum[0][cl]);
#pragma unroll
                for (int g = 1; g < RC_GROUPS; ++g) {
                    const float4 y = *reinterpret_cast<const float4*>(&s_sum[g][cl]);
                    x.x += y.x; x.y += y.y; x.z += y.z; x.w += y.w;
                }
#pragma unroll
                for (int k = 0; k < RC_OPW; ++k) {
                    const int o = wave + RC_WAVES * k;
                    if (o < n_out) {
                        const float4 w = *reinterpret_cast<const float4*>(W_s + (size_t)o * d_model + col0 + cl);
                        acc[k] += x.x * w.x + x.y * w.y + x.z * w.z + x.w * w.w;
                    }
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < RC_OPW; ++k) {
        float v = acc[k];
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
        if (lane == 0) s_out[wave + RC_WAVES * k] = v;
    }
    __syncthreads();
    if (tid < H) {
        const float inv = 1.f / (float)C;
        const float s0 = s_out[2 * tid] * inv, s1 = s_out[2 * tid + 1] * inv;
        if (scores != nullptr) {
            float* dst = scores + (((size_t)b * n_chunks + c) * H + tid) * 2;
            dst[0] = s0; dst[1] = s1;
        }
        if (mask_c != nullptr) mask_c[((size_t)b * H + tid) * n_chunks + c] = s0 >= s1 ? 1 : 0;
        if (w_nla != nullptr) {   // the same linear map as a source of merge weights (Section 5, ablation (v))
            float a0 = s0, a1 = s1;
            if (act == 0) {          // the softmax over the pair, as in Eq. 22
                const float m = fmaxf(s0, s1);
                const float e0 = expf(s0 - m), e1 = expf(s1 - m);
                a0 = e0 / (e0 + e1); a1 = e1 / (e0 + e1);
            } else if (act == 1) {   // a sigmoid of each
                a0 = 1.f / (1.f + expf(-s0)); a1 = 1.f / (1.f + expf(-s1));
            }
            w_nla[((size_t)b * H + tid) * n_chunks + c] = a0;
            w_la[((size_t)b * H + tid) * n_chunks + c] = a1;
        }
    }
}

// X [B,L,d_model] (dtype), W_s [H,2,d_model] f32 -> scores [B,L/C,H,2] f32 (optional), mask_c [B,H,L/C] u8
// w_nla, w_la [B,H,L/C] f32 (optional): the scores passed through the activation `act` of the merge weights
nats_status launch_route_chunks(int B, int L, int C, int d_model, int H, int dtype, const void* X, const float* W_s,
                                float* scores, uint8_t* mask_c, float* w_nla, float* w_la, int act, hipStream_t st) {
    dim3 grid((unsigned)(B * (L / C)));
    if (dtype == NATS_BF16)
        hipLaunchKernelGGL(route_chunks_kernel<bf16_t>, grid, dim3(RC_THREADS), 0, st, (const bf16_t*)X, W_s, scores,
                           mask_c, L, C, d_model, H, w_nla, w_la, act);
    else
        hipLaunchKernelGGL(route_chunks_kernel<float>, grid, dim3(RC_THREADS), 0, st, (const float*)X, W_s, scores,
                           mask_c, L, C, d_model, H, w_nla, w_la, act);
    return check_launch("route_chunks");
}

}  // namespace nats
