// Linear branch in fp32 arithmetic: the token-recurrent Gated DeltaNet update of
// Section 4.3 (Eq. 19), written for linear tokens only (Eq. 14), decayed at every
// token (Eq. 20), read by every query, o_t = la_scale * S_t q_t (Eq. 5 / Eq. 10):
//     S <- alpha_t S ;  if m_t == 0:  S <- S + beta_t (v_t - S k_t) k_t^T ;  o_t = S q_t.
// Rows of S (index d_v) evolve independently: four adjacent lanes own one row of S in
// registers (a quarter of its d_k columns each, the two dot products of a token finished by
// two shuffles); k_t, q_t, alpha_t, beta_t are the same for all rows and are staged through
// LDS a tile of tokens at a time (broadcast reads).
//
// This is the NATS_MATH_FP32 path (tight-tolerance fp32 workloads); the bf16
// throughput path is the chunkwise MFMA kernel.  VALU-bound: 6 d FLOP per row-token.
#include "nats_common.h"

namespace nats {

constexpr int REC_ROWS = 64;      // state rows per block
constexpr int REC_THREADS = 256;  // 4 adjacent lanes share a row, each owns a quarter of its d_k columns
constexpr int REC_TT = 32;        // tokens staged per tile

template <typename T, int D>
__global__ __launch_bounds__(REC_THREADS) void gdn_recurrent_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const float* __restrict__ alpha, const float* __restrict__ beta, const uint8_t* __restrict__ mask,
    const float* __restrict__ S0, float* __restrict__ S_final, float* __restrict__ O_la,
    float* __restrict__ snap, int L, float la_scale, int linear_op, int freeze_on_softmax, int G,
    int no_inner_output, int RC) {
    constexpr int DP = D / 4;       // columns of a row per lane
    constexpr int DPP = DP + 4;     // padded quarter stride: the four quarters land in different banks
    __shared__ __align__(16) float s_k[REC_TT][4 * DPP];
    __shared__ __align__(16) float s_q[REC_TT][4 * DPP];
    __shared__ float s_v[REC_TT][REC_ROWS];
    __shared__ float s_a[REC_TT], s_b[REC_TT];

    const int bh = blockIdx.y;
    const int tid = threadIdx.x, r = tid >> 2, part = tid & 3;
    const int row = blockIdx.x * REC_ROWS + r;  // d_v index of this lane's row
    // bh counts output heads: the G heads of a group are row blocks of one wide state, fed by their own value
    // columns and by the queries, keys, gates and mask of linear head bh / G (Section 4.3)
    const size_t base = (size_t)bh * L, lin = (size_t)(bh / G) * L;
    auto row_sum = [](float x) { return lane_group_sum<4>(x); };   // over a row's 4 lanes

    float S[DP];
    if (S0 != nullptr) {
        const float* src = S0 + ((size_t)bh * D + row) * D + part * DP;
#pragma unroll
        for (int c = 0; c < DP; c += 4) {
            float4 x = *reinterpret_cast<const float4*>(src + c);
            S[c] = x.x; S[c + 1] = x.y; S[c + 2] = x.z; S[c + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int c = 0; c < DP; ++c) S[c] = 0.f;
    }

    // Routing per chunk (snap != nullptr; mask holds one byte per chunk of RC tokens, 64 or 128): every token
    // of a chunk is written (the intra-chunk part is computed for every chunk); at the end of a softmax
    // chunk the row goes back to its value at the chunk's start, kept in snap, times the chunk's decay.
    const bool chunk_mask = snap != nullptr;
    float* my_snap = chunk_mask ? snap + ((size_t)bh * D + row) * D + part * DP : nullptr;
    const uint8_t* mask_c = mask + (size_t)(bh / G) * (L / RC);
    float chunk_decay = 1.f;
    // no_inner_output (routing per chunk only): the output reads the state carried into the chunk, decayed up to
    // the query, and nothing the chunk's own tokens wrote; that state lives in Sc beside the provisional one
    float Sc[DP];
#pragma unroll
    for (int c = 0; c < DP; ++c) Sc[c] = S[c];

    constexpr int EPL = Vec16<T>::N;
    for (int t0 = 0; t0 < L; t0 += REC_TT) {
        __syncthreads();
        // stage k, q (all D columns, quarters padded apart) and this block's slice of v for REC_TT tokens
        for (int e = tid * EPL; e < REC_TT * D; e += REC_THREADS * EPL) {
            const int i = e / D, c = e % D;
            const int pq = c / DP, pc = c % DP;   // EPL divides DP: a 16-byte group stays inside one quarter
            float tmp[EPL];
            Vec16<T>::load(K + (lin + t0 + i) * D + c, tmp);
#pragma unroll
            for (int j = 0; j < EPL; ++j) s_k[i][pq * DPP + pc + j] = tmp[j];
            Vec16<T>::load(Q + (lin + t0 + i) * D + c, tmp);
#pragma unroll
            for (int j = 0; j < EPL; ++j) s_q[i][pq * DPP + pc + j] = tmp[j];
        }
        for (int e = tid * EPL; e < REC_TT * REC_ROWS; e += REC_THREADS * EPL) {
            const int i = e / REC_ROWS, c = e % REC_ROWS;
            float tmp[EPL];
            Vec16<T>::load(V + (base + t0 + i) * D + blockIdx.x * REC_ROWS + c, tmp);
#pragma unroll
            for (int j = 0; j < EPL; ++j) s_v[i][c + j] = tmp[j];
        }
        if (tid < REC_TT) {
            // variant without decay on softmax tokens (routing per token): their alpha counts as 1
            s_a[tid] = (freeze_on_softmax && !chunk_mask && mask[lin + t0 + tid]) ? 1.f : alpha[lin + t0 + tid];
            // routing per token: softmax tokens never write
            s_b[tid] = (!chunk_mask && mask[lin + t0 + tid]) ? 0.f : beta[lin + t0 + tid];
        }
        __syncthreads();

        for (int i = 0; i < REC_TT; ++i) {
            const float a = s_a[i], b = s_b[i];
            const float* kr = &s_k[i][part * DPP];
            const float* qr = &s_q[i][part * DPP];
            float o = 0.f;
            if (chunk_mask && ((t0 + i) & (RC - 1)) == 0) {   // chunk start (uniform)
#pragma unroll
                for (int c = 0; c < DP; c += 4)
                    *reinterpret_cast<float4*>(my_snap + c) = make_float4(S[c], S[c + 1], S[c + 2], S[c + 3]);
                chunk_decay = 1.f;
                if (no_inner_output) {
#pragma unroll
                    for (int c = 0; c < DP; ++c) Sc[c] = S[c];
                }
            }
            chunk_decay *= a;
            if (b != 0.f) {  // uniform across the block
                float pred = 0.f;
#pragma unroll
                for (int c = 0; c < DP; c += 4) {
                    const float4 k4 = *reinterpret_cast<const float4*>(kr + c);
                    S[c] *= a; S[c + 1] *= a; S[c + 2] *= a; S[c + 3] *= a;
                    pred += S[c] * k4.x + S[c + 1] * k4.y + S[c + 2] * k4.z + S[c + 3] * k4.w;
                }
                pred = row_sum(pred);
                // gated linear attention (linear_op != 0) writes beta v k^T as it is: no correction by the state
                const float delta = b * (s_v[i][r] - (linear_op == 0 ? pred : 0.f));
#pragma unroll
                for (int c = 0; c < DP; c += 4) {
                    const float4 k4 = *reinterpret_cast<const float4*>(kr + c);
                    const float4 q4 = *reinterpret_cast<const float4*>(qr + c);
                    S[c] += delta * k4.x; S[c + 1] += delta * k4.y;
                    S[c + 2] += delta * k4.z; S[c + 3] += delta * k4.w;
                    o += S[c] * q4.x + S[c + 1] * q4.y + S[c + 2] * q4.z + S[c + 3] * q4.w;
                }
            } else {
#pragma unroll
                for (int c = 0; c < DP; c += 4) {
                    const float4 q4 = *reinterpret_cast<const float4*>(qr + c);
                    S[c] *= a; S[c + 1] *= a; S[c + 2] *= a; S[c + 3] *= a;
                    o += S[c] * q4.x + S[c + 1] * q4.y + S[c + 2] * q4.z + S[c + 3] * q4.w;
                }
            }
            if (no_inner_output) {   // uniform
                o = 0.f;
#pragma unroll
                for (int c = 0; c < DP; c += 4) {
                    const float4 q4 = *reinterpret_cast<const float4*>(qr + c);
                    Sc[c] *= a; Sc[c + 1] *= a; Sc[c + 2] *= a; Sc[c + 3] *= a;
                    o += Sc[c] * q4.x + Sc[c + 1] * q4.y + Sc[c + 2] * q4.z + Sc[c + 3] * q4.w;
                }
            }
            o = row_sum(o);
            if (part == 0) O_la[(base + t0 + i) * D + row] = la_scale * o;
            if (chunk_mask && ((t0 + i) & (RC - 1)) == RC - 1 && mask_c[(t0 + i) / RC]) {   // end of a softmax chunk
                if (freeze_on_softmax) chunk_decay = 1.f;   // variant: a softmax chunk leaves the state as it found it
#pragma unroll
                for (int c = 0; c < DP; c += 4) {
                    const float4 x = *reinterpret_cast<const float4*>(my_snap + c);
                    S[c] = chunk_decay * x.x; S[c + 1] = chunk_decay * x.y;
                    S[c + 2] = chunk_decay * x.z; S[c + 3] = chunk_decay * x.w;
                }
            }
        }
    }
    if (S_final != nullptr) {
        float* dst = S_final + ((size_t)bh * D + row) * D + part * DP;
#pragma unroll
        for (int c = 0; c < DP; c += 4)
            *reinterpret_cast<float4*>(dst + c) = make_float4(S[c], S[c + 1], S[c + 2], S[c + 3]);
    }
}

template <typename T>
static void launch_rec(const FwdPlan& pl, const void* Q, const void* K, const void* V, const float* alpha,
                       const float* beta, const uint8_t* mask, const float* S0, float* S_final,
                       float* O_la, float* snap, hipStream_t st) {
    dim3 grid(pl.d / REC_ROWS, pl.BHG);
    if (pl.d == 64)
        hipLaunchKernelGGL((gdn_recurrent_kernel<T, 64>), grid, dim3(REC_THREADS), 0, st, (const T*)Q,
                           (const T*)K, (const T*)V, alpha, beta, mask, S0, S_final, O_la, snap, pl.L, pl.la_scale,
                           pl.linear_op, pl.freeze_on_softmax, pl.G, pl.inner_chunk == 1, pl.RC);
    else
        hipLaunchKernelGGL((gdn_recurrent_kernel<T, 128>), grid, dim3(REC_THREADS), 0, st, (const T*)Q,
                           (const T*)K, (const T*)V, alpha, beta, mask, S0, S_final, O_la, snap, pl.L, pl.la_scale,
                           pl.linear_op, pl.freeze_on_softmax, pl.G, pl.inner_chunk == 1, pl.RC);
}

nats_status launch_gdn_recurrent(const FwdPlan& pl, const void* Q, const void* K, const void* V,
                                 const float* alpha, const float* beta, const uint8_t* mask,
                                 const float* S0, float* S_final, float* O_la, float* snap, hipStream_t st) {
    if (pl.dtype == NATS_BF16)
        launch_rec<bf16_t>(pl, Q, K, V, alpha, beta, mask, S0, S_final, O_la, snap, st);
    else
        launch_rec<float>(pl, Q, K, V, alpha, beta, mask, S0, S_final, O_la, snap, st);
    return check_launch("gdn_recurrent");
}

}  // namespace nats
