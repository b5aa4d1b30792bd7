// Softmax branch over the compacted keys, fp32 arithmetic, with the merge epilogue.
//   o_nla[t] = softmax_{c < cnt[t]}(scale * q_t . Kc[c]) Vc        (Eq. 11 under the mask of Eq. 12:
//   the keys visible to query t are exactly the first cnt[t] rows of the compacted cache)
//   O[t] = O_la[t] + o_nla[t]                                       (Section 4.1), or
//   O[t] = w_nla RMSNorm(o_nla[t]) + w_la RMSNorm(O_la[t])          (Eq. 21)
// Rows with cnt[t] == 0 give o_nla = 0, lse = -inf.
//
// A block owns 64 consecutive queries; 4 adjacent lanes share one query row and
// each keeps a quarter of q and of the output accumulator in registers.  Key/value
// tiles of SM_BN compacted rows are staged in LDS as fp32; all lanes with the same
// quarter read the same LDS address (broadcast).  Online max/sum in blocks of 8 keys.
//
// This is the NATS_MATH_FP32 path; the bf16 throughput path is the MFMA flash kernel.
#include <math.h>

#include "nats_common.h"

namespace nats {

constexpr int SM_BM = 64;       // queries per block
constexpr int SM_THREADS = 256; // 4 lanes per query
constexpr int SM_BN = 32;       // compacted keys per LDS tile
constexpr int SM_KB = 8;        // keys per online-softmax step

template <typename T, int D>
__global__ __launch_bounds__(SM_THREADS) void softmax_fp32_kernel(
    const T* __restrict__ Q, const T* __restrict__ Kc, const T* __restrict__ Vc,
    const T* __restrict__ K, const T* __restrict__ V, int chunk_routing, const int32_t* __restrict__ cnt, const float* __restrict__ O_la, const float* __restrict__ w_nla,
    const float* __restrict__ w_la, T* __restrict__ O, float* __restrict__ O_nla_out,
    float* __restrict__ lse_out, int L, float scale, int combine_mode, float eps, int G, int qk_per_out_head,
    int own_chunk) {
    constexpr int DP = D / 4;       // elements of a row per lane
    constexpr int DPP = DP + 4;     // padded quarter stride (floats): quarters land in different banks
    constexpr int EPL = Vec16<T>::N;
    __shared__ __align__(16) float s_k[SM_BN][4 * DPP];
    __shared__ __align__(16) float s_v[SM_BN][4 * DPP];

    const int bh = blockIdx.y;
    const int q0 = (gridDim.x - 1 - blockIdx.x) * SM_BM;   // later queries see more keys: the long blocks go first
    const int tid = threadIdx.x;
    const int r = tid >> 2, part = tid & 3;
    const int t = q0 + r;
    // bh counts output heads; the G heads of a group share the counts of linear head bh / G, and take their
    // queries (and the raw keys of their own chunk) from it unless the softmax heads have their own
    const size_t tokb = (size_t)bh * L, tokb_lin = (size_t)(bh / G) * L;
    const size_t tokb_qk = qk_per_out_head ? tokb : tokb_lin;
    const size_t row_off = (tokb + t) * D + part * DP;

    float q[DP], acc[DP];
#pragma unroll
    for (int c = 0; c < DP; c += EPL) Vec16<T>::load(Q + (tokb_qk + t) * D + part * DP + c, q + c);
#pragma unroll
    for (int c = 0; c < DP; ++c) { q[c] *= scale; acc[c] = 0.f; }
    float m_run = -INFINITY, l_run = 0.f;

    // Routing per token: the first cnt[t] compacted rows are visible.  Routing per chunk (chunk_routing = tokens
    // per routing chunk, 64 or 128): a block's 64 queries lie in one chunk, which starts at cs; they see the
    // compacted rows of earlier chunks, cnt at the last token before the chunk, and then, causally, the chunk's own
    // rows of K and V.
    const int cs = chunk_routing ? (q0 & ~(chunk_routing - 1)) : 0;
    const int my_cnt = chunk_routing ? (cs > 0 ? cnt[tokb_lin + cs - 1] : 0) : cnt[tokb_lin + t];
    const int n_hi = chunk_routing ? my_cnt : cnt[tokb_lin + q0 + SM_BM - 1];  // cnt is non-decreasing: the tile's bound

    // One tile of SM_BN rows of (Ks, Vs) starting at row0, the first n_rows of which exist; this
    // query sees the first `mine` of them.
    auto tile = [&](const T* Ks, size_t kbase, const T* Vs, int row0, int n_rows, int mine) {
        __syncthreads();
        for (int e = tid * EPL; e < SM_BN * D; e += SM_THREADS * EPL) {
            const int i = e / D, c = e % D;
            float tk[EPL], tv[EPL];
            if (i < n_rows) {
                Vec16<T>::load(Ks + (kbase + row0 + i) * D + c, tk);
                Vec16<T>::load(Vs + (tokb + row0 + i) * D + c, tv);
            } else {
#pragma unroll
                for (int j = 0; j < EPL; ++j) { tk[j] = 0.f; tv[j] = 0.f; }
            }
            const int pq = c / DP, pc = c % DP;   // EPL divides DP: a 16-byte group stays in one quarter
#pragma unroll
            for (int j = 0; j < EPL; ++j) {
                s_k[i][pq * DPP + pc + j] = tk[j];
                s_v[i][pq * DPP + pc + j] = tv[j];
            }
        }
        __syncthreads();

        for (int kb = 0; kb < SM_BN; kb += SM_KB) {
            if (kb >= mine) break;
            float s[SM_KB];
#pragma unroll
            for (int j = 0; j < SM_KB; ++j) {
                const float* kr = &s_k[kb + j][part * DPP];
                float dot = 0.f;
#pragma unroll
                for (int c = 0; c < DP; c += 4) {
                    const float4 k4 = *reinterpret_cast<const float4*>(kr + c);
                    dot += q[c] * k4.x + q[c + 1] * k4.y + q[c + 2] * k4.z + q[c + 3] * k4.w;
                }
                dot = lane_group_sum<4>(dot);
                s[j] = (kb + j < mine) ? dot : -INFINITY;
            }
            float bm = s[0];
#pragma unroll
            for (int j = 1; j < SM_KB; ++j) bm = fmaxf(bm, s[j]);
            const float m_new = fmaxf(m_run, bm);      // finite: row kb is visible
            const float corr = expf(m_run - m_new);    // exp(-inf) = 0 on the first step
            float p[SM_KB], psum = 0.f;
#pragma unroll
            for (int j = 0; j < SM_KB; ++j) { p[j] = expf(s[j] - m_new); psum += p[j]; }
            l_run = l_run * corr + psum;
            m_run = m_new;
#pragma unroll
            for (int c = 0; c < DP; ++c) acc[c] *= corr;
#pragma unroll
            for (int j = 0; j < SM_KB; ++j) {
                const float* vr = &s_v[kb + j][part * DPP];
#pragma unroll
                for (int c = 0; c < DP; c += 4) {
                    const float4 v4 = *reinterpret_cast<const float4*>(vr + c);
                    acc[c] += p[j] * v4.x; acc[c + 1] += p[j] * v4.y;
                    acc[c + 2] += p[j] * v4.z; acc[c + 3] += p[j] * v4.w;
                }
            }
        }
    };
    for (int c0 = 0; c0 < n_hi; c0 += SM_BN) tile(Kc, tokb, Vc, c0, min(SM_BN, n_hi - c0), my_cnt - c0);
    if (chunk_routing && own_chunk)   // the chunk's own rows cs .. q0 + 63 of K and V: query t sees rows <= t
        for (int row0 = cs; row0 < q0 + SM_BM; row0 += SM_BN) tile(K, tokb_qk, V, row0, SM_BN, t + 1 - row0);

    // ---- epilogue: normalise, optional branch outputs, merge, store -----------------------
    const float inv_l = (l_run > 0.f) ? 1.f / l_run : 0.f;
#pragma unroll
    for (int c = 0; c < DP; ++c) acc[c] *= inv_l;
    if (lse_out != nullptr && part == 0)
        lse_out[(size_t)bh * L + t] = (l_run > 0.f) ? m_run + logf(l_run) : -INFINITY;
    if (O_nla_out != nullptr) {
#pragma unroll
        for (int c = 0; c < DP; c += 4)
            *reinterpret_cast<float4*>(O_nla_out + row_off + c) =
                make_float4(acc[c], acc[c + 1], acc[c + 2], acc[c + 3]);
    }
    if (O == nullptr) return;   // the caller wanted the branch output and lse only (backward pass)
    float la[DP];
#pragma unroll
    for (int c = 0; c < DP; c += 4) {
        const float4 x = *reinterpret_cast<const float4*>(O_la + row_off + c);
        la[c] = x.x; la[c + 1] = x.y; la[c + 2] = x.z; la[c + 3] = x.w;
    }
    float out[DP];
    if (combine_mode == 0) {
#pragma unroll
        for (int c = 0; c < DP; ++c) out[c] = la[c] + acc[c];
    } else if (combine_mode == 1) {   // Eq. 21: each branch normalised, then weighted
        float ss_la = 0.f, ss_nla = 0.f;
#pragma unroll
        for (int c = 0; c < DP; ++c) { ss_la += la[c] * la[c]; ss_nla += acc[c] * acc[c]; }
        ss_la = lane_group_sum<4>(ss_la);
        ss_nla = lane_group_sum<4>(ss_nla);
        const float wn = (w_nla ? w_nla[(size_t)bh * L + t] : 0.5f) / sqrtf(ss_nla / D + eps);
        const float wl = (w_la ? w_la[(size_t)bh * L + t] : 0.5f) / sqrtf(ss_la / D + eps);
#pragma unroll
        for (int c = 0; c < DP; ++c) out[c] = wn * acc[c] + wl * la[c];
    } else {                          // one normalisation of the (weighted) sum
        const float wn = w_nla ? w_nla[(size_t)bh * L + t] : 1.f, wl = w_la ? w_la[(size_t)bh * L + t] : 1.f;
        float ss = 0.f;
#pragma unroll
        for (int c = 0; c < DP; ++c) { out[c] = wn * acc[c] + wl * la[c]; ss += out[c] * out[c]; }
        ss = lane_group_sum<4>(ss);
        const float inv = 1.f / sqrtf(ss / D + eps);
#pragma unroll
        for (int c = 0; c < DP; ++c) out[c] *= inv;
    }
#pragma unroll
    for (int c = 0; c < DP; c += EPL) Vec16<T>::store(O + row_off + c, out + c);
}

template <typename T>
static void launch_sm(const FwdPlan& pl, const void* Q, const void* Kc, const void* Vc, const void* K,
                      const void* V, const int32_t* cnt,
                      const float* O_la, const float* w_nla, const float* w_la, void* O, float* O_nla_out,
                      float* lse_out, hipStream_t st) {
    dim3 grid(pl.L / SM_BM, pl.BHG);
    if (pl.d == 64)
        hipLaunchKernelGGL((softmax_fp32_kernel<T, 64>), grid, dim3(SM_THREADS), 0, st, (const T*)Q,
                           (const T*)Kc, (const T*)Vc, (const T*)K, (const T*)V, pl.routing == NATS_ROUTE_CHUNK ? pl.RC : 0, cnt,
                           O_la, w_nla, w_la, (T*)O, O_nla_out, lse_out,
                           pl.L, pl.softmax_scale, pl.combine_mode, pl.rms_eps, pl.G, pl.qk_per_out_head, pl.inner_chunk != 2);
    else
        hipLaunchKernelGGL((softmax_fp32_kernel<T, 128>), grid, dim3(SM_THREADS), 0, st, (const T*)Q,
                           (const T*)Kc, (const T*)Vc, (const T*)K, (const T*)V, pl.routing == NATS_ROUTE_CHUNK ? pl.RC : 0, cnt,
                           O_la, w_nla, w_la, (T*)O, O_nla_out, lse_out,
                           pl.L, pl.softmax_scale, pl.combine_mode, pl.rms_eps, pl.G, pl.qk_per_out_head, pl.inner_chunk != 2);
}

nats_status launch_softmax_fp32(const FwdPlan& pl, const void* Q, const void* Kc, const void* Vc,
                                const void* K, const void* V, const int32_t* cnt, const float* O_la, const float* w_nla,
                                const float* w_la, void* O, float* O_nla_out, float* lse_out,
                                hipStream_t st) {
    if (pl.dtype == NATS_BF16)
        launch_sm<bf16_t>(pl, Q, Kc, Vc, K, V, cnt, O_la, w_nla, w_la, O, O_nla_out, lse_out, st);
    else
        launch_sm<float>(pl, Q, Kc, Vc, K, V, cnt, O_la, w_nla, w_la, O, O_nla_out, lse_out, st);
    return check_launch("softmax_fp32");
}

}  // namespace nats
