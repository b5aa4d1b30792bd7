// Backward of the softmax branch over the compacted keys (Section 4.2), fp32 arithmetic.
// With P_ic = exp(scale q_i . Kc[c] - lse_i) for the rows c < cnt[i] that query i sees (Eq. 11-12),
// dP_ic = do_i . Vc[c] and D_i = do_i . o_nla_i:
//     dS_ic = P_ic (dP_ic - D_i)                 (Eq. 15: this is also the gradient of the mask entry)
//     dq_i  = scale sum_c dS_ic Kc[c]
//     dKc_c = scale sum_i dS_ic q_i,   dVc_c = sum_i P_ic do_i,   g_c = sum_i dS_ic   (Eq. 15 column sum;
//                                                                  Eq. 16 adds the columns of a chunk)
// and the rows of dKc, dVc, g go back to the token positions idx[c] they were gathered from.
//
// Two kernels, both laid out like the fp32 forward kernel (4 adjacent lanes share a row and own a
// quarter of its d elements; the other operand is staged in LDS as fp32 and read as a broadcast):
//   softmax_bwd_dq : a block owns 64 queries and walks the key tiles they see; also writes D_i
//   softmax_bwd_dkv: a block owns 64 compacted keys and walks the queries from the first one that can
//                    see its first key to the end of the sequence
// Nothing is accumulated across blocks: results are deterministic.
#include <math.h>

#include "nats_common.h"

namespace nats {

constexpr int SB_ROWS = 64;      // rows (queries or keys) per block
constexpr int SB_THREADS = 256;  // 4 lanes per row
constexpr int SB_TILE = 32;      // rows of the other operand per LDS tile

template <typename T, int D>
__global__ __launch_bounds__(SB_THREADS) void softmax_bwd_dq_kernel(
    const T* __restrict__ Q, const T* __restrict__ Kc, const T* __restrict__ Vc, const T* __restrict__ dO,
    const int32_t* __restrict__ cnt, const float* __restrict__ O_nla, const float* __restrict__ lse,
    float* __restrict__ Dvec, float* __restrict__ dQ, int L, float scale) {
    constexpr int DP = D / 4, DPP = DP + 4, EPL = Vec16<T>::N;
    __shared__ __align__(16) float s_k[SB_TILE][4 * DPP];
    __shared__ __align__(16) float s_v[SB_TILE][4 * DPP];
    const int bh = blockIdx.y, q0 = blockIdx.x * SB_ROWS, tid = threadIdx.x;
    const int r = tid >> 2, part = tid & 3, t = q0 + r;
    const size_t tokb = (size_t)bh * L;
    const size_t row_off = (tokb + t) * D + part * DP;

    float q[DP], dout[DP], acc[DP];
#pragma unroll
    for (int c = 0; c < DP; c += EPL) { Vec16<T>::load(Q + row_off + c, q + c); Vec16<T>::load(dO + row_off + c, dout + c); }
    float Di = 0.f;
#pragma unroll
    for (int c = 0; c < DP; c += 4) {
        const float4 o = *reinterpret_cast<const float4*>(O_nla + row_off + c);
        Di += dout[c] * o.x + dout[c + 1] * o.y + dout[c + 2] * o.z + dout[c + 3] * o.w;
    }
    Di += __shfl_xor(Di, 1);
    Di += __shfl_xor(Di, 2);
    if (part == 0) Dvec[tokb + t] = Di;
#pragma unroll
    for (int c = 0; c < DP; ++c) { q[c] *= scale; acc[c] = 0.f; }
    const float lse_t = lse[tokb + t];
    const int my_cnt = cnt[tokb + t];
    const int n_hi = cnt[tokb + q0 + SB_ROWS - 1];   // cnt is non-decreasing: the block's bound

    for (int c0 = 0; c0 < n_hi; c0 += SB_TILE) {
        const int n_rows = min(SB_TILE, n_hi - c0), mine = my_cnt - c0;
        __syncthreads();
        for (int e = tid * EPL; e < SB_TILE * D; e += SB_THREADS * EPL) {
            const int i = e / D, c = e % D;
            float tk[EPL], tv[EPL];
            if (i < n_rows) {
                const size_t src = (tokb + c0 + i) * D + c;
                Vec16<T>::load(Kc + src, tk);
                Vec16<T>::load(Vc + src, tv);
            } else {
#pragma unroll
                for (int j = 0; j < EPL; ++j) { tk[j] = 0.f; tv[j] = 0.f; }
            }
            const int pq = c / DP, pc = c % DP;
#pragma unroll
            for (int j = 0; j < EPL; ++j) { s_k[i][pq * DPP + pc + j] = tk[j]; s_v[i][pq * DPP + pc + j] = tv[j]; }
        }
        __syncthreads();
        for (int j = 0; j < SB_TILE; ++j) {
            if (j >= n_rows) break;                  // uniform
            const float* kr = &s_k[j][part * DPP];
            const float* vr = &s_v[j][part * DPP];
            float s = 0.f, dp = 0.f;
#pragma unroll
            for (int c = 0; c < DP; c += 4) {
                const float4 k4 = *reinterpret_cast<const float4*>(kr + c);
                const float4 v4 = *reinterpret_cast<const float4*>(vr + c);
                s += q[c] * k4.x + q[c + 1] * k4.y + q[c + 2] * k4.z + q[c + 3] * k4.w;
                dp += dout[c] * v4.x + dout[c + 1] * v4.y + dout[c + 2] * v4.z + dout[c + 3] * v4.w;
            }
            s += __shfl_xor(s, 1); s += __shfl_xor(s, 2);
            dp += __shfl_xor(dp, 1); dp += __shfl_xor(dp, 2);
            const float p = (j < mine) ? expf(s - lse_t) : 0.f;   // a row that sees nothing has mine <= 0
            const float ds = p * (dp - Di);
#pragma unroll
            for (int c = 0; c < DP; c += 4) {
                const float4 k4 = *reinterpret_cast<const float4*>(kr + c);
                acc[c] += ds * k4.x; acc[c + 1] += ds * k4.y; acc[c + 2] += ds * k4.z; acc[c + 3] += ds * k4.w;
            }
        }
    }
#pragma unroll
    for (int c = 0; c < DP; c += 4)
        *reinterpret_cast<float4*>(dQ + row_off + c) =
            make_float4(scale * acc[c], scale * acc[c + 1], scale * acc[c + 2], scale * acc[c + 3]);
}

template <typename T, int D>
__global__ __launch_bounds__(SB_THREADS) void softmax_bwd_dkv_kernel(
    const T* __restrict__ Q, const T* __restrict__ Kc, const T* __restrict__ Vc, const T* __restrict__ dO,
    const int32_t* __restrict__ cnt, const int32_t* __restrict__ idx, const int32_t* __restrict__ n_s,
    const float* __restrict__ lse, const float* __restrict__ Dvec, float* __restrict__ dk_part,
    float* __restrict__ dv_part, float* __restrict__ g_part, int L, float scale) {
    constexpr int DP = D / 4, DPP = DP + 4, EPL = Vec16<T>::N;
    __shared__ __align__(16) float s_q[SB_TILE][4 * DPP];
    __shared__ __align__(16) float s_do[SB_TILE][4 * DPP];
    __shared__ float s_lse[SB_TILE], s_D[SB_TILE];
    __shared__ int s_cnt[SB_TILE];
    const int bh = blockIdx.y, c0 = blockIdx.x * SB_ROWS, tid = threadIdx.x;
    const int n_keys = n_s[bh];
    if (c0 >= n_keys) return;                          // uniform: this tile holds no key
    const int kr = tid >> 2, part = tid & 3, c = c0 + kr;
    const bool valid = c < n_keys;
    const size_t tokb = (size_t)bh * L;
    const size_t key_off = (tokb + (valid ? c : c0)) * D + part * DP;

    float k[DP], v[DP], dk[DP], dv[DP];
#pragma unroll
    for (int e = 0; e < DP; e += EPL) { Vec16<T>::load(Kc + key_off + e, k + e); Vec16<T>::load(Vc + key_off + e, v + e); }
#pragma unroll
    for (int e = 0; e < DP; ++e) { k[e] *= scale; dk[e] = 0.f; dv[e] = 0.f; }
    float g = 0.f;

    // The queries that see the tile's first key, in tiles; the blocks of the tile (blockIdx.z) take equal shares
    // of them: the first key tile of a head is seen by every query, and one block walking all of them was the
    // whole kernel's run time.
    const int i_first = idx[tokb + c0] & ~(SB_TILE - 1);
    const int n_tiles = (L - i_first) / SB_TILE, seg = blockIdx.z, n_seg = gridDim.z;
    const int i_lo = i_first + (int)((long long)n_tiles * seg / n_seg) * SB_TILE;
    const int i_hi = i_first + (int)((long long)n_tiles * (seg + 1) / n_seg) * SB_TILE;
    for (int i0 = i_lo; i0 < i_hi; i0 += SB_TILE) {
        __syncthreads();
        for (int e = tid * EPL; e < SB_TILE * D; e += SB_THREADS * EPL) {
            const int i = e / D, col = e % D;
            float tq[EPL], td[EPL];
            const size_t src = (tokb + i0 + i) * D + col;     // L is a multiple of the tile
            Vec16<T>::load(Q + src, tq);
            Vec16<T>::load(dO + src, td);
            const int pq = col / DP, pc = col % DP;
#pragma unroll
            for (int j = 0; j < EPL; ++j) { s_q[i][pq * DPP + pc + j] = tq[j]; s_do[i][pq * DPP + pc + j] = td[j]; }
        }
        if (tid < SB_TILE) {
            s_lse[tid] = lse[tokb + i0 + tid];
            s_D[tid] = Dvec[tokb + i0 + tid];
            s_cnt[tid] = cnt[tokb + i0 + tid];
        }
        __syncthreads();
        for (int i = 0; i < SB_TILE; ++i) {
            if (s_cnt[i] <= c0) continue;              // uniform: this query sees none of the tile's keys
            const float* qr = &s_q[i][part * DPP];
            const float* dr = &s_do[i][part * DPP];
            float s = 0.f, dp = 0.f;
#pragma unroll
            for (int e = 0; e < DP; e += 4) {
                const float4 q4 = *reinterpret_cast<const float4*>(qr + e);
                const float4 d4 = *reinterpret_cast<const float4*>(dr + e);
                s += k[e] * q4.x + k[e + 1] * q4.y + k[e + 2] * q4.z + k[e + 3] * q4.w;
                dp += v[e] * d4.x + v[e + 1] * d4.y + v[e + 2] * d4.z + v[e + 3] * d4.w;
            }
            s += __shfl_xor(s, 1); s += __shfl_xor(s, 2);
            dp += __shfl_xor(dp, 1); dp += __shfl_xor(dp, 2);
            const float p = (valid && c < s_cnt[i]) ? expf(s - s_lse[i]) : 0.f;
            const float ds = p * (dp - s_D[i]);
            g += ds;
#pragma unroll
            for (int e = 0; e < DP; e += 4) {
                const float4 q4 = *reinterpret_cast<const float4*>(qr + e);
                const float4 d4 = *reinterpret_cast<const float4*>(dr + e);
                dk[e] += ds * q4.x; dk[e + 1] += ds * q4.y; dk[e + 2] += ds * q4.z; dk[e + 3] += ds * q4.w;
                dv[e] += p * d4.x; dv[e + 1] += p * d4.y; dv[e + 2] += p * d4.z; dv[e + 3] += p * d4.w;
            }
        }
    }
    if (valid) {   // this segment's share, by compacted key; a second kernel adds the shares up in order
        const size_t row = ((size_t)seg * gridDim.y + bh) * L + c;
#pragma unroll
        for (int e = 0; e < DP; e += 4) {
            *reinterpret_cast<float4*>(dk_part + row * D + part * DP + e) = make_float4(dk[e], dk[e + 1], dk[e + 2], dk[e + 3]);
            *reinterpret_cast<float4*>(dv_part + row * D + part * DP + e) = make_float4(dv[e], dv[e + 1], dv[e + 2], dv[e + 3]);
        }
        if (part == 0) g_part[row] = g;
    }
}

// Adds the segments' shares of a compacted key up, in order, and writes the rows of dK, dV (and g_nla) of the
// token the key was gathered from (its linear-branch gradient is zero).  One thread per key and 4 columns.
template <int D>
__global__ __launch_bounds__(256) void softmax_bwd_dkv_combine_kernel(
    const float* __restrict__ dk_part, const float* __restrict__ dv_part, const float* __restrict__ g_part,
    const int32_t* __restrict__ idx, const int32_t* __restrict__ n_s, float* __restrict__ dK, float* __restrict__ dV,
    float* __restrict__ g_nla, int L, int n_seg, float scale) {
    constexpr int TPK = D / 4;                 // threads per key
    const int bh = blockIdx.y, c = blockIdx.x * (256 / TPK) + threadIdx.x / TPK, col = (threadIdx.x % TPK) * 4;
    if (c >= n_s[bh]) return;
    const size_t tokb = (size_t)bh * L;
    float4 k = make_float4(0.f, 0.f, 0.f, 0.f), v = k;
    float g = 0.f;
    for (int s = 0; s < n_seg; ++s) {
        const size_t row = ((size_t)s * gridDim.y + bh) * L + c;
        const float4 a = *reinterpret_cast<const float4*>(dk_part + row * D + col);
        const float4 b = *reinterpret_cast<const float4*>(dv_part + row * D + col);
        k.x += a.x; k.y += a.y; k.z += a.z; k.w += a.w;
        v.x += b.x; v.y += b.y; v.z += b.z; v.w += b.w;
        g += g_part[row];
    }
    const size_t dst = (tokb + idx[tokb + c]) * D + col;
    *reinterpret_cast<float4*>(dK + dst) = make_float4(scale * k.x, scale * k.y, scale * k.z, scale * k.w);
    *reinterpret_cast<float4*>(dV + dst) = v;
    if (col == 0 && g_nla != nullptr) g_nla[tokb + idx[tokb + c]] = g;
}

template <typename T>
static void launch_sb(const FwdPlan& pl, const void* Q, const void* Kc, const void* Vc, const void* dO,
                      const int32_t* cnt, const int32_t* idx, const int32_t* n_s, const float* O_nla, const float* lse,
                      float* Dvec, float* dQ, float* dK, float* dV, float* g_nla, bool dkv, hipStream_t st) {
    dim3 grid(pl.L / SB_ROWS, pl.BH, dkv ? BWD_DKV_SEGMENTS : 1);
#define NATS_SB_LAUNCH(DD)                                                                                          \
    if (!dkv)                                                                                                        \
        hipLaunchKernelGGL((softmax_bwd_dq_kernel<T, DD>), grid, dim3(SB_THREADS), 0, st, (const T*)Q, (const T*)Kc, \
                           (const T*)Vc, (const T*)dO, cnt, O_nla, lse, Dvec, dQ, pl.L, pl.softmax_scale);           \
    else                                                                                                             \
        hipLaunchKernelGGL((softmax_bwd_dkv_kernel<T, DD>), grid, dim3(SB_THREADS), 0, st, (const T*)Q,              \
                           (const T*)Kc, (const T*)Vc, (const T*)dO, cnt, idx, n_s, lse, Dvec, dK, dV, g_nla, pl.L,  \
                           pl.softmax_scale)
    if (pl.d == 64) NATS_SB_LAUNCH(64);
    else NATS_SB_LAUNCH(128);
#undef NATS_SB_LAUNCH
}

// dQ [B,H,L,d] f32 is written (not accumulated); also Dvec [B,H,L]
nats_status launch_softmax_bwd_dq(const FwdPlan& pl, const void* Q, const void* Kc, const void* Vc, const void* dO,
                                  const int32_t* cnt, const float* O_nla, const float* lse, float* Dvec, float* dQ,
                                  hipStream_t st) {
    if (pl.dtype == NATS_BF16)
        launch_sb<bf16_t>(pl, Q, Kc, Vc, dO, cnt, nullptr, nullptr, O_nla, lse, Dvec, dQ, nullptr, nullptr, nullptr, false, st);
    else
        launch_sb<float>(pl, Q, Kc, Vc, dO, cnt, nullptr, nullptr, O_nla, lse, Dvec, dQ, nullptr, nullptr, nullptr, false, st);
    return check_launch("softmax_bwd_dq");
}

// the rows idx[c] of dK, dV [B,H,L,d] f32 (and of g_nla [B,H,L], optional) are overwritten; other rows are left alone.
// dk_part, dv_part: BWD_DKV_SEGMENTS * BH * L * d floats, g_part: BWD_DKV_SEGMENTS * BH * L floats (scratch)
nats_status launch_softmax_bwd_dkv(const FwdPlan& pl, const void* Q, const void* Kc, const void* Vc, const void* dO,
                                   const int32_t* cnt, const int32_t* idx, const int32_t* n_s, const float* lse,
                                   const float* Dvec, float* dK, float* dV, float* g_nla, float* dk_part, float* dv_part,
                                   float* g_part, hipStream_t st) {
    if (pl.dtype == NATS_BF16)
        launch_sb<bf16_t>(pl, Q, Kc, Vc, dO, cnt, idx, n_s, nullptr, lse, const_cast<float*>(Dvec), nullptr, dk_part, dv_part,
                          g_part, true, st);
    else
        launch_sb<float>(pl, Q, Kc, Vc, dO, cnt, idx, n_s, nullptr, lse, const_cast<float*>(Dvec), nullptr, dk_part, dv_part,
                         g_part, true, st);
    nats_status rc = check_launch("softmax_bwd_dkv");
    if (rc != NATS_OK) return rc;
    if (pl.d == 64) {
        dim3 grid((pl.L + 15) / 16, pl.BH);   // 256 / (64 / 4) keys per block
        hipLaunchKernelGGL((softmax_bwd_dkv_combine_kernel<64>), grid, dim3(256), 0, st, dk_part, dv_part, g_part, idx, n_s,
                           dK, dV, g_nla, pl.L, BWD_DKV_SEGMENTS, pl.softmax_scale);
    } else {
        dim3 grid((pl.L + 7) / 8, pl.BH);     // 256 / (128 / 4) keys per block
        hipLaunchKernelGGL((softmax_bwd_dkv_combine_kernel<128>), grid, dim3(256), 0, st, dk_part, dv_part, g_part, idx, n_s,
                           dK, dV, g_nla, pl.L, BWD_DKV_SEGMENTS, pl.softmax_scale);
    }
    return check_launch("softmax_bwd_dkv_combine");
}

}  // namespace nats
