// Softmax branch over the compacted keys on MFMA, with the merge epilogue.
//   o_nla[t] = softmax_{c < cnt[t]}(scale * q_t . Kc[c]) Vc      (Eq. 11 under the column mask of
//   Eq. 12: query t sees exactly the first cnt[t] rows of the compacted key/value cache)
//   O[t] = O_la[t] + o_nla[t]  (Section 4.1)   or   w_nla RMSNorm(o_nla[t]) + w_la RMSNorm(O_la[t])  (Eq. 21)
//
// Flash-style: a block owns FL_BM = 128 consecutive queries (4 wavefronts x 32), walks the
// key tiles of 64 compacted rows that its last query can see, and keeps running max / sum /
// output in registers.  Everything is computed transposed so that no operand has to be
// re-laid out between the two products:
//   S^T [key x query] = Kc Q^T     bf16 MFMA (inputs exact), A = K tile from LDS, B = Q held in registers
//   O^T [d_v x query] += V^T P^T   fp16 MFMA, A = V^T tile from LDS (written transposed, fp16, by the
//                                  compaction kernel), B = P^T straight from the S^T accumulators:
//                                  a result tile gives each lane 4 consecutive keys of one query, and two
//                                  such tiles fill the 8 contraction slots of one lane (the V^T fragment
//                                  is read with the same slot -> key map).
// A query is one MFMA column, so its max / sum live in the 4 lanes {l, l+16, l+32, l+48}:
// two xor-shuffles per reduction.  P is rounded to fp16 (2^-12), not bf16: with few visible
// keys a single p v term dominates and bf16's 2^-9 would exceed the parity bar.
//
// MFMA-bound on its tiles: 4 d FLOP per visible (query, key) pair.
#include <math.h>

#include "mfma_util.h"
#include "nats_common.h"

namespace nats {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));

constexpr int FL_THREADS = 256;
constexpr int FL_NQ = 2;                 // 16-query MFMA columns per wavefront
constexpr int FL_BM = 4 * 16 * FL_NQ;    // queries per block
constexpr int FL_BN = 64;                // compacted keys per tile

__device__ __forceinline__ f32x4 mfma16_bf16(uint4 a, uint4 b, f32x4 c) {
    union { uint4 u; bf16x8_t v; } ua, ub;
    ua.u = a; ub.u = b;
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(ua.v, ub.v, c, 0, 0, 0);
}

__device__ __forceinline__ float quad_max(float x) {   // over lanes l, l^16, l^32, l^48
    x = fmaxf(x, __shfl_xor(x, 16));
    return fmaxf(x, __shfl_xor(x, 32));
}
__device__ __forceinline__ float quad_sum(float x) {
    x += __shfl_xor(x, 16);
    return x + __shfl_xor(x, 32);
}

template <int D>
__global__ __launch_bounds__(FL_THREADS) void flash_softmax_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ Kc, const half_t* __restrict__ VhT,
    const int32_t* __restrict__ cnt, const float* __restrict__ O_la, const float* __restrict__ w_nla,
    const float* __restrict__ w_la, bf16_t* __restrict__ O, float* __restrict__ O_nla_out,
    float* __restrict__ lse_out, int L, float scale, int combine_mode, float eps) {
    constexpr int RS = D + LDS_PAD;      // K tile rows (bf16 elements)
    constexpr int TS = FL_BN + LDS_PAD;  // V^T tile rows (fp16 elements)
    constexpr int KS_D = D / 32;
    constexpr int DT = D / 16;           // 16-row d_v tiles
    __shared__ __align__(16) uint16_t Ks[FL_BN * RS];
    __shared__ __align__(16) half_t Vs[D * TS];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    const int bh = blockIdx.y;
    const int q0 = blockIdx.x * FL_BM;
    const size_t tokbase = (size_t)bh * L;
    const float scale2 = scale * 1.44269504088896341f;   // logits in base-2 units

    // ---- this wavefront's queries: fragments of Q^T (B operand) and visible-key counts ----------
    uint4 qf[FL_NQ][KS_D];
    int my_cnt[FL_NQ], q_row[FL_NQ];
    int wave_hi = 0;
#pragma unroll
    for (int nq = 0; nq < FL_NQ; ++nq) {
        const int q = q0 + (wave * FL_NQ + nq) * 16 + l16;
        q_row[nq] = q;
        const bool live = q < L;
        my_cnt[nq] = live ? cnt[tokbase + q] : 0;
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks)
            qf[nq][ks] = live ? *reinterpret_cast<const uint4*>(Q + (tokbase + q) * D + 32 * ks + 8 * lq)
                              : make_uint4(0, 0, 0, 0);
        wave_hi = max(wave_hi, my_cnt[nq]);
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) wave_hi = max(wave_hi, __shfl_xor(wave_hi, off));
    const int q_last = min(q0 + FL_BM, L) - 1;
    const int n_hi = cnt[tokbase + q_last];   // cnt is non-decreasing: bound for the whole block

    f32x4 accO[FL_NQ][DT];
    float m_run[FL_NQ], l_run[FL_NQ];
#pragma unroll
    for (int nq = 0; nq < FL_NQ; ++nq) {
        m_run[nq] = -INFINITY;
        l_run[nq] = 0.f;
#pragma unroll
        for (int t = 0; t < DT; ++t) accO[nq][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const int n_tiles = (n_hi + FL_BN - 1) / FL_BN;
    for (int kt = 0; kt < n_tiles; ++kt) {
        __syncthreads();
        {   // stage K tile (bf16 rows) and V^T tile (fp16, [d_v][key]) -- straight 16-byte copies
            const bf16_t* Kt = Kc + (tokbase + (size_t)kt * FL_BN) * D;
            for (int e = tid; e < FL_BN * D / 8; e += FL_THREADS) {
                const int row = e / (D / 8), c8 = e % (D / 8);
                *reinterpret_cast<uint4*>(Ks + row * RS + c8 * 8) =
                    *reinterpret_cast<const uint4*>(Kt + row * D + c8 * 8);
            }
            const half_t* Vt = VhT + (tokbase + (size_t)kt * FL_BN) * D;   // tile kt: [D][64]
            for (int e = tid; e < D * FL_BN / 8; e += FL_THREADS) {
                const int row = e >> 3, c8 = e & 7;
                *reinterpret_cast<uint4*>(Vs + row * TS + c8 * 8) =
                    *reinterpret_cast<const uint4*>(Vt + row * FL_BN + c8 * 8);
            }
        }
        __syncthreads();
        if (kt * FL_BN >= wave_hi) continue;   // nothing visible to this wavefront in this tile (uniform)

        // ---- S^T = K Q^T for 64 keys x 16*FL_NQ queries ------------------------------------------
        f32x4 accS[FL_NQ][4];
#pragma unroll
        for (int nq = 0; nq < FL_NQ; ++nq)
#pragma unroll
            for (int m = 0; m < 4; ++m) accS[nq][m] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks)
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const uint4 fk = *reinterpret_cast<const uint4*>(Ks + (16 * m + l16) * RS + 32 * ks + 8 * lq);
#pragma unroll
                for (int nq = 0; nq < FL_NQ; ++nq) accS[nq][m] = mfma16_bf16(fk, qf[nq][ks], accS[nq][m]);
            }

        // ---- online softmax per query column; P^T fragments ------------------------------------------
        half8 pf[FL_NQ][2];
#pragma unroll
        for (int nq = 0; nq < FL_NQ; ++nq) {
            float tmax = -INFINITY;
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int c = kt * FL_BN + 16 * m + 4 * lq + j;
                    const float s = (c < my_cnt[nq]) ? accS[nq][m][j] * scale2 : -INFINITY;
                    accS[nq][m][j] = s;
                    tmax = fmaxf(tmax, s);
                }
            tmax = quad_max(tmax);
            const float m_new = fmaxf(m_run[nq], tmax);
            const bool any = m_new > -INFINITY;
            const float corr = any ? __builtin_amdgcn_exp2f(m_run[nq] - m_new) : 1.f;
            float psum = 0.f;
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float p = any ? __builtin_amdgcn_exp2f(accS[nq][m][j] - m_new) : 0.f;
                    accS[nq][m][j] = p;
                    psum += p;
                }
            psum = quad_sum(psum);
            l_run[nq] = l_run[nq] * corr + psum;
            m_run[nq] = m_new;
#pragma unroll
            for (int t = 0; t < DT; ++t) {
                accO[nq][t][0] *= corr; accO[nq][t][1] *= corr; accO[nq][t][2] *= corr; accO[nq][t][3] *= corr;
            }
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {   // contraction step s2: slots 0-3 <- key tile 2 s2, 4-7 <- 2 s2 + 1
                const half4 lo = to_half4(accS[nq][2 * s2]), hi = to_half4(accS[nq][2 * s2 + 1]);
                pf[nq][s2] = half8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
            }
        }

        // ---- O^T += V^T P^T -----------------------------------------------------------------------
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const half_t* vrow = Vs + (16 * t + l16) * TS + 32 * s2 + 4 * lq;
                const half4 lo = lds_read4(vrow), hi = lds_read4(vrow + 16);
                const half8 fv = half8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
#pragma unroll
                for (int nq = 0; nq < FL_NQ; ++nq) accO[nq][t] = mfma16(fv, pf[nq][s2], accO[nq][t]);
            }
    }

    // ---- epilogue: normalise, optional branch outputs, merge with the linear branch, store --------
#pragma unroll
    for (int nq = 0; nq < FL_NQ; ++nq) {
        const int q = q_row[nq];
        if (q >= L) continue;
        const float l = l_run[nq];
        const float inv_l = l > 0.f ? 1.f / l : 0.f;
        if (lse_out != nullptr && lq == 0)
            lse_out[tokbase + q] = l > 0.f ? (m_run[nq] + log2f(l)) * 0.69314718055994531f : -INFINITY;
        float ss_la = 0.f, ss_nla = 0.f;
        float4 la[DT];
#pragma unroll
        for (int t = 0; t < DT; ++t) {
            accO[nq][t][0] *= inv_l; accO[nq][t][1] *= inv_l; accO[nq][t][2] *= inv_l; accO[nq][t][3] *= inv_l;
            const size_t off = (tokbase + q) * D + 16 * t + 4 * lq;
            la[t] = *reinterpret_cast<const float4*>(O_la + off);
            if (O_nla_out != nullptr)
                *reinterpret_cast<float4*>(O_nla_out + off) =
                    make_float4(accO[nq][t][0], accO[nq][t][1], accO[nq][t][2], accO[nq][t][3]);
            ss_la += la[t].x * la[t].x + la[t].y * la[t].y + la[t].z * la[t].z + la[t].w * la[t].w;
            ss_nla += accO[nq][t][0] * accO[nq][t][0] + accO[nq][t][1] * accO[nq][t][1] +
                      accO[nq][t][2] * accO[nq][t][2] + accO[nq][t][3] * accO[nq][t][3];
        }
        float wn = 1.f, wl = 1.f;
        if (combine_mode != 0) {
            ss_la = quad_sum(ss_la);
            ss_nla = quad_sum(ss_nla);
            wn = (w_nla ? w_nla[tokbase + q] : 0.5f) / sqrtf(ss_nla / D + eps);
            wl = (w_la ? w_la[tokbase + q] : 0.5f) / sqrtf(ss_la / D + eps);
        }
#pragma unroll
        for (int t = 0; t < DT; ++t) {
            const float o0 = wn * accO[nq][t][0] + wl * la[t].x, o1 = wn * accO[nq][t][1] + wl * la[t].y;
            const float o2 = wn * accO[nq][t][2] + wl * la[t].z, o3 = wn * accO[nq][t][3] + wl * la[t].w;
            uint2 w;
            w.x = (uint32_t)f32_to_bf16_bits(o0) | ((uint32_t)f32_to_bf16_bits(o1) << 16);
            w.y = (uint32_t)f32_to_bf16_bits(o2) | ((uint32_t)f32_to_bf16_bits(o3) << 16);
            *reinterpret_cast<uint2*>(O + (tokbase + q) * D + 16 * t + 4 * lq) = w;
        }
    }
}

nats_status launch_flash_softmax(const FwdPlan& pl, const void* Q, const void* Kc, const void* VhT,
                                 const int32_t* cnt, const float* O_la, const float* w_nla,
                                 const float* w_la, void* O, float* O_nla_out, float* lse_out,
                                 hipStream_t st) {
    dim3 grid((pl.L + FL_BM - 1) / FL_BM, pl.BH);
    if (pl.d == 64)
        hipLaunchKernelGGL((flash_softmax_kernel<64>), grid, dim3(FL_THREADS), 0, st, (const bf16_t*)Q,
                           (const bf16_t*)Kc, (const half_t*)VhT, cnt, O_la, w_nla, w_la, (bf16_t*)O,
                           O_nla_out, lse_out, pl.L, pl.softmax_scale, pl.combine_mode, pl.rms_eps);
    else
        hipLaunchKernelGGL((flash_softmax_kernel<128>), grid, dim3(FL_THREADS), 0, st, (const bf16_t*)Q,
                           (const bf16_t*)Kc, (const half_t*)VhT, cnt, O_la, w_nla, w_la, (bf16_t*)O,
                           O_nla_out, lse_out, pl.L, pl.softmax_scale, pl.combine_mode, pl.rms_eps);
    return check_launch("flash_softmax");
}

}  // namespace nats
