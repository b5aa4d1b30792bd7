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
// For bf16 tensors the second kernel has a form on MFMA (below): its products run on the matrix cores with
// operands that are exact (the bf16 inputs) or split into two fp16 terms (P and dS), so that it meets the same bar.
#include <math.h>

#include "mfma_util.h"
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
    const int bh = blockIdx.y, q0 = (gridDim.x - 1 - blockIdx.x) * SB_ROWS, tid = threadIdx.x;   // long blocks first
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
    Di = lane_group_sum<4>(Di);
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
            s = lane_group_sum<4>(s);
            dp = lane_group_sum<4>(dp);
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
    float* __restrict__ dv_part, float* __restrict__ g_part, int L, float scale, int BH, int n_seg) {
    constexpr int DP = D / 4, DPP = DP + 4, EPL = Vec16<T>::N;
    __shared__ __align__(16) float s_q[SB_TILE][4 * DPP];
    __shared__ __align__(16) float s_do[SB_TILE][4 * DPP];
    __shared__ float s_lse[SB_TILE], s_D[SB_TILE];
    __shared__ int s_cnt[SB_TILE];
    // one-dimensional grid, the key tile slowest (see the MFMA kernel below)
    const int seg = blockIdx.x % n_seg, bh = (blockIdx.x / n_seg) % BH, c0 = (blockIdx.x / n_seg / BH) * SB_ROWS;
    const int tid = threadIdx.x;
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

    // The queries that see the tile's first key, in tiles; the blocks of the tile take equal shares
    // of them: the first key tile of a head is seen by every query, and one block walking all of them was the
    // whole kernel's run time.
    const int i_first = idx[tokb + c0] & ~(SB_TILE - 1);
    const int n_tiles = (L - i_first) / SB_TILE;
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
            s = lane_group_sum<4>(s);
            dp = lane_group_sum<4>(dp);
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
        const size_t row = ((size_t)seg * BH + bh) * L + c;
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
    float* __restrict__ g_nla, int L, int n_seg, float scale, int accumulate) {
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
    if (accumulate) {   // routing per chunk: the token's rows already hold its shares from inside its chunk
        const float4 k0 = *reinterpret_cast<const float4*>(dK + dst), v0 = *reinterpret_cast<const float4*>(dV + dst);
        *reinterpret_cast<float4*>(dK + dst) = make_float4(k0.x + scale * k.x, k0.y + scale * k.y, k0.z + scale * k.z, k0.w + scale * k.w);
        *reinterpret_cast<float4*>(dV + dst) = make_float4(v0.x + v.x, v0.y + v.y, v0.z + v.z, v0.w + v.w);
    } else {
        *reinterpret_cast<float4*>(dK + dst) = make_float4(scale * k.x, scale * k.y, scale * k.z, scale * k.w);
        *reinterpret_cast<float4*>(dV + dst) = v;
    }
    if (col == 0 && g_nla != nullptr) g_nla[tokb + idx[tokb + c]] = g;
}

// ---- dKc, dVc, g on MFMA, bf16 tensors ---------------------------------------------------------------------
// A block owns 64 compacted keys, wavefront w the 16 keys of tile w, and walks the queries that can see them
// in tiles of 64 (its share of them).  Per query tile, with everything a wavefront needs of P and dS
// staying in its own registers:
//   S [q][key] = Q K^T,  dP[q][key] = dO V^T     bf16 MFMA, inputs exact; A = the Q / dO tile (LDS, row-major),
//                                                 B = the wavefront's K / V rows, held in registers
//   P = exp(scale S - lse_q) under the column mask,  dS = P (dP - D_q),  g += column sums of dS      (fp32)
//   dV^T[d][key] += dO^T P,  dK^T[d][key] += Q^T dS   fp16 MFMA; B = P / dS straight from the accumulators: a
//       result tile gives a lane 4 consecutive queries of one key, and two tiles fill the 8 contraction slots of
//       a lane; A = the transposed dO / Q tile (LDS, fp16, columns stored in that slot order).  P and dS enter
//       as hi + lo, two fp16 terms each (two products): their rounding then costs 2^-22, not 2^-11.
constexpr int SBM_QT = 64;       // queries per tile

__device__ __forceinline__ f32x4 sbm_mfma_bf16(u32x4 a, u32x4 b, f32x4 c) {
    typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
}

// column of query q (0..63) in the transposed tiles: the 8 queries {16 (2 mp) + 4 lq + j, 16 (2 mp + 1) + 4 lq + j},
// j < 4, are the contraction slots of lane quarter lq in step mp, and sit side by side
__device__ __forceinline__ int sbm_col(int q) {
    const int mt = q >> 4, lq = (q >> 2) & 3, j = q & 3;
    return (mt >> 1) * 32 + lq * 8 + (mt & 1) * 4 + j;
}
// element (d, col) of a transposed tile [D][TS]: the 8-column groups are xor-swizzled with d / 8, so that the 2-byte
// writes of lanes that hold different d of one query spread over the banks
__device__ __forceinline__ int sbm_at(int d, int col, int TS) {
    return d * TS + ((((col >> 3) ^ (d >> 3)) & 7) << 3) + (col & 7);
}

template <int D>
constexpr int sbm_lds_bytes() { return 2 * SBM_QT * (D + LDS_PAD) * 2 + 2 * D * (SBM_QT + LDS_PAD) * 2 + 3 * SBM_QT * 4; }

template <int D>
__global__ __launch_bounds__(256, 2) void softmax_bwd_dkv_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ Kc, const bf16_t* __restrict__ Vc,
    const bf16_t* __restrict__ dO, const int32_t* __restrict__ cnt, const int32_t* __restrict__ idx,
    const int32_t* __restrict__ n_s, const float* __restrict__ lse, const float* __restrict__ Dvec,
    float* __restrict__ dk_part, float* __restrict__ dv_part, float* __restrict__ g_part, int L, float scale, int BH,
    int n_seg) {
    constexpr int RS = D + LDS_PAD, TS = SBM_QT + LDS_PAD;
    constexpr int KS_D = D / 32, MD = D / 16, NPC = SBM_QT * D / 8 / 256;
    extern __shared__ __align__(16) unsigned char sbm_smem[];
    uint16_t* Qs = reinterpret_cast<uint16_t*>(sbm_smem);                    // bf16, row-major [64][RS]
    uint16_t* dOs = Qs + SBM_QT * RS;
    half_t* QT = reinterpret_cast<half_t*>(dOs + SBM_QT * RS);                // fp16, transposed [D][TS]
    half_t* dOT = QT + D * TS;
    float* s_lse2 = reinterpret_cast<float*>(dOT + D * TS);
    float* s_D = s_lse2 + SBM_QT;
    int* s_cnt = reinterpret_cast<int*>(s_D + SBM_QT);

    // One-dimensional grid, the key tile slowest: the tiles that hold keys (the first ones) are dispatched first,
    // the heaviest of all (tile 0, seen by every query) at the very front; the empty ones follow and exit at once.
    // (With the key tile as the fastest dimension the few working blocks sat between thousands of empty ones,
    // each of which claims a block's LDS and registers before it can exit: 1.2 ms instead of 0.35.)
    const int seg = blockIdx.x % n_seg, bh = (blockIdx.x / n_seg) % BH, c0 = (blockIdx.x / n_seg / BH) * 64;
    const int tid = threadIdx.x;
    const int n_keys = n_s[bh];
    if (c0 >= n_keys) return;                          // uniform: this tile holds no key
    const int lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
    const int c = c0 + 16 * wave + l16;                // this lane's key
    const bool valid = c < n_keys;
    const size_t tokb = (size_t)bh * L;
    const float LOG2E = 1.44269504088896341f;
    const float scale2 = scale * LOG2E;

    // the wavefront's rows of Kc and Vc as B operands (row of an invalid key: the tile's first, masked below)
    u32x4 kf[KS_D], vf[KS_D];
    {
        const size_t row = (tokb + (valid ? c : c0)) * D + 8 * lq;
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) {
            kf[ks] = *reinterpret_cast<const u32x4*>(Kc + row + 32 * ks);
            vf[ks] = *reinterpret_cast<const u32x4*>(Vc + row + 32 * ks);
        }
    }
    f32x4 accK[MD], accV[MD];
#pragma unroll
    for (int md = 0; md < MD; ++md) { accK[md] = f32x4{0.f, 0.f, 0.f, 0.f}; accV[md] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    float g = 0.f;

    // the queries that see the tile's first key, in tiles; the blocks of the tile take equal shares of them
    const int i_first = idx[tokb + c0] & ~(SBM_QT - 1);
    const int n_tiles = (L - i_first) / SBM_QT;
    const int i_lo = i_first + (int)((long long)n_tiles * seg / n_seg) * SBM_QT;
    const int i_hi = i_first + (int)((long long)n_tiles * (seg + 1) / n_seg) * SBM_QT;
#pragma unroll 1
    for (int i0 = i_lo; i0 < i_hi; i0 += SBM_QT) {
        __syncthreads();   // the previous tile has been read by everyone
        // (fetching the next tile into registers during the products, as the dQ kernel does, costs this kernel more
        // in registers, which it has none to spare of, than the exposed load costs: 0.26 against 0.22 ms)
#pragma unroll
        for (int i = 0; i < NPC; ++i) {
            const int e = tid + 256 * i, q = e / (D / 8), c8 = e % (D / 8);
            const size_t src = (tokb + i0 + q) * D + 8 * c8;     // L is a multiple of the tile
            const u32x4 rq = *reinterpret_cast<const u32x4*>(Q + src);
            const u32x4 rd = *reinterpret_cast<const u32x4*>(dO + src);
            *reinterpret_cast<u32x4*>(Qs + q * RS + 8 * c8) = rq;
            *reinterpret_cast<u32x4*>(dOs + q * RS + 8 * c8) = rd;
            const half8 hq = bf16x8_to_half8(rq), hd = bf16x8_to_half8(rd);
            const int col = sbm_col(q);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                QT[sbm_at(8 * c8 + j, col, TS)] = hq[j];
                dOT[sbm_at(8 * c8 + j, col, TS)] = hd[j];
            }
        }
        if (tid < SBM_QT) {
            s_lse2[tid] = lse[tokb + i0 + tid] * LOG2E;
            s_D[tid] = Dvec[tokb + i0 + tid];
            s_cnt[tid] = cnt[tokb + i0 + tid];
        }
        __syncthreads();

        // ---- S and dP for 64 queries x this wavefront's 16 keys -----------------------------------------
        f32x4 accS[4], accP[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) { accS[mt] = f32x4{0.f, 0.f, 0.f, 0.f}; accP[mt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks)
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                const u32x4 fq = *reinterpret_cast<const u32x4*>(Qs + (16 * mt + l16) * RS + 32 * ks + 8 * lq);
                const u32x4 fd = *reinterpret_cast<const u32x4*>(dOs + (16 * mt + l16) * RS + 32 * ks + 8 * lq);
                accS[mt] = sbm_mfma_bf16(fq, kf[ks], accS[mt]);   // rows: queries 16 mt + 4 lq + j, col: key l16
                accP[mt] = sbm_mfma_bf16(fd, vf[ks], accP[mt]);
            }
        // ---- P, dS (fp32), split into two fp16 terms; column sums of dS ---------------------------------
        half8 p_hi[2], p_lo[2], s_hi[2], s_lo[2];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
            const float4 l4 = *reinterpret_cast<const float4*>(s_lse2 + 16 * mt + 4 * lq);
            const float4 d4 = *reinterpret_cast<const float4*>(s_D + 16 * mt + 4 * lq);
            const int4 c4 = *reinterpret_cast<const int4*>(s_cnt + 16 * mt + 4 * lq);
            const float lq4[4] = {l4.x, l4.y, l4.z, l4.w}, dq4[4] = {d4.x, d4.y, d4.z, d4.w};
            const int cq4[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float p = (valid && c < cq4[j]) ? __builtin_amdgcn_exp2f(scale2 * accS[mt][j] - lq4[j]) : 0.f;
                const float ds = p * (accP[mt][j] - dq4[j]);
                g += ds;
                const half_t ph = (half_t)p, sh = f32_to_half_sat(ds);
                const int slot = 4 * (mt & 1) + j;
                p_hi[mt >> 1][slot] = ph;
                p_lo[mt >> 1][slot] = (half_t)(p - (float)ph);
                s_hi[mt >> 1][slot] = sh;
                s_lo[mt >> 1][slot] = (half_t)(ds - (float)sh);
            }
        }
        // ---- dV^T += dO^T P,  dK^T += Q^T dS  (rows d = 16 md + 4 lq + j, col key l16) -------------------
#pragma unroll
        for (int md = 0; md < MD; ++md)
#pragma unroll
            for (int mp = 0; mp < 2; ++mp) {
                const half8 ad = lds_read8(dOT + sbm_at(16 * md + l16, 32 * mp + 8 * lq, TS));
                const half8 aq = lds_read8(QT + sbm_at(16 * md + l16, 32 * mp + 8 * lq, TS));
                accV[md] = mfma16(ad, p_hi[mp], accV[md]);
                accV[md] = mfma16(ad, p_lo[mp], accV[md]);
                accK[md] = mfma16(aq, s_hi[mp], accK[md]);
                accK[md] = mfma16(aq, s_lo[mp], accK[md]);
            }
    }
    // this segment's share, by compacted key; a second kernel adds the shares up in order
    g += lane_xor16(g, lane);
    g += lane_xor32(g, lane);
    if (valid) {
        const size_t row = ((size_t)seg * BH + bh) * L + c;
#pragma unroll
        for (int md = 0; md < MD; ++md) {
            *reinterpret_cast<float4*>(dk_part + row * D + 16 * md + 4 * lq) =
                make_float4(accK[md][0], accK[md][1], accK[md][2], accK[md][3]);
            *reinterpret_cast<float4*>(dv_part + row * D + 16 * md + 4 * lq) =
                make_float4(accV[md][0], accV[md][1], accV[md][2], accV[md][3]);
        }
        if (lq == 0) g_part[row] = g;
    }
}

// ---- dQ and D on MFMA, bf16 tensors: the mirror image of the kernel above ----------------------------------------
// A block owns 64 queries, wavefront w the 16 queries of tile w (their Q and dO rows are its B operands, in
// registers), and walks the key tiles its last query sees.  Per key tile:
//   S^T [key][q] = K Q^T,  dP^T[key][q] = V dO^T     bf16 MFMA, A = the K / V tile (LDS, row-major)
//   P, dS (fp32, as above; a query is one MFMA column, so lse, D and the count are per-lane scalars)
//   dQ^T[d][q] += K^T dS^T      fp16 MFMA, A = the transposed K tile (LDS, columns in slot order),
//                               B = dS straight from the accumulators, as two fp16 terms
template <int D>
__global__ __launch_bounds__(256, 2) void softmax_bwd_dq_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ Kc, const bf16_t* __restrict__ Vc,
    const bf16_t* __restrict__ dO, const int32_t* __restrict__ cnt, const float* __restrict__ O_nla,
    const float* __restrict__ lse, float* __restrict__ Dvec, float* __restrict__ dQ, int L, float scale) {
    constexpr int RS = D + LDS_PAD, TS = 64 + LDS_PAD;
    constexpr int KS_D = D / 32, MD = D / 16, NPC = 64 * D / 8 / 256;
    __shared__ __align__(16) uint16_t Ks[64 * RS], Vs[64 * RS];   // bf16, row-major
    __shared__ __align__(16) half_t KT[D * TS];                    // fp16, transposed
    __shared__ float s_D[64];

    const int bh = blockIdx.y, q0 = ((int)gridDim.x - 1 - (int)blockIdx.x) * 64, tid = threadIdx.x;   // long blocks first
    const int lane = tid & 63, wave = tid >> 6, l16 = lane & 15, lq = lane >> 4;
    const size_t tokb = (size_t)bh * L;
    const float LOG2E = 1.44269504088896341f;
    const float scale2 = scale * LOG2E;

    // D_i = do_i . o_i: four lanes per query, as in the fp32 kernel
    {
        const int r = tid >> 2, part = tid & 3;
        const size_t off = (tokb + q0 + r) * D + part * (D / 4);
        float Di = 0.f;
#pragma unroll
        for (int c = 0; c < D / 4; c += 8) {
            float dv[8];
            Vec16<bf16_t>::load(dO + off + c, dv);
            const float4 o0 = *reinterpret_cast<const float4*>(O_nla + off + c);
            const float4 o1 = *reinterpret_cast<const float4*>(O_nla + off + c + 4);
            Di += dv[0] * o0.x + dv[1] * o0.y + dv[2] * o0.z + dv[3] * o0.w + dv[4] * o1.x + dv[5] * o1.y + dv[6] * o1.z +
                  dv[7] * o1.w;
        }
        Di = lane_group_sum<4>(Di);
        if (part == 0) { s_D[r] = Di; Dvec[tokb + q0 + r] = Di; }
    }
    // this lane's query (an MFMA column): its rows of Q and dO as B operands, its scalars
    const int qi = q0 + 16 * wave + l16;
    u32x4 qf[KS_D], dof[KS_D];
#pragma unroll
    for (int ks = 0; ks < KS_D; ++ks) {
        qf[ks] = *reinterpret_cast<const u32x4*>(Q + (tokb + qi) * D + 32 * ks + 8 * lq);
        dof[ks] = *reinterpret_cast<const u32x4*>(dO + (tokb + qi) * D + 32 * ks + 8 * lq);
    }
    const float lse2_q = lse[tokb + qi] * LOG2E;
    const int cnt_q = cnt[tokb + qi];
    const int n_hi = cnt[tokb + q0 + 63];   // cnt is non-decreasing: the block's bound
    __syncthreads();
    const float D_q = s_D[16 * wave + l16];

    f32x4 accQ[MD];
#pragma unroll
    for (int md = 0; md < MD; ++md) accQ[md] = f32x4{0.f, 0.f, 0.f, 0.f};

    // A key tile is fetched into registers while the tile before it is multiplied.
    u32x4 rk[NPC], rv[NPC];
    auto fetch_tile = [&](int c0) {
#pragma unroll
        for (int i = 0; i < NPC; ++i) {
            const int e = tid + 256 * i, key = e / (D / 8), c8 = e % (D / 8);
            rk[i] = u32x4{0u, 0u, 0u, 0u};
            rv[i] = u32x4{0u, 0u, 0u, 0u};
            if (c0 + key < n_hi) {   // rows past the block's bound are not initialised: they enter as zeros
                const size_t src = (tokb + c0 + key) * D + 8 * c8;
                rk[i] = *reinterpret_cast<const u32x4*>(Kc + src);
                rv[i] = *reinterpret_cast<const u32x4*>(Vc + src);
            }
        }
    };
    if (n_hi > 0) fetch_tile(0);
#pragma unroll 1
    for (int c0 = 0; c0 < n_hi; c0 += 64) {
        __syncthreads();   // the previous tile has been read by everyone
#pragma unroll
        for (int i = 0; i < NPC; ++i) {
            const int e = tid + 256 * i, key = e / (D / 8), c8 = e % (D / 8);
            *reinterpret_cast<u32x4*>(Ks + key * RS + 8 * c8) = rk[i];
            *reinterpret_cast<u32x4*>(Vs + key * RS + 8 * c8) = rv[i];
            const half8 hk = bf16x8_to_half8(rk[i]);
            const int col = sbm_col(key);
#pragma unroll
            for (int j = 0; j < 8; ++j) KT[sbm_at(8 * c8 + j, col, TS)] = hk[j];
        }
        __syncthreads();
        if (c0 + 64 < n_hi) fetch_tile(c0 + 64);
        f32x4 accS[4], accP[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) { accS[mt] = f32x4{0.f, 0.f, 0.f, 0.f}; accP[mt] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks)
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) {
                const u32x4 fk = *reinterpret_cast<const u32x4*>(Ks + (16 * mt + l16) * RS + 32 * ks + 8 * lq);
                const u32x4 fv = *reinterpret_cast<const u32x4*>(Vs + (16 * mt + l16) * RS + 32 * ks + 8 * lq);
                accS[mt] = sbm_mfma_bf16(fk, qf[ks], accS[mt]);   // rows: keys 16 mt + 4 lq + j, col: query l16
                accP[mt] = sbm_mfma_bf16(fv, dof[ks], accP[mt]);
            }
        half8 s_hi[2], s_lo[2];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = c0 + 16 * mt + 4 * lq + j;
                const float p = (c < cnt_q) ? __builtin_amdgcn_exp2f(scale2 * accS[mt][j] - lse2_q) : 0.f;
                const float ds = p * (accP[mt][j] - D_q);
                const half_t sh = f32_to_half_sat(ds);
                const int slot = 4 * (mt & 1) + j;
                s_hi[mt >> 1][slot] = sh;
                s_lo[mt >> 1][slot] = (half_t)(ds - (float)sh);
            }
#pragma unroll
        for (int md = 0; md < MD; ++md)
#pragma unroll
            for (int mp = 0; mp < 2; ++mp) {
                const half8 ak = lds_read8(KT + sbm_at(16 * md + l16, 32 * mp + 8 * lq, TS));
                accQ[md] = mfma16(ak, s_hi[mp], accQ[md]);   // rows d = 16 md + 4 lq + j, col query l16
                accQ[md] = mfma16(ak, s_lo[mp], accQ[md]);
            }
    }
#pragma unroll
    for (int md = 0; md < MD; ++md)
        *reinterpret_cast<float4*>(dQ + (tokb + qi) * D + 16 * md + 4 * lq) =
            make_float4(scale * accQ[md][0], scale * accQ[md][1], scale * accQ[md][2], scale * accQ[md][3]);
}

template <typename T>
static void launch_sb(const FwdPlan& pl, const void* Q, const void* Kc, const void* Vc, const void* dO,
                      const int32_t* cnt, const int32_t* idx, const int32_t* n_s, const float* O_nla, const float* lse,
                      float* Dvec, float* dQ, float* dK, float* dV, float* g_nla, bool dkv, hipStream_t st) {
    dim3 grid(pl.L / SB_ROWS, pl.BH);
    if (dkv) grid = dim3((unsigned)((size_t)(pl.L / SB_ROWS) * pl.BH * BWD_DKV_SEGMENTS));
#define NATS_SB_LAUNCH(DD)                                                                                          \
    if (!dkv)                                                                                                        \
        hipLaunchKernelGGL((softmax_bwd_dq_kernel<T, DD>), grid, dim3(SB_THREADS), 0, st, (const T*)Q, (const T*)Kc, \
                           (const T*)Vc, (const T*)dO, cnt, O_nla, lse, Dvec, dQ, pl.L, pl.softmax_scale);           \
    else                                                                                                             \
        hipLaunchKernelGGL((softmax_bwd_dkv_kernel<T, DD>), grid, dim3(SB_THREADS), 0, st, (const T*)Q,              \
                           (const T*)Kc, (const T*)Vc, (const T*)dO, cnt, idx, n_s, lse, Dvec, dK, dV, g_nla, pl.L,  \
                           pl.softmax_scale, pl.BH, BWD_DKV_SEGMENTS)
    if (pl.d == 64) NATS_SB_LAUNCH(64);
    else NATS_SB_LAUNCH(128);
#undef NATS_SB_LAUNCH
}

// dQ [B,H,L,d] f32 is written (not accumulated); also Dvec [B,H,L]
nats_status launch_softmax_bwd_dq(const FwdPlan& pl, const void* Q, const void* Kc, const void* Vc, const void* dO,
                                  const int32_t* cnt, const float* O_nla, const float* lse, float* Dvec, float* dQ,
                                  hipStream_t st) {
    if (pl.dtype == NATS_BF16) {   // the MFMA form
        dim3 grid(pl.L / 64, pl.BH);
        if (pl.d == 64)
            hipLaunchKernelGGL((softmax_bwd_dq_mfma_kernel<64>), grid, dim3(256), 0, st, (const bf16_t*)Q, (const bf16_t*)Kc,
                               (const bf16_t*)Vc, (const bf16_t*)dO, cnt, O_nla, lse, Dvec, dQ, pl.L, pl.softmax_scale);
        else
            hipLaunchKernelGGL((softmax_bwd_dq_mfma_kernel<128>), grid, dim3(256), 0, st, (const bf16_t*)Q, (const bf16_t*)Kc,
                               (const bf16_t*)Vc, (const bf16_t*)dO, cnt, O_nla, lse, Dvec, dQ, pl.L, pl.softmax_scale);
    } else
        launch_sb<float>(pl, Q, Kc, Vc, dO, cnt, nullptr, nullptr, O_nla, lse, Dvec, dQ, nullptr, nullptr, nullptr, false, st);
    return check_launch("softmax_bwd_dq");
}

// the rows idx[c] of dK, dV [B,H,L,d] f32 (and of g_nla [B,H,L], optional) are overwritten; other rows are left alone.
// dk_part, dv_part: BWD_DKV_SEGMENTS * BH * L * d floats, g_part: BWD_DKV_SEGMENTS * BH * L floats (scratch)
nats_status launch_softmax_bwd_dkv(const FwdPlan& pl, const void* Q, const void* Kc, const void* Vc, const void* dO,
                                   const int32_t* cnt, const int32_t* idx, const int32_t* n_s, const float* lse,
                                   const float* Dvec, float* dK, float* dV, float* g_nla, float* dk_part, float* dv_part,
                                   float* g_part, hipStream_t st) {
    if (pl.dtype == NATS_BF16) {   // the MFMA form
        dim3 grid((unsigned)((size_t)(pl.L / 64) * pl.BH * BWD_DKV_SEGMENTS));
        // the LDS-size attribute is per function and device: set once per device, not per launch
        static bool attr_done[2][64] = {};
        int dev = 0;
        (void)hipGetDevice(&dev);
        dev = (dev >= 0 && dev < 64) ? dev : 0;
        if (pl.d == 64) {
            auto kern = softmax_bwd_dkv_mfma_kernel<64>;
            if (!attr_done[0][dev]) {
                if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        sbm_lds_bytes<64>()) != hipSuccess)
                    return check_launch("softmax_bwd_dkv (LDS attribute)");
                attr_done[0][dev] = true;
            }
            hipLaunchKernelGGL(kern, grid, dim3(256), sbm_lds_bytes<64>(), st, (const bf16_t*)Q, (const bf16_t*)Kc,
                               (const bf16_t*)Vc, (const bf16_t*)dO, cnt, idx, n_s, lse, Dvec, dk_part, dv_part, g_part,
                               pl.L, pl.softmax_scale, pl.BH, BWD_DKV_SEGMENTS);
        } else {
            auto kern = softmax_bwd_dkv_mfma_kernel<128>;
            if (!attr_done[1][dev]) {
                if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                        sbm_lds_bytes<128>()) != hipSuccess)
                    return check_launch("softmax_bwd_dkv (LDS attribute)");
                attr_done[1][dev] = true;
            }
            hipLaunchKernelGGL(kern, grid, dim3(256), sbm_lds_bytes<128>(), st, (const bf16_t*)Q, (const bf16_t*)Kc,
                               (const bf16_t*)Vc, (const bf16_t*)dO, cnt, idx, n_s, lse, Dvec, dk_part, dv_part, g_part,
                               pl.L, pl.softmax_scale, pl.BH, BWD_DKV_SEGMENTS);
        }
    } else
        launch_sb<float>(pl, Q, Kc, Vc, dO, cnt, idx, n_s, nullptr, lse, const_cast<float*>(Dvec), nullptr, dk_part, dv_part,
                         g_part, true, st);
    nats_status rc = check_launch("softmax_bwd_dkv");
    if (rc != NATS_OK) return rc;
    if (pl.d == 64) {
        dim3 grid((pl.L + 15) / 16, pl.BH);   // 256 / (64 / 4) keys per block
        hipLaunchKernelGGL((softmax_bwd_dkv_combine_kernel<64>), grid, dim3(256), 0, st, dk_part, dv_part, g_part, idx, n_s,
                           dK, dV, g_nla, pl.L, BWD_DKV_SEGMENTS, pl.softmax_scale, pl.routing == NATS_ROUTE_CHUNK);
    } else {
        dim3 grid((pl.L + 7) / 8, pl.BH);     // 256 / (128 / 4) keys per block
        hipLaunchKernelGGL((softmax_bwd_dkv_combine_kernel<128>), grid, dim3(256), 0, st, dk_part, dv_part, g_part, idx, n_s,
                           dK, dV, g_nla, pl.L, BWD_DKV_SEGMENTS, pl.softmax_scale, pl.routing == NATS_ROUTE_CHUNK);
    }
    return check_launch("softmax_bwd_dkv_combine");
}

// ---- routing per chunk -------------------------------------------------------------------------------------
// Compacted rows a query sees: with routing per token the first cnt[t]; with routing per chunk those of earlier
// chunks, cnt at the last token before the query's chunk.  Written out once so that the kernels above, which take
// "rows visible to query t" as an array, serve both routings unchanged.
__global__ __launch_bounds__(256) void visible_rows_kernel(const int32_t* __restrict__ cnt, int32_t* __restrict__ vis, int L,
                                                          size_t n_tok) {
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= n_tok) return;
    const size_t cs = t - (t % L) % 64;          // first token of the query's chunk
    vis[t] = (cs % L) > 0 ? cnt[cs - 1] : 0;
}

// The inner part of every chunk (routing per chunk): query i of a chunk also attends to the chunk's own tokens
// j <= i, whatever the chunk's type; no mask stands on these columns, so they add to dQ, dK, dV but not to the score
// gradient.  One block per (chunk, batch*head), the 64 x 64 causal block in fp32:
//   p_ij = exp(scale q_i.k_j - lse_i),  ds_ij = p_ij (do_i.v_j - D_i)        (lse_i, D_i: of the whole row)
//   dQ_i += scale sum_j ds_ij k_j;   dK_j += scale sum_i ds_ij q_i;   dV_j += sum_i p_ij do_i
// Rows of Q, K, V, dO pass through LDS 64 columns at a time.  Thread (i = tid / 4, quarter = tid % 4) owns 16
// entries of a 64 x 64 result.  Accumulates into dQ, dK, dV (no other kernel runs beside it).
constexpr int OC_TS = 65;
constexpr int OC_LDS_BYTES = 4 * 64 * OC_TS * 4;
template <typename T, int D>
__global__ __launch_bounds__(256) void softmax_bwd_own_chunk_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, const T* __restrict__ dO,
    const float* __restrict__ lse, const float* __restrict__ Dvec, float* __restrict__ dQ, float* __restrict__ dK,
    float* __restrict__ dV, int L, float scale) {
    constexpr int TS = OC_TS;   // row stride (floats) of the 64 x 64 tiles
    extern __shared__ __align__(16) unsigned char oc_smem[];
    float* s_x = reinterpret_cast<float*>(oc_smem);
    float* s_y = s_x + 64 * TS;
    float* s_p = s_y + 64 * TS;
    float* s_ds = s_p + 64 * TS;
    const int bh = blockIdx.y, c0 = blockIdx.x * 64, tid = threadIdx.x;
    const size_t rowb = (size_t)bh * L + c0;
    const int i = tid >> 2, qt = tid & 3;
    // loads columns [dc, dc + 64) of 64 rows of a tensor into a tile
    auto load_tile = [&](const T* src, float* dst, int dc) {
        for (int e = tid; e < 64 * 64; e += 256) {
            const int r = e >> 6, c = e & 63;
            dst[r * TS + c] = to_float(src[(rowb + r) * D + dc + c]);
        }
    };
    float acc_s[16], acc_dp[16];
#pragma unroll
    for (int m = 0; m < 16; ++m) { acc_s[m] = 0.f; acc_dp[m] = 0.f; }
    for (int dc = 0; dc < D; dc += 64) {
        __syncthreads();
        load_tile(Q, s_x, dc);
        load_tile(K, s_y, dc);
        __syncthreads();
        for (int c = 0; c < 64; ++c) {
            const float x = s_x[i * TS + c];
#pragma unroll
            for (int m = 0; m < 16; ++m) acc_s[m] += x * s_y[(qt + 4 * m) * TS + c];
        }
        __syncthreads();
        load_tile(dO, s_x, dc);
        load_tile(V, s_y, dc);
        __syncthreads();
        for (int c = 0; c < 64; ++c) {
            const float x = s_x[i * TS + c];
#pragma unroll
            for (int m = 0; m < 16; ++m) acc_dp[m] += x * s_y[(qt + 4 * m) * TS + c];
        }
    }
    {
        const float l = lse[rowb + i], Di = Dvec[rowb + i];
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            const int j = qt + 4 * m;
            const float p = j <= i ? expf(scale * acc_s[m] - l) : 0.f;
            s_p[i * TS + j] = p;
            s_ds[i * TS + j] = p * (acc_dp[m] - Di);
        }
    }
    for (int dc = 0; dc < D; dc += 64) {
        float out[16];
        // dQ_i[c] += scale sum_j ds_ij K_j[c]
        __syncthreads();
        load_tile(K, s_y, dc);
        load_tile(Q, s_x, dc);
        __syncthreads();
#pragma unroll
        for (int m = 0; m < 16; ++m) out[m] = 0.f;
        for (int j = 0; j < 64; ++j) {
            const float w = s_ds[i * TS + j];
#pragma unroll
            for (int m = 0; m < 16; ++m) out[m] += w * s_y[j * TS + qt + 4 * m];
        }
#pragma unroll
        for (int m = 0; m < 16; ++m) dQ[(rowb + i) * D + dc + qt + 4 * m] += scale * out[m];
        // dK_j[c] += scale sum_i ds_ij Q_i[c]      (this thread's row index now counts keys)
#pragma unroll
        for (int m = 0; m < 16; ++m) out[m] = 0.f;
        for (int q = 0; q < 64; ++q) {
            const float w = s_ds[q * TS + i];
#pragma unroll
            for (int m = 0; m < 16; ++m) out[m] += w * s_x[q * TS + qt + 4 * m];
        }
#pragma unroll
        for (int m = 0; m < 16; ++m) dK[(rowb + i) * D + dc + qt + 4 * m] += scale * out[m];
        // dV_j[c] += sum_i p_ij dO_i[c]
        __syncthreads();
        load_tile(dO, s_x, dc);
        __syncthreads();
#pragma unroll
        for (int m = 0; m < 16; ++m) out[m] = 0.f;
        for (int q = 0; q < 64; ++q) {
            const float w = s_p[q * TS + i];
#pragma unroll
            for (int m = 0; m < 16; ++m) out[m] += w * s_x[q * TS + qt + 4 * m];
        }
#pragma unroll
        for (int m = 0; m < 16; ++m) dV[(rowb + i) * D + dc + qt + 4 * m] += out[m];
    }
}

// The same on fp32 matrix instructions, for bf16 tensors: the four 64 x D tiles stay in LDS as they are (bf16,
// widened when read), S = Q K^T and dP = dO V^T by 16 x 16 tiles below the diagonal (wavefront w: query tile w), then
// p and scale x ds through LDS as fp32, and dQ_w = ds_w K, dK_w = ds^T Q, dV_w = p^T dO (wavefront w: key tile w).
constexpr int OCM_PS = 68;   // row stride (floats) of the p and ds tiles
template <int D>
__global__ __launch_bounds__(256) void softmax_bwd_own_chunk_mfma_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V, const bf16_t* __restrict__ dO,
    const float* __restrict__ lse, const float* __restrict__ Dvec, float* __restrict__ dQ, float* __restrict__ dK,
    float* __restrict__ dV, int L, float scale) {
    constexpr int RS = D + 8, PS = OCM_PS, NP = 64 * D / 8 / 256;
    extern __shared__ __align__(16) unsigned char oc_smem[];
    uint16_t* Qs = reinterpret_cast<uint16_t*>(oc_smem);
    uint16_t* Ks = Qs + 64 * RS;
    uint16_t* Vs = Ks + 64 * RS;
    uint16_t* Os = Vs + 64 * RS;
    float* s_p = reinterpret_cast<float*>(Os + 64 * RS);
    float* s_ds = s_p + 64 * PS;
    const int bh = blockIdx.y, c0 = blockIdx.x * 64, tid = threadIdx.x;
    const int lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6), l16 = lane & 15, lq = lane >> 4;
    const size_t rowb = (size_t)bh * L + c0;
    {
        u32x4 r[4][NP];
        const bf16_t* src[4] = {Q, K, V, dO};
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int i = 0; i < NP; ++i) r[a][i] = reinterpret_cast<const u32x4*>(src[a] + rowb * D)[tid + 256 * i];
        uint16_t* dst[4] = {Qs, Ks, Vs, Os};
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int e = tid + 256 * i;
                *reinterpret_cast<u32x4*>(dst[a] + (e / (D / 8)) * RS + (e % (D / 8)) * 8) = r[a][i];
            }
    }
    float lq4[4], dq4[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        lq4[j] = lse[rowb + 16 * w + 4 * lq + j] * 1.44269504088896341f;
        dq4[j] = Dvec[rowb + 16 * w + 4 * lq + j];
    }
    const float scale2 = scale * 1.44269504088896341f;
    __syncthreads();
    for (int tb = 0; tb <= w; ++tb) {
        f32x4 accS = {0.f, 0.f, 0.f, 0.f}, accD = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
        for (int kt = 0; kt < D / 16; ++kt) {
            accS = mac16(ldb4(Qs + (16 * w + l16) * RS + 16 * kt + 4 * lq), ldb4(Ks + (16 * tb + l16) * RS + 16 * kt + 4 * lq), accS);
            accD = mac16(ldb4(Os + (16 * w + l16) * RS + 16 * kt + 4 * lq), ldb4(Vs + (16 * tb + l16) * RS + 16 * kt + 4 * lq), accD);
        }
        const int key = 16 * tb + l16;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int q = 16 * w + 4 * lq + j;
            const float p = key <= q ? __builtin_amdgcn_exp2f(scale2 * accS[j] - lq4[j]) : 0.f;   // base-2 units
            s_p[q * PS + key] = p;
            s_ds[q * PS + key] = scale * p * (accD[j] - dq4[j]);
        }
    }
    __syncthreads();
    // The old values of dQ, dK, dV that the results are added to: asked for up front, all at once (a read inside
    // the loop below would cost a trip to memory per column tile).
    constexpr int NKT = D / 16;
    float oq[NKT][4], ok[NKT][4], ov[NKT][4];
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const size_t off = (rowb + 16 * w + 4 * lq + j) * D + 16 * kt + l16;
            oq[kt][j] = dQ[off];
            ok[kt][j] = dK[off];
            ov[kt][j] = dV[off];
        }
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt) {
        f32x4 aq = {oq[kt][0], oq[kt][1], oq[kt][2], oq[kt][3]}, ak = {ok[kt][0], ok[kt][1], ok[kt][2], ok[kt][3]};
        f32x4 av = {ov[kt][0], ov[kt][1], ov[kt][2], ov[kt][3]};
        for (int tb = 0; tb <= w; ++tb)     // dQ of query tile w: keys of the tiles up to it
            aq = mac16(ld4(s_ds + (16 * w + l16) * PS + 16 * tb + 4 * lq), ldbcol(Ks + (16 * tb + 4 * lq) * RS + 16 * kt + l16, RS), aq);
        for (int ta = w; ta < 4; ++ta) {    // dK, dV of key tile w: queries of the tiles from it on
            ak = mac16(ld4col(s_ds + (16 * ta + 4 * lq) * PS + 16 * w + l16, PS), ldbcol(Qs + (16 * ta + 4 * lq) * RS + 16 * kt + l16, RS), ak);
            av = mac16(ld4col(s_p + (16 * ta + 4 * lq) * PS + 16 * w + l16, PS), ldbcol(Os + (16 * ta + 4 * lq) * RS + 16 * kt + l16, RS), av);
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const size_t off = (rowb + 16 * w + 4 * lq + j) * D + 16 * kt + l16;
            dQ[off] = aq[j];
            dK[off] = ak[j];
            dV[off] = av[j];
        }
    }
}

nats_status launch_visible_rows(const FwdPlan& pl, const int32_t* cnt, int32_t* vis, hipStream_t st) {
    const size_t n_tok = (size_t)pl.BH * pl.L;
    hipLaunchKernelGGL(visible_rows_kernel, dim3((unsigned)((n_tok + 255) / 256)), dim3(256), 0, st, cnt, vis, pl.L, n_tok);
    return check_launch("visible_rows");
}

nats_status launch_softmax_bwd_own_chunk(const FwdPlan& pl, const void* Q, const void* K, const void* V, const void* dO,
                                         const float* lse, const float* Dvec, float* dQ, float* dK, float* dV,
                                         hipStream_t st) {
    dim3 grid(pl.L / 64, pl.BH);
    // more than 64 KB of LDS: the limit is raised per kernel (cheap, so done at every launch)
#define NATS_OC_LAUNCH(TT, DD)                                                                                       \
    do {                                                                                                             \
        auto kern = softmax_bwd_own_chunk_kernel<TT, DD>;                                                            \
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,    \
                                OC_LDS_BYTES) != hipSuccess)                                                         \
            return check_launch("softmax_bwd_own_chunk (LDS attribute)");                                            \
        hipLaunchKernelGGL(kern, grid, dim3(256), OC_LDS_BYTES, st, (const TT*)Q, (const TT*)K, (const TT*)V,        \
                           (const TT*)dO, lse, Dvec, dQ, dK, dV, pl.L, pl.softmax_scale);                           \
    } while (0)
#define NATS_OCM_LAUNCH(DD)                                                                                          \
    do {                                                                                                             \
        auto kern = softmax_bwd_own_chunk_mfma_kernel<DD>;                                                           \
        constexpr int lds = 4 * 64 * (DD + 8) * 2 + 2 * 64 * OCM_PS * 4;                                             \
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,    \
                                lds) != hipSuccess)                                                                  \
            return check_launch("softmax_bwd_own_chunk (LDS attribute)");                                            \
        hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, (const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V,     \
                           (const bf16_t*)dO, lse, Dvec, dQ, dK, dV, pl.L, pl.softmax_scale);                       \
    } while (0)
    if (pl.dtype == NATS_BF16) { if (pl.d == 64) NATS_OCM_LAUNCH(64); else NATS_OCM_LAUNCH(128); }
    else { if (pl.d == 64) NATS_OC_LAUNCH(float, 64); else NATS_OC_LAUNCH(float, 128); }
#undef NATS_OC_LAUNCH
#undef NATS_OCM_LAUNCH
    return check_launch("softmax_bwd_own_chunk");
}

}  // namespace nats
