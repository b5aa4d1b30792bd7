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
//                                  such tiles fill the 8 contraction slots of one lane (the V^T tile's
//                                  columns are stored in that slot order).
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
constexpr int FL_VAHEAD = 6;             // V^T fragment reads in flight ahead of their matrix instructions
constexpr int FL_OCC = 2;                // blocks per CU the kernel is built for
constexpr int FL_BM = 4 * 16 * FL_NQ;    // queries per block
constexpr int FL_BN = 64;                // compacted keys per tile

__device__ __forceinline__ f32x4 mfma16_bf16(u32x4 a, u32x4 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, a), __builtin_bit_cast(bf16x8_t, b), c,
                                                   0, 0, 0);
}

// Reductions over the four lanes l, l^16, l^32, l^48 that share a query column, with gfx950's row
// swaps instead of trips through LDS: v_permlane32_swap exchanges the upper half of its first
// operand with the lower half of its second, v_permlane16_swap the odd 16-lane rows of the first
// with the even rows of the second; given the same value twice, the two results hold a lane's own
// value and its partner's.
__device__ __forceinline__ float quad_max(float x) {
    const auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}

__device__ __forceinline__ float quad_sum(float x) {
    const auto a = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const auto b = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// The epilogue reads the linear branch's output (fp16), merges (Section 4.1 sum, Eq. 21 or its ablation) and
// stores O.
// chunk_routing: routing per chunk (a template parameter: the per-token kernel carries none of its code)
// STATS: what the backward pass needs from this branch's forward, to fp32 accuracy: the weights enter the second
// product (and their sum) as the sum of two fp16 terms, and only O_nla_out (fp32) and lse_out are written; no merge.
// MERGED: the merges other than the plain sum (combine_mode 1, 2) and Eq. 22; the plain sum's instantiation carries
// none of their code.
template <int D, bool chunk_routing, bool STATS, bool MERGED>
__global__ __launch_bounds__(FL_THREADS, FL_OCC) void flash_softmax_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ Kc, const half_t* __restrict__ VhT,
    const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const int32_t* __restrict__ cnt, const half_t* __restrict__ O_la, const float* __restrict__ w_nla,
    const float* __restrict__ w_la, bf16_t* __restrict__ O,
    float* __restrict__ O_nla_out, float* __restrict__ lse_out, int L, float scale, int combine_mode_arg,
    float eps, int BH, int G, int qk_per_out_head, int own_chunk, const float* __restrict__ W_out, int weight_act,
    int heads_out) {
    const int combine_mode = MERGED ? combine_mode_arg : 0;
    constexpr int RS = D + LDS_PAD;      // K / Q tile rows (bf16 elements)
    constexpr int TS = FL_BN + LDS_PAD;  // V^T tile rows (fp16 elements)
    constexpr int OS = D + 4;            // output staging rows (fp32 elements)
    constexpr int KS_D = D / 32;
    constexpr int DT = D / 16;           // 16-row d_v tiles
    // one LDS region, three tenants: the Q tile (prologue), the K and V^T tiles (main loop), the
    // per-wavefront output staging (epilogue)
    constexpr int TILE_BYTES = FL_BN * RS * 2 + D * TS * 2;
    constexpr int Q_BYTES = FL_BM * RS * 2;
    constexpr int O_BYTES = 4 * 16 * OS * 4;
    constexpr int LDS_BYTES = TILE_BYTES > Q_BYTES ? (TILE_BYTES > O_BYTES ? TILE_BYTES : O_BYTES)
                                                   : (Q_BYTES > O_BYTES ? Q_BYTES : O_BYTES);
    __shared__ __align__(16) unsigned char smem[LDS_BYTES];
    uint16_t* Ks = reinterpret_cast<uint16_t*>(smem);
    half_t* Vs = reinterpret_cast<half_t*>(smem + FL_BN * RS * 2);
    uint16_t* Qst = reinterpret_cast<uint16_t*>(smem);
    float* Ot = reinterpret_cast<float*>(smem);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    // One-dimensional grid over (batch, head) pairs (padded to a multiple of 8) and query tiles.  Later
    // tiles see more keys and are dispatched first, so that the long blocks do not form the tail.
    // Routing per token: tile-major, the blocks of one tile side by side, one per pair; a pair's blocks
    // then always land on the same XCD and share its L2 for the compacted keys (measured 71 against 85
    // microseconds on the headline shape).  Routing per chunk, where every block also streams its own
    // 128 rows of K and V: pair-major, neighbouring blocks read neighbouring rows (136 against 149).
    const int bh8 = (BH + 7) & ~7;
    const int n_tiles_g = gridDim.x / bh8;
    const int bh = chunk_routing ? blockIdx.x / n_tiles_g : blockIdx.x % bh8;
    const int tile = n_tiles_g - 1 - (chunk_routing ? blockIdx.x % n_tiles_g : blockIdx.x / bh8);
    if (bh >= BH) return;
    const int q0 = tile * FL_BM;
    const size_t tokbase = (size_t)bh * L;                 // bh counts output heads (BH of them)
    const size_t tokbase_lin = (size_t)(bh / G) * L;       // the linear head whose mask the group shares: cnt
    const size_t tokbase_qk = qk_per_out_head ? tokbase : tokbase_lin;   // queries and raw keys of the softmax branch
    const float scale2 = scale * 1.44269504088896341f;   // logits in base-2 units

    // ---- prologue: the block's Q rows, coalesced, through LDS into B-operand fragments ------------
    constexpr int NQP = FL_BM * D / 8 / FL_THREADS;   // 16-byte pieces per thread of the Q tile
    constexpr int NKP = FL_BN * D / 8 / FL_THREADS;   // ... of a K tile and of a V^T tile
    // Every global load of the prologue is issued before the first use of any of them, so that the
    // block pays one memory latency here, not one per dependent step: the per-query counts, the count
    // that bounds the block, the Q tile and key tile 0 (which exists for every sequence: the
    // compacted buffers have capacity L >= 64 rows; its contents are not used if nothing is visible).
    const int q_last = min(q0 + FL_BM, L) - 1;
    // Compacted rows visible to a query: routing per token, the first cnt[t]; routing per chunk, those of
    // earlier chunks, i.e. cnt at the last token before the query's chunk (the chunk's own tokens come
    // from K and V after the compacted tiles, see below).
    auto visible_rows = [&](int t) __attribute__((always_inline)) -> int {
        if (!chunk_routing) return cnt[tokbase_lin + t];
        const int cs = t & ~(FL_BN - 1);
        return cs > 0 ? cnt[tokbase_lin + cs - 1] : 0;
    };
    int my_cnt[FL_NQ];
#pragma unroll
    for (int nq = 0; nq < FL_NQ; ++nq) {
        const int ql = (wave * FL_NQ + nq) * 16 + l16;
        my_cnt[nq] = visible_rows(min(q0 + ql, L - 1));
    }
    const int n_hi = visible_rows(q_last);    // non-decreasing in t: bound for the whole block
    u32x4 kreg[NKP], vreg[NKP];               // next K / V^T tile on its way from global memory to LDS
    auto load_tile = [&](int kt) __attribute__((always_inline)) {
        const u32x4* Kt = reinterpret_cast<const u32x4*>(Kc + (tokbase + (size_t)kt * FL_BN) * D);
        const u32x4* Vt = reinterpret_cast<const u32x4*>(VhT + (tokbase + (size_t)kt * FL_BN) * D);   // [D][64]
#pragma unroll
        for (int i = 0; i < NKP; ++i) {   // both tiles are contiguous in global memory
            kreg[i] = Kt[tid + FL_THREADS * i];
            vreg[i] = Vt[tid + FL_THREADS * i];
        }
    };
    // routing per chunk: the dc-th chunk of this block's queries, rows of K and V as they are (V row-major)
    auto load_own_chunk = [&](int dc) __attribute__((always_inline)) {
        const size_t t0 = min(q0 + dc * FL_BN, L - FL_BN);
        const u32x4* Kt = reinterpret_cast<const u32x4*>(K + (tokbase_qk + t0) * D);
        const u32x4* Vt = reinterpret_cast<const u32x4*>(V + (tokbase + t0) * D);
#pragma unroll
        for (int i = 0; i < NKP; ++i) {
            kreg[i] = Kt[tid + FL_THREADS * i];
            vreg[i] = Vt[tid + FL_THREADS * i];
        }
    };
    {
        u32x4 qreg[NQP];
#pragma unroll
        for (int i = 0; i < NQP; ++i) {
            const int e = tid + FL_THREADS * i;
            const int row = e / (D / 8), c8 = e % (D / 8);
            qreg[i] = *reinterpret_cast<const u32x4*>(Q + (tokbase_qk + min(q0 + row, L - 1)) * D + c8 * 8);
        }
        if (!chunk_routing) load_tile(0);
#pragma unroll
        for (int i = 0; i < NQP; ++i) {
            const int e = tid + FL_THREADS * i;
            *reinterpret_cast<u32x4*>(Qst + (e / (D / 8)) * RS + (e % (D / 8)) * 8) = qreg[i];
        }
    }
    const int n_tiles = (n_hi + FL_BN - 1) / FL_BN;
    // The tiles of this block in order: n_tiles compacted ones, then (routing per chunk) the chunks the
    // block's own queries lie in.  Tile i + 1 is loaded while tile i is used.
    // (own_chunk = 0: the variant in which only the linear operation computes the inner part of a chunk)
    const int n_own = (chunk_routing && own_chunk) ? (min(q0 + FL_BM, L) - q0) / FL_BN : 0;
    const int n_all = n_tiles + n_own;
    auto load_any = [&](int i) __attribute__((always_inline)) {
        if (i < n_tiles) load_tile(i); else load_own_chunk(i - n_tiles);
    };
    if (chunk_routing) load_any(0);   // which kind tile 0 is depends on the counts just read
    __syncthreads();
    u32x4 qf[FL_NQ][KS_D];
    int wave_hi = 0, wave_lo = 0x7fffffff;   // most and fewest keys visible to a query of this wavefront
#pragma unroll
    for (int nq = 0; nq < FL_NQ; ++nq) {
        const int ql = (wave * FL_NQ + nq) * 16 + l16;
        if (q0 + ql >= L) my_cnt[nq] = 0;   // rows past the end see nothing
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks)
            qf[nq][ks] = *reinterpret_cast<const u32x4*>(Qst + ql * RS + 32 * ks + 8 * lq);
        wave_hi = max(wave_hi, my_cnt[nq]);
        wave_lo = min(wave_lo, my_cnt[nq]);
    }
    wave_hi = wave_extreme_i32<true>(wave_hi);
    wave_lo = wave_extreme_i32<false>(wave_lo);

    f32x4 accO[FL_NQ][DT];
    float m_run[FL_NQ];
    f32x4 accL[FL_NQ];   // running sum of the weights, the same value in every row
#pragma unroll
    for (int nq = 0; nq < FL_NQ; ++nq) {
        m_run[nq] = -INFINITY;
        accL[nq] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int t = 0; t < DT; ++t) accO[nq][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    for (int kt = 0; kt < n_all; ++kt) {
        const bool own = kt >= n_tiles;      // one of the block's own chunks (uniform)
        const int dc = kt - n_tiles;
        __syncthreads();   // the previous tile (or the Q tile) is no longer read
#pragma unroll
        for (int i = 0; i < NKP; ++i) {   // registers -> LDS: K rows [key][d], V^T rows [d_v][key]
            const int e = tid + FL_THREADS * i;
            *reinterpret_cast<u32x4*>(Ks + (e / (D / 8)) * RS + (e % (D / 8)) * 8) = kreg[i];
            if (!own) {
                *reinterpret_cast<u32x4*>(Vs + (e >> 3) * TS + (e & 7) * 8) = vreg[i];
            } else {   // a piece of row `key` of V: transposed here, columns in the order the compaction kernel uses
                const int key = e / (D / 8), c8 = e % (D / 8);
                const half8 hv = bf16x8_to_half8(vreg[i]);
#pragma unroll
                for (int j = 0; j < 8; ++j) Vs[(c8 * 8 + j) * TS + vht_col(key)] = hv[j];
            }
        }
        __syncthreads();
        load_any(kt + 1 < n_all ? kt + 1 : kt);   // next tile in flight during this tile's products
        // keys of this tile visible to each of this lane's queries (may be <= 0 or >= 64)
        int vis[FL_NQ];
        bool full_tile, skip;
        if (!own) {
#pragma unroll
            for (int nq = 0; nq < FL_NQ; ++nq) vis[nq] = my_cnt[nq] - kt * FL_BN;
            full_tile = (kt + 1) * FL_BN <= wave_lo;
            skip = kt * FL_BN >= wave_hi;     // nothing visible to this wavefront in this tile (uniform)
        } else {
#pragma unroll
            for (int nq = 0; nq < FL_NQ; ++nq) {   // causal inside the chunk, the token itself included
                const int ql = (wave * FL_NQ + nq) * 16 + l16;
                vis[nq] = (q0 + ql < L) ? ql - dc * FL_BN + 1 : 0;
            }
            full_tile = false;
            skip = (wave * FL_NQ * 16) / FL_BN != dc;   // this wavefront's queries lie in another chunk (uniform)
        }
        if (skip) continue;

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
                const u32x4 fk = *reinterpret_cast<const u32x4*>(Ks + (16 * m + l16) * RS + 32 * ks + 8 * lq);
#pragma unroll
                for (int nq = 0; nq < FL_NQ; ++nq) accS[nq][m] = mfma16_bf16(fk, qf[nq][ks], accS[nq][m]);
            }
        // issue order: K fragments several reads ahead of the matrix instructions that take them
        __builtin_amdgcn_sched_group_barrier(0x100, FL_VAHEAD, 0);
#pragma unroll
        for (int i = 0; i < KS_D * 4; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, FL_NQ, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }

        // ---- online softmax per query column; P^T fragments ------------------------------------------
        // VALU work is what bounds this loop, so it is kept to one fused multiply-add, one exponential,
        // half a maximum and half a conversion per logit: masking only in tiles that are not visible in
        // full to every query of the wavefront; the sums of the weights are left to the matrix cores (see
        // below); the running maximum is raised only when the tile's maximum exceeds it by more than 2^8
        // (the weights then stay below 2^8, exact enough in fp16 and far from overflow), so rescaling of
        // the accumulators is rare and skipped by the whole wavefront.
        half8 pf[FL_NQ][2], pr[FL_NQ][2];   // pr (STATS): what rounding to fp16 left of the weights
#pragma unroll
        for (int nq = 0; nq < FL_NQ; ++nq) {
            if (!full_tile) {
#pragma unroll
                for (int m = 0; m < 4; ++m)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        if (16 * m + 4 * lq + j >= vis[nq]) accS[nq][m][j] = -INFINITY;
                    }
            }
            // Logits relative to the running maximum as it stands: the fused multiply-add's result feeds the
            // tile maximum and, unless the maximum is raised, the exponential as it is.
            const float m_old = m_run[nq];
            const float m_sub = m_old > -INFINITY ? m_old : 0.f;   // nothing visible yet: weights exp2(-inf) = 0
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j) accS[nq][m][j] = __builtin_fmaf(accS[nq][m][j], scale2, -m_sub);
            float tz = -INFINITY;
#pragma unroll
            for (int m = 0; m < 4; ++m)
                tz = fmaxf(fmaxf(tz, fmaxf(accS[nq][m][0], accS[nq][m][1])), fmaxf(accS[nq][m][2], accS[nq][m][3]));
            tz = quad_max(tz);
            const float tmax = tz + m_sub;
            const bool raise = tmax > m_old + 8.f;   // also true for the first visible key (m_old = -inf)
            if (__any(raise)) {
                const float corr = raise ? __builtin_amdgcn_exp2f(m_old - tmax) : 1.f;   // exp2(-inf) = 0
                const float delta = raise ? tz : 0.f;
                m_run[nq] = raise ? tmax : m_old;
#pragma unroll
                for (int m = 0; m < 4; ++m)
#pragma unroll
                    for (int j = 0; j < 4; ++j) accS[nq][m][j] -= delta;
                accL[nq][0] *= corr; accL[nq][1] *= corr; accL[nq][2] *= corr; accL[nq][3] *= corr;
#pragma unroll
                for (int t = 0; t < DT; ++t) {
                    accO[nq][t][0] *= corr; accO[nq][t][1] *= corr; accO[nq][t][2] *= corr; accO[nq][t][3] *= corr;
                }
            }
#pragma unroll
            for (int m = 0; m < 4; ++m)
#pragma unroll
                for (int j = 0; j < 4; ++j) accS[nq][m][j] = __builtin_amdgcn_exp2f(accS[nq][m][j]);
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {   // contraction step s2: slots 0-3 <- key tile 2 s2, 4-7 <- 2 s2 + 1
                const f32x4 lo = accS[nq][2 * s2], hi = accS[nq][2 * s2 + 1];   // weights <= 2^8: no clamp needed
                pf[nq][s2] = half8{(half_t)lo[0], (half_t)lo[1], (half_t)lo[2], (half_t)lo[3],
                                   (half_t)hi[0], (half_t)hi[1], (half_t)hi[2], (half_t)hi[3]};
                if (STATS) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        pr[nq][s2][j] = (half_t)(lo[j] - (float)pf[nq][s2][j]);
                        pr[nq][s2][4 + j] = (half_t)(hi[j] - (float)pf[nq][s2][4 + j]);
                    }
                }
            }
        }

        // ---- O^T += V^T P^T -----------------------------------------------------------------------
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                // the tile's columns were stored in contraction-slot order by the compaction kernel
                const half8 fv = lds_read8(Vs + (16 * t + l16) * TS + 32 * s2 + 8 * lq);
#pragma unroll
                for (int nq = 0; nq < FL_NQ; ++nq) {
                    accO[nq][t] = mfma16(fv, pf[nq][s2], accO[nq][t]);
                    if (STATS) accO[nq][t] = mfma16(fv, pr[nq][s2], accO[nq][t]);
                }
            }
        // The sums of the weights come from the same products: a 16-row tile of ones above V^T puts, in
        // every accumulator row, the sum over the keys of the fp16 weights that multiply V.
        {
            const half8 ones = half8{(half_t)1.f, (half_t)1.f, (half_t)1.f, (half_t)1.f,
                                     (half_t)1.f, (half_t)1.f, (half_t)1.f, (half_t)1.f};
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int nq = 0; nq < FL_NQ; ++nq) {
                    accL[nq] = mfma16(ones, pf[nq][s2], accL[nq]);
                    if (STATS) accL[nq] = mfma16(ones, pr[nq][s2], accL[nq]);
                }
        }
        // Issue order of this block: V^T fragments several reads ahead of the matrix instructions that take
        // them (the compiler's own order waits for every other read just before its use).
        if (!STATS) {
            __builtin_amdgcn_sched_group_barrier(0x100, FL_VAHEAD, 0);
#pragma unroll
            for (int i = 0; i < DT * 2; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, FL_NQ, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
        }
    }
    __syncthreads();   // tiles are dead: the region becomes the output staging

    if (!STATS && O_nla_out == nullptr) {
        // No fp32 copy of the branch's rows asked for: the normalised rows are staged as fp16, both 16-query groups
        // of the wavefront at once, so that all LDS writes, then all LDS reads, then all stores (16 bytes per lane,
        // full rows) are in flight together.  Read back, a row lies in D / 8 adjacent lanes beside the linear
        // branch's row (fp16 as well): the plain sum adds them; Eq. 21 and its ablation take the rows' mean squares
        // with sums over those lanes.
        constexpr int HS = D + 8;                 // staged row, fp16 elements
        constexpr int LPR_H = D / 8;              // lanes per row
        constexpr int RPP_H = 64 / LPR_H;         // rows per pass
        static_assert(4 * FL_NQ * 16 * HS * 2 <= LDS_BYTES, "fp16 output staging must fit the tile region");
        half_t* Oh = reinterpret_cast<half_t*>(smem) + wave * (FL_NQ * 16 * HS);
        // Eq. 22 here (W_out given: [heads_out][2][D] f32): the two logits of a query are dot products of its row with
        // the head's two weight vectors, and the query's row is still in this lane group's registers as the first
        // product's operand (lane (l16, lq) holds columns 32 ks + 8 lq .. + 7 of query l16): 8 D / 16 multiply-adds per
        // lane, a sum over the four lanes of the query, the activation; the weights go through LDS to the lanes that
        // merge the row.
        __shared__ float s_w[MERGED ? 2 : 1][MERGED ? FL_BM : 1];
        const bool fused_w = MERGED && combine_mode != 0 && W_out != nullptr;
        u32x4 la_rows[FL_NQ * 16 / RPP_H];   // the linear branch's rows (fp16), asked for up front (before the
        // weights' dot products below, which cover part of their latency)
        float wn_row[FL_NQ * 16 / RPP_H], wl_row[FL_NQ * 16 / RPP_H];   // the rows' weights (Eq. 21 and its ablation)
        const float w_default = combine_mode == 1 ? 0.5f : 1.f;
#pragma unroll
        for (int pass = 0; pass < FL_NQ * 16 / RPP_H; ++pass) {
            const int q = q0 + wave * FL_NQ * 16 + pass * RPP_H + lane / LPR_H;
            const size_t tok = tokbase + (q < L ? q : 0);
            la_rows[pass] = *reinterpret_cast<const u32x4*>(O_la + tok * D + 8 * (lane % LPR_H));
            wn_row[pass] = (combine_mode != 0 && !fused_w && w_nla != nullptr) ? w_nla[tok] : w_default;
            wl_row[pass] = (combine_mode != 0 && !fused_w && w_la != nullptr) ? w_la[tok] : w_default;
        }
        if (fused_w) {
            const float* w0 = W_out + (size_t)(bh % heads_out) * 2 * D;
            float lg[FL_NQ][2];
#pragma unroll
            for (int nq = 0; nq < FL_NQ; ++nq) lg[nq][0] = lg[nq][1] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks) {
                float wv[2][8];
#pragma unroll
                for (int k = 0; k < 2; ++k) {
                    const float4 x = *reinterpret_cast<const float4*>(w0 + k * D + 32 * ks + 8 * lq);
                    const float4 y = *reinterpret_cast<const float4*>(w0 + k * D + 32 * ks + 8 * lq + 4);
                    wv[k][0] = x.x; wv[k][1] = x.y; wv[k][2] = x.z; wv[k][3] = x.w;
                    wv[k][4] = y.x; wv[k][5] = y.y; wv[k][6] = y.z; wv[k][7] = y.w;
                }
#pragma unroll
                for (int nq = 0; nq < FL_NQ; ++nq)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float qa = __uint_as_float(qf[nq][ks][j] << 16), qb = __uint_as_float(qf[nq][ks][j] & 0xffff0000u);
                        lg[nq][0] += qa * wv[0][2 * j] + qb * wv[0][2 * j + 1];
                        lg[nq][1] += qa * wv[1][2 * j] + qb * wv[1][2 * j + 1];
                    }
            }
#pragma unroll
            for (int nq = 0; nq < FL_NQ; ++nq) {
                const float a = quad_sum(lg[nq][0]), b = quad_sum(lg[nq][1]);
                float wa, wb;
                if (weight_act == 0) {          // Eq. 22: softmax over the two logits
                    const float m = fmaxf(a, b);
                    const float ea = expf(a - m), eb = expf(b - m);
                    const float inv = 1.f / (ea + eb);
                    wa = ea * inv;
                    wb = eb * inv;
                } else if (weight_act == 1) {   // sigmoid weights
                    wa = 1.f / (1.f + expf(-a));
                    wb = 1.f / (1.f + expf(-b));
                } else {                        // linear weights
                    wa = a;
                    wb = b;
                }
                if (lq == 0) {
                    s_w[0][(wave * FL_NQ + nq) * 16 + l16] = wa;
                    s_w[1][(wave * FL_NQ + nq) * 16 + l16] = wb;
                }
            }
        }
#pragma unroll
        for (int nq = 0; nq < FL_NQ; ++nq) {
            const int q = q0 + (wave * FL_NQ + nq) * 16 + l16;
            const float l = accL[nq][0];
            const float inv_l = l > 0.f ? 1.f / l : 0.f;
            if (lse_out != nullptr && lq == 0 && q < L)
                lse_out[tokbase + q] = l > 0.f ? (m_run[nq] + __builtin_amdgcn_logf(l)) * 0.69314718055994531f : -INFINITY;
#pragma unroll
            for (int t = 0; t < DT; ++t)
                *reinterpret_cast<half4*>(Oh + (nq * 16 + l16) * HS + 16 * t + 4 * lq) =
                    to_half4(f32x4{accO[nq][t][0] * inv_l, accO[nq][t][1] * inv_l, accO[nq][t][2] * inv_l,
                                   accO[nq][t][3] * inv_l});
        }
        __builtin_amdgcn_wave_barrier();   // LDS operations of one wavefront complete in order
        u32x4 rows[FL_NQ * 16 / RPP_H];
#pragma unroll
        for (int pass = 0; pass < FL_NQ * 16 / RPP_H; ++pass) {
            rows[pass] = *reinterpret_cast<const u32x4*>(Oh + (pass * RPP_H + lane / LPR_H) * HS + 8 * (lane % LPR_H));
            if (fused_w) {   // this wavefront's own queries: written above by this wavefront
                wn_row[pass] = s_w[0][wave * FL_NQ * 16 + pass * RPP_H + lane / LPR_H];
                wl_row[pass] = s_w[1][wave * FL_NQ * 16 + pass * RPP_H + lane / LPR_H];
            }
        }
#pragma unroll
        for (int pass = 0; pass < FL_NQ * 16 / RPP_H; ++pass) {
            const int q = q0 + wave * FL_NQ * 16 + pass * RPP_H + lane / LPR_H;
            const half8 a = __builtin_bit_cast(half8, rows[pass]), b = __builtin_bit_cast(half8, la_rows[pass]);
            float o[8];
            if (combine_mode == 0) {   // O = O_la + O_nla (Section 4.1), rounded to bf16 once
#pragma unroll
                for (int j = 0; j < 8; ++j) o[j] = (float)a[j] + (float)b[j];
            } else {                   // (every lane of a row takes part in the row's sums: no lane leaves before them)
                float ssn = 0.f, ssl = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    ssn += (float)a[j] * (float)a[j];
                    ssl += (float)b[j] * (float)b[j];
                }
                float wn = wn_row[pass], wl = wl_row[pass];
                // (the hardware's reciprocal square root, one ulp: the rows are rounded to bf16 right after)
                if (combine_mode == 1) {   // Eq. 21: each branch normalised, then weighted
                    wn *= __builtin_amdgcn_rsqf(lane_group_sum<LPR_H>(ssn) * (1.f / D) + eps);
                    wl *= __builtin_amdgcn_rsqf(lane_group_sum<LPR_H>(ssl) * (1.f / D) + eps);
                }
                float ss = 0.f;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    o[j] = wn * (float)a[j] + wl * (float)b[j];
                    ss += o[j] * o[j];
                }
                if (combine_mode == 2) {   // one normalisation of the weighted sum
                    const float inv = __builtin_amdgcn_rsqf(lane_group_sum<LPR_H>(ss) * (1.f / D) + eps);
#pragma unroll
                    for (int j = 0; j < 8; ++j) o[j] *= inv;
                }
            }
            if (q >= L) continue;
            u32x4 w;
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = pack_bf16x2(o[2 * j], o[2 * j + 1]);
            *reinterpret_cast<u32x4*>(O + (tokbase + q) * D + 8 * (lane % LPR_H)) = w;
        }
        return;
    }

    // ---- epilogue: normalise; transpose each 16-query x D result through LDS so that every global
    //      access below is a full row segment; merge with the linear branch; store ------------------
    constexpr int LPR = D / 4;            // lanes per output row (float4 each)
    constexpr int RPP = 64 / LPR;         // rows per pass of a wavefront
    float* Ow = Ot + wave * 16 * OS;
    half4 lah_all[FL_NQ][16 / RPP];       // the linear branch's rows, all loads issued up front
#pragma unroll
    for (int nq = 0; nq < FL_NQ; ++nq)
#pragma unroll
        for (int pass = 0; pass < 16 / RPP; ++pass) {
            const int q = q0 + (wave * FL_NQ + nq) * 16 + pass * RPP + lane / LPR;
            lah_all[nq][pass] = half4{0, 0, 0, 0};
            if (!STATS)
                lah_all[nq][pass] =
                    *reinterpret_cast<const half4*>(O_la + (tokbase + (q < L ? q : 0)) * D + 4 * (lane % LPR));
        }
#pragma unroll
    for (int nq = 0; nq < FL_NQ; ++nq) {
        const int qbase = q0 + (wave * FL_NQ + nq) * 16;
        const float l = accL[nq][0];
        const float inv_l = l > 0.f ? 1.f / l : 0.f;
        if (lse_out != nullptr && lq == 0 && qbase + l16 < L)
            lse_out[tokbase + qbase + l16] =
                l > 0.f ? (m_run[nq] + __builtin_amdgcn_logf(l)) * 0.69314718055994531f : -INFINITY;
#pragma unroll
        for (int t = 0; t < DT; ++t)
            *reinterpret_cast<float4*>(Ow + l16 * OS + 16 * t + 4 * lq) =
                make_float4(accO[nq][t][0] * inv_l, accO[nq][t][1] * inv_l, accO[nq][t][2] * inv_l,
                            accO[nq][t][3] * inv_l);
        __builtin_amdgcn_wave_barrier();   // LDS operations of one wavefront complete in order
#pragma unroll
        for (int pass = 0; pass < 16 / RPP; ++pass) {
            const int row = pass * RPP + lane / LPR, c4 = lane % LPR;
            const int q = qbase + row;
            const bool live = q < L;
            const float4 x = *reinterpret_cast<const float4*>(Ow + row * OS + 4 * c4);
            const size_t off = (tokbase + (live ? q : 0)) * D + 4 * c4;
            if (O_nla_out != nullptr && live) *reinterpret_cast<float4*>(O_nla_out + off) = x;
            if (STATS) continue;
            const half4 lah = lah_all[nq][pass];
            const float la0 = (float)lah[0], la1 = (float)lah[1], la2 = (float)lah[2], la3 = (float)lah[3];
            float4 xs = x;
            if (combine_mode == 0) {   // the plain sum takes this branch's rows as fp16, as the path above does: same bits
                const half4 xh = to_half4(f32x4{x.x, x.y, x.z, x.w});
                xs = make_float4((float)xh[0], (float)xh[1], (float)xh[2], (float)xh[3]);
            }
            float wn = 1.f, wl = 1.f;
            if (combine_mode == 1) {          // Eq. 21: each branch normalised, then weighted
                const float ss_nla = lane_group_sum<LPR>(x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w);
                const float ss_la = lane_group_sum<LPR>(la0 * la0 + la1 * la1 + la2 * la2 + la3 * la3);
                wn = (w_nla ? w_nla[tokbase + (live ? q : 0)] : 0.5f) / sqrtf(ss_nla / D + eps);
                wl = (w_la ? w_la[tokbase + (live ? q : 0)] : 0.5f) / sqrtf(ss_la / D + eps);
            } else if (combine_mode == 2) {   // one normalisation of the (weighted) sum
                wn = w_nla ? w_nla[tokbase + (live ? q : 0)] : 1.f;
                wl = w_la ? w_la[tokbase + (live ? q : 0)] : 1.f;
            }
            float o0 = wn * xs.x + wl * la0, o1 = wn * xs.y + wl * la1, o2 = wn * xs.z + wl * la2, o3 = wn * xs.w + wl * la3;
            if (combine_mode == 2) {
                const float inv = 1.f / sqrtf(lane_group_sum<LPR>(o0 * o0 + o1 * o1 + o2 * o2 + o3 * o3) / D + eps);
                o0 *= inv; o1 *= inv; o2 *= inv; o3 *= inv;
            }
            if (live) {
                uint2 w;
                w.x = pack_bf16x2(o0, o1);
                w.y = pack_bf16x2(o2, o3);
                *reinterpret_cast<uint2*>(O + off) = w;
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
}

template <int D>
static void launch_fl(const FwdPlan& pl, const void* Q, const void* Kc, const void* VhT, const void* K,
                      const void* V, const int32_t* cnt,
                      const void* O_la, const float* w_nla, const float* w_la, void* O,
                      float* O_nla_out, float* lse_out, const float* W_out, hipStream_t st) {
    dim3 grid((unsigned)(((pl.L + FL_BM - 1) / FL_BM) * ((pl.BHG + 7) & ~7)));
    if (O == nullptr) {   // the backward pass's call: branch output and log-sum-exp only
        if (pl.routing == NATS_ROUTE_CHUNK)
            hipLaunchKernelGGL((flash_softmax_kernel<D, true, true, false>), grid, dim3(FL_THREADS), 0, st, (const bf16_t*)Q,
                               (const bf16_t*)Kc, (const half_t*)VhT, (const bf16_t*)K, (const bf16_t*)V, cnt, nullptr,
                               nullptr, nullptr, nullptr, O_nla_out, lse_out, pl.L, pl.softmax_scale, 0, pl.rms_eps, pl.BHG,
                               pl.G, pl.qk_per_out_head, pl.inner_chunk != 2, nullptr, 0, 1);
        else
            hipLaunchKernelGGL((flash_softmax_kernel<D, false, true, false>), grid, dim3(FL_THREADS), 0, st, (const bf16_t*)Q,
                               (const bf16_t*)Kc, (const half_t*)VhT, (const bf16_t*)K, (const bf16_t*)V, cnt, nullptr,
                               nullptr, nullptr, nullptr, O_nla_out, lse_out, pl.L, pl.softmax_scale, 0, pl.rms_eps, pl.BHG,
                               pl.G, pl.qk_per_out_head, pl.inner_chunk != 2, nullptr, 0, 1);
        return;
    }
    if (pl.combine_mode != 0) {   // Eq. 21, its ablation, Eq. 22: the instantiation with their code
        if (pl.routing == NATS_ROUTE_CHUNK)
            hipLaunchKernelGGL((flash_softmax_kernel<D, true, false, true>), grid, dim3(FL_THREADS), 0, st, (const bf16_t*)Q,
                               (const bf16_t*)Kc, (const half_t*)VhT, (const bf16_t*)K, (const bf16_t*)V, cnt,
                               (const half_t*)O_la, w_nla, w_la, (bf16_t*)O, O_nla_out, lse_out, pl.L,
                               pl.softmax_scale, pl.combine_mode, pl.rms_eps, pl.BHG, pl.G, pl.qk_per_out_head, pl.inner_chunk != 2,
                               W_out, pl.weight_act, pl.H * pl.G);
        else
            hipLaunchKernelGGL((flash_softmax_kernel<D, false, false, true>), grid, dim3(FL_THREADS), 0, st, (const bf16_t*)Q,
                               (const bf16_t*)Kc, (const half_t*)VhT, (const bf16_t*)K, (const bf16_t*)V, cnt,
                               (const half_t*)O_la, w_nla, w_la, (bf16_t*)O, O_nla_out, lse_out, pl.L,
                               pl.softmax_scale, pl.combine_mode, pl.rms_eps, pl.BHG, pl.G, pl.qk_per_out_head, pl.inner_chunk != 2,
                               W_out, pl.weight_act, pl.H * pl.G);
        return;
    }
    if (pl.routing == NATS_ROUTE_CHUNK)
        hipLaunchKernelGGL((flash_softmax_kernel<D, true, false, false>), grid, dim3(FL_THREADS), 0, st, (const bf16_t*)Q,
                           (const bf16_t*)Kc, (const half_t*)VhT, (const bf16_t*)K, (const bf16_t*)V, cnt,
                           (const half_t*)O_la, w_nla, w_la, (bf16_t*)O, O_nla_out, lse_out, pl.L,
                           pl.softmax_scale, pl.combine_mode, pl.rms_eps, pl.BHG, pl.G, pl.qk_per_out_head, pl.inner_chunk != 2,
                           W_out, pl.weight_act, pl.H * pl.G);
    else
        hipLaunchKernelGGL((flash_softmax_kernel<D, false, false, false>), grid, dim3(FL_THREADS), 0, st, (const bf16_t*)Q,
                           (const bf16_t*)Kc, (const half_t*)VhT, (const bf16_t*)K, (const bf16_t*)V, cnt,
                           (const half_t*)O_la, w_nla, w_la, (bf16_t*)O, O_nla_out, lse_out, pl.L,
                           pl.softmax_scale, pl.combine_mode, pl.rms_eps, pl.BHG, pl.G, pl.qk_per_out_head, pl.inner_chunk != 2,
                           W_out, pl.weight_act, pl.H * pl.G);
}

// reads O_la (fp16, the linear branch's rows), merges, writes O.  O = NULL: no merge, O_nla_out and lse_out (both
// required then) to fp32 accuracy.  W_out (or NULL): the merge weights made here from the kernel's queries by
// Eq. 22 instead of read from w_nla, w_la; only with O_nla_out = NULL, and Q must be the tensor Eq. 22 reads.
nats_status launch_flash_softmax(const FwdPlan& pl, const void* Q, const void* Kc, const void* VhT,
                                 const void* K, const void* V, const int32_t* cnt, const void* O_la, const float* w_nla,
                                 const float* w_la, void* O, float* O_nla_out, float* lse_out, hipStream_t st,
                                 const float* W_out) {
    if (W_out != nullptr && (O_nla_out != nullptr || O == nullptr)) {
        set_error("flash_softmax: weights by Eq. 22 inside the kernel need the merge without the fp32 side output");
        return NATS_ERR_UNSUPPORTED;
    }
    if (pl.d == 64) launch_fl<64>(pl, Q, Kc, VhT, K, V, cnt, O_la, w_nla, w_la, O, O_nla_out, lse_out, W_out, st);
    else launch_fl<128>(pl, Q, Kc, VhT, K, V, cnt, O_la, w_nla, w_la, O, O_nla_out, lse_out, W_out, st);
    return check_launch("flash_softmax");
}

}  // namespace nats
