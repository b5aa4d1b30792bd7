// Backward of the linear branch by chunks of 64 tokens, on fp32 matrix instructions (Section 4.2; the recurrence is
// Eq. 19 with the decay of Eq. 20, written for linear tokens only, Eq. 14).
//
// One chunk, with the state S0 [d_v][d_k] at its start, b' = beta (0 for a softmax token), gamma_r the product of the
// chunk's alphas up to token r, Gamma_ri = gamma_r / gamma_i, kd_i = gamma_C / gamma_i:
//     At = strict lower (Gamma . K K^T),  P = lower (Gamma . Q K^T),  T = (I + diag(b') At)^-1
//     R = V - diag(gamma) K S0^T,   U = T diag(b') R,   Uh = R - At U  (= v_t - Sd k_t, the residual of Eq. 19),
//     O = la (diag(gamma) Q S0^T + P U),   S1 = gamma_C S0 + U^T diag(kd) K.
// Given dO' = la dO and dS1 (from the chunks behind):
//     dU = P^T dO' + diag(kd) K dS1^T,   dRt = T^T dU,   dR = diag(b') dRt = dV,   dbeta_r = Uh_r . dRt_r
//     dS0 = gamma_C dS1 + dO'^T diag(gamma) Q - dR^T diag(gamma) K
//     dP = lower (dO' U^T),   dAt = - strict lower (dR U^T)
//     dQ = diag(gamma) dO' S0 + (dP . Gamma) K
//     dK = (dP . Gamma)^T Q + ((dAt . Gamma) + (dAt . Gamma)^T) K + diag(kd) U dS1 - diag(gamma) dR S0
//     d ln gamma_r = sum_i (dAt_ri At_ri + dP_ri P_ri) - sum_r' (dAt_r'r At_r'r + dP_r'r P_r'r)
//                    + gamma_r (Q_r . (dO' S0)_r - K_r . (dR S0)_r) - E_r,      E_i = kd_i K_i . (U dS1)_i
//     d ln gamma_C += sum_i E_i + gamma_C <dS1, S0>;     dalpha_t = (sum over r >= t of d ln gamma_r) / alpha_t.
// (The gated operation without the delta rule has At = 0, T = I, R = V: the terms that come from K S0^T drop.)
//
// Four kinds of kernel: the operands of every chunk (parallel over chunks), the states at the chunk starts (forwards
// along the sequence), the state gradients (backwards along it), and the gradients of every chunk from those
// (parallel over chunks).  Columns of V (rows of the state) never mix along the sequence, so the two sequential
// kernels split every (batch, head) into slices of 16 value columns, one block each.
//
// Matrix instruction used throughout: v_mfma_f32_16x16x4_f32 through mac16 (sixteen contraction indices in four
// instructions, a lane's A operands four consecutive elements of a row: one 16-byte LDS read when the buffer is
// contiguous along the contraction index).
#include <type_traits>

#include "nats_common.h"
#include "mfma_util.h"

namespace nats {

constexpr int CB_C = 64;          // chunk
constexpr int CB_MS = CB_C + 4;   // row stride (floats) of a 64 x 64 operand in LDS
constexpr int CB_NV = 16;         // value columns per block of the sequential kernels

struct ChunkOps {   // per chunk: Tm, At, Pm [64][64] f32 row-major;  per token: g2 (log2 of gamma), gam, kd, bp;  per chunk: gamC
    float *Tm, *At, *Pm, *g2, *gam, *kd, *bp, *gamC;
};

// a 16-byte word of T as it came from memory -> floats (8 for bf16, 4 for fp32)
__device__ __forceinline__ void unpack16(const u32x4 w, float (&out)[8], bf16_t) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        out[2 * q] = __uint_as_float(w[q] << 16);
        out[2 * q + 1] = __uint_as_float(w[q] & 0xffff0000u);
    }
}
__device__ __forceinline__ void unpack16(const u32x4 w, float (&out)[4], float) {
#pragma unroll
    for (int q = 0; q < 4; ++q) out[q] = __uint_as_float(w[q]);
}

// ---- operands of a chunk ---------------------------------------------------------------------------------------------
// One block per (chunk, batch*head).  Products in fp32 from the inputs as given (bf16 converts exactly); the inverse
// by 16 x 16 blocks: forward substitution on the diagonal, matrix instructions below it.
template <typename T, int D>
__global__ __launch_bounds__(256) void gdn_bwd_prep_kernel(const T* __restrict__ Q, const T* __restrict__ K,
                                                           const float* __restrict__ alpha, const float* __restrict__ beta,
                                                           const uint8_t* __restrict__ mask, const ChunkOps o, const int L,
                                                           const int BH, const int freeze_on_softmax, const int linear_op,
                                                           const int chunk_mask) {
    constexpr int KS = D + 4, E = Vec16<T>::N, NP = CB_C * D / E / 256;
    extern __shared__ __align__(16) float cb_smem[];
    float* Ks = cb_smem;
    float* Qs = cb_smem + CB_C * KS;
    float* As = Qs;                         // after the products: diag(b') At, [64][CB_MS]
    float* s_g = cb_smem + 2 * CB_C * KS;   // log2 gamma
    float* s_bp = s_g + CB_C;
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const int n_chunks = L / CB_C;
    const int bh = blockIdx.x % BH, chunk = blockIdx.x / BH;
    const size_t gc = (size_t)bh * n_chunks + chunk, tok0 = (size_t)bh * L + (size_t)chunk * CB_C;
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const int e = tid + 256 * i, row = e / (D / E), c = (e % (D / E)) * E;
        float tmp[E];
        Vec16<T>::load(K + (tok0 + row) * D + c, tmp);
#pragma unroll
        for (int j = 0; j < E; j += 4) *reinterpret_cast<float4*>(Ks + row * KS + c + j) = make_float4(tmp[j], tmp[j + 1], tmp[j + 2], tmp[j + 3]);
        Vec16<T>::load(Q + (tok0 + row) * D + c, tmp);
#pragma unroll
        for (int j = 0; j < E; j += 4) *reinterpret_cast<float4*>(Qs + row * KS + c + j) = make_float4(tmp[j], tmp[j + 1], tmp[j + 2], tmp[j + 3]);
    }
    if (w == 0) {
        // Routing per token: a softmax token writes nothing (b' = 0) and, in the variant without decay there, its
        // alpha counts as 1.  Routing per chunk (mask: one byte per chunk): every token writes inside its chunk, and
        // a softmax chunk hands on only (its decay) x (the state at its start): kd = 0, and the carried decay is 1
        // in the variant without decay (inside the chunk the decays still act on the provisional state).
        const bool soft = !chunk_mask && mask[tok0 + lane] != 0;
        const bool soft_chunk = chunk_mask && mask[gc] != 0;
        const float a = (freeze_on_softmax && soft) ? 1.f : alpha[tok0 + lane];
        float g = __builtin_amdgcn_logf(fmaxf(a, 1e-30f));   // log2; inclusive scan over the 64 lanes
        g += dpp_move<0x111>(g);
        g += dpp_move<0x112>(g);
        g += dpp_move<0x114>(g);
        g += dpp_move<0x118>(g);
        g += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(g), 0x142, 0xA, 0xF, false));
        g += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(g), 0x143, 0xC, 0xF, false));
        const float gC = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(g), 63));
        const float gam = __builtin_amdgcn_exp2f(g);
        const float bp = soft ? 0.f : beta[tok0 + lane];
        s_g[lane] = g;
        s_bp[lane] = bp;
        o.g2[tok0 + lane] = g;
        o.gam[tok0 + lane] = gam;
        o.kd[tok0 + lane] = soft_chunk ? 0.f : __builtin_amdgcn_exp2f(gC - g);
        o.bp[tok0 + lane] = bp;
        if (lane == 63) o.gamC[gc] = (freeze_on_softmax && soft_chunk) ? 1.f : gam;
    }
    __syncthreads();
    // the 10 lower tiles (a, b), b <= a, of K K^T and Q K^T: tile t of the list to wavefront t % 4
    float* Ato = o.At + gc * (CB_C * CB_C);
    float* Pmo = o.Pm + gc * (CB_C * CB_C);
    float* Tmo = o.Tm + gc * (CB_C * CB_C);
    f32x4 keepA[3];
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        const int t = w + 4 * s;   // uniform
        keepA[s] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (t < 10) {
            const int a = (0x3333222110 >> (4 * t)) & 15, b = (0x3210210100 >> (4 * t)) & 15;
            f32x4 accK = {0.f, 0.f, 0.f, 0.f}, accQ = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
            for (int kt = 0; kt < D / 16; ++kt) {
                const float4 bk = ld4(Ks + (16 * b + l16) * KS + 16 * kt + 4 * lq);
                accK = mac16(ld4(Ks + (16 * a + l16) * KS + 16 * kt + 4 * lq), bk, accK);
                accQ = mac16(ld4(Qs + (16 * a + l16) * KS + 16 * kt + 4 * lq), bk, accQ);
            }
            const int i = 16 * b + l16;
            const float gi = s_g[i];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = 16 * a + 4 * lq + j;
                const float G = __builtin_amdgcn_exp2f(s_g[r] - gi);
                const float at = (i < r && linear_op == 0) ? G * accK[j] : 0.f;
                Ato[r * CB_C + i] = at;
                Pmo[r * CB_C + i] = (i <= r) ? G * accQ[j] : 0.f;
                keepA[s][j] = s_bp[r] * at;
            }
        }
    }
    // the 6 tiles above the diagonal are zeros (T's come out of the substitution below)
    for (int z = w; z < 6; z += 4) {
        const int a = (0x211000 >> (4 * z)) & 15, b = (0x332321 >> (4 * z)) & 15;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int off = (16 * a + 4 * lq + j) * CB_C + 16 * b + l16;
            Ato[off] = 0.f;
            Pmo[off] = 0.f;
        }
    }
    __syncthreads();   // the Q tile is dead: its region takes diag(b') At
#pragma unroll
    for (int s = 0; s < 3; ++s) {
        const int t = w + 4 * s;
        if (t < 10) {
            const int a = (0x3333222110 >> (4 * t)) & 15, b = (0x3210210100 >> (4 * t)) & 15;
#pragma unroll
            for (int j = 0; j < 4; ++j) As[(16 * a + 4 * lq + j) * CB_MS + 16 * b + l16] = keepA[s][j];
        }
    }
    __syncthreads();
    // T = (I + A)^-1, unit lower triangular, by 16 x 16 blocks (K's region, dead since the products, holds T).
    // (a) Diagonal blocks: wavefront b inverts I + A_bb by forward substitution, lane j < 16 owns column j:
    //     T[r][j] = [r == j] - sum over i < r of A[r][i] T[i][j]  (entries above the diagonal come out as exact zeros).
    float* Ts = Ks;   // [64][CB_MS]
    if (lane < 16) {
        const float* Ab = As + (16 * w) * CB_MS + 16 * w;
        float col[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float acc = 0.f;
#pragma unroll
            for (int i4 = 0; i4 < (r + 3) / 4; ++i4) {
                const float4 a4 = ld4(Ab + r * CB_MS + 4 * i4);
                acc += a4.x * col[4 * i4];
                if (4 * i4 + 1 < r) acc += a4.y * col[4 * i4 + 1];
                if (4 * i4 + 2 < r) acc += a4.z * col[4 * i4 + 2];
                if (4 * i4 + 3 < r) acc += a4.w * col[4 * i4 + 3];
            }
            col[r] = ((r == lane) ? 1.f : 0.f) - acc;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) Ts[(16 * w + r) * CB_MS + 16 * w + lane] = col[r];
    }
    __syncthreads();
    // (b) Blocks below the diagonal: T_ab = - T_aa sum over b <= k < a of A_ak T_kb.  Wavefront b owns block column b
    //     and walks down it; the sum's result tile is the right operand of the product with T_aa as it sits in
    //     registers.
    for (int ta = w + 1; ta < 4; ++ta) {
        f32x4 X = {0.f, 0.f, 0.f, 0.f};
        for (int k = w; k < ta; ++k)
            X = mac16(ld4(As + (16 * ta + l16) * CB_MS + 16 * k + 4 * lq), ld4col(Ts + (16 * k + 4 * lq) * CB_MS + 16 * w + l16, CB_MS), X);
        const f32x4 Y = mac16(ld4(Ts + (16 * ta + l16) * CB_MS + 16 * ta + 4 * lq), make_float4(X[0], X[1], X[2], X[3]),
                              f32x4{0.f, 0.f, 0.f, 0.f});
#pragma unroll
        for (int j = 0; j < 4; ++j) Ts[(16 * ta + 4 * lq + j) * CB_MS + 16 * w + l16] = -Y[j];
        __builtin_amdgcn_wave_barrier();   // LDS operations of one wavefront complete in order
    }
    __syncthreads();
    // (c) out, 16 bytes per thread and step; the tiles above the diagonal were never written: zeros
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int e = tid + 256 * i, r = e / 16, c4 = (e % 16) * 4;
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        if ((c4 >> 4) <= (r >> 4)) t = ld4(Ts + r * CB_MS + c4);
        *reinterpret_cast<float4*>(Tmo + r * CB_C + c4) = t;
    }
}

// ---- the states along the sequence -------------------------------------------------------------------------------------
// DIR 0: forwards, the state S^T [d_k][16] of the block's 16 value columns; leaves S0 of every chunk (ck), U and Uh.
// DIR 1: backwards, the gradient of that state; leaves dS1 of every chunk (ck), dV, the block's share of dbeta and the
// gradient of the initial state.  Wavefront w owns the chunk's tokens 16 w .. 16 w + 15 in everything that is one
// row per token, and D / 64 of the state's 16 x 16 tiles.
template <typename T>
struct SeqArgs {
    const T *K, *Q, *X;            // X: V (DIR 0) or dO (DIR 1), [BH][L][D]
    ChunkOps o;
    const uint8_t* mask;
    const float* S_init;           // DIR 0: [BH][D][D] or NULL
    float* ck;                     // [BH][L/64][D][D]
    float *Ug, *Uh;                // [BH][L][D]: DIR 0 writes both, DIR 1 reads Uh
    float *dV, *dbeta_part, *dS0;  // DIR 1
    int L, BH;
    float la_scale;
    int delta;                     // 1: delta rule; 0: gated linear attention
};

// Eight wavefronts: four compute (as above), four only move the next chunk's operands from global memory to LDS.
// A burst of loads of this size keeps a wavefront at the issue of its memory instructions for about as long as a
// whole phase of the chunk's products takes, and there is one block per CU with nothing else to fill the time:
// so the wavefronts that multiply issue no global loads at all.  What is staged has two places in LDS where that
// fits (K, Q and the per-token vectors; At forwards), so the next chunk is written while this one is multiplied;
// T and (backwards) P have one place and are replaced once their last reader of the chunk is past, behind the
// second barrier.
// With fp32 tensors the backward direction has room for one place only: there the staged operands are replaced
// between the third barrier and a fourth.
template <typename T, int D, int DIR>
struct SeqLds {
    static constexpr bool two = !(DIR == 1 && sizeof(T) == 4);   // two places for K, Q and the small operands
    static constexpr int NB = two ? 2 : 1;
    static constexpr int MS = CB_MS;
    // K and Q in LDS: fp32 forwards (the moving wavefronts widen bf16 once: widening at every read costs the
    // multiplying wavefronts more than the second place saves); backwards, where two places for K and Q in fp32 do
    // not fit, in the tensors' own type (bf16 is widened when read)
    static constexpr bool wide = DIR == 0 || sizeof(T) == 4;
    static constexpr int KE_BYTES = wide ? 4 : 2;
    static constexpr int KS = D + (wide ? 4 : 8);                // row stride of K, Q (elements)
    static constexpr int KQ_BYTES = CB_C * KS * KE_BYTES * (DIR ? 2 : 1);   // K, then (DIR 1) Q
    static constexpr int M_BYTES = CB_C * MS * 4;
    static constexpr int NB2 = DIR ? 1 : NB;                     // places of M2: At (DIR 0) as K; P (DIR 1) one
    static constexpr int B_BYTES = CB_NV * MS * 4;               // a [16 v][MS] operand with tokens as contraction index
    // small operands of a chunk: Xt, Gt (256 floats), and (DIR 1) dO' and diag(gamma) dO'
    static constexpr int SM_BYTES = B_BYTES + 256 * 4 + (DIR ? 2 * B_BYTES : 0);
    static constexpr int o_kq = 0;
    static constexpr int o_m1 = o_kq + NB * KQ_BYTES;
    static constexpr int o_m2 = o_m1 + M_BYTES;
    static constexpr int o_sm = o_m2 + NB2 * M_BYTES;
    static constexpr int o_st = o_sm + NB * SM_BYTES;
    static constexpr int o_b = o_st + CB_NV * (D + 4) * 4;       // DIR 0: B0, B1, B2;  DIR 1: B2, B3
    static constexpr int bytes = o_b + (DIR ? 2 : 3) * B_BYTES;
};

__device__ __forceinline__ float4 ldk4(const float* p) { return ld4(p); }
__device__ __forceinline__ float4 ldk4(const uint16_t* p) { return ldb4(p); }
__device__ __forceinline__ float4 ldkcol(const float* p, int rs) { return ld4col(p, rs); }
__device__ __forceinline__ float4 ldkcol(const uint16_t* p, int rs) { return ldbcol(p, rs); }

template <typename T, int D, int DIR>
__global__ __launch_bounds__(512) void gdn_chunk_seq_kernel(const SeqArgs<T> a) {
    using LY = SeqLds<T, D, DIR>;
    using KE = typename std::conditional<LY::wide, float, uint16_t>::type;   // K, Q in LDS
    constexpr int KS = LY::KS, SS = D + 4, NP = CB_C * D * (int)sizeof(T) / 16 / 256, KT = D / 64, MS = CB_MS, NB = LY::NB;
    constexpr int EPW = 16 / (int)sizeof(T);   // elements of a 16-byte word
    extern __shared__ __align__(16) float cb_smem[];
    unsigned char* lds = reinterpret_cast<unsigned char*>(cb_smem);
    auto Ksb = [&](int i) { return reinterpret_cast<KE*>(lds + LY::o_kq + i * LY::KQ_BYTES); };
    auto Qsb = [&](int i) { return Ksb(i) + CB_C * KS; };                               // DIR 1
    float* M1 = reinterpret_cast<float*>(lds + LY::o_m1);                                 // T
    auto M2b = [&](int i) { return reinterpret_cast<float*>(lds + LY::o_m2 + (DIR ? 0 : i) * LY::M_BYTES); };   // At / P
    auto Xtb = [&](int i) { return reinterpret_cast<float*>(lds + LY::o_sm + i * LY::SM_BYTES); };   // V or Uh, [16 v][MS]
    auto Gtb = [&](int i) { return Xtb(i) + CB_NV * MS; };       // gam, kd, bp [64] each, gamC, then (DIR 1) 64 mask bytes
    auto B0b = [&](int i) { return Gtb(i) + 256; };              // DIR 1: dO' with the tokens as contraction index
    auto B1b = [&](int i) { return B0b(i) + CB_NV * MS; };       // DIR 1: diag(gamma) dO'
    float* St = reinterpret_cast<float*>(lds + LY::o_st);       // state, [16 v][SS]
    float* Bx = reinterpret_cast<float*>(lds + LY::o_b);        // exchange between the wavefronts, [16 v][MS] each
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave >= 4;
    const int w = wave & 3, lt = tid & 255;
    const int l16 = lane & 15, lq = lane >> 4;
    const int bh = blockIdx.x % a.BH, slice = blockIdx.x / a.BH, v0 = CB_NV * slice;
    const int L = a.L, n_chunks = L / CB_C;
    const size_t n_tok = (size_t)a.BH * L;
    const float delta = a.delta ? 1.f : 0.f;

    // The two kinds of wavefront run loops of their own with the same number of barriers (a barrier counts
    // arrivals, wherever in the code they come from): what one kind keeps in registers across a chunk then takes
    // no registers from the other.
    if (loader) {
        u32x4 kreg[NP], qreg[DIR ? NP : 1];
        float4 m1reg[4], m2reg[4], gate4 = make_float4(0.f, 0.f, 0.f, 0.f), g4n = gate4;
        T xvn[4];
        float uhn[4] = {0.f, 0.f, 0.f, 0.f}, gCn = 0.f;
        uint32_t linn = 0;
        auto fetch = [&](int c) {   // as it comes from memory: a conversion here would wait for the load
            const size_t gc = (size_t)bh * n_chunks + c, tok0 = (size_t)bh * L + (size_t)c * CB_C;
#pragma unroll
            for (int i = 0; i < NP; ++i) {   // a chunk's rows are contiguous
                kreg[i] = reinterpret_cast<const u32x4*>(a.K + tok0 * D)[lt + 256 * i];
                if (DIR) qreg[i] = reinterpret_cast<const u32x4*>(a.Q + tok0 * D)[lt + 256 * i];
            }
            if (lt < 48) gate4 = ld4((lt < 16 ? a.o.gam : lt < 32 ? a.o.kd : a.o.bp) + tok0 + 4 * (lt & 15));
            if (lt == 48) gCn = a.o.gamC[gc];
            if (DIR && a.mask != nullptr && lt >= 64 && lt < 80)   // NULL: routing per chunk, every token of a chunk writes
                linn = *reinterpret_cast<const uint32_t*>(a.mask + tok0 + 4 * (lt - 64));
            const size_t t4 = tok0 + 16 * w + 4 * lq;
            if (DIR) g4n = ld4(a.o.gam + t4);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                xvn[j] = a.X[(t4 + j) * D + v0 + l16];
                if (DIR) uhn[j] = a.Uh[(t4 + j) * D + v0 + l16];
            }
            const float* m1 = a.o.Tm + gc * (CB_C * CB_C);
            const float* m2 = (DIR ? a.o.Pm : a.o.At) + gc * (CB_C * CB_C);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                m2reg[i] = ld4(m2 + 4 * (lt + 256 * i));
                m1reg[i] = ld4(m1 + 4 * (lt + 256 * i));
            }
        };
        auto put_kq_small = [&](int nb) {
            KE* Ks = Ksb(nb);
            KE* Qs = Qsb(nb);
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int e = lt + 256 * i, row = e / (D / EPW), cc = (e % (D / EPW)) * EPW;
                if (sizeof(KE) == sizeof(T)) {   // as they are
                    *reinterpret_cast<u32x4*>(Ks + row * KS + cc) = kreg[i];
                    if (DIR) *reinterpret_cast<u32x4*>(Qs + row * KS + cc) = qreg[i];
                } else {                          // bf16 widened here (forwards only: no Q)
                    float kf[EPW];
                    unpack16(kreg[i], kf, T{});
#pragma unroll
                    for (int j = 0; j < EPW; j += 4)
                        *reinterpret_cast<float4*>(reinterpret_cast<float*>(Ks) + row * KS + cc + j) = make_float4(kf[j], kf[j + 1], kf[j + 2], kf[j + 3]);
                }
            }
            float* Gt = Gtb(nb);
            if (lt < 48) *reinterpret_cast<float4*>(Gt + 4 * lt) = gate4;
            if (lt == 48) Gt[3 * CB_C] = gCn;
            if (DIR && lt >= 64 && lt < 80) reinterpret_cast<uint32_t*>(Gt + 3 * CB_C + 4)[lt - 64] = linn;
            if (DIR == 0) {
                *reinterpret_cast<float4*>(Xtb(nb) + l16 * MS + 16 * w + 4 * lq) =
                    make_float4(to_float(xvn[0]), to_float(xvn[1]), to_float(xvn[2]), to_float(xvn[3]));
            } else {   // Uh; dO' and diag(gamma) dO' with the tokens as contraction index
                *reinterpret_cast<float4*>(Xtb(nb) + l16 * MS + 16 * w + 4 * lq) = make_float4(uhn[0], uhn[1], uhn[2], uhn[3]);
                float4 x, y;
                x.x = a.la_scale * to_float(xvn[0]); x.y = a.la_scale * to_float(xvn[1]);
                x.z = a.la_scale * to_float(xvn[2]); x.w = a.la_scale * to_float(xvn[3]);
                y.x = g4n.x * x.x; y.y = g4n.y * x.y; y.z = g4n.z * x.z; y.w = g4n.w * x.w;
                *reinterpret_cast<float4*>(B0b(nb) + l16 * MS + 16 * w + 4 * lq) = x;
                *reinterpret_cast<float4*>(B1b(nb) + l16 * MS + 16 * w + 4 * lq) = y;
            }
        };
        auto put_m = [&](float* M, const float4 (&r)[4]) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int e = lt + 256 * i, row = e / 16, c4 = (e % 16) * 4;
                *reinterpret_cast<float4*>(M + row * MS + c4) = r[i];
            }
        };
        // Chunk ci + 1 is written to LDS behind the second barrier of chunk ci (by then its loads, issued a chunk
        // earlier, have long arrived, and the readers of T and P are past), and the loads of chunk ci + 2 are issued
        // right after: the first two barriers of a chunk never wait for these wavefronts.
        auto chunk_at = [&](int ci) { return DIR ? n_chunks - 1 - ci : ci; };
        fetch(chunk_at(0));
        put_kq_small(0);
        put_m(M2b(0), m2reg);
        put_m(M1, m1reg);
        if (n_chunks > 1) fetch(chunk_at(1));
        __syncthreads();
        for (int ci = 0; ci < n_chunks; ++ci) {
            const int nb = (ci + 1) % NB;
            const bool more = ci + 1 < n_chunks;
            __syncthreads();
            __syncthreads();
            if (more) {
                if (LY::two) put_kq_small(nb);
                put_m(M2b(nb), m2reg);
                put_m(M1, m1reg);
            }
            if (LY::two && ci + 2 < n_chunks) fetch(chunk_at(ci + 2));
            __syncthreads();
            if (!LY::two) {   // one place for K, Q and the per-token vectors: replaced between the third barrier and a fourth
                if (more) put_kq_small(0);
                if (ci + 2 < n_chunks) fetch(chunk_at(ci + 2));
                __syncthreads();
            }
        }
        return;
    }

    // the state: tiles kt = KT w + t, element [k = 16 kt + 4 lq + j][v = l16]
    f32x4 Sacc[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t) {
        const int kt = KT * w + t;
        float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
        if (DIR == 0 && a.S_init != nullptr) s = ld4(a.S_init + ((size_t)bh * D + v0 + l16) * D + 16 * kt + 4 * lq);
        Sacc[t] = f32x4{s.x, s.y, s.z, s.w};
        *reinterpret_cast<float4*>(St + l16 * SS + 16 * kt + 4 * lq) = s;
    }
    __syncthreads();

    for (int ci = 0; ci < n_chunks; ++ci) {
        const int c = DIR ? n_chunks - 1 - ci : ci, cb = ci % NB;
        const size_t gc = (size_t)bh * n_chunks + c;
        const size_t t4 = (size_t)bh * L + (size_t)c * CB_C + 16 * w + 4 * lq;   // the lane's first token
        const KE* Ks = Ksb(cb);
        const KE* Qs = Qsb(cb);
        const float* M2 = M2b(cb);
        const float* Gt = Gtb(cb);
        // exchange buffers: DIR 0: B0 = b' R, B1 = U, B2 = kd U;  DIR 1: B0, B1 staged (dO', gamma dO'), B2 = dU, B3 = -gamma dR
        float* B0 = DIR ? B0b(cb) : Bx;
        float* B1 = DIR ? B1b(cb) : Bx + CB_NV * MS;
        float* B2 = DIR ? Bx : Bx + 2 * CB_NV * MS;
        float* B3 = Bx + CB_NV * MS;   // DIR 1
        float gg[4], kk[4], bb[4], xv[4], R[4];
        {
            const float4 g4 = ld4(Gt + 16 * w + 4 * lq), kd4 = ld4(Gt + CB_C + 16 * w + 4 * lq);
            const float4 bp4 = ld4(Gt + 2 * CB_C + 16 * w + 4 * lq), x4 = ld4(Xtb(cb) + l16 * MS + 16 * w + 4 * lq);
            gg[0] = g4.x; gg[1] = g4.y; gg[2] = g4.z; gg[3] = g4.w;
            kk[0] = kd4.x; kk[1] = kd4.y; kk[2] = kd4.z; kk[3] = kd4.w;
            bb[0] = bp4.x; bb[1] = bp4.y; bb[2] = bp4.z; bb[3] = bp4.w;
            xv[0] = x4.x; xv[1] = x4.y; xv[2] = x4.z; xv[3] = x4.w;
        }
        const float gC = Gt[3 * CB_C];
        const uint32_t lin = DIR ? reinterpret_cast<const uint32_t*>(Gt + 3 * CB_C + 4)[4 * w + lq] : 0u;
        // ---- 1: the state seen by the wavefront's tokens: K_w S^T --------------------------------------------
        {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
            for (int kt = 0; kt < D / 16; ++kt)
                acc = mac16(ldk4(Ks + (16 * w + l16) * KS + 16 * kt + 4 * lq), ld4(St + l16 * SS + 16 * kt + 4 * lq), acc);
            if (DIR == 0) {
                float4 br;
#pragma unroll
                for (int j = 0; j < 4; ++j) R[j] = xv[j] - delta * gg[j] * acc[j];
                br.x = bb[0] * R[0]; br.y = bb[1] * R[1]; br.z = bb[2] * R[2]; br.w = bb[3] * R[3];
                *reinterpret_cast<float4*>(B0 + l16 * MS + 16 * w + 4 * lq) = br;
            } else {
                // dU = P^T dO' + diag(kd) K dS1^T: rows of P behind the wavefront's tokens
                f32x4 accP = {0.f, 0.f, 0.f, 0.f};
                for (int ta = w; ta < 4; ++ta)
                    accP = mac16(ld4col(M2 + (16 * ta + 4 * lq) * MS + 16 * w + l16, MS), ld4(B0 + l16 * MS + 16 * ta + 4 * lq), accP);
                float4 du;
                du.x = kk[0] * acc[0] + accP[0]; du.y = kk[1] * acc[1] + accP[1];
                du.z = kk[2] * acc[2] + accP[2]; du.w = kk[3] * acc[3] + accP[3];
                *reinterpret_cast<float4*>(B2 + l16 * MS + 16 * w + 4 * lq) = du;
            }
        }
        __syncthreads();
        // ---- 2: through the inverse ------------------------------------------------------------------------
        if (DIR == 0) {
            f32x4 U = {0.f, 0.f, 0.f, 0.f};
            for (int tb = 0; tb <= w; ++tb)
                U = mac16(ld4(M1 + (16 * w + l16) * MS + 16 * tb + 4 * lq), ld4(B0 + l16 * MS + 16 * tb + 4 * lq), U);
            *reinterpret_cast<float4*>(B1 + l16 * MS + 16 * w + 4 * lq) = make_float4(U[0], U[1], U[2], U[3]);
            *reinterpret_cast<float4*>(B2 + l16 * MS + 16 * w + 4 * lq) = make_float4(kk[0] * U[0], kk[1] * U[1], kk[2] * U[2], kk[3] * U[3]);
#pragma unroll
            for (int j = 0; j < 4; ++j) a.Ug[(t4 + j) * D + v0 + l16] = U[j];
        } else {
            f32x4 Rt = {0.f, 0.f, 0.f, 0.f};
            for (int ta = w; ta < 4; ++ta)
                Rt = mac16(ld4col(M1 + (16 * ta + 4 * lq) * MS + 16 * w + l16, MS), ld4(B2 + l16 * MS + 16 * ta + 4 * lq), Rt);
            float4 ng;
            float dr[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                dr[j] = bb[j] * Rt[j];
                a.dV[(t4 + j) * D + v0 + l16] = dr[j];
                const float sdb = lane_group_sum<16>(xv[j] * Rt[j]);   // xv: Uh
                if (l16 == 0) a.dbeta_part[(size_t)slice * n_tok + t4 + j] = ((lin >> (8 * j)) & 0xff) ? 0.f : sdb;
            }
            ng.x = -delta * gg[0] * dr[0]; ng.y = -delta * gg[1] * dr[1]; ng.z = -delta * gg[2] * dr[2]; ng.w = -delta * gg[3] * dr[3];
            *reinterpret_cast<float4*>(B3 + l16 * MS + 16 * w + 4 * lq) = ng;
        }
        __syncthreads();
        // ---- 3: the chunk's contribution to the state ------------------------------------------------------------
        if (DIR == 0) {
            f32x4 AU = {0.f, 0.f, 0.f, 0.f};
            for (int tb = 0; tb <= w; ++tb)
                AU = mac16(ld4(M2 + (16 * w + l16) * MS + 16 * tb + 4 * lq), ld4(B1 + l16 * MS + 16 * tb + 4 * lq), AU);
#pragma unroll
            for (int j = 0; j < 4; ++j) a.Uh[(t4 + j) * D + v0 + l16] = R[j] - AU[j];
        }
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            const int kt = KT * w + t;
            *reinterpret_cast<float4*>(a.ck + (gc * D + v0 + l16) * D + 16 * kt + 4 * lq) =
                make_float4(Sacc[t][0], Sacc[t][1], Sacc[t][2], Sacc[t][3]);
            Sacc[t][0] *= gC; Sacc[t][1] *= gC; Sacc[t][2] *= gC; Sacc[t][3] *= gC;
        }
#pragma unroll 2
        for (int tb = 0; tb < 4; ++tb) {   // token tiles outside: their operands serve all of the wavefront's state tiles
            const float4 b2 = ld4((DIR ? B1 : B2) + l16 * MS + 16 * tb + 4 * lq);
            const float4 b3 = DIR ? ld4(B3 + l16 * MS + 16 * tb + 4 * lq) : b2;
#pragma unroll
            for (int t = 0; t < KT; ++t) {
                const int kt = KT * w + t;
                if (DIR == 0) {
                    Sacc[t] = mac16(ldkcol(Ks + (16 * tb + 4 * lq) * KS + 16 * kt + l16, KS), b2, Sacc[t]);
                } else {
                    Sacc[t] = mac16(ldkcol(Qs + (16 * tb + 4 * lq) * KS + 16 * kt + l16, KS), b2, Sacc[t]);
                    Sacc[t] = mac16(ldkcol(Ks + (16 * tb + 4 * lq) * KS + 16 * kt + l16, KS), b3, Sacc[t]);
                }
            }
        }
        // the state for the next chunk's first phase (nothing reads it in between)
#pragma unroll
        for (int t = 0; t < KT; ++t)
            *reinterpret_cast<float4*>(St + l16 * SS + 16 * (KT * w + t) + 4 * lq) = make_float4(Sacc[t][0], Sacc[t][1], Sacc[t][2], Sacc[t][3]);
        __syncthreads();   // every read of the chunk's operands is done, the new state is in place
        if (!LY::two) __syncthreads();   // one place for the staged operands: they are replaced in between
    }
    if (DIR == 1 && a.dS0 != nullptr) {
#pragma unroll
        for (int t = 0; t < KT; ++t)
            *reinterpret_cast<float4*>(a.dS0 + ((size_t)bh * D + v0 + l16) * D + 16 * (KT * w + t) + 4 * lq) =
                make_float4(Sacc[t][0], Sacc[t][1], Sacc[t][2], Sacc[t][3]);
    }
}

template <typename T, int D, int DIR>
constexpr size_t seq_lds_bytes() { return SeqLds<T, D, DIR>::bytes; }
template <int D>
constexpr size_t prep_lds_bytes() { return sizeof(float) * (2 * (size_t)CB_C * (D + 4) + 2 * CB_C); }

// ---- the gradients of a chunk -------------------------------------------------------------------------------------------
// One block per (chunk, batch*head), d / 16 wavefronts; wavefront w owns the columns 16 w .. 16 w + 15 of dQ and dK
// (all 64 rows: four accumulator tiles each) and of the three products with the states that feed them.  Three LDS
// regions are filled in turn:   A: S0, then U with dS1 (64 rows at a time), then K with Q;   B: dO', then dP . Gamma;
// C: dR, then the symmetric (dAt . Gamma) + (dAt . Gamma)^T.  Sums over rows, columns or wavefronts go through small
// per-tile or per-wavefront arrays that one wavefront adds up in a fixed order (no atomics).
template <typename T>
struct GradArgs {
    const T *Q, *K, *dO;
    ChunkOps o;
    const float *alpha;
    const uint8_t* mask;
    const float *ck, *dck, *Ug, *dR, *dbeta_part;
    float *dQ, *dK, *dalpha, *dbeta, *g_nla;
    float* dscore_la;   // optional, routing per chunk: Eq. 17 per chunk
    int L, BH;
    float la_scale;
    int delta, freeze_on_softmax, chunk_mask;
};

template <typename T, int D>
__global__ __launch_bounds__(D * 4) void gdn_chunk_grads_kernel(const GradArgs<T> a) {
    constexpr int NW = D / 16, NT = 64 * NW, KS = D + 4, MS = CB_MS, E = Vec16<T>::N;
    constexpr int HALF = CB_C * KS;            // floats of a [64][KS] tile
    constexpr int NS0 = D * D / 4 / NT;        // 16-byte pieces of a state per thread
    constexpr int NSH = 64 * D / 4 / NT;       // ... of 64 rows of it (or of a [64][D] fp32 tile)
    extern __shared__ __align__(16) float cb_smem[];
    float* RA = cb_smem;
    float* RAhi = RA + HALF;
    float* RB = RA + 2 * HALF;
    float* RC = RB + HALF;
    float* s_g2 = RC + HALF;
    float* s_gam = s_g2 + CB_C;
    float* s_kd = s_gam + CB_C;
    float* rs = s_kd + CB_C;                   // [4 column tiles][64 rows]: row sums of dAt . At + dP . P per tile
    float* cs = rs + 4 * CB_C;                 // [4 row tiles][64 columns]: column sums
    float* gk = cs + 4 * CB_C;                 // [NW][64]: the state terms of d ln gamma, per wavefront's columns
    float* ge = gk + NW * CB_C;                // [NW]: the sum of E_r over the chunk, likewise
    float* s_dot = ge + NW * CB_C;             // [NW]: <dS1, S0>
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const int n_chunks = a.L / CB_C;
    const int bh = blockIdx.x % a.BH, chunk = blockIdx.x / a.BH;
    const size_t gc = (size_t)bh * n_chunks + chunk, tok0 = (size_t)bh * a.L + (size_t)chunk * CB_C;
    const float delta = a.delta ? 1.f : 0.f;

    // The block's global loads: what stage 1 needs goes out first; the later stages' operands are asked for from
    // inside stage 1's product loop, a few loads per step (the issue of a load costs a wavefront 100 cycles and more
    // while the CU's miss queue is full; between matrix instructions the SIMD's other wavefront fills that time),
    // and wait in registers (one block per CU: nothing else would hide their latency).
    constexpr int NPT = 64 * D / E / NT;       // 16-byte words of a [64][D] tile of T per thread
    auto put_rows_f32 = [&](float* dst, const float4 (&r)[NSH]) {   // [64][D] fp32 -> LDS rows of KS
#pragma unroll
        for (int i = 0; i < NSH; ++i) {
            const int e = tid + NT * i, row = e / (D / 4), c4 = (e % (D / 4)) * 4;
            *reinterpret_cast<float4*>(dst + row * KS + c4) = r[i];
        }
    };
    auto put_rows_T = [&](float* dst, const u32x4 (&r)[NPT], float scale) {
#pragma unroll
        for (int i = 0; i < NPT; ++i) {
            const int e = tid + NT * i, row = e / (D / E), c = (e % (D / E)) * E;
            float tmp[E];
            unpack16(r[i], tmp, T{});
#pragma unroll
            for (int j = 0; j < E; j += 4)
                *reinterpret_cast<float4*>(dst + row * KS + c + j) = make_float4(scale * tmp[j], scale * tmp[j + 1], scale * tmp[j + 2], scale * tmp[j + 3]);
        }
    };
    float4 s0reg[NS0], dRreg[NSH], Ureg[NSH], dS1a[NSH], dS1b[NSH];
    u32x4 dOreg[NPT], Kreg[NPT], Qreg[NPT];
    const float* dS1g = a.dck + gc * ((size_t)D * D);
    constexpr int NTL = (10 + NW - 1) / NW;   // lower 16 x 16 tiles of a 64 x 64 operand per wavefront
    float atv[NTL][4], pmv[NTL][4];           // At and P where this lane will hold dAt and dP
    float gate_in = 0.f;   // threads 0..191: one of g2, gam, kd of the chunk's tokens
    if (tid < 3 * CB_C) gate_in = (tid < CB_C ? a.o.g2 : tid < 2 * CB_C ? a.o.gam : a.o.kd)[tok0 + (tid & 63)];
    {
        const float* S0g = a.ck + gc * ((size_t)D * D);
#pragma unroll
        for (int i = 0; i < NS0; ++i) s0reg[i] = ld4(S0g + 4 * (size_t)(tid + NT * i));   // rows of D floats: contiguous
#pragma unroll
        for (int i = 0; i < NPT; ++i) dOreg[i] = reinterpret_cast<const u32x4*>(a.dO + tok0 * D)[tid + NT * i];
#pragma unroll
        for (int i = 0; i < NSH; ++i) dRreg[i] = ld4(a.dR + tok0 * D + 4 * (size_t)(tid + NT * i));
    }
    auto issue_later = [&](int step) {   // step: a compile-time constant where it is called
        if (step == 0) {
#pragma unroll
            for (int i = 0; i < NSH; ++i) Ureg[i] = ld4(a.Ug + tok0 * D + 4 * (size_t)(tid + NT * i));
        } else if (step == 1) {
#pragma unroll
            for (int i = 0; i < NSH; ++i) dS1a[i] = ld4(dS1g + 4 * (size_t)(tid + NT * i));
        } else if (step == 2) {
#pragma unroll
            for (int i = 0; i < NSH; ++i) dS1b[i] = (D > 64) ? ld4(dS1g + (size_t)64 * D + 4 * (size_t)(tid + NT * i)) : make_float4(0.f, 0.f, 0.f, 0.f);
        } else if (step == 3) {
#pragma unroll
            for (int i = 0; i < NPT; ++i) {
                Kreg[i] = reinterpret_cast<const u32x4*>(a.K + tok0 * D)[tid + NT * i];
                Qreg[i] = reinterpret_cast<const u32x4*>(a.Q + tok0 * D)[tid + NT * i];
            }
        } else if (step == 4) {
#pragma unroll
            for (int s = 0; s < NTL; ++s) {
                const int t = w + NW * s < 10 ? w + NW * s : 0;
                const int ta = (0x3333222110 >> (4 * t)) & 15, tb = (0x3210210100 >> (4 * t)) & 15;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const size_t off = gc * (CB_C * CB_C) + (16 * ta + 4 * lq + j) * CB_C + 16 * tb + l16;
                    atv[s][j] = a.o.At[off];
                    pmv[s][j] = a.o.Pm[off];
                }
            }
        }
    };
    // ---- stage 1: S0, dO', dR ------------------------------------------------------------------------------
#pragma unroll
    for (int i = 0; i < NS0; ++i) {
        const int e = tid + NT * i, row = e / (D / 4), c4 = (e % (D / 4)) * 4;
        *reinterpret_cast<float4*>(RA + row * KS + c4) = s0reg[i];
    }
    put_rows_T(RB, dOreg, a.la_scale);
    put_rows_f32(RC, dRreg);
    if (tid < 3 * CB_C) s_g2[tid] = gate_in;   // s_g2, s_gam, s_kd lie one behind the other
    for (int e = tid; e < 8 * CB_C; e += NT) rs[e] = 0.f;   // rs and cs
    __syncthreads();
    f32x4 Gdq[4], Gdk[4], Gu[4];
#pragma unroll
    for (int ta = 0; ta < 4; ++ta) {
        Gdq[ta] = f32x4{0.f, 0.f, 0.f, 0.f};
        Gdk[ta] = f32x4{0.f, 0.f, 0.f, 0.f};
        Gu[ta] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
#pragma unroll
    for (int kv = 0; kv < D / 16; ++kv) {
        issue_later(kv);
        const float4 bs = ld4col(RA + (16 * kv + 4 * lq) * KS + 16 * w + l16, KS);
#pragma unroll
        for (int ta = 0; ta < 4; ++ta) {
            Gdq[ta] = mac16(ld4(RB + (16 * ta + l16) * KS + 16 * kv + 4 * lq), bs, Gdq[ta]);
            Gdk[ta] = mac16(ld4(RC + (16 * ta + l16) * KS + 16 * kv + 4 * lq), bs, Gdk[ta]);
        }
    }
#pragma unroll
    for (int step = D / 16; step < 5; ++step) issue_later(step);
    __syncthreads();
    // ---- stage 2: U and the first 64 rows of dS1; dP and dAt ---------------------------------------------------
    float dot = 0.f;
    put_rows_f32(RA, Ureg);
    put_rows_f32(RAhi, dS1a);
#pragma unroll
    for (int i = 0; i < NSH; ++i)
        dot += dS1a[i].x * s0reg[i].x + dS1a[i].y * s0reg[i].y + dS1a[i].z * s0reg[i].z + dS1a[i].w * s0reg[i].w;
    __syncthreads();
#pragma unroll 2
    for (int kv = 0; kv < 4; ++kv) {
        const float4 bs = ld4col(RAhi + (16 * kv + 4 * lq) * KS + 16 * w + l16, KS);
#pragma unroll
        for (int ta = 0; ta < 4; ++ta) Gu[ta] = mac16(ld4(RA + (16 * ta + l16) * KS + 16 * kv + 4 * lq), bs, Gu[ta]);
    }
    f32x4 DPv[NTL], DAv[NTL];
#pragma unroll
    for (int s = 0; s < NTL; ++s) {
        const int t = w + NW * s;   // uniform
        if (t < 10) {
            const int ta = (0x3333222110 >> (4 * t)) & 15, tb = (0x3210210100 >> (4 * t)) & 15;
            f32x4 accP = {0.f, 0.f, 0.f, 0.f}, accA = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
            for (int kv = 0; kv < D / 16; ++kv) {
                const float4 bu = ld4(RA + (16 * tb + l16) * KS + 16 * kv + 4 * lq);
                accP = mac16(ld4(RB + (16 * ta + l16) * KS + 16 * kv + 4 * lq), bu, accP);
                accA = mac16(ld4(RC + (16 * ta + l16) * KS + 16 * kv + 4 * lq), bu, accA);
            }
            const int i = 16 * tb + l16;
            const float gi = s_g2[i];
            float csum = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = 16 * ta + 4 * lq + j;
                const float G = __builtin_amdgcn_exp2f(s_g2[r] - gi);
                const float dp = (i <= r) ? accP[j] : 0.f, da = (i < r) ? -delta * accA[j] : 0.f;   // no At without the delta rule
                const float e = da * atv[s][j] + dp * pmv[s][j];
                const float rsum = lane_group_sum<16>(e);
                if (l16 == 0) rs[tb * CB_C + r] = rsum;
                csum += e;
                DPv[s][j] = dp * G;
                DAv[s][j] = da * G;
            }
            csum += lane_xor16(csum, lane);
            csum += lane_xor32(csum, lane);
            if (lq == 0) cs[ta * CB_C + i] = csum;
        }
    }
    __syncthreads();
    // ---- stage 3: the two 64 x 64 operands take the places of dO' and dR; the rest of dS1 ------------------------
#pragma unroll
    for (int s = 0; s < NTL; ++s) {
        const int t = w + NW * s;
        if (t < 10) {
            const int ta = (0x3333222110 >> (4 * t)) & 15, tb = (0x3210210100 >> (4 * t)) & 15;
            const int i = 16 * tb + l16;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int r = 16 * ta + 4 * lq + j;
                RB[r * MS + i] = DPv[s][j];
                if (i < r) {
                    RC[r * MS + i] = DAv[s][j];
                    RC[i * MS + r] = DAv[s][j];
                } else if (i == r) {
                    RC[r * MS + i] = 0.f;
                }
            }
        }
    }
    if (D > 64) {
        put_rows_f32(RAhi, dS1b);
#pragma unroll
        for (int i = 0; i < NSH; ++i) {
            const float4 x = dS1b[i], y = s0reg[(NS0 > NSH ? NSH : 0) + i];
            dot += x.x * y.x + x.y * y.y + x.z * y.z + x.w * y.w;
        }
        __syncthreads();
#pragma unroll 2
        for (int kv = 4; kv < D / 16; ++kv) {
            const float4 bs = ld4col(RAhi + (16 * (kv - 4) + 4 * lq) * KS + 16 * w + l16, KS);
#pragma unroll
            for (int ta = 0; ta < 4; ++ta) Gu[ta] = mac16(ld4(RA + (16 * ta + l16) * KS + 16 * kv + 4 * lq), bs, Gu[ta]);
        }
    }
    __syncthreads();
    // ---- stage 4: K and Q ----------------------------------------------------------------------------------------
    put_rows_T(RA, Kreg, 1.f);
    put_rows_T(RAhi, Qreg, 1.f);
    {   // <dS1, S0>: the wavefront's sum
        float x = lane_group_sum<64>(dot);
        if (lane == 0) s_dot[w] = x;
    }
    __syncthreads();
    f32x4 dQa[4], dKa[4];
    float4 kcs[4], qcs[4];   // K and Q: rows 4 lq + j of every token tile, the wavefront's own columns
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
        kcs[tb] = ld4col(RA + (16 * tb + 4 * lq) * KS + 16 * w + l16, KS);
        qcs[tb] = ld4col(RAhi + (16 * tb + 4 * lq) * KS + 16 * w + l16, KS);
    }
    float esum = 0.f;   // E_r is needed only as its sum over the chunk
#pragma unroll
    for (int ta = 0; ta < 4; ++ta) {
        const float kq[4] = {kcs[ta].x, kcs[ta].y, kcs[ta].z, kcs[ta].w}, qq[4] = {qcs[ta].x, qcs[ta].y, qcs[ta].z, qcs[ta].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = 16 * ta + 4 * lq + j;
            const float gam = s_gam[r], kd = s_kd[r];
            const float eu = kd * kq[j] * Gu[ta][j];
            const float x = gam * (qq[j] * Gdq[ta][j] - delta * kq[j] * Gdk[ta][j]) - eu;
            const float xs = lane_group_sum<16>(x);
            esum += eu;
            if (l16 == 0) gk[w * CB_C + r] = xs;
            dQa[ta][j] = gam * Gdq[ta][j];
            dKa[ta][j] = kd * Gu[ta][j] - delta * gam * Gdk[ta][j];
        }
    }
    esum = lane_group_sum<64>(esum);
    if (lane == 0) ge[w] = esum;
    // the softmax branch's share of dQ, which the result is added to: asked for before the products below
    float oldq[4][4];
#pragma unroll
    for (int ta = 0; ta < 4; ++ta)
#pragma unroll
        for (int j = 0; j < 4; ++j) oldq[ta][j] = a.dQ[(tok0 + 16 * ta + 4 * lq + j) * D + 16 * w + l16];
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
        const float4 kc = kcs[tb], qc = qcs[tb];
#pragma unroll
        for (int ta = 0; ta < 4; ++ta) {
            if (tb <= ta) dQa[ta] = mac16(ld4(RB + (16 * ta + l16) * MS + 16 * tb + 4 * lq), kc, dQa[ta]);
            dKa[ta] = mac16(ld4(RC + (16 * ta + l16) * MS + 16 * tb + 4 * lq), kc, dKa[ta]);
            // (dP . Gamma)^T Q: rows tb of dP (as contraction index) against the columns of tile ta
            if (tb >= ta) dKa[ta] = mac16(ld4col(RB + (16 * tb + 4 * lq) * MS + 16 * ta + l16, MS), qc, dKa[ta]);
        }
    }
#pragma unroll
    for (int ta = 0; ta < 4; ++ta) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const size_t off = (tok0 + 16 * ta + 4 * lq + j) * D + 16 * w + l16;
            a.dQ[off] = oldq[ta][j] + dQa[ta][j];
            a.dK[off] = dKa[ta][j];
        }
    }
    __syncthreads();
    // ---- the gates: d ln gamma of every token, its sum from the back, dalpha; dbeta ----------------------------
    if (w == 0) {
        const int r = 63 - lane;   // reversed, so that the inclusive scan below sums from the chunk's end
        float dl = 0.f, et = 0.f;
#pragma unroll
        for (int q = 0; q < 4; ++q) dl += rs[q * CB_C + r];
#pragma unroll
        for (int q = 0; q < 4; ++q) dl -= cs[q * CB_C + r];
#pragma unroll
        for (int q = 0; q < NW; ++q) { dl += gk[q * CB_C + r]; et += ge[q]; }
        float dt = 0.f;
#pragma unroll
        for (int q = 0; q < NW; ++q) dt += s_dot[q];
        // the decay carried over the chunk: not a function of the alphas for a softmax chunk in the variant without decay
        const bool carry_fixed = a.chunk_mask && a.freeze_on_softmax && a.mask[gc] != 0;
        if (r == 63) dl += et + (carry_fixed ? 0.f : a.o.gamC[gc] * dt);
        // Eq. 17 for a chunk: <dS1, what the chunk added to the carried state> = sum_i kd_i K_i . (U dS1)_i (kd = 0 for
        // a softmax chunk)
        if (lane == 0 && a.dscore_la != nullptr) a.dscore_la[gc] = et;
        dl += dpp_move<0x111>(dl);
        dl += dpp_move<0x112>(dl);
        dl += dpp_move<0x114>(dl);
        dl += dpp_move<0x118>(dl);
        dl += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(dl), 0x142, 0xA, 0xF, false));
        dl += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(dl), 0x143, 0xC, 0xF, false));
        const size_t t = tok0 + r;
        const bool frozen = a.freeze_on_softmax && !a.chunk_mask && a.mask[t] != 0;   // its alpha counted as 1
        a.dalpha[t] = frozen ? 0.f : dl / fmaxf(a.alpha[t], 1e-30f);
        float db = 0.f;
        const size_t n_tok = (size_t)a.BH * a.L;
#pragma unroll
        for (int q = 0; q < NW; ++q) db += a.dbeta_part[(size_t)q * n_tok + t];
        a.dbeta[t] = db;
        if (a.g_nla != nullptr) a.g_nla[t] = 0.f;
    }
}

template <int D>
constexpr size_t grads_lds_bytes() {
    return sizeof(float) * (4 * (size_t)CB_C * (D + 4) + 3 * CB_C + 8 * CB_C + 2 * (D / 16) * CB_C + 64);
}


// ---- the linear branch's output rows from what the forward-by-chunks leaves ---------------------------------------------
// O = la (diag(gamma) Q S0^T + P U) for every chunk at once, fp32: S0 the state at the chunk's start (ck), U the rows
// gdn_chunk_seq_kernel<.., 0> wrote, P and gamma from the chunk's operands.  Needed where the backward pass must know
// the branch's rows (the merges that normalise them, Eq. 21).  One block per (chunk, batch*head); wavefront w owns a
// quarter of the value columns for all 64 tokens, so every element of S0 and U is read once per block, straight
// from memory as the right operand; Q and P, which every wavefront reads whole, go through LDS.
template <int D>
__global__ __launch_bounds__(256) void gdn_chunk_out_kernel(const float* __restrict__ Q, const ChunkOps o,
                                                           const float* __restrict__ ck, const float* __restrict__ Ug,
                                                           float* __restrict__ O_la, const int L, const int BH,
                                                           const float la_scale) {
    constexpr int KS = D + 4, MS = CB_MS, VW = D / 4, VT = VW / 16;   // value columns per wavefront, in tiles of 16
    __shared__ __align__(16) float Qs[CB_C * KS];
    __shared__ __align__(16) float Ps[CB_C * MS];
    __shared__ float s_gam[CB_C];
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
    const int n_chunks = L / CB_C;
    const int bh = blockIdx.x % BH, chunk = blockIdx.x / BH;
    const size_t gc = (size_t)bh * n_chunks + chunk, tok0 = (size_t)bh * L + (size_t)chunk * CB_C;
    for (int e = tid; e < CB_C * D / 4; e += 256) {
        const int row = e / (D / 4), c4 = (e % (D / 4)) * 4;
        *reinterpret_cast<float4*>(Qs + row * KS + c4) = ld4(Q + (tok0 + row) * D + c4);
    }
    for (int e = tid; e < CB_C * CB_C / 4; e += 256) {
        const int row = e / 16, c4 = (e % 16) * 4;
        *reinterpret_cast<float4*>(Ps + row * MS + c4) = ld4(o.Pm + gc * (CB_C * CB_C) + row * CB_C + c4);
    }
    if (tid < CB_C) s_gam[tid] = o.gam[tok0 + tid];
    __syncthreads();
    const float* S0 = ck + gc * (size_t)D * D;
    f32x4 acc[4][VT];
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int vt = 0; vt < VT; ++vt) acc[tt][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
    // Q S0^T: A = Q[token l16 of tile tt][k], B = S0[v = l16 of tile vt][k]
#pragma unroll 2
    for (int kt = 0; kt < D / 16; ++kt) {
        float4 b[VT];
#pragma unroll
        for (int vt = 0; vt < VT; ++vt) b[vt] = ld4(S0 + (size_t)(VW * w + 16 * vt + l16) * D + 16 * kt + 4 * lq);
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) {
            const float4 a = ld4(Qs + (16 * tt + l16) * KS + 16 * kt + 4 * lq);
#pragma unroll
            for (int vt = 0; vt < VT; ++vt) acc[tt][vt] = mac16(a, b[vt], acc[tt][vt]);
        }
    }
    // rows scaled by gamma (a lane holds tokens 16 tt + 4 lq + j of value column l16)
#pragma unroll
    for (int tt = 0; tt < 4; ++tt) {
        const float4 g4 = ld4(s_gam + 16 * tt + 4 * lq);
        const float g[4] = {g4.x, g4.y, g4.z, g4.w};
#pragma unroll
        for (int vt = 0; vt < VT; ++vt)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc[tt][vt][j] *= g[j];
    }
    // + P U: A = P[token][i], B = U[i = 16 tb + 4 lq + j][v]; P is lower triangular: tiles tb <= tt
#pragma unroll
    for (int tb = 0; tb < 4; ++tb) {
        float4 b[VT];
#pragma unroll
        for (int vt = 0; vt < VT; ++vt)
            b[vt] = ld4col(Ug + (tok0 + 16 * tb + 4 * lq) * D + VW * w + 16 * vt + l16, D);
#pragma unroll
        for (int tt = tb; tt < 4; ++tt) {
            const float4 a = ld4(Ps + (16 * tt + l16) * MS + 16 * tb + 4 * lq);
#pragma unroll
            for (int vt = 0; vt < VT; ++vt) acc[tt][vt] = mac16(a, b[vt], acc[tt][vt]);
        }
    }
#pragma unroll
    for (int tt = 0; tt < 4; ++tt)
#pragma unroll
        for (int vt = 0; vt < VT; ++vt)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                O_la[(tok0 + 16 * tt + 4 * lq + j) * D + VW * w + 16 * vt + l16] = la_scale * acc[tt][vt][j];
}

static ChunkOps chunk_ops(const FwdPlan& pl, float* base) {
    const size_t n_tok = (size_t)pl.BH * pl.L, n_ch = n_tok / CB_C;
    ChunkOps o;
    o.Tm = base;
    o.At = o.Tm + n_ch * CB_C * CB_C;
    o.Pm = o.At + n_ch * CB_C * CB_C;
    o.g2 = o.Pm + n_ch * CB_C * CB_C;
    o.gam = o.g2 + n_tok;
    o.kd = o.gam + n_tok;
    o.bp = o.kd + n_tok;
    o.gamC = o.bp + n_tok;
    return o;
}
size_t chunk_ops_floats(const FwdPlan& pl) {
    const size_t n_tok = (size_t)pl.BH * pl.L, n_ch = n_tok / CB_C;
    return 3 * n_ch * CB_C * CB_C + 4 * n_tok + align_up(n_ch, 64);
}

template <typename T, int D>
static bool launch_prep_t(const FwdPlan& pl, const void* Q, const void* K, const float* alpha, const float* beta,
                          const uint8_t* mask, const ChunkOps& o, hipStream_t st) {
    auto kern = gdn_bwd_prep_kernel<T, D>;
    constexpr size_t lds = prep_lds_bytes<D>();
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
        hipSuccess) return false;
    hipLaunchKernelGGL(kern, dim3((unsigned)(pl.BH * (pl.L / CB_C))), dim3(256), lds, st, (const T*)Q,
                       (const T*)K, alpha, beta, mask, o, pl.L, pl.BH, pl.freeze_on_softmax, pl.linear_op,
                       pl.routing == NATS_ROUTE_CHUNK);
    return true;
}

// ops: chunk_ops_floats(pl) floats.  Either routing.
nats_status launch_gdn_bwd_prep(const FwdPlan& pl, const void* Q, const void* K, const float* alpha, const float* beta,
                                const uint8_t* mask, float* ops, hipStream_t st) {
    const ChunkOps o = chunk_ops(pl, ops);
    bool ok;
    if (pl.dtype == NATS_BF16) ok = pl.d == 64 ? launch_prep_t<bf16_t, 64>(pl, Q, K, alpha, beta, mask, o, st)
                                               : launch_prep_t<bf16_t, 128>(pl, Q, K, alpha, beta, mask, o, st);
    else ok = pl.d == 64 ? launch_prep_t<float, 64>(pl, Q, K, alpha, beta, mask, o, st)
                         : launch_prep_t<float, 128>(pl, Q, K, alpha, beta, mask, o, st);
    if (!ok) { set_error("gdn_bwd_prep: the kernel's LDS size was refused"); return NATS_ERR_HIP; }
    return check_launch("gdn_bwd_prep");
}

template <typename T, int D, int DIR>
static bool launch_seq_t(const FwdPlan& pl, const SeqArgs<T>& a, hipStream_t st) {
    auto kern = gdn_chunk_seq_kernel<T, D, DIR>;
    constexpr size_t lds = seq_lds_bytes<T, D, DIR>();
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
        hipSuccess) return false;
    hipLaunchKernelGGL(kern, dim3((unsigned)(pl.BH * (D / CB_NV))), dim3(512), lds, st, a);
    return true;
}
template <typename T, int DIR>
static bool launch_seq_d(const FwdPlan& pl, const SeqArgs<T>& a, hipStream_t st) {
    return pl.d == 64 ? launch_seq_t<T, 64, DIR>(pl, a, st) : launch_seq_t<T, 128, DIR>(pl, a, st);
}

// The states at the chunk starts, ck [BH][L/64][d][d], with U and Uh [BH][L][d] of every chunk.
nats_status launch_gdn_chunk_states(const FwdPlan& pl, const void* K, const void* V, float* ops, const float* S_init,
                                    float* ck, float* Ug, float* Uh, hipStream_t st) {
    bool ok;
    if (pl.dtype == NATS_BF16) {
        const SeqArgs<bf16_t> a{(const bf16_t*)K, nullptr, (const bf16_t*)V, chunk_ops(pl, ops), nullptr, S_init, ck, Ug, Uh,
                                nullptr, nullptr, nullptr, pl.L, pl.BH, pl.la_scale, pl.linear_op == 0};
        ok = launch_seq_d<bf16_t, 0>(pl, a, st);
    } else {
        const SeqArgs<float> a{(const float*)K, nullptr, (const float*)V, chunk_ops(pl, ops), nullptr, S_init, ck, Ug, Uh,
                               nullptr, nullptr, nullptr, pl.L, pl.BH, pl.la_scale, pl.linear_op == 0};
        ok = launch_seq_d<float, 0>(pl, a, st);
    }
    if (!ok) { set_error("gdn_chunk_states: the kernel's LDS size was refused"); return NATS_ERR_HIP; }
    return check_launch("gdn_chunk_states");
}

// O_la [BH][L][d] f32 from ops (after launch_gdn_bwd_prep), ck and Ug (after launch_gdn_chunk_states).  fp32 tensors.
nats_status launch_gdn_chunk_out(const FwdPlan& pl, const void* Q, float* ops, const float* ck, const float* Ug,
                                 float* O_la, hipStream_t st) {
    if (pl.dtype != NATS_F32) { set_error("gdn_chunk_out: fp32 tensors only"); return NATS_ERR_UNSUPPORTED; }
    const ChunkOps o = chunk_ops(pl, ops);
    const dim3 grid((unsigned)(pl.BH * (pl.L / CB_C)));
    if (pl.d == 64)
        hipLaunchKernelGGL(gdn_chunk_out_kernel<64>, grid, dim3(256), 0, st, (const float*)Q, o, ck, Ug, O_la, pl.L, pl.BH,
                           pl.la_scale);
    else
        hipLaunchKernelGGL(gdn_chunk_out_kernel<128>, grid, dim3(256), 0, st, (const float*)Q, o, ck, Ug, O_la, pl.L, pl.BH,
                           pl.la_scale);
    return check_launch("gdn_chunk_out");
}

// The state gradients behind every chunk, dck [BH][L/64][d][d]; dV (every row), dbeta_part [d/16][BH][L], dS0 (or NULL).
nats_status launch_gdn_chunk_state_grads(const FwdPlan& pl, const void* Q, const void* K, const void* dO,
                                         const uint8_t* mask, float* ops, float* dck, float* Uh, float* dV,
                                         float* dbeta_part, float* dS0, hipStream_t st) {
    const uint8_t* tok_mask = pl.routing == NATS_ROUTE_CHUNK ? nullptr : mask;
    bool ok;
    if (pl.dtype == NATS_BF16) {
        const SeqArgs<bf16_t> a{(const bf16_t*)K, (const bf16_t*)Q, (const bf16_t*)dO, chunk_ops(pl, ops), tok_mask, nullptr, dck,
                                nullptr, Uh, dV, dbeta_part, dS0, pl.L, pl.BH, pl.la_scale, pl.linear_op == 0};
        ok = launch_seq_d<bf16_t, 1>(pl, a, st);
    } else {
        const SeqArgs<float> a{(const float*)K, (const float*)Q, (const float*)dO, chunk_ops(pl, ops), tok_mask, nullptr, dck,
                               nullptr, Uh, dV, dbeta_part, dS0, pl.L, pl.BH, pl.la_scale, pl.linear_op == 0};
        ok = launch_seq_d<float, 1>(pl, a, st);
    }
    if (!ok) { set_error("gdn_chunk_state_grads: the kernel's LDS size was refused"); return NATS_ERR_HIP; }
    return check_launch("gdn_chunk_state_grads");
}

template <typename T, int D>
static bool launch_grads_t(const FwdPlan& pl, const GradArgs<T>& a, hipStream_t st) {
    auto kern = gdn_chunk_grads_kernel<T, D>;
    constexpr size_t lds = grads_lds_bytes<D>();
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) !=
        hipSuccess) return false;
    hipLaunchKernelGGL(kern, dim3((unsigned)(pl.BH * (pl.L / CB_C))), dim3(D * 4), lds, st, a);
    return true;
}

// dQ += the linear branch's share; dK, dalpha, dbeta = it; g_nla (optional) cleared.  ck, dck: the states and state
// gradients per chunk; Ug, dR (= the linear branch's dV) [BH][L][d]; dbeta_part [d/16][BH][L].
nats_status launch_gdn_chunk_grads(const FwdPlan& pl, const void* Q, const void* K, const void* dO, const float* alpha,
                                   const uint8_t* mask, float* ops, const float* ck, const float* dck, const float* Ug,
                                   const float* dR, const float* dbeta_part, float* dQ, float* dK, float* dalpha,
                                   float* dbeta, float* g_nla, float* dscore_la, hipStream_t st) {
    bool ok;
    if (pl.dtype == NATS_BF16) {
        const GradArgs<bf16_t> a{(const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)dO, chunk_ops(pl, ops), alpha, mask, ck, dck,
                                 Ug, dR, dbeta_part, dQ, dK, dalpha, dbeta, g_nla, dscore_la, pl.L, pl.BH, pl.la_scale,
                                 pl.linear_op == 0, pl.freeze_on_softmax, pl.routing == NATS_ROUTE_CHUNK};
        ok = pl.d == 64 ? launch_grads_t<bf16_t, 64>(pl, a, st) : launch_grads_t<bf16_t, 128>(pl, a, st);
    } else {
        const GradArgs<float> a{(const float*)Q, (const float*)K, (const float*)dO, chunk_ops(pl, ops), alpha, mask, ck, dck,
                                Ug, dR, dbeta_part, dQ, dK, dalpha, dbeta, g_nla, dscore_la, pl.L, pl.BH, pl.la_scale,
                                pl.linear_op == 0, pl.freeze_on_softmax, pl.routing == NATS_ROUTE_CHUNK};
        ok = pl.d == 64 ? launch_grads_t<float, 64>(pl, a, st) : launch_grads_t<float, 128>(pl, a, st);
    }
    if (!ok) { set_error("gdn_chunk_grads: the kernel's LDS size was refused"); return NATS_ERR_HIP; }
    return check_launch("gdn_chunk_grads");
}

}  // namespace nats
