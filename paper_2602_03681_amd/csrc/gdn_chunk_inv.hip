// Chunkwise Gated DeltaNet, step 1 of 2: the part of a chunk that depends neither on the running
// state nor on the values (Section 3, Eq. 6-7 applied to the update rule of Eq. 19, with Eq. 14 /
// Eq. 20 folded in as  b'_t = beta_t (1 - m_t)  and decay at every token).
//
// For one chunk of C = 64 tokens, with g_r = sum_{i<=r} log alpha_i (inside the chunk), gam_r = exp(g_r):
//   D[r,i]  = exp(g_r - g_i)                       (i <= r)
//   A       = strict_lower( diag(b') (K K^T . D) )
//   T       = (I + A)^{-1}                         (unit lower triangular; fp32, blocks of 16)
//   T''     = T diag(b')                           (stored, fp16)
//   P       = (Q K^T) . D  (i <= r, zero above the diagonal)   (stored, fp16)
//   gam_r,  kd_r = gam_C / gam_r,  gam_C           (stored, fp32)
// The state-carrying kernel then needs only the raw K, Q, V beside these:
//   U  = T'' (V - diag(gam) K S0^T)
//   O  = diag(gam) Q S0^T + P U
//   S1 = gam_C S0 + U^T diag(kd) K.
// (The products T diag(b' gam) K and T diag(b') V of the usual chunkwise form are never stored: they are
// as large as K and V themselves, and writing and re-reading them cost more than the whole recurrence.)
//
// Output format, fp16, "fragment-major": both matrices are written in the order in which a wavefront of
// the state-carrying kernel reads them as MFMA operands (row of the lane, 8 contraction slots), so that
// a fragment is one contiguous 1 KiB.  With lane = 16 lq + l16, token tile tw = 0..3 and fragment number
// f = tri_frag(tw, ks) (the two fragments above the diagonal, tw < 2 with ks = 1, are left out: 6 per matrix):
//   TF [chunk][f][lane][s < 8] = T''[r = 16 tw + l16][i = 32 ks + 16 (s / 4) + 4 lq + s % 4]
//   PF [chunk][f][lane][s < 8] = P  [r = 16 tw + l16][i = 32 ks + 16 (s / 4) + 4 lq + s % 4]
//   gamv[chunk][64], kdv[chunk][64], gamC[chunk]   (fp32)
// The contraction slots of a lane stand for tokens 4 lq .. 4 lq + 3 of two neighbouring 16-token tiles:
// that is how a lane holds two accumulator tiles of a product over tokens, so the other operand of such a
// product (R, U of the state-carrying kernel) goes from the accumulators into the next matrix instruction
// without leaving the registers.
//
// One block per chunk and (batch, head) (a one-dimensional grid, chunk-major), 4 wavefronts.  K K^T and
// Q K^T run on MFMA with fp16 operands (bf16 inputs convert exactly) and fp32 accumulation.  The
// triangular inverse is blocked 16x16: substitution inside the four diagonal blocks (one per wavefront),
// fp32 MFMA for the blocks below them.
#include <math.h>

#include "mfma_util.h"
#include "nats_common.h"
#include "scan_compact_block.h"

namespace nats {

constexpr int INV_THREADS = 256;
constexpr int INV_OCC = 5;             // blocks per CU (96 registers, 32 KB of LDS each)
constexpr int CH = 64;                 // chunk size
constexpr int AT = 20;                 // fp32 row stride of a 16x16 tile of A or T in LDS (rows stay 16-byte aligned)
constexpr int AT_TILE = 16 * AT + 16;  // floats per tile; the 16 extra shift the next tile by 16 banks
constexpr int N_TRI = 10;              // 16x16 tiles on and below the diagonal of a 64x64 matrix

// A and T are lower triangular: only the tiles (a, b), b <= a, exist, row by row
__device__ __forceinline__ int tri_tile(int a, int b) { return ((a * (a + 1)) / 2 + b) * AT_TILE; }

// LDS plan (bytes): the K tile (fp16 [64][d+8]) is dead once A and P are complete, and T takes its place.
template <int D>
struct InvLds {
    static constexpr int RS = D + LDS_PAD;
    static constexpr int tri_bytes = N_TRI * AT_TILE * 4;
    static constexpr int k_bytes = CH * RS * 2;
    static constexpr int r1_bytes = k_bytes > tri_bytes ? k_bytes : tri_bytes;
    static constexpr int o_as = r1_bytes;
    static constexpr int o_gate = o_as + tri_bytes;
    static constexpr int bytes = o_gate + 4 * CH * 4;
};

// offset (in halves) of element (r, i) of a 64 x 64 operand in the fragment-major layout above; i a multiple of 4,
// (r, i) not in the two fragments that are left out
__device__ __forceinline__ int frag_off(int r, int i) {
    return ((tri_frag(r >> 4, i >> 5) * 64) + 16 * ((i >> 2) & 3) + (r & 15)) * 8 + 4 * ((i >> 4) & 1) + (i & 3);
}

// Block column B of T = (I + A)^-1 below its diagonal block, by one wavefront: T_aB = -T_aa sum_{B <= k < a} A_ak T_kB.
// As, Ts: the lower 16x16 tiles in LDS (the diagonal blocks of T are complete).
template <int B>
__device__ __forceinline__ void inv_block_column(const float* As, float* Ts, const int l16, const int lq) {
    f32x4 X[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) X[a] = f32x4{0.f, 0.f, 0.f, 0.f};
    f32x4 tkb;   // T_kB as the right operand: rows 4 lq + j, column l16
    {
        const float* Tbb = Ts + tri_tile(B, B) + (4 * lq) * AT + l16;
#pragma unroll
        for (int j = 0; j < 4; ++j) tkb[j] = Tbb[j * AT];
    }
#pragma unroll
    for (int k = B; k < 3; ++k) {
#pragma unroll
        for (int a = k + 1; a < 4; ++a) {
            const float4 af = *reinterpret_cast<const float4*>(As + tri_tile(a, k) + l16 * AT + 4 * lq);
            X[a] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.x, tkb[0], X[a], 0, 0, 0);
            X[a] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.y, tkb[1], X[a], 0, 0, 0);
            X[a] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.z, tkb[2], X[a], 0, 0, 0);
            X[a] = __builtin_amdgcn_mfma_f32_16x16x4f32(af.w, tkb[3], X[a], 0, 0, 0);
        }
        const int a = k + 1;   // this block's sum is complete
        const float4 tf = *reinterpret_cast<const float4*>(Ts + tri_tile(a, a) + l16 * AT + 4 * lq);
        f32x4 Y = {0.f, 0.f, 0.f, 0.f};
        Y = __builtin_amdgcn_mfma_f32_16x16x4f32(tf.x, X[a][0], Y, 0, 0, 0);
        Y = __builtin_amdgcn_mfma_f32_16x16x4f32(tf.y, X[a][1], Y, 0, 0, 0);
        Y = __builtin_amdgcn_mfma_f32_16x16x4f32(tf.z, X[a][2], Y, 0, 0, 0);
        Y = __builtin_amdgcn_mfma_f32_16x16x4f32(tf.w, X[a][3], Y, 0, 0, 0);
        float* Tab = Ts + tri_tile(a, B) + (4 * lq) * AT + l16;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            tkb[j] = -Y[j];   // the next step's right operand as it sits in the registers
            Tab[j * AT] = tkb[j];
        }
    }
}

struct InvArgs {
    const bf16_t *Q, *K;
    const float *alpha, *beta;
    const uint8_t* mask;
    int L, chunk_mask;
    half_t *TF, *PF;
    float *gamv, *kdv, *gamC;
    int BH, linear_op, freeze_on_softmax, no_inner_output;
};

// one block of the inversion: block_id counts (chunk, batch*head padded to a multiple of 8)
template <int D>
__device__ __forceinline__ void gdn_chunk_inv_block(const InvArgs& a, const int block_id, unsigned char* smem) {
    const bf16_t* __restrict__ Q = a.Q;
    const bf16_t* __restrict__ K = a.K;
    const float* __restrict__ alpha = a.alpha;
    const float* __restrict__ beta = a.beta;
    const uint8_t* __restrict__ mask = a.mask;
    const int L = a.L, chunk_mask = a.chunk_mask, BH = a.BH, linear_op = a.linear_op;
    const int freeze_on_softmax = a.freeze_on_softmax, no_inner_output = a.no_inner_output;
    half_t* __restrict__ TF = a.TF;
    half_t* __restrict__ PF = a.PF;
    float* __restrict__ gamv = a.gamv;
    float* __restrict__ kdv = a.kdv;
    float* __restrict__ gamC = a.gamC;
    using Lds = InvLds<D>;
    constexpr int RS = Lds::RS;
    constexpr int NPC = CH * D / 8 / INV_THREADS;   // 16-byte pieces of a [64][D] tile per thread
    constexpr int KS_D = D / 32;
    half_t* Ks = reinterpret_cast<half_t*>(smem);              // [64][RS]
    float* Ts = reinterpret_cast<float*>(smem);                // lower tiles   (after Ks)
    float* As = reinterpret_cast<float*>(smem + Lds::o_as);    // lower tiles
    float* s_g2 = reinterpret_cast<float*>(smem + Lds::o_gate);  // cumulative log2-decay
    float* s_gam = s_g2 + CH;
    float* s_bp = s_gam + CH;
    float* s_gdec = s_bp + CH;

    const int tid = threadIdx.x;
    const int n_chunks = L / CH;
    // One-dimensional grid, chunk-major: all (batch, head) pairs of a chunk side by side (padded to a
    // multiple of 8, so that a pair's blocks land on the XCD whose L2 the recurrence blocks of that pair use).
    const int bh8 = (BH + 7) & ~7;
    const int bh = block_id % bh8;
    if (bh >= BH) return;
    const int chunk = block_id / bh8;
    const size_t gc = (size_t)bh * n_chunks + chunk;  // global chunk id
    const size_t tok0 = (size_t)bh * L + (size_t)chunk * CH;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lq = lane >> 4;

    // ---- K tile: coalesced 16-byte loads (a [64][D] tile is contiguous in global memory) ----
    // ---- Q: MFMA fragments straight from global memory.  Wavefront w multiplies query tile a0 = 3 - w
    //      (wavefront 3 also tile 3); lane (l16, lq) holds, per step ks, the 8 elements
    //      d_k = (D/4) lq + 8 ks + j of token 16 a + l16 (any contraction order does, as long as both
    //      operands use it).
    u32x4 rk[NPC], q0[KS_D], q1[KS_D];
    {
        const u32x4* Kg = reinterpret_cast<const u32x4*>(K + tok0 * D);
#pragma unroll
        for (int i = 0; i < NPC; ++i) rk[i] = Kg[tid + INV_THREADS * i];
        const int qa0 = 3 - wave, qa1 = (wave == 3) ? 3 : qa0;
        const bf16_t* Qc = Q + (tok0 + l16) * D + (D / 4) * lq;
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) {
            q0[ks] = *reinterpret_cast<const u32x4*>(Qc + (size_t)(16 * qa0) * D + 8 * ks);
            q1[ks] = *reinterpret_cast<const u32x4*>(Qc + (size_t)(16 * qa1) * D + 8 * ks);
        }
    }
    // ---- gates: cumulative log-decay and write strengths -------------------------------
    if (wave == 0) {
        // variant without decay on softmax tokens (routing per token): their alpha counts as 1
        const float a = (freeze_on_softmax && !chunk_mask && mask[tok0 + lane]) ? 1.f : alpha[tok0 + lane];
        float g = __builtin_amdgcn_logf(fmaxf(a, 1e-30f));   // log2
        // inclusive scan over the 64 lanes on DPP moves (no LDS): inside the 16-lane rows by shifts of 1, 2, 4, 8
        // (a lane without a source adds 0), then lane 15 of rows 0 and 2 into rows 1 and 3, then lane 31 into
        // the upper half
        g += dpp_move<0x111>(g);
        g += dpp_move<0x112>(g);
        g += dpp_move<0x114>(g);
        g += dpp_move<0x118>(g);
        g += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(g), 0x142, 0xA, 0xF, false));   // row_bcast15
        g += __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(g), 0x143, 0xC, 0xF, false));   // row_bcast31
        const float gC = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(g), 63));
        const float gam = __builtin_amdgcn_exp2f(g);
        s_g2[lane] = g;
        s_gam[lane] = gam;
        // Routing per token: a softmax token writes nothing (b' = 0).  Routing per chunk: every token
        // writes inside its chunk (the intra-chunk part is computed for every chunk), and a softmax
        // chunk hands nothing on: its kd is zero, so the state only takes the chunk's decay.
        const bool soft_chunk = chunk_mask && mask[gc] != 0;
        const float kd = soft_chunk ? 0.f : __builtin_amdgcn_exp2f(gC - g);
        s_gdec[lane] = kd;
        s_bp[lane] = (!chunk_mask && mask[tok0 + lane]) ? 0.f : beta[tok0 + lane];
        gamv[gc * CH + lane] = gam;
        kdv[gc * CH + lane] = kd;
        // the decay the recurrence applies to the state it carries over this chunk (1 for a softmax chunk in
        // the variant without decay there: inside the chunk the decays still act on the provisional state)
        if (lane == 63) gamC[gc] = (freeze_on_softmax && soft_chunk) ? 1.f : gam;
    }
#pragma unroll
    for (int i = 0; i < NPC; ++i) {
        const int e = tid + INV_THREADS * i;
        const int row = e / (D / 8), c8 = e % (D / 8);
        *reinterpret_cast<half8*>(Ks + row * RS + c8 * 8) = bf16x8_to_half8(rk[i]);
    }
    // the query fragments in fp16 (wavefronts 0..2 use one tile for all their products)
    half8 hq0[KS_D], hq1[KS_D];
#pragma unroll
    for (int ks = 0; ks < KS_D; ++ks) hq0[ks] = bf16x8_to_half8(q0[ks]);
    if (wave == 3) {
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) hq1[ks] = bf16x8_to_half8(q1[ks]);
    } else {
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) hq1[ks] = hq0[ks];
    }
    __syncthreads();

    // ---- K K^T -> A (LDS, fp32) and (Q K^T . D) -> P (global), lower 16x16 tiles ----------
    const int a0 = 3 - wave, a1 = (wave == 3) ? 3 : a0;
    {
        // 16x16 tile products (a, b), b <= a: wavefront w takes (a0, 0), (a1, 1) [wavefront 3: (3, 3)] and, for
        // w < 2, (a0, 2); the third slot of wavefronts 2 and 3 repeats their first product and is not stored.
        // The three run as one straight-line sequence with separate accumulators, so that the LDS reads and
        // MFMA chains of one fill the latencies of the others.
        constexpr int NJ = 3;
        const int ja[NJ] = {a0, a1, a0};
        const int jb[NJ] = {0, (wave == 3) ? 3 : 1, (wave < 2) ? 2 : 0};
        half_t* Pc = PF + gc * TRI_FRAG_HALFS;
        f32x4 accK[NJ], accP[NJ];
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            accK[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
            accP[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) {
            const int ko = (D / 4) * lq + 8 * ks;
            const half8 fa0 = lds_read8(Ks + (16 * a0 + l16) * RS + ko);
            const half8 fa1 = lds_read8(Ks + (16 * a1 + l16) * RS + ko);
            const half8 fb0 = lds_read8(Ks + (16 * jb[0] + l16) * RS + ko);
            const half8 fb1 = lds_read8(Ks + (16 * jb[1] + l16) * RS + ko);
            const half8 fb2 = lds_read8(Ks + (16 * jb[2] + l16) * RS + ko);
            accK[0] = mfma16(fa0, fb0, accK[0]);   // rows: tokens of block a, cols: tokens of block b
            accP[0] = mfma16(fb0, hq0[ks], accP[0]);   // rows: key tokens i of block b, cols: query tokens r of block a
            accK[1] = mfma16(fa1, fb1, accK[1]);
            accP[1] = mfma16(fb1, hq1[ks], accP[1]);
            accK[2] = mfma16(fa0, fb2, accK[2]);
            accP[2] = mfma16(fb2, hq0[ks], accP[2]);
        }
        // every gate value first, then the stores: LDS reads are not moved across LDS writes
        float gi[NJ], gr[NJ];
        float4 gr4[NJ], bp4[NJ], gi4[NJ];
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            gi[jj] = s_g2[16 * jb[jj] + l16];
            gr[jj] = s_g2[16 * ja[jj] + l16];
            gr4[jj] = *reinterpret_cast<const float4*>(s_g2 + 16 * ja[jj] + 4 * lq);
            bp4[jj] = *reinterpret_cast<const float4*>(s_bp + 16 * ja[jj] + 4 * lq);
            gi4[jj] = *reinterpret_cast<const float4*>(s_g2 + 16 * jb[jj] + 4 * lq);
        }
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            if (jj == 2 && wave >= 2) continue;   // uniform per wavefront
            const int a = ja[jj], b = jb[jj];
            {   // A[r][i], r = 16a + 4 lq + j, i = 16b + l16
                float* At = As + tri_tile(a, b) + (4 * lq) * AT + l16;
                const float g4[4] = {gr4[jj].x, gr4[jj].y, gr4[jj].z, gr4[jj].w};
                const float b4[4] = {bp4[jj].x, bp4[jj].y, bp4[jj].z, bp4[jj].w};
                const int i = 16 * b + l16;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = 16 * a + 4 * lq + j;
                    // gated linear attention (no delta rule): A = 0, so T = (I + A)^-1 = I below
                    At[j * AT] = (i < r && linear_op == 0)
                                     ? b4[j] * accK[jj][j] * __builtin_amdgcn_exp2f(g4[j] - gi[jj]) : 0.f;
                }
            }
            {   // P[r][i], r = 16a + l16, i = 16b + 4 lq + j
                const int r = 16 * a + l16;
                const float g4[4] = {gi4[jj].x, gi4[jj].y, gi4[jj].z, gi4[jj].w};
                f32x4 pv;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = 16 * b + 4 * lq + j;
                    // no_inner_output: the variant in which the linear branch's output reads the carried state only
                    pv[j] = (i <= r && !no_inner_output) ? accP[jj][j] * __builtin_amdgcn_exp2f(gr[jj] - g4[j]) : 0.f;
                }
                *reinterpret_cast<half4*>(Pc + frag_off(r, 16 * b + 4 * lq)) = to_half4(pv);
            }
        }
        // the tiles of P above the diagonal inside the stored fragments are zeros: (0,1) and (2,3)
        if (wave < 2) {
            const int a = 2 * wave, b = a + 1;
            half4 zero = {0, 0, 0, 0};
            *reinterpret_cast<half4*>(Pc + frag_off(16 * a + l16, 16 * b + 4 * lq)) = zero;
        }
    }
    __syncthreads();   // A complete; the K tile is dead from here on: its region becomes T

    // ---- T = (I + A)^{-1}, unit lower triangular, by 16x16 blocks in fp32 ------------------------
    // (a) diagonal blocks: wavefront b inverts I + A_bb by forward substitution; lane j < 16 owns
    //     column j, row r needs rows < r of the same column
    if (lane < 16) {
        const float* At = As + tri_tile(wave, wave);
        float* Tt = Ts + tri_tile(wave, wave);
        // col[r] = [r == lane] - sum_{i < r} A[r][i] col[i].  The terms are taken oldest first, in two chains, and the
        // term of col[r - 1] last: only that product and the subtraction wait for the previous row, everything else
        // of a row is computed while earlier rows finish.
        float col[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float a_row[16];
#pragma unroll
            for (int i4 = 0; i4 < (r + 3) / 4; ++i4) {
                const float4 a4 = *reinterpret_cast<const float4*>(At + r * AT + 4 * i4);
                a_row[4 * i4] = a4.x;
                a_row[4 * i4 + 1] = a4.y;
                a_row[4 * i4 + 2] = a4.z;
                a_row[4 * i4 + 3] = a4.w;
            }
            float s0 = 0.f, s1 = 0.f;
#pragma unroll
            for (int i = 0; i + 1 < r; ++i) {   // i <= r - 2
                if (i & 1) s1 = fmaf(a_row[i], col[i], s1);
                else s0 = fmaf(a_row[i], col[i], s0);
            }
            float acc = s0 + s1;
            if (r > 0) acc = fmaf(a_row[r > 0 ? r - 1 : 0], col[r > 0 ? r - 1 : 0], acc);
            col[r] = ((r == lane) ? 1.f : 0.f) - acc;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) Tt[r * AT + lane] = col[r];
    }
    __syncthreads();
    // (b) blocks below the diagonal: T_ab = -T_aa sum_{b <= k < a} A_ak T_kb.  Wavefront b owns block
    //     column b and walks down it; products are 16x16x16 in fp32 MFMA (four 16x16x4 steps).  Step j of a
    //     product contracts over the indices 4 lq + j (lq: the lane's quarter): then the left operand is one
    //     16-byte read per lane, and a result tile, which a lane holds as rows 4 lq + j, is the right operand
    //     of the next product as it sits in registers.
    //     The partial sums of the blocks further down take each T_kb as soon as it exists, so that only the two
    //     products that finish a block (A_{k+1,k} T_kb and T_{k+1,k+1} X) stand between T_kb and T_{k+1,b}.
    if (wave == 0) inv_block_column<0>(As, Ts, l16, lq);
    else if (wave == 1) inv_block_column<1>(As, Ts, l16, lq);
    else if (wave == 2) inv_block_column<2>(As, Ts, l16, lq);
    __syncthreads();   // T complete
    // (c) T'' = T diag(b'), fp16, straight to global memory in fragment order: thread e writes the 4-element
    //     piece e of the chunk's 6 KiB, so a wavefront's store is one contiguous run.
    {
        half_t* Tc = TF + gc * TRI_FRAG_HALFS;
        constexpr int QPT = TRI_FRAG_HALFS / 4 / INV_THREADS;   // pieces of 4 per thread
        static_assert(QPT * 4 * INV_THREADS == TRI_FRAG_HALFS, "whole pieces");
#pragma unroll
        for (int k = 0; k < QPT; ++k) {
            const int e = tid + INV_THREADS * k;         // piece index: (f * 64 + lane') * 2 + half
            const int ln = (e >> 1) & 63, f = e >> 7;    // f = tri_frag(tw, ks)
            const int tw = f < 2 ? f : (f + 2) >> 1, ks = f < 2 ? 0 : f & 1;
            const int r = 16 * tw + (ln & 15), i = 32 * ks + 16 * (e & 1) + 4 * (ln >> 4);
            const int a = r >> 4, b = i >> 4;
            const float4 bp = *reinterpret_cast<const float4*>(s_bp + i);
            float4 t = {0.f, 0.f, 0.f, 0.f};
            if (b <= a) t = *reinterpret_cast<const float4*>(Ts + tri_tile(a, b) + (r & 15) * AT + (i & 15));
            f32x4 t4;
            t4[0] = (i <= r) ? t.x * bp.x : 0.f;
            t4[1] = (i + 1 <= r) ? t.y * bp.y : 0.f;
            t4[2] = (i + 2 <= r) ? t.z * bp.z : 0.f;
            t4[3] = (i + 3 <= r) ? t.w * bp.w : 0.f;
            *reinterpret_cast<half4*>(Tc + 4 * e) = to_half4(t4);
        }
    }
}

// The grid: first the blocks of the mask scan and compaction (the softmax branch's inputs, which nothing of the linear
// branch needs: a few hundred blocks, each a chain of memory latencies, that would otherwise stand alone on the
// stream for as long as a fifth of this kernel), then one block per chunk and (batch, head).
template <int D>
__global__ __launch_bounds__(INV_THREADS, INV_OCC) void gdn_chunk_inv_kernel(const InvArgs a, const ScanArgs<bf16_t> sc,
                                                                       const int scan_segs, const int scan_blocks) {
    static_assert(INV_THREADS == SCAN_THREADS, "the two kinds of block share one launch");
    static_assert(InvLds<D>::bytes >= SCAN_LDS_INTS * 4, "and one piece of LDS");
    __shared__ __align__(16) unsigned char smem[InvLds<D>::bytes];
    if ((int)blockIdx.x < scan_blocks) {
        scan_compact_block<bf16_t>(sc, blockIdx.x % scan_segs, blockIdx.x / scan_segs, reinterpret_cast<int*>(smem));
        return;
    }
    gdn_chunk_inv_block<D>(a, blockIdx.x - scan_blocks, smem);
}

// per chunk: TF, PF (TRI_FRAG_HALFS fp16 each), gamv, kdv (64 fp32 each), gamC (1 fp32); layouts above.
// The same launch carries the mask scan and compaction (arguments as launch_scan_compact).
nats_status launch_gdn_chunk_inv(const FwdPlan& pl, const void* Q, const void* K, const float* alpha,
                                 const float* beta, const uint8_t* mask, void* TF, void* PF, float* gamv,
                                 float* kdv, float* gamC, const void* K_sm, const void* V, int32_t* cnt, int32_t* idx,
                                 int32_t* n_s, void* Kc, void* Vc, void* Kc_user, void* Vc_user, int cap_user, void* VhT,
                                 hipStream_t st) {
    const InvArgs a{(const bf16_t*)Q, (const bf16_t*)K, alpha, beta, mask, pl.L, pl.routing == NATS_ROUTE_CHUNK,
                    (half_t*)TF, (half_t*)PF, gamv, kdv, gamC, pl.BH, pl.linear_op, pl.freeze_on_softmax,
                    pl.inner_chunk == 1};
    const ScanArgs<bf16_t> sc{mask, (const bf16_t*)K_sm, (const bf16_t*)V, pl.L, pl.d, cnt, idx, n_s, (bf16_t*)Kc,
                              (bf16_t*)Vc, (bf16_t*)Kc_user, (bf16_t*)Vc_user, cap_user, (half_t*)VhT,
                              pl.routing == NATS_ROUTE_CHUNK ? 6 : 0, pl.G, pl.qk_per_out_head};   // (this path: routing chunks of 64)
    const int scan_segs = (pl.L + SCAN_SEG - 1) / SCAN_SEG, scan_blocks = scan_segs * pl.BHG;
    dim3 grid((unsigned)(scan_blocks + (pl.L / CH) * ((pl.BH + 7) & ~7)));
    if (pl.d == 64) hipLaunchKernelGGL(gdn_chunk_inv_kernel<64>, grid, dim3(INV_THREADS), 0, st, a, sc, scan_segs, scan_blocks);
    else hipLaunchKernelGGL(gdn_chunk_inv_kernel<128>, grid, dim3(INV_THREADS), 0, st, a, sc, scan_segs, scan_blocks);
    return check_launch("gdn_chunk_inv");
}

}  // namespace nats
