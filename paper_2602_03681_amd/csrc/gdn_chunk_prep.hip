// Chunkwise Gated DeltaNet, step 1 of 2: everything inside a chunk that does not depend
// on the running state (Section 3, Eq. 6-7 applied to the update rule of Eq. 19, with
// Eq. 14 / Eq. 20 folded in as  b'_t = beta_t (1 - m_t)  and decay at every token).
//
// For one chunk of C = 64 tokens, with g_r = sum_{i<=r} log alpha_i (inside the chunk):
//   D[r,i]  = exp(g_r - g_i)                       (i <= r)
//   A       = strict_lower( diag(b') (K K^T . D) )
//   T       = (I + A)^{-1}                         (unit lower triangular; fp32, blocks of 16)
//   W       = T diag(b' exp(g)) K                  (stored negated)
//   U~      = T diag(b') V
//   P       = (Q K^T) . D  (i <= r, zero above the diagonal)
//   Kd      = diag(exp(g_C - g)) K
//   Qg      = diag(exp(g)) Q
//   gam_C   = exp(g_C)
// so that the state-carrying kernel only needs
//   U = U~ - W S0^T,  O = Qg S0^T + P U,  S1 = gam_C S0 + U^T Kd.
//
// Output format ("fragment-major", fp16): every operand is written in the order in which the
// wavefronts of the state-carrying kernel load their MFMA fragments, so that each of their
// loads is one contiguous 1 KiB (64 lanes x 16 bytes).  With lane = 16 lq + l16 and w = 0..3:
//   WF  [chunk][w][ks < d/32][lane][8] = -W [tok = 16w + l16][d_k = (d/4) lq + 8 ks + j]
//   QF  same shape                     =  Qg[tok = 16w + l16][d_k = (d/4) lq + 8 ks + j]
//   KdF [chunk][w][ms < d/64][ks < 2][lane][8] = Kd[tok = 16 lq + 8 ks + j][d_k = 16 (d/64 w + ms) + l16]
//   PF  [chunk][w][ks < 2][lane][8]    =  P [r = 16w + l16][i = 16 lq + 8 ks + j]
//   UtF [chunk][vt < d/16][w][lane][4] =  U~[tok = 16w + 4 lq + j][d_v = 16 vt + l16]
//   gamC[chunk]                        (fp32)
//
// One block per chunk and (batch, head) (a one-dimensional grid, chunk-major), 4 wavefronts.  All matrix products run on
// MFMA with fp16 operands / fp32 accumulation; products are arranged (transposed where
// needed) so that every result tile is stored as 4 consecutive fp16 along the layout the
// consumer reads.  The triangular inverse is blocked 16x16: substitution inside the four
// diagonal blocks (one per wavefront), fp32 MFMA for the blocks below them.
#include <math.h>

#include "mfma_util.h"
#include "nats_common.h"

#ifndef NATS_MARK
#define NATS_MARK(i) do {} while (0)   // phase timestamps, only in debug harness builds
#endif

namespace nats {

constexpr int PREP_THREADS = 256;
constexpr int CH = 64;                 // chunk size
constexpr int AT = 20;                 // fp32 row stride of a 16x16 tile of A or T in LDS (rows stay 16-byte aligned)
constexpr int AT_TILE = 16 * AT + 16;  // floats per tile; the 16 extra shift the next tile by 16 banks
constexpr int N_TRI = 10;              // 16x16 tiles on and below the diagonal of a 64x64 matrix
constexpr float LOG2E = 1.44269504088896341f;

// A and T are lower triangular: only the tiles (a, b), b <= a, exist, row by row
__device__ __forceinline__ int tri_tile(int a, int b) { return ((a * (a + 1)) / 2 + b) * AT_TILE; }

// LDS plan (bytes).  Regions are reused as their first tenants die, to keep a block under a third of the
// CU's 160 KiB: the kernel is bound by latencies (global loads, LDS round trips, barriers), and three blocks
// per CU fill each other's gaps.  Q never enters LDS: every wavefront loads its fragments from global memory.
//   R1  : K tile, fp16 [64][d+8]                         (until A and P are complete)
//         -> T, fp32 lower tiles                         (triangular inverse)
//         -> V^T fp16 [d][72]                            (last phase; V waits in registers until then)
//   R2  : K^T fp16 [d][72]                               (whole chunk)
//   R3  : A, fp32 lower tiles -> T'' = T diag(b') fp16 [64][72]
//   gates: 4 x 64 fp32 + 2 x 64 fp16
template <int D>
struct PrepLds {
    static constexpr int RS = D + LDS_PAD, TS = CH + LDS_PAD;
    static constexpr int tri_bytes = N_TRI * AT_TILE * 4;
    static constexpr int k_bytes = CH * RS * 2, vt_bytes = D * TS * 2, tpp_bytes = CH * TS * 2;
    static constexpr int r1_bytes =
        k_bytes > vt_bytes ? (k_bytes > tri_bytes ? k_bytes : tri_bytes) : (vt_bytes > tri_bytes ? vt_bytes : tri_bytes);
    static constexpr int o_kst = r1_bytes;
    static constexpr int o_as = o_kst + vt_bytes;
    static constexpr int o_gate = o_as + (tri_bytes > tpp_bytes ? tri_bytes : tpp_bytes);
    static constexpr int bytes = o_gate + 4 * CH * 4 + 2 * CH * 2;
    static_assert(3 * bytes <= 160 * 1024, "three blocks per CU");
};

// Transposed tiles [d][tok] are written 2 bytes at a time by lanes that hold different d of the
// same token; an xor swizzle of the 8-token group index with (d / 8) spreads those writes over
// the banks.  Readers fetch 8 consecutive tokens (16 bytes) starting at a multiple of 8.
__device__ __forceinline__ int swz_t(int drow, int tok, int TS) {
    return drow * TS + ((((tok >> 3) ^ (drow >> 3)) & 7) << 3) + (tok & 7);
}

#ifndef NATS_PREP_CPB
#define NATS_PREP_CPB 1
#endif
constexpr int PREP_CPB = NATS_PREP_CPB;   // chunks per block

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

// h[j] *= s[j], two elements per instruction
__device__ __forceinline__ half8 mul8(half8 h, half8 s) {
#pragma unroll
    for (int j = 0; j < 8; j += 2) {
        const half2_t pr = half2_t{h[j], h[j + 1]} * half2_t{s[j], s[j + 1]};
        h[j] = pr[0]; h[j + 1] = pr[1];
    }
    return h;
}

template <int D>
__global__ __launch_bounds__(PREP_THREADS, 3) void gdn_chunk_prep_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const float* __restrict__ alpha, const float* __restrict__ beta, const uint8_t* __restrict__ mask,
    int L, int chunk_mask, half_t* __restrict__ WF, half_t* __restrict__ QF, half_t* __restrict__ KdF,
    half_t* __restrict__ UtF, half_t* __restrict__ PF, float* __restrict__ gamC, int BH, int linear_op,
    int freeze_on_softmax) {
    using Lds = PrepLds<D>;
    constexpr int RS = Lds::RS, TS = Lds::TS;
    constexpr int NPC = CH * D / 8 / PREP_THREADS;   // 16-byte pieces of a [64][D] tile per thread
    constexpr int KS_D = D / 32;
    extern __shared__ __align__(16) unsigned char smem[];
    half_t* Ks = reinterpret_cast<half_t*>(smem);              // [64][RS]
    float* Ts = reinterpret_cast<float*>(smem);                // lower tiles   (after Ks)
    half_t* VsT = reinterpret_cast<half_t*>(smem);             // [D][TS]       (after T)
    half_t* KsT = reinterpret_cast<half_t*>(smem + Lds::o_kst);  // [D][TS]
    float* As = reinterpret_cast<float*>(smem + Lds::o_as);    // lower tiles
    half_t* Tpp = reinterpret_cast<half_t*>(smem + Lds::o_as); // [64][TS]  T diag(b')  (after A)
    float* s_g2 = reinterpret_cast<float*>(smem + Lds::o_gate);  // cumulative log2-decay
    float* s_gam = s_g2 + CH;
    float* s_bp = s_gam + CH;
    float* s_gdec = s_bp + CH;
    half_t* s_gdec_h = reinterpret_cast<half_t*>(s_gdec + CH);   // fp16 copies of gam_C / gam and gam
    half_t* s_gam_h = s_gdec_h + CH;

    const int tid0 = threadIdx.x;
    const int n_chunks = L / CH;
    // One-dimensional grid, chunk-major: all (batch, head) pairs of a chunk side by side (padded to a
    // multiple of 8, so that a pair's blocks land on the XCD whose L2 the recurrence blocks of that pair
    // use), the chunks back to front: what the recurrence reads first is then what was written last and is
    // still in the caches (its time per chunk is 1.05 microseconds while all operands fit the memory-side
    // cache, 1.3 beyond; on the headline shape this order brought it from 1.31 to 1.20).
    // A block takes PREP_CPB chunks of one pair, one after the other, and issues the global loads of K and Q
    // of the next chunk while it works on the current one.
    const int bh8 = (BH + 7) & ~7;
    const int bh = blockIdx.x % bh8;
    if (bh >= BH) return;
    int chunk = n_chunks - 1 - (blockIdx.x / bh8) * PREP_CPB;
    // The thread's indices are re-derived inside the chunk loop from a value the compiler cannot see through:
    // otherwise it hoists every LDS address of the body out of the loop and runs out of registers.
    int tid = tid0;

    NATS_MARK(0);
    // ---- K and V tiles: coalesced 16-byte loads (a [64][D] tile is contiguous in global memory) ----
    // ---- Q: MFMA fragments straight from global memory.  Wavefront w multiplies query tile a0 = 3 - w
    //      (wavefront 3 also tile 3) and writes that tile of Qg; lane (l16, lq) holds, per step ks, the 8
    //      elements d_k = (D/4) lq + 8 ks + j of token 16 a + l16, which is the order Qg is stored in.
    u32x4 rk[NPC], rv[NPC], q0[KS_D], q1[KS_D];
    auto load_k = [&](int c) __attribute__((always_inline)) {
        const u32x4* Kg = reinterpret_cast<const u32x4*>(K + ((size_t)bh * L + (size_t)c * CH) * D);
#pragma unroll
        for (int i = 0; i < NPC; ++i) rk[i] = Kg[tid + PREP_THREADS * i];
    };
    auto load_v = [&](int c) __attribute__((always_inline)) {
        const u32x4* Vg = reinterpret_cast<const u32x4*>(V + ((size_t)bh * L + (size_t)c * CH) * D);
#pragma unroll
        for (int i = 0; i < NPC; ++i) rv[i] = Vg[tid + PREP_THREADS * i];
    };
    auto load_q = [&](int c) __attribute__((always_inline)) {
        const int wv = tid >> 6, ln = tid & 63;
        const int qa0 = 3 - wv, qa1 = (wv == 3) ? 3 : qa0;
        const bf16_t* Qc = Q + ((size_t)bh * L + (size_t)c * CH + (ln & 15)) * D + (D / 4) * (ln >> 4);
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) {
            q0[ks] = *reinterpret_cast<const u32x4*>(Qc + (size_t)(16 * qa0) * D + 8 * ks);
            q1[ks] = *reinterpret_cast<const u32x4*>(Qc + (size_t)(16 * qa1) * D + 8 * ks);
        }
    };
    load_k(chunk);
    load_q(chunk);
#pragma unroll 1
    for (int it = 0; it < PREP_CPB && chunk >= 0; ++it, --chunk) {
    const size_t gc = (size_t)bh * n_chunks + chunk;  // global chunk id
    const size_t tok0 = (size_t)bh * L + (size_t)chunk * CH;
    const bool more = it + 1 < PREP_CPB && chunk > 0;   // another chunk follows in this block (uniform)
    asm volatile("" : "+v"(tid));
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l16 = lane & 15, lq = lane >> 4;
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
        s_g2[lane] = g;
        s_gam[lane] = __builtin_amdgcn_exp2f(g);
        // Routing per token: a softmax token writes nothing (b' = 0).  Routing per chunk: every token
        // writes inside its chunk (the intra-chunk part is computed for every chunk), and a softmax
        // chunk hands nothing on: its Kd is zero, so the state only takes the chunk's decay.
        const bool soft_chunk = chunk_mask && mask[gc] != 0;
        s_gdec[lane] = soft_chunk ? 0.f : __builtin_amdgcn_exp2f(gC - g);
        s_gdec_h[lane] = (half_t)s_gdec[lane];
        s_gam_h[lane] = (half_t)s_gam[lane];
        s_bp[lane] = (!chunk_mask && mask[tok0 + lane]) ? 0.f : beta[tok0 + lane];
    }
    // K row-major + transposed (swizzled); V stays in registers for now
#pragma unroll
    for (int i = 0; i < NPC; ++i) {
        const int e = tid + PREP_THREADS * i;
        const int row = e / (D / 8), c8 = e % (D / 8);
        const half8 hk = bf16x8_to_half8(rk[i]);
        *reinterpret_cast<half8*>(Ks + row * RS + c8 * 8) = hk;
#pragma unroll
        for (int j = 0; j < 8; ++j) KsT[swz_t(c8 * 8 + j, row, TS)] = hk[j];
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
    NATS_MARK(1);

    // ---- K K^T -> A (LDS, fp32) and (Q K^T . D) -> P (global), lower 16x16 tiles ----------
    const int a0 = 3 - wave, a1 = (wave == 3) ? 3 : a0;
    {
        // 16x16 tile products (a, b), b <= a: wavefront w takes (a0, 0), (a1, 1) [wavefront 3: (3, 3)] and, for
        // w < 2, (a0, 2); the third slot of wavefronts 2 and 3 repeats their first product and is not stored.
        // The three run as one straight-line sequence with separate accumulators, so that the LDS reads and
        // MFMA chains of one fill the latencies of the others.
        // P[r = 16a + l16][i = 16b + 4 lq + j] -> PF[w = a][ks = lq / 2][lane = 16 b + l16][4 (lq % 2) + j]
        constexpr int NJ = 3;
        const int ja[NJ] = {a0, a1, a0};
        const int jb[NJ] = {0, (wave == 3) ? 3 : 1, (wave < 2) ? 2 : 0};
        half_t* Pc = PF + gc * (CH * CH);
        f32x4 accK[NJ], accP[NJ];
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            accK[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
            accP[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) {
            // contraction order of the query fragments; any order does as long as both operands use it
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
                    pv[j] = (i <= r) ? accP[jj][j] * __builtin_amdgcn_exp2f(gr[jj] - g4[j]) : 0.f;
                }
                *reinterpret_cast<half4*>(Pc + (((a * 2 + (lq >> 1)) * 64) + 16 * b + l16) * 8 + 4 * (lq & 1)) =
                    to_half4(pv);
            }
        }
        // the 6 tiles of P above the diagonal are zeros: (0,1) (0,2) (0,3) (1,2) (1,3) (2,3)
        for (int z = wave; z < 6; z += 4) {
            const int a = (0x211000 >> (4 * z)) & 15, b = (0x332321 >> (4 * z)) & 15;
            half4 zero = {0, 0, 0, 0};
            *reinterpret_cast<half4*>(Pc + (((a * 2 + (lq >> 1)) * 64) + 16 * b + l16) * 8 + 4 * (lq & 1)) = zero;
        }
    }
    __syncthreads();   // A complete; the K tile is dead from here on: its region becomes T
    NATS_MARK(2);

    // V of this chunk and K of the next one are asked for here, where the registers of the products above
    // are free; they arrive while the triangular inverse runs
    load_v(chunk);
    if (more) load_k(chunk - 1);
    // ---- Kd and Qg in fragment order, straight to global (coalesced 16-byte stores) ---------------
    {
        half8* Kd = reinterpret_cast<half8*>(KdF + gc * (size_t)(D * CH));
        // scaling in packed fp16 (two elements per instruction): the factors gam_C / gam_r and gam_r are
        // in (0, 1], so nothing overflows, and the second rounding costs 2^-12 relative
        for (int e = tid; e < D * CH / 8; e += PREP_THREADS) {   // e = ((w * MS + ms) * 2 + ks) * 64 + lane
            const int ln = e & 63, ks = (e >> 6) & 1, wm = e >> 7;   // wm = w * MS + ms
            const int dk = 16 * wm + (ln & 15), t0 = 16 * (ln >> 4) + 8 * ks;
            Kd[e] = mul8(lds_read8(KsT + swz_t(dk, t0, TS)), lds_read8(s_gdec_h + t0));
        }
        // QF[w = a0][ks][lane][8]: the query fragments as they sit in registers, times gam of their token
        half8* Qg = reinterpret_cast<half8*>(QF + gc * (size_t)(CH * D)) + (size_t)a0 * KS_D * 64 + lane;
        const half_t g = s_gam_h[16 * a0 + l16];
        const half8 g8 = {g, g, g, g, g, g, g, g};
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) Qg[ks * 64] = mul8(hq0[ks], g8);
        if (more) load_q(chunk - 1);
        // the decay the recurrence applies to the state it carries over this chunk (1 for a softmax chunk in
        // the variant without decay there: inside the chunk the decays still act on the provisional state)
        if (tid == 0) gamC[gc] = (freeze_on_softmax && chunk_mask && mask[gc] != 0) ? 1.f : s_gam[CH - 1];
    }
    NATS_MARK(8);
    // ---- T = (I + A)^{-1}, unit lower triangular, by 16x16 blocks in fp32 ------------------------
    // (a) diagonal blocks: wavefront b inverts I + A_bb by forward substitution; lane j < 16 owns
    //     column j, row r needs rows < r of the same column
    if (lane < 16) {
        const float* At = As + tri_tile(wave, wave);
        float* Tt = Ts + tri_tile(wave, wave);
        float col[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) col[r] = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float acc = 0.f;
#pragma unroll
            for (int i4 = 0; i4 < (r + 3) / 4; ++i4) {   // A[r][i] is 0 for i >= r, col[i] is 0 there too
                const float4 a4 = *reinterpret_cast<const float4*>(At + r * AT + 4 * i4);
                acc += a4.x * col[4 * i4] + a4.y * col[4 * i4 + 1] + a4.z * col[4 * i4 + 2] +
                       a4.w * col[4 * i4 + 3];
            }
            col[r] = ((r == lane) ? 1.f : 0.f) - acc;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) Tt[r * AT + lane] = col[r];
    }
    __syncthreads();
    NATS_MARK(3);
    // (b) blocks below the diagonal: T_ab = -T_aa sum_{b <= k < a} A_ak T_kb.  Wavefront b owns block
    //     column b and walks down it; products are 16x16x16 in fp32 MFMA (four 16x16x4 steps).  Step j of a
    //     product contracts over the indices 4 lq + j (lq: the lane's quarter): then the left operand is one
    //     16-byte read per lane, and a result tile, which a lane holds as rows 4 lq + j, is the right operand
    //     of the next product as it sits in registers.
    {
        const int b = wave;
        for (int a = b + 1; a < 4; ++a) {
            f32x4 X = {0.f, 0.f, 0.f, 0.f};
            for (int k = b; k < a; ++k) {
                const float4 af = *reinterpret_cast<const float4*>(As + tri_tile(a, k) + l16 * AT + 4 * lq);
                const float* Tkb = Ts + tri_tile(k, b) + (4 * lq) * AT + l16;
                X = __builtin_amdgcn_mfma_f32_16x16x4f32(af.x, Tkb[0], X, 0, 0, 0);
                X = __builtin_amdgcn_mfma_f32_16x16x4f32(af.y, Tkb[AT], X, 0, 0, 0);
                X = __builtin_amdgcn_mfma_f32_16x16x4f32(af.z, Tkb[2 * AT], X, 0, 0, 0);
                X = __builtin_amdgcn_mfma_f32_16x16x4f32(af.w, Tkb[3 * AT], X, 0, 0, 0);
            }
            const float4 tf = *reinterpret_cast<const float4*>(Ts + tri_tile(a, a) + l16 * AT + 4 * lq);
            f32x4 Y = {0.f, 0.f, 0.f, 0.f};
            Y = __builtin_amdgcn_mfma_f32_16x16x4f32(tf.x, X[0], Y, 0, 0, 0);
            Y = __builtin_amdgcn_mfma_f32_16x16x4f32(tf.y, X[1], Y, 0, 0, 0);
            Y = __builtin_amdgcn_mfma_f32_16x16x4f32(tf.z, X[2], Y, 0, 0, 0);
            Y = __builtin_amdgcn_mfma_f32_16x16x4f32(tf.w, X[3], Y, 0, 0, 0);
            float* Tab = Ts + tri_tile(a, b) + (4 * lq) * AT + l16;
#pragma unroll
            for (int j = 0; j < 4; ++j) Tab[j * AT] = -Y[j];
            __builtin_amdgcn_wave_barrier();   // LDS operations of one wavefront complete in order
        }
    }
    __syncthreads();   // T complete; A is dead from here on: its region becomes T''
    NATS_MARK(9);
    // (c) operand form T'' = T diag(b'), fp16, row-major [r][i]: four columns per thread.  All reads first,
    //     then all writes: the compiler cannot tell that T'' does not overlap T, and would otherwise wait for
    //     every write before the next read.  (W takes its factor gam from K below.)
    {
        constexpr int QPT = CH * CH / 4 / PREP_THREADS;   // groups of 4 per thread
        f32x4 t4[QPT];
#pragma unroll
        for (int k = 0; k < QPT; ++k) {
            const int e = tid + PREP_THREADS * k, r = e >> 4, g = e & 15;
            const int a = r >> 4, b = g >> 2;
            const float4 bp = *reinterpret_cast<const float4*>(s_bp + 4 * g);
            float4 t = {0.f, 0.f, 0.f, 0.f};
            if (b <= a) t = *reinterpret_cast<const float4*>(Ts + tri_tile(a, b) + (r & 15) * AT + 4 * (g & 3));
            const int i = 4 * g;
            t4[k][0] = (i <= r) ? t.x * bp.x : 0.f;
            t4[k][1] = (i + 1 <= r) ? t.y * bp.y : 0.f;
            t4[k][2] = (i + 2 <= r) ? t.z * bp.z : 0.f;
            t4[k][3] = (i + 3 <= r) ? t.w * bp.w : 0.f;
        }
#pragma unroll
        for (int k = 0; k < QPT; ++k) {
            const int e = tid + PREP_THREADS * k, r = e >> 4, g = e & 15;
            *reinterpret_cast<half4*>(Tpp + r * TS + 4 * g) = to_half4(t4[k]);
        }
    }
    __syncthreads();   // T is dead from here on: its region becomes V^T
    NATS_MARK(10);
#pragma unroll
    for (int i = 0; i < NPC; ++i) {
        const int e = tid + PREP_THREADS * i;
        const int row = e / (D / 8), c8 = e % (D / 8);
        const half8 hv = bf16x8_to_half8(rv[i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) VsT[swz_t(c8 * 8 + j, row, TS)] = hv[j];
    }
    NATS_MARK(4);
    __syncthreads();
    NATS_MARK(5);

    // ---- W^T = (diag(gam) K)^T T''^T  and  U~ = T'' V ------------------------------------------
    {
        half_t* Wc = WF + gc * (size_t)(CH * D);
        half_t* Uc = UtF + gc * (size_t)(D * CH);
        // T'' fragments (token tile n, k-step ks <= n / 2: T is lower triangular) and the factors gam of the
        // tokens of a k-step (zero without the delta rule: W = 0 there)
        half8 ft[4][2], gf[2];
#pragma unroll
        for (int n = 0; n < 4; ++n)
#pragma unroll
            for (int ks = 0; ks <= n / 2; ++ks) ft[n][ks] = lds_read8(Tpp + (16 * n + l16) * TS + 32 * ks + 8 * lq);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            gf[ks] = lds_read8(s_gam_h + 32 * ks + 8 * lq);
            if (linear_op != 0) gf[ks] = half8{0, 0, 0, 0, 0, 0, 0, 0};
        }
#pragma unroll
        for (int mi = 0; mi < D / 64; ++mi) {
            const int m = wave * (D / 64) + mi;  // 16-wide tile index along d_k (W) / d_v (U~)
            half8 fk[2], fv[2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int ko = 32 * ks + 8 * lq;
                fk[ks] = mul8(lds_read8(KsT + swz_t(16 * m + l16, ko, TS)), gf[ks]);
                fv[ks] = lds_read8(VsT + swz_t(16 * m + l16, ko, TS));
            }
#pragma unroll
            for (int n = 0; n < 4; ++n) {        // 16-token tile
                f32x4 accW = {0.f, 0.f, 0.f, 0.f}, accU = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks <= n / 2; ++ks) {
                    accW = mfma16(fk[ks], ft[n][ks], accW);   // rows d_k = 16m + 4lq + j, col token r = 16n + l16
                    accU = mfma16(ft[n][ks], fv[ks], accU);   // rows token r = 16n + 4lq + j, col d_v = 16m + l16
                }
                f32x4 neg = {-accW[0], -accW[1], -accW[2], -accW[3]};
                // -W[tok = 16n + l16][d_k = 16m + 4 lq + j] -> WF[w = n][ks'][lane = 16 lq' + l16][j0 + j]
                const int dk0 = 16 * m + 4 * lq;
                const int lq2 = dk0 / (D / 4), ks2 = (dk0 % (D / 4)) / 8, j0 = dk0 & 7;
                *reinterpret_cast<half4*>(Wc + (((n * KS_D + ks2) * 64) + 16 * lq2 + l16) * 8 + j0) = to_half4(neg);
                // U~[tok = 16n + 4 lq + j][d_v = 16m + l16] -> UtF[vt = m][w = n][lane][j]
                *reinterpret_cast<half4*>(Uc + ((m * 4 + n) * 64 + lane) * 4) = to_half4(accU);
            }
        }
    }
    NATS_MARK(6);
    __syncthreads();   // also: the LDS regions are free for the block's next chunk
    NATS_MARK(7);
    }
}

// per chunk: WF, QF, KdF, UtF (64 * d fp16 each), PF (64 * 64 fp16), gamC (1 fp32); layouts above
nats_status launch_gdn_chunk_prep(const FwdPlan& pl, const void* Q, const void* K, const void* V,
                                  const float* alpha, const float* beta, const uint8_t* mask, void* WF,
                                  void* QF, void* KdF, void* UtF, void* PF, float* gamC, hipStream_t st) {
    dim3 grid((unsigned)(((pl.L / CH + PREP_CPB - 1) / PREP_CPB) * ((pl.BH + 7) & ~7)));
    // the LDS-size attribute is per function and device: set once per device, not per launch
    static bool attr_done[2][64] = {};
    int dev = 0;
    (void)hipGetDevice(&dev);
    dev = (dev >= 0 && dev < 64) ? dev : 0;
    if (pl.d == 64) {
        auto kern = gdn_chunk_prep_kernel<64>;
        if (!attr_done[0][dev]) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    PrepLds<64>::bytes) != hipSuccess)
                return check_launch("gdn_chunk_prep (LDS attribute)");
            attr_done[0][dev] = true;
        }
        hipLaunchKernelGGL(kern, grid, dim3(PREP_THREADS), PrepLds<64>::bytes, st, (const bf16_t*)Q,
                           (const bf16_t*)K, (const bf16_t*)V, alpha, beta, mask, pl.L, pl.routing == NATS_ROUTE_CHUNK, (half_t*)WF, (half_t*)QF,
                           (half_t*)KdF, (half_t*)UtF, (half_t*)PF, gamC, pl.BH, pl.linear_op, pl.freeze_on_softmax);
    } else {
        auto kern = gdn_chunk_prep_kernel<128>;
        if (!attr_done[1][dev]) {
            if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    PrepLds<128>::bytes) != hipSuccess)
                return check_launch("gdn_chunk_prep (LDS attribute)");
            attr_done[1][dev] = true;
        }
        hipLaunchKernelGGL(kern, grid, dim3(PREP_THREADS), PrepLds<128>::bytes, st, (const bf16_t*)Q,
                           (const bf16_t*)K, (const bf16_t*)V, alpha, beta, mask, pl.L, pl.routing == NATS_ROUTE_CHUNK, (half_t*)WF, (half_t*)QF,
                           (half_t*)KdF, (half_t*)UtF, (half_t*)PF, gamC, pl.BH, pl.linear_op, pl.freeze_on_softmax);
    }
    return check_launch("gdn_chunk_prep");
}

}  // namespace nats
