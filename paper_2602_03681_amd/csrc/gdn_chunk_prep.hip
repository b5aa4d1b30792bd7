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
constexpr int CH = 64;        // chunk size
constexpr int AS_STRIDE = 68; // fp32 row stride of the A and T matrices in LDS
constexpr float LOG2E = 1.44269504088896341f;

// LDS plan (bytes).  Regions are reused as their first tenants die, to keep a block under half
// of the CU's 160 KiB so that two blocks overlap each other's latency-bound phases:
//   R12 : K and Q tiles, fp16 [64][d+8] each           (until Qg is written)
//         -> T fp32 [64][68] at 0, T' fp16 [64][72] at 25600   (triangular inverse, then operand form)
//         -> V^T fp16 [d][72] at 0                      (last phase; V waits in registers until then)
//   R3  : K^T fp16 [d][72]                              (whole kernel)
//   R5  : A fp32 [64][68] -> T'' fp16 [64][72]
//   Xs  : 4 x 16x16 fp32 scratch of the block inverse;  gates: 4 x 64 fp32
template <int D>
struct PrepLds {
    static constexpr int RS = D + LDS_PAD, TS = CH + LDS_PAD;
    static constexpr int kq_bytes = 2 * CH * RS * 2;
    static constexpr int tp_off = 25600;
    static constexpr int r12_bytes = (kq_bytes > tp_off + CH * TS * 2) ? kq_bytes : tp_off + CH * TS * 2;
    static constexpr int o_kst = r12_bytes;
    static constexpr int o_as = o_kst + D * TS * 2;
    static constexpr int o_xs = o_as + CH * AS_STRIDE * 4;
    static constexpr int o_gate = o_xs + 4 * 256 * 4;
    static constexpr int bytes = o_gate + 4 * CH * 4 + 2 * CH * 2;
    static_assert(CH * AS_STRIDE * 4 <= tp_off, "T and T' overlap");
    static_assert(D * TS * 2 <= tp_off, "V^T and T' overlap");
};

// Transposed tiles [d][tok] are written 2 bytes at a time by lanes that hold different d of the
// same token; an xor swizzle of the 8-token group index with (d / 8) spreads those writes over
// the banks.  Readers fetch 8 consecutive tokens (16 bytes) starting at a multiple of 8.
__device__ __forceinline__ int swz_t(int drow, int tok, int TS) {
    return drow * TS + ((((tok >> 3) ^ (drow >> 3)) & 7) << 3) + (tok & 7);
}

#ifndef NATS_PREP_CPB
#define NATS_PREP_CPB 2
#endif
constexpr int PREP_CPB = NATS_PREP_CPB;   // chunks per block

template <int D>
__global__ __launch_bounds__(PREP_THREADS, 2) void gdn_chunk_prep_kernel(
    const bf16_t* __restrict__ Q, const bf16_t* __restrict__ K, const bf16_t* __restrict__ V,
    const float* __restrict__ alpha, const float* __restrict__ beta, const uint8_t* __restrict__ mask,
    int L, int chunk_mask, half_t* __restrict__ WF, half_t* __restrict__ QF, half_t* __restrict__ KdF,
    half_t* __restrict__ UtF, half_t* __restrict__ PF, float* __restrict__ gamC, int BH, int linear_op,
    int freeze_on_softmax) {
    using Lds = PrepLds<D>;
    constexpr int RS = Lds::RS, TS = Lds::TS;
    constexpr int NPC = CH * D / 8 / PREP_THREADS;   // 16-byte pieces of a [64][D] tile per thread
    extern __shared__ __align__(16) unsigned char smem[];
    half_t* Ks = reinterpret_cast<half_t*>(smem);              // [64][RS]
    half_t* Qs = Ks + CH * RS;                                 // [64][RS]
    float* Ts = reinterpret_cast<float*>(smem);                // [64][AS_STRIDE]   (after Ks, Qs)
    half_t* Tp = reinterpret_cast<half_t*>(smem + Lds::tp_off);  // [64][TS]  T diag(b' gam)
    half_t* VsT = reinterpret_cast<half_t*>(smem);             // [D][TS]   (after T)
    half_t* KsT = reinterpret_cast<half_t*>(smem + Lds::o_kst);  // [D][TS]
    float* As = reinterpret_cast<float*>(smem + Lds::o_as);    // [64][AS_STRIDE]
    half_t* Tpp = reinterpret_cast<half_t*>(smem + Lds::o_as); // [64][TS]  T diag(b')  (after A)
    float* Xs = reinterpret_cast<float*>(smem + Lds::o_xs);    // [4][256]
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
    // A block takes PREP_CPB chunks of one pair, one after the other, and issues the global loads of the next
    // chunk while it works on the current one (K and Q as soon as their registers are free, V later): with
    // two blocks per CU (LDS) there are not enough wavefronts to hide that latency otherwise.
    const int bh8 = (BH + 7) & ~7;
    const int bh = blockIdx.x % bh8;
    if (bh >= BH) return;
    int chunk = n_chunks - 1 - (blockIdx.x / bh8) * PREP_CPB;
    // The thread's indices are re-derived inside the chunk loop from a value the compiler cannot see through:
    // otherwise it hoists every LDS address of the body out of the loop and runs out of registers.
    int tid = tid0;

    NATS_MARK(0);
    // ---- tiles: coalesced 16-byte loads (a [64][D] tile is contiguous in global memory) --------
    u32x4 rk[NPC], rq[NPC], rv[NPC];
    auto load_kq = [&](int c) __attribute__((always_inline)) {
        const size_t t0 = (size_t)bh * L + (size_t)c * CH;
        const u32x4* Kg = reinterpret_cast<const u32x4*>(K + t0 * D);
        const u32x4* Qg = reinterpret_cast<const u32x4*>(Q + t0 * D);
#pragma unroll
        for (int i = 0; i < NPC; ++i) {
            rk[i] = Kg[tid + PREP_THREADS * i];
            rq[i] = Qg[tid + PREP_THREADS * i];
        }
    };
    auto load_v = [&](int c) __attribute__((always_inline)) {
        const u32x4* Vg = reinterpret_cast<const u32x4*>(V + ((size_t)bh * L + (size_t)c * CH) * D);
#pragma unroll
        for (int i = 0; i < NPC; ++i) rv[i] = Vg[tid + PREP_THREADS * i];
    };
    load_kq(chunk);
    load_v(chunk);
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
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float up = __shfl_up(g, off);
            if (lane >= off) g += up;
        }
        const float gC = __shfl(g, 63);
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
    // K row-major + transposed (swizzled), Q row-major; V stays in registers for now
#pragma unroll
    for (int i = 0; i < NPC; ++i) {
        const int e = tid + PREP_THREADS * i;
        const int row = e / (D / 8), c8 = e % (D / 8);
        const half8 hk = bf16x8_to_half8(rk[i]);
        *reinterpret_cast<half8*>(Ks + row * RS + c8 * 8) = hk;
        *reinterpret_cast<half8*>(Qs + row * RS + c8 * 8) = bf16x8_to_half8(rq[i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) KsT[swz_t(c8 * 8 + j, row, TS)] = hk[j];
    }
    if (more) load_kq(chunk - 1);
    __syncthreads();
    NATS_MARK(1);

    // ---- K K^T -> A (LDS, fp32) and (Q K^T . D) -> P (global), lower 16x16 tiles ----------
    {
        // 16x16 tile jobs (a, b), one hex digit per job: the 10 lower tiles (products), then the 6
        // upper tiles, which are stored as zeros (the consumer contracts over all 64 tokens)
        constexpr uint64_t JA = 0x2110003333222110ull;  // a of job 0 in the lowest digit
        constexpr uint64_t JB = 0x3323213210210100ull;
        half_t* Pc = PF + gc * (CH * CH);
        // P[r = 16a + l16][i = 16b + 4 lq + j] -> PF[w = a][ks = lq / 2][lane = 16 b + l16][4 (lq % 2) + j]
        // A wavefront's product jobs (job = wave, wave + 4, wave + 8 < 10) run as one straight-line
        // sequence with separate accumulators, so that the LDS reads and MFMA chains of one job fill
        // the latencies of the others; the third slot of wavefronts 2 and 3 repeats job 0 and is not stored.
        constexpr int NJ = 3;
        int ja[NJ], jb[NJ];
        f32x4 accK[NJ], accP[NJ];
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            const int job = (wave + 4 * jj < 10) ? wave + 4 * jj : 0;
            ja[jj] = (int)((JA >> (4 * job)) & 15);
            jb[jj] = (int)((JB >> (4 * job)) & 15);
            accK[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
            accP[jj] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int ks = 0; ks < D / 32; ++ks)
#pragma unroll
            for (int jj = 0; jj < NJ; ++jj) {
                const int ko = 32 * ks + 8 * lq;
                const half8 fa = lds_read8(Ks + (16 * ja[jj] + l16) * RS + ko);
                const half8 fb = lds_read8(Ks + (16 * jb[jj] + l16) * RS + ko);
                const half8 fq = lds_read8(Qs + (16 * ja[jj] + l16) * RS + ko);
                accK[jj] = mfma16(fa, fb, accK[jj]);  // rows: tokens of block a, cols: tokens of block b
                accP[jj] = mfma16(fb, fq, accP[jj]);  // rows: key tokens i of block b, cols: query tokens r of block a
            }
#pragma unroll
        for (int jj = 0; jj < NJ; ++jj) {
            if (wave + 4 * jj >= 10) continue;   // uniform per wavefront
            const int a = ja[jj], b = jb[jj];
            half_t* dst = Pc + (((a * 2 + (lq >> 1)) * 64) + 16 * b + l16) * 8 + 4 * (lq & 1);
            {   // A[r][i], r = 16a + 4 lq + j, i = 16b + l16
                const int i = 16 * b + l16;
                const float gi = s_g2[i];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int r = 16 * a + 4 * lq + j;
                    // gated linear attention (no delta rule): A = 0, so T = (I + A)^-1 = I below
                    As[r * AS_STRIDE + i] =
                        (i < r && linear_op == 0) ? s_bp[r] * accK[jj][j] * __builtin_amdgcn_exp2f(s_g2[r] - gi) : 0.f;
                }
            }
            {   // P[r][i], r = 16a + l16, i = 16b + 4 lq + j
                const int r = 16 * a + l16;
                const float gr = s_g2[r];
                f32x4 pv;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int i = 16 * b + 4 * lq + j;
                    pv[j] = (i <= r) ? accP[jj][j] * __builtin_amdgcn_exp2f(gr - s_g2[i]) : 0.f;
                }
                *reinterpret_cast<half4*>(dst) = to_half4(pv);
            }
        }
        // the 6 upper tiles (jobs 10..15) of P are zeros
        for (int job = 10 + wave; job < 16; job += 4) {
            const int a = (int)((JA >> (4 * job)) & 15), b = (int)((JB >> (4 * job)) & 15);
            half4 z = {0, 0, 0, 0};
            *reinterpret_cast<half4*>(Pc + (((a * 2 + (lq >> 1)) * 64) + 16 * b + l16) * 8 + 4 * (lq & 1)) = z;
        }
    }
    __syncthreads();
    NATS_MARK(2);

    // ---- Kd and Qg in fragment order, straight to global (coalesced 16-byte stores) ---------------
    {
        constexpr int KS_D = D / 32;
        half8* Kd = reinterpret_cast<half8*>(KdF + gc * (size_t)(D * CH));
        // scaling in packed fp16 (two elements per instruction): the factors gam_C / gam_r and gam_r are
        // in (0, 1], so nothing overflows, and the second rounding costs 2^-12 relative
        typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
        for (int e = tid; e < D * CH / 8; e += PREP_THREADS) {   // e = ((w * MS + ms) * 2 + ks) * 64 + lane
            const int ln = e & 63, ks = (e >> 6) & 1, wm = e >> 7;   // wm = w * MS + ms
            const int dk = 16 * wm + (ln & 15), t0 = 16 * (ln >> 4) + 8 * ks;
            half8 h = lds_read8(KsT + swz_t(dk, t0, TS));
            const half8 sc = lds_read8(s_gdec_h + t0);
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
                const half2_t pr = half2_t{h[j], h[j + 1]} * half2_t{sc[j], sc[j + 1]};
                h[j] = pr[0]; h[j + 1] = pr[1];
            }
            Kd[e] = h;
        }
        half8* Qg = reinterpret_cast<half8*>(QF + gc * (size_t)(CH * D));
        for (int e = tid; e < CH * D / 8; e += PREP_THREADS) {   // e = (w * KS_D + ks) * 64 + lane
            const int ln = e & 63, ks = (e >> 6) % KS_D, w = (e >> 6) / KS_D;
            const int tok = 16 * w + (ln & 15), dk = (D / 4) * (ln >> 4) + 8 * ks;
            half8 h = lds_read8(Qs + tok * RS + dk);
            const half_t g = s_gam_h[tok];
#pragma unroll
            for (int j = 0; j < 8; j += 2) {
                const half2_t pr = half2_t{h[j], h[j + 1]} * half2_t{g, g};
                h[j] = pr[0]; h[j + 1] = pr[1];
            }
            Qg[e] = h;
        }
        // the decay the recurrence applies to the state it carries over this chunk (1 for a softmax chunk in
        // the variant without decay there: inside the chunk the decays still act on the provisional state)
        if (tid == 0) gamC[gc] = (freeze_on_softmax && chunk_mask && mask[gc] != 0) ? 1.f : s_gam[CH - 1];
    }
    __syncthreads();   // K and Q tiles are dead from here on: their region becomes T
    // ---- T = (I + A)^{-1}, unit lower triangular, by 16x16 blocks in fp32 ------------------------
    // (a) diagonal blocks: wavefront b inverts I + A_bb by forward substitution; lane j < 16 owns
    //     column j, row r needs rows < r of the same column
    if (lane < 16) {
        const int b = wave;
        float col[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) col[r] = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float acc = 0.f;
#pragma unroll
            for (int i4 = 0; i4 < (r + 3) / 4; ++i4) {   // A[r][i] is 0 for i >= r, col[i] is 0 there too
                const float4 a4 = *reinterpret_cast<const float4*>(As + (16 * b + r) * AS_STRIDE + 16 * b + 4 * i4);
                acc += a4.x * col[4 * i4] + a4.y * col[4 * i4 + 1] + a4.z * col[4 * i4 + 2] +
                       a4.w * col[4 * i4 + 3];
            }
            col[r] = ((r == lane) ? 1.f : 0.f) - acc;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) Ts[(16 * b + r) * AS_STRIDE + 16 * b + lane] = col[r];
    }
    __syncthreads();
    NATS_MARK(3);
    // (b) blocks below the diagonal: T_ab = -T_aa sum_{b <= k < a} A_ak T_kb.  Wavefront b owns block
    //     column b and walks down it; products are 16x16x16 in fp32 MFMA (16x16x4 steps).  A result
    //     tile is in row-quad layout while the next product wants it as a B operand (one row per
    //     lane quad), so it takes one trip through a per-wavefront LDS scratch.
    {
        const int b = wave;
        float* Xw = Xs + wave * 256;
        for (int a = b + 1; a < 4; ++a) {
            f32x4 X = {0.f, 0.f, 0.f, 0.f};
            for (int k = b; k < a; ++k) {
#pragma unroll
                for (int s4 = 0; s4 < 4; ++s4) {
                    const float af = As[(16 * a + l16) * AS_STRIDE + 16 * k + 4 * s4 + lq];
                    const float bf = Ts[(16 * k + 4 * s4 + lq) * AS_STRIDE + 16 * b + l16];
                    X = __builtin_amdgcn_mfma_f32_16x16x4f32(af, bf, X, 0, 0, 0);
                }
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) Xw[(4 * lq + j) * 16 + l16] = X[j];
            __builtin_amdgcn_wave_barrier();   // LDS operations of one wavefront complete in order
            f32x4 Y = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s4 = 0; s4 < 4; ++s4) {
                const float af = Ts[(16 * a + l16) * AS_STRIDE + 16 * a + 4 * s4 + lq];
                const float bf = Xw[(4 * s4 + lq) * 16 + l16];
                Y = __builtin_amdgcn_mfma_f32_16x16x4f32(af, bf, Y, 0, 0, 0);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) Ts[(16 * a + 4 * lq + j) * AS_STRIDE + 16 * b + l16] = -Y[j];
            __builtin_amdgcn_wave_barrier();
        }
    }
    __syncthreads();   // T complete; A is dead from here on: its region becomes T''
    // (c) operand forms T diag(b' gam) and T diag(b'), fp16, row-major [r][i]
    for (int e = tid; e < CH * CH; e += PREP_THREADS) {
        const int r = e >> 6, i = e & 63;
        const float t = (i <= r) ? Ts[r * AS_STRIDE + i] : 0.f;
        const float bp = s_bp[i];
        Tpp[r * TS + i] = f32_to_half_sat(t * bp);
        Tp[r * TS + i] = linear_op == 0 ? f32_to_half_sat(t * bp * s_gam[i]) : (half_t)0.f;   // W = 0 without the delta rule
    }
    __syncthreads();   // T is dead from here on: its region becomes V^T
#pragma unroll
    for (int i = 0; i < NPC; ++i) {
        const int e = tid + PREP_THREADS * i;
        const int row = e / (D / 8), c8 = e % (D / 8);
        const half8 hv = bf16x8_to_half8(rv[i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) VsT[swz_t(c8 * 8 + j, row, TS)] = hv[j];
    }
    if (more) load_v(chunk - 1);
    NATS_MARK(4);
    __syncthreads();
    NATS_MARK(5);

    // ---- W^T = K^T (T diag(b' gam))^T  and  U~ = (T diag(b')) V ------------------------------
    {
        constexpr int KS_D = D / 32;
        half_t* Wc = WF + gc * (size_t)(CH * D);
        half_t* Uc = UtF + gc * (size_t)(D * CH);
#pragma unroll
        for (int mi = 0; mi < D / 64; ++mi) {
            const int m = wave * (D / 64) + mi;  // 16-wide tile index along d_k (W) / d_v (U~)
#pragma unroll
            for (int n = 0; n < 4; ++n) {        // 16-token tile; T is lower triangular: k-steps 0..n/2
                f32x4 accW = {0.f, 0.f, 0.f, 0.f}, accU = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks <= n / 2; ++ks) {
                    const int ko = 32 * ks + 8 * lq;
                    const half8 fk = lds_read8(KsT + swz_t(16 * m + l16, ko, TS));
                    const half8 fv = lds_read8(VsT + swz_t(16 * m + l16, ko, TS));
                    const half8 ft = lds_read8(Tp + (16 * n + l16) * TS + ko);
                    const half8 ftt = lds_read8(Tpp + (16 * n + l16) * TS + ko);
                    accW = mfma16(fk, ft, accW);   // rows d_k = 16m + 4lq + j, col token r = 16n + l16
                    accU = mfma16(ftt, fv, accU);  // rows token r = 16n + 4lq + j, col d_v = 16m + l16
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
