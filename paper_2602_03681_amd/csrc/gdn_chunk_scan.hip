// Chunkwise Gated DeltaNet, step 2 of 2: the recurrence over chunks (Section 3, Eq. 6-7;
// update rule Eq. 19 with Eq. 14 / Eq. 20 folded into the per-chunk operands).
// With the per-chunk operands of the preparation kernel (W negated, U~ and Kd transposed):
//   U  = U~ - W S0^T                          [C x d_v]
//   O  = la_scale (Qg S0^T + P U)             [C x d_v]   (linear-branch output, Eq. 7 / Eq. 10; Qg = diag(gam) Q)
//   S1 = gam_C S0 + U^T Kd                    [d_v x d_k]
// The rows of S (index d_v) never mix, so a block owns a slice of BV values of d_v for one
// (batch, head) and walks the chunks in order; the grid is (d / BV) * (B*H) blocks.
//
// The state lives transposed, S^T [d_k x BV], as fp32 MFMA accumulators spread over four
// wavefronts (each owns d_k/4 rows) and never leaves registers in fp32; an fp16 copy of S in LDS
// is the B operand of the products that read it, and the fp16 copy of U is the B operand of the
// state update.  A block has two groups of four wavefronts: the first carries the dependent chain
// (U, then S1), the second produces the output (Qg S0^T + P U) from the same two LDS copies and
// merges / stores it one step later, so that only the products that read U stand between the two
// barriers of a step.  Phase 1 splits the chunk's tokens over a group's wavefronts, phase 2 splits
// d_k, so every A operand is private to one wavefront: it is loaded from global memory straight
// into MFMA fragment registers, three chunks ahead of use and one load at a time between the
// matrix instructions, and LDS carries only the two exchanged copies.  Where CUs would idle
// anyway, one extra block per (batch, head) touches the operands a dozen chunks ahead so that those
// loads hit in L2.  Per chunk: two block barriers (U ready, S ready).
//
// MFMA work per chunk and block: (2 d + 2 d + 2 C + 2 d) C BV FLOP; the path is bound by the
// length of the dependent chain (L / C steps), not by MFMA throughput.
#include <stdlib.h>

#include <algorithm>

#include "mfma_util.h"
#include "nats_common.h"

#ifndef NATS_MARK
#define NATS_MARK(i) do {} while (0)   // phase timestamps, only in debug harness builds
#define NATS_MARK_STEP (-1)
#endif

#ifndef NATS_SCAN_BV128
#define NATS_SCAN_BV128 32          // d_v values per block for d = 128
#endif
#ifndef NATS_SCAN_HELPER_PARTS
#define NATS_SCAN_HELPER_PARTS 4    // most prefetch helpers per (batch, head)
#endif
#ifndef NATS_SCAN_HELPER_LIMIT
#define NATS_SCAN_HELPER_LIMIT 256  // prefetch helpers only while compute blocks + helpers stay within the CUs
#endif

namespace nats {

constexpr int SCAN_THREADS_G = 512;   // 8 wavefronts: 4 carry the state, 4 produce the output
constexpr int CS = 64;                // chunk size
#ifndef PF_HELPER_AHEAD
#define PF_HELPER_AHEAD 12
#endif
constexpr int PF_HELPER_FIRST = 4;    // first chunk a prefetch helper touches (earlier ones are already in flight)

template <int D, int BV>
struct ScanLds {
    // The fp16 copies of S and U are the B operands of every product here: a lane (l16, quad lq) reads 16
    // bytes of row l16 at a column that depends on lq.  On gfx950 such reads run at the full LDS rate
    // (about 200 B/clk measured, against 128) when the four quads' addresses are equal modulo 256
    // bytes and the 16 rows of a quad fall on 16 different 16-byte slots modulo 256.  So each copy
    // is stored as four planes, one per quad (d_k / (D/4) for S, tok / 16 for U), whose size is a
    // multiple of 256 bytes and whose rows are an odd number of 16-byte slots long.
    static constexpr int SP = D / 4 + LDS_PAD;          // halves per row of a state plane  [BV][SP]
    static constexpr int UP = 16 + LDS_PAD;             // halves per row of a U plane      [BV][UP]
    static constexpr int S_PLANE = BV * SP, U_PLANE = BV * UP;
    static_assert((S_PLANE * 2) % 256 == 0 && (U_PLANE * 2) % 256 == 0, "planes must be 256-byte multiples");
    static_assert(((SP * 2 / 16) & 1) == 1 && ((UP * 2 / 16) & 1) == 1, "rows must be an odd number of 16-byte slots");
    static constexpr int o_S = 0;                       // state copy, fp16
    static constexpr int o_U = o_S + 4 * S_PLANE;       // U^T, fp16
    static constexpr int n_half = o_U + 4 * U_PLANE;
    // element (row v, d_k) of the state copy / (row v, token) of the U copy, in halves from the copy's base
    __device__ static __forceinline__ int s_at(int v, int dk) { return (dk / (D / 4)) * S_PLANE + v * SP + dk % (D / 4); }
    __device__ static __forceinline__ int u_at(int v, int tok) { return (tok / 16) * U_PLANE + v * UP + tok % 16; }
    static constexpr int OSTR = BV + 4;                 // fp32 row stride of the output staging tiles
    static constexpr int n_ost = 4 * 16 * OSTR;         // [4 wavefronts][16 tok][OSTR]
};

template <int N> struct HalfVec;
template <> struct HalfVec<8> { typedef half8 type; };
template <> struct HalfVec<4> { typedef half4 type; };

// Operands of one chunk for one wavefront, as MFMA fragments in registers.  Every A operand of a
// step is private to a wavefront (phase 1 splits the chunk's tokens, phase 2 splits d_k), so
// fragments are loaded straight from global memory and never staged in LDS; the preparation
// kernel wrote them in fragment order, so each load below is one contiguous 1 KiB per wavefront.
// The contraction slots of a lane (quad lq, step ks, slot j) stand for
//   d_k = (D/4) lq + 8 ks + j   in the products over d_k,   tok = 16 lq + 8 ks + j   over tokens,
// and the B operands (fp16 copies of S and U in LDS) are read with the same maps.
template <int D, int BV>
struct ChainStage {   // wavefront w of the state-carrying group
    static constexpr int KS_D = D / 32, MS = D / 64, NT = BV / 16;
    half8 w[KS_D];      // -W   rows tok = 16 w + l16
    half8 kd[MS][2];    // Kd^T rows d_k = 16 (MS w + ms) + l16
    half4 ut[NT];       // U~   rows tok = 16 w + 4 lq + j, col v = 16 nt + l16
    float gC;           // decay of the whole chunk
    __device__ __forceinline__ void load(const half_t* __restrict__ WF, const half_t* __restrict__ KdF,
                                         const half_t* __restrict__ UtF, const float* __restrict__ gamC,
                                         size_t gc, int v0, int w4, int lane) {
#pragma unroll
        for (int i = 0; i < N_PIECES; ++i) load_piece(i, WF, KdF, UtF, gamC, gc, v0, w4, lane);
    }
    // The loads of a stage one at a time, so that a step can spread them between its matrix
    // instructions: pieces [0, KS_D) -W, [KS_D, KS_D + NT) U~, then the chunk decay, then Kd.
    static constexpr int N_P1 = KS_D + NT + 1;          // pieces phase 1 of the step needs
    static constexpr int N_PIECES = N_P1 + 2 * MS;
    __device__ __forceinline__ void load_piece(int i, const half_t* __restrict__ WF, const half_t* __restrict__ KdF,
                                               const half_t* __restrict__ UtF, const float* __restrict__ gamC,
                                               size_t gc, int v0, int w4, int lane) {
        if (i < KS_D) {
            w[i] = (reinterpret_cast<const half8*>(WF) + ((gc * 4 + w4) * KS_D) * 64 + lane)[i * 64];
        } else if (i < KS_D + NT) {
            const int nt = i - KS_D;
            ut[nt] = (reinterpret_cast<const half4*>(UtF) + ((gc * (D / 16) + v0 / 16) * 4 + w4) * 64 + lane)[nt * 4 * 64];
        } else if (i == KS_D + NT) {
            gC = gamC[gc];
        } else {
            const int m = i - N_P1;
            kd[m / 2][m % 2] = (reinterpret_cast<const half8*>(KdF) + ((gc * 4 + w4) * MS * 2) * 64 + lane)[m * 64];
        }
    }
};

template <int D, int BV>
struct OutStage {     // wavefront w of the output group
    static constexpr int KS_D = D / 32, VPL = BV / 4;
    typedef typename HalfVec<VPL>::type hvec;
    half8 q[KS_D];      // Qg   rows tok = 16 w + l16
    half8 p[2];         // P    rows r = 16 w + l16
    hvec onla;          // softmax-branch output, row 16 w + lane / 4, columns v0 + VPL (lane % 4) ..
    // onla_row: pointer to this lane's VPL values of row (16 w + lane / 4) of the chunk, or nullptr
    __device__ __forceinline__ void load(const half_t* __restrict__ QF, const half_t* __restrict__ PF,
                                         const half_t* onla_row, size_t gc, int w4, int lane) {
#pragma unroll
        for (int i = 0; i < N_PIECES; ++i) load_piece(i, QF, PF, onla_row, gc, w4, lane);
    }
    // one load at a time (see ChainStage): pieces [0, KS_D) Qg, then P, then the softmax-branch row piece
    static constexpr int N_PIECES = KS_D + 3;
    __device__ __forceinline__ void load_piece(int i, const half_t* __restrict__ QF, const half_t* __restrict__ PF,
                                               const half_t* onla_row, size_t gc, int w4, int lane) {
        if (i < KS_D) {
            q[i] = (reinterpret_cast<const half8*>(QF) + ((gc * 4 + w4) * KS_D) * 64 + lane)[i * 64];
        } else if (i < KS_D + 2) {
            p[i - KS_D] = (reinterpret_cast<const half8*>(PF) + ((gc * 4 + w4) * 2) * 64 + lane)[(i - KS_D) * 64];
        } else if (onla_row != nullptr) {
            onla = *reinterpret_cast<const hvec*>(onla_row);
        }
    }
};

// MERGE = false: the output group stores the linear branch's output as fp16 (O_la_h) for the softmax
//                kernel's merge epilogue.
// MERGE = true : it reads the softmax branch's output (O_nla_h, fp16), adds it and stores O (bf16):
//                the plain-sum merge of Section 4.1, done where the linear output is in registers.
template <int D, int BV, bool MERGE>
__global__ __launch_bounds__(SCAN_THREADS_G) void gdn_chunk_scan_kernel(
    const half_t* __restrict__ WF, const half_t* __restrict__ QF, const half_t* __restrict__ KdF,
    const half_t* __restrict__ UtF, const half_t* __restrict__ PF, const float* __restrict__ gamC,
    const float* __restrict__ S0, float* __restrict__ S_final, half_t* __restrict__ O_la_h,
    float* __restrict__ O_la_f32, const half_t* __restrict__ O_nla_h, bf16_t* __restrict__ O,
    int32_t* __restrict__ progress, int n_compute, int L, int BH, float la_scale) {
    using Lds = ScanLds<D, BV>;
    constexpr int NT = BV / 16;       // 16-wide tiles along the d_v slice
    constexpr int MS = D / 64;        // 16-row d_k tiles of S^T owned by one wavefront
    constexpr int KS_D = D / 32;      // contraction steps over d_k
    __shared__ __align__(16) half_t sh[Lds::n_half];
    __shared__ __align__(16) float ost_all[Lds::n_ost];
    half_t* Ss = sh + Lds::o_S;
    half_t* Us = sh + Lds::o_U;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int w4 = wave & 3;                 // index inside the group: token tile (phase 1), d_k quarter (phase 2)
    const bool is_chain = wave < 4;          // wavefronts 0-3 carry the state, 4-7 produce the output
    const int l16 = lane & 15, lq = lane >> 4;
    // Block -> (batch*head, d_v slice).  Workgroups are dealt round-robin to the 8 XCDs, each with
    // its own L2; the slices of one (batch, head) read the same operands, so they are given ids
    // that are congruent modulo 8 and therefore share one L2.
    constexpr int NSL = D / BV;
    const int n_chunks = L / CS;
    if ((int)blockIdx.x >= n_compute) {
        // ---- prefetch helper: one block per (batch, head) on an otherwise idle CU of the same XCD.
        // A CU can keep only so many cache-line misses in flight, so with HBM latency the compute
        // blocks cannot pull their 60 KB per chunk fast enough by themselves.  The helper reads one
        // word of every 64 bytes of the chunks they will need a few steps from now, so that their
        // loads hit in L2.  It follows the published chunk counter and never blocks anyone: every
        // wait is bounded, and the compute blocks never wait for a helper.
        // Several helpers may serve one (batch, head): helper part p of n_parts takes every n_parts-th of a
        // wavefront's chunks.  (One CU cannot keep enough misses in flight to fetch a pair's 72 KB per step
        // from HBM: with one helper, 3 of every 8 chunks arrived in time.)
        const int n_helper = 8 * ((BH + 7) / 8);
        const int hid = ((int)blockIdx.x - n_compute) % n_helper, part = ((int)blockIdx.x - n_compute) / n_helper;
        const int n_parts = ((int)gridDim.x - n_compute) / n_helper;
        const int hbh = (hid >> 3) * 8 + (hid & 7);
        if (hbh >= BH) return;
        constexpr int AHEAD = PF_HELPER_AHEAD;       // chunks of lead over the consumer
        constexpr int SEG = 64 / (int)sizeof(half_t);
        const size_t hgc0 = (size_t)hbh * n_chunks;
        float sink = 0.f;
        for (int c = PF_HELPER_FIRST + wave + part * (SCAN_THREADS_G / 64); c < n_chunks; c += n_parts * (SCAN_THREADS_G / 64)) {
            int spins = 0, done = 0;
            while (true) {
                done = __hip_atomic_load(progress + hbh * PROG_STRIDE, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (c <= done + AHEAD || ++spins > 2000) break;
                // sleep roughly one consumer step per chunk of excess lead: few polls per chunk
                for (int e = min(c - done - AHEAD, 16); e > 0; --e) __builtin_amdgcn_s_sleep(24);
            }
            if (spins > 2000) break;                 // the consumer is not advancing: stop helping
            if (c <= done + 2) continue;             // too late to be useful for this chunk
            const size_t gc = hgc0 + c;
            const half_t* bases[5] = {WF + gc * (size_t)(CS * D), QF + gc * (size_t)(CS * D),
                                      KdF + gc * (size_t)(D * CS), UtF + gc * (size_t)(D * CS),
                                      MERGE ? O_nla_h + ((size_t)hbh * L + (size_t)c * CS) * D : WF + gc * (size_t)(CS * D)};
#pragma unroll
            for (int a = 0; a < 5; ++a)
#pragma unroll
                for (int i = 0; i < CS * D / SEG / 64; ++i)
                    sink += (float)bases[a][(size_t)(i * 64 + lane) * SEG];
            const half_t* pb = PF + gc * (size_t)(CS * CS);
#pragma unroll
            for (int i = 0; i < CS * CS / SEG / 64; ++i) sink += (float)pb[(size_t)(i * 64 + lane) * SEG];
        }
        asm volatile("" ::"v"(sink));   // keeps the loads alive; the values are not used
        return;
    }
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int bh = (slot / NSL) * 8 + xcd;
    if (bh >= BH) return;
    const int v0 = (slot % NSL) * BV;
    const size_t gc0 = (size_t)bh * n_chunks;
    const size_t tokb = (size_t)bh * L;
    constexpr int PF_DIST = 3;
    const bool publisher = progress != nullptr && is_chain && v0 == 0 && tid == 0;   // reports progress
    // Both groups run the same barrier sequence (two per chunk).  Loads are issued PF_DIST chunks
    // ahead of use through PF_DIST + 1 rotating register stages; they are unconditional (the tail re-loads the
    // last chunk), so that the compiler's load-wait counts stay exact and never include the loads issued
    // after the one being waited for.

    if (is_chain) {
        // ---- state: S^T tiles (rows d_k, cols v) as fp32 accumulators; fp16 copy S[v][d_k] in LDS -----
        f32x4 accS[MS][NT];
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int dk = 16 * (MS * w4 + ms) + 4 * lq, v = v0 + 16 * nt + l16;
                if (S0 != nullptr) {
                    const float4 x = *reinterpret_cast<const float4*>(S0 + ((size_t)bh * D + v) * D + dk);
                    accS[ms][nt] = f32x4{x.x, x.y, x.z, x.w};
                } else {
                    accS[ms][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
                *reinterpret_cast<half4*>(Ss + Lds::s_at(16 * nt + l16, dk)) = to_half4(accS[ms][nt]);
            }
        ChainStage<D, BV> stA, stB, stC, stD;
        stA.load(WF, KdF, UtF, gamC, gc0, v0, w4, lane);
        stB.load(WF, KdF, UtF, gamC, gc0 + min(1, n_chunks - 1), v0, w4, lane);
        stC.load(WF, KdF, UtF, gamC, gc0 + min(2, n_chunks - 1), v0, w4, lane);
        __syncthreads();   // initial state copy visible

        int c_pub = 0;
        auto step = [&](int c, const ChainStage<D, BV>& cur, ChainStage<D, BV>& nxt) __attribute__((always_inline)) {
            if (c == NATS_MARK_STEP) NATS_MARK(0);
            // The published chunk number lives in a vector register of its own: a temporary for the store's data
            // would be a register with a load in flight, and the store would wait for every load before it.
            asm volatile("" : "+v"(c_pub));
            if (publisher) __hip_atomic_store(progress + bh * PROG_STRIDE, c_pub, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            c_pub += 1;
            // The loads for chunk c + PF_DIST are issued one at a time between the matrix instructions of
            // this step: issued in a burst they queue in the CU's vector-memory path (about 16 cycles
            // per 1 KiB load, shared with the output group) and stall the wavefront that carries the
            // dependent chain for hundreds of cycles.
            using CS_t = ChainStage<D, BV>;
            const size_t gcn = gc0 + min(c + PF_DIST, n_chunks - 1);
            int piece = 0;
            auto one_load = [&]() __attribute__((always_inline)) {
                __builtin_amdgcn_sched_barrier(0);
                if (piece < CS_t::N_PIECES) nxt.load_piece(piece, WF, KdF, UtF, gamC, gcn, v0, w4, lane);
                ++piece;
                __builtin_amdgcn_sched_barrier(0);
            };
            // phase 1: U = U~ - W S0^T for this wavefront's 16 tokens
            half8 fs[KS_D][NT];
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) fs[ks][nt] = lds_read8(Ss + Lds::s_at(16 * nt + l16, (D / 4) * lq + 8 * ks));
            f32x4 accU[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                accU[nt] = f32x4{(float)cur.ut[nt][0], (float)cur.ut[nt][1], (float)cur.ut[nt][2], (float)cur.ut[nt][3]};
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    accU[nt] = mfma16(cur.w[ks], fs[ks][nt], accU[nt]);
                    if (piece < CS_t::N_P1) one_load();
                }
            // decay of the state, off the dependent chain (phase 1 reads the fp16 copy in LDS)
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    accS[ms][nt][0] *= cur.gC; accS[ms][nt][1] *= cur.gC;
                    accS[ms][nt][2] *= cur.gC; accS[ms][nt][3] *= cur.gC;
                }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                *reinterpret_cast<half4*>(Us + Lds::u_at(16 * nt + l16, 16 * w4 + 4 * lq)) = to_half4(accU[nt]);
            while (piece < CS_t::N_P1) one_load();
            if (c == NATS_MARK_STEP) NATS_MARK(1);
            __syncthreads();   // U complete; the old state copy has been read by everyone
            if (c == NATS_MARK_STEP) NATS_MARK(2);
            // phase 2: S^T = gam_C S^T + Kd^T U for this wavefront's quarter of d_k
            half8 fu[2][NT];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) fu[ks][nt] = lds_read8(Us + Lds::u_at(16 * nt + l16, 16 * lq + 8 * ks));
#pragma unroll
            for (int ms = 0; ms < MS; ++ms) {
#pragma unroll
                for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        accS[ms][nt] = mfma16(cur.kd[ms][ks], fu[ks][nt], accS[ms][nt]);
                        one_load();
                    }
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    *reinterpret_cast<half4*>(Ss + Lds::s_at(16 * nt + l16, 16 * (MS * w4 + ms) + 4 * lq)) =
                        to_half4(accS[ms][nt]);
            }
            while (piece < CS_t::N_PIECES) one_load();
            if (c == NATS_MARK_STEP) NATS_MARK(3);
            __syncthreads();   // new state copy visible; U copy free again
            if (c == NATS_MARK_STEP) NATS_MARK(4);
        };
        // step(c, stage holding chunk c, stage to refill with chunk c + PF_DIST).  Four unconditional steps per
        // trip: every path into the loop header then has the same loads in flight, in the same order (three
        // stages' worth), and the compiler's wait counts are exact.  A conditional step inside the loop makes it
        // merge paths with fewer loads in flight and wait for all of them, also for those just issued.
        int c = 0;
        for (; c + 4 <= n_chunks; c += 4) {
            step(c, stA, stD);
            step(c + 1, stB, stA);
            step(c + 2, stC, stB);
            step(c + 3, stD, stC);
        }
        if (c < n_chunks) step(c, stA, stD);
        if (c + 1 < n_chunks) step(c + 1, stB, stA);
        if (c + 2 < n_chunks) step(c + 2, stC, stB);
        if (S_final != nullptr) {
#pragma unroll
            for (int ms = 0; ms < MS; ++ms)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const int dk = 16 * (MS * w4 + ms) + 4 * lq, v = v0 + 16 * nt + l16;
                    *reinterpret_cast<float4*>(S_final + ((size_t)bh * D + v) * D + dk) =
                        make_float4(accS[ms][nt][0], accS[ms][nt][1], accS[ms][nt][2], accS[ms][nt][3]);
                }
        }
    } else {
        constexpr int VPL = BV / 4;   // merged output: a lane stores VPL consecutive d_v of one token
        // this lane's piece of the softmax-branch output for chunk cc (row 16 w4 + lane / 4)
        auto onla_ptr = [&](int cc) __attribute__((always_inline)) -> const half_t* {
            return MERGE ? O_nla_h + (tokb + (size_t)cc * CS + 16 * w4 + (lane >> 2)) * D + v0 + VPL * (lane & 3)
                         : nullptr;
        };
        OutStage<D, BV> stA, stB, stC, stD;
        stA.load(QF, PF, onla_ptr(0), gc0, w4, lane);
        stB.load(QF, PF, onla_ptr(min(1, n_chunks - 1)), gc0 + min(1, n_chunks - 1), w4, lane);
        stC.load(QF, PF, onla_ptr(min(2, n_chunks - 1)), gc0 + min(2, n_chunks - 1), w4, lane);
        __syncthreads();   // initial state copy visible

        // The result rows of a chunk leave through a staging tile in LDS that is private to the
        // wavefront (transposed there so that a lane owns VPL consecutive d_v of one token and every
        // global access is a full row segment).  Between the two barriers of a step stand only the
        // products that read U and the writes into that tile: the dependent chain waits at the second
        // barrier.  Reading the tile back, the merge and the store of chunk c - 1 come at the start of step c.
        constexpr int OSTR = Lds::OSTR;
        float* Ost = ost_all + w4 * 16 * OSTR;
        using OS_t = OutStage<D, BV>;
        // st: the stage that holds chunk cprev's piece of the softmax-branch output
        auto store_rows = [&](int cprev, const OS_t& st) __attribute__((always_inline)) {
            const int row = lane >> 2, piece = lane & 3;
            const size_t off = (tokb + (size_t)cprev * CS + 16 * w4 + row) * D + v0 + VPL * piece;
            float ola[VPL];
#pragma unroll
            for (int i = 0; i < VPL; i += 4) {
                const float4 x = *reinterpret_cast<const float4*>(Ost + row * OSTR + VPL * piece + i);
                ola[i] = x.x; ola[i + 1] = x.y; ola[i + 2] = x.z; ola[i + 3] = x.w;
            }
            if (O_la_f32 != nullptr) {
#pragma unroll
                for (int i = 0; i < VPL; i += 4)
                    *reinterpret_cast<float4*>(O_la_f32 + off + i) = make_float4(ola[i], ola[i + 1], ola[i + 2], ola[i + 3]);
            }
            uint32_t packed[VPL / 2];
            if (MERGE) {   // add the softmax branch's row piece, store bf16
#pragma unroll
                for (int i = 0; i < VPL; i += 2)
                    packed[i / 2] = pack_bf16x2(ola[i] + (float)st.onla[i], ola[i + 1] + (float)st.onla[i + 1]);
            } else {       // the linear branch's rows as fp16 for the softmax kernel's merge epilogue
#pragma unroll
                for (int i = 0; i < VPL; i += 2) {
                    typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
                    const half2_t h = half2_t{f32_to_half_sat(ola[i]), f32_to_half_sat(ola[i + 1])};
                    packed[i / 2] = __builtin_bit_cast(uint32_t, h);
                }
            }
            void* dst = MERGE ? static_cast<void*>(O + off) : static_cast<void*>(O_la_h + off);
            if (VPL == 8)
                *reinterpret_cast<u32x4*>(dst) = u32x4{packed[0], packed[1], packed[VPL / 2 - 2], packed[VPL / 2 - 1]};
            else
                *reinterpret_cast<uint2*>(dst) = make_uint2(packed[0], packed[1]);
        };

        auto step = [&](int c, const OS_t& cur, OS_t& nxt) __attribute__((always_inline)) {
            const int cn = min(c + PF_DIST, n_chunks - 1);
            const half_t* onla_n = onla_ptr(cn);
            int piece = 0;
            auto one_load = [&]() __attribute__((always_inline)) {
                __builtin_amdgcn_sched_barrier(0);
                if (piece < OS_t::N_PIECES) nxt.load_piece(piece, QF, PF, onla_n, gc0 + cn, w4, lane);
                ++piece;
                __builtin_amdgcn_sched_barrier(0);
            };
            // rows of the previous chunk first: the chain group's reads of the state copy get the LDS to themselves
            // for a few hundred cycles.  (Moving them behind the first barrier, where this group has time to
            // spare, changed nothing: the two groups share the SIMDs.)
            if (c > 0) {
                store_rows(c - 1, nxt);
                __builtin_amdgcn_sched_barrier(0);
            }
            // phase 1: Qg S0^T for this wavefront's 16 tokens
            half8 fs[KS_D][NT];
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) fs[ks][nt] = lds_read8(Ss + Lds::s_at(16 * nt + l16, (D / 4) * lq + 8 * ks));
            f32x4 accO[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) accO[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    accO[nt] = mfma16(cur.q[ks], fs[ks][nt], accO[nt]);
                    if (ks > 0 || nt == NT - 1) one_load();
                }
            while (piece < OS_t::N_PIECES) one_load();
            __syncthreads();   // U complete
            // phase 2: + P U, then the result tile into the staging rows
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const half8 fu = lds_read8(Us + Lds::u_at(16 * nt + l16, 16 * lq + 8 * ks));
                    accO[nt] = mfma16(cur.p[ks], fu, accO[nt]);
                }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int j = 0; j < 4; ++j) Ost[(4 * lq + j) * OSTR + 16 * nt + l16] = la_scale * accO[nt][j];
            __syncthreads();   // U copy free again
        };
        // step(c, stage holding chunk c, stage to refill with chunk c + PF_DIST, which held chunk c - 1);
        // the same loop shape as the other group's (same barriers, exact wait counts)
        int c = 0;
        for (; c + 4 <= n_chunks; c += 4) {
            step(c, stA, stD);
            step(c + 1, stB, stA);
            step(c + 2, stC, stB);
            step(c + 3, stD, stC);
        }
        if (c < n_chunks) step(c, stA, stD);
        if (c + 1 < n_chunks) step(c + 1, stB, stA);
        if (c + 2 < n_chunks) step(c + 2, stC, stB);
        // rows of the last chunk
        switch ((n_chunks - 1) & 3) {
            case 0: store_rows(n_chunks - 1, stA); break;
            case 1: store_rows(n_chunks - 1, stB); break;
            case 2: store_rows(n_chunks - 1, stC); break;
            default: store_rows(n_chunks - 1, stD); break;
        }
    }
}

template <int D, int BV>
static nats_status launch_scan_t(const FwdPlan& pl, const void* WF, const void* QF, const void* KdF,
                                 const void* UtF, const void* PF, const float* gamC, const float* S0,
                                 float* S_final, void* O_la_h, float* O_la_f32, const void* O_nla_h, void* O,
                                 int32_t* progress, hipStream_t st) {
    const int n_compute = 8 * ((pl.BH + 7) / 8) * (D / BV);   // see the block -> (bh, slice) map in the kernel
    // prefetch helpers only where CUs would otherwise idle (one compute block fills a CU)
    const int n_helper = 8 * ((pl.BH + 7) / 8);
    static const bool helpers_off = getenv("NATS_NO_PREFETCH_HELPERS") != nullptr;   // A/B switch, read once
    const bool helpers = progress != nullptr && n_compute + n_helper <= NATS_SCAN_HELPER_LIMIT && !helpers_off;
    // as many helpers per (batch, head) as idle CUs allow, at most NATS_SCAN_HELPER_PARTS
    const int n_parts = helpers ? std::min(NATS_SCAN_HELPER_PARTS, (NATS_SCAN_HELPER_LIMIT - n_compute) / n_helper) : 0;
    dim3 grid(n_compute + n_parts * n_helper);
    if (O_nla_h != nullptr)
        hipLaunchKernelGGL((gdn_chunk_scan_kernel<D, BV, true>), grid, dim3(SCAN_THREADS_G), 0, st,
                           (const half_t*)WF, (const half_t*)QF, (const half_t*)KdF, (const half_t*)UtF,
                           (const half_t*)PF, gamC, S0, S_final, (half_t*)nullptr, O_la_f32,
                           (const half_t*)O_nla_h, (bf16_t*)O, progress, n_compute, pl.L, pl.BH, pl.la_scale);
    else
        hipLaunchKernelGGL((gdn_chunk_scan_kernel<D, BV, false>), grid, dim3(SCAN_THREADS_G), 0, st,
                           (const half_t*)WF, (const half_t*)QF, (const half_t*)KdF, (const half_t*)UtF,
                           (const half_t*)PF, gamC, S0, S_final, (half_t*)O_la_h, O_la_f32,
                           (const half_t*)nullptr, (bf16_t*)nullptr, progress, n_compute, pl.L, pl.BH, pl.la_scale);
    return check_launch("gdn_chunk_scan");
}

// O_nla_h == nullptr: writes O_la_h (fp16) for the softmax kernel to merge.  Otherwise merges
// (plain sum) with O_nla_h and writes O.
nats_status launch_gdn_chunk_scan(const FwdPlan& pl, const void* WF, const void* QF, const void* KdF,
                                  const void* UtF, const void* PF, const float* gamC, const float* S0,
                                  float* S_final, void* O_la_h, float* O_la_f32, const void* O_nla_h, void* O,
                                  int32_t* progress, hipStream_t st) {
    if (pl.d == 64)
        return launch_scan_t<64, 16>(pl, WF, QF, KdF, UtF, PF, gamC, S0, S_final, O_la_h, O_la_f32, O_nla_h, O,
                                     progress, st);
    return launch_scan_t<128, NATS_SCAN_BV128>(pl, WF, QF, KdF, UtF, PF, gamC, S0, S_final, O_la_h, O_la_f32,
                                               O_nla_h, O, progress, st);
}

}  // namespace nats
