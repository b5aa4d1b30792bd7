// Chunkwise Gated DeltaNet, step 2 of 2: the recurrence over chunks (Section 3, Eq. 6-7; update rule
// Eq. 19 with Eq. 14 / Eq. 20 folded into the per-chunk gates), on the raw K, Q, V and the per-chunk
// T'' = (I + A)^-1 diag(b'), P = (Q K^T) . D and gates of the inversion kernel:
//   R  = V - diag(gam) K S0^T                 [C x d_v]
//   U  = T'' R                                [C x d_v]
//   O  = la_scale (diag(gam) Q S0^T + P U)    [C x d_v]   (linear-branch output, Eq. 7 / Eq. 10)
//   S1 = gam_C S0 + U^T diag(kd) K            [d_v x d_k]
//
// The chunk recurrence is affine in the state: S1 = S0 M + N with M (d_k x d_k) and N (d_v x d_k) that do
// not depend on S0.  So the sequence is cut into segments that run side by side:
//   pass 1   segment 0 runs the recurrence from the initial state, outputs included.  For every middle
//            segment the same recurrence runs twice without outputs: from the zero state (the end state is the
//            segment's N) and on the d_k unit rows with V = 0 (the end state is the segment's M); the two runs
//            share one block, which reads K, T'' and the gates once for both;
//   fix-up   (gdn_seg_fix) S_start[s + 1] = S_start[s] M_s + N_s along the few segments of a (batch, head);
//   pass 2   every later segment runs the recurrence from its start state, outputs included.
// A (batch, head) with L / 64 chunks then costs about 2 L / (64 n_seg) dependent steps instead of L / 64, for
// 2 (n_seg - 2) / n_seg more state products.
//
// One block = one (batch, head, segment), 8 wavefronts in two groups (a block with outputs: a state group and a
// staging group; a block of the two output-free runs: a state group for each, see PAIR below).
//   The four STATE wavefronts each own a quarter of the d_v rows and everything that is indexed by d_v: their
// slice of the state (S^T tiles in fp32 MFMA accumulators), of R, U and of the output.  The rows of S never mix,
// so the whole dependent chain  S0 -> K S0^T -> R -> U = T'' R -> S1  of a slice runs inside one wavefront, and
// every link stays in registers: a lane holds two 16-row accumulator tiles of a product as rows 4 lq .. 4 lq + 3
// of each, and the contraction slots of the next product's operand are defined as exactly those 8 rows (the
// operands that come from memory are laid out to match: K, Q rows by the block's other group, T'' and P by the
// inversion kernel).  No barrier and no LDS round trip stands inside the chain.
//   The four STAGING wavefronts prepare what all d_v slices share, one chunk ahead, in a double-buffered LDS
// set: the K and Q tiles (contiguous loads, converted to fp16 once, columns permuted into the slot order above),
// T'', P and the gates.  (K^T scaled by kd, the operand of the state update, is made by the state wavefronts
// from the K tile, a (contraction step, column half) share each: a product with a 0/1 selector hands a row-major
// fragment back in the accumulator layout, exactly.)  They also store the output rows (fp16; the
// softmax kernel, which runs afterwards, merges the two branches), which the state wavefronts leave in an LDS
// tile (computed transposed, S0 Q^T and U^T P^T, so that a lane holds four consecutive d_v of a token): whole
// rows of 2 d bytes go out.
//   Two block barriers per chunk: one before the output tile is overwritten, one when the next operand set is
// complete.
#include <algorithm>
#include <type_traits>

#include "mfma_util.h"
#include "nats_common.h"

namespace nats {

constexpr int SEG_THREADS = 512;
constexpr int SEG_GROUP = 256;   // threads of a group (state / staging)
constexpr int SC = 64;           // chunk size

template <int D>
struct SegLds {
    static constexpr int SS = D + LDS_PAD;     // halves per row of the K, Q tiles [64][SS] and of the output tile
    static constexpr int TS = SC + LDS_PAD;    // halves per row of Kd^T [d_k][TS]
    // one operand set (halves)
    static constexpr int o_Kt = 0;
    static constexpr int o_Qt = o_Kt + SC * SS;
    static constexpr int o_T = o_Qt + SC * SS;         // T'' in fragment order (the 6 fragments on and below the diagonal)
    static constexpr int o_P = o_T + TRI_FRAG_HALFS;   // P in fragment order, times la_scale
    static constexpr int o_G = o_P + TRI_FRAG_HALFS;   // fp32: gam[64], gam_C at [64], kd[64] from [68]
    static constexpr int G_KD = 68;
    static constexpr int SET = o_G + 2 * 132;          // 132 floats
    static constexpr int o_Kd = 2 * SET;               // Kd^T [d_k][TS]: written and read inside one step
    static constexpr int o_Out = o_Kd + D * TS;        // output tile [64][SS], fp16
    static constexpr int n_half = o_Out + SC * SS;
    static constexpr int bytes = n_half * 2;
    static_assert(bytes <= 160 * 1024, "one block per CU");
    static_assert(SET % 8 == 0, "sets stay 16-byte aligned");
};

// LDS of a block that runs the two output-free roles of a segment side by side (no Q, P, output tile): two operand
// sets, and Kd^T per group and chunk parity, so that one barrier per chunk is enough.
template <int D>
struct PairLds {
    static constexpr int SS = SegLds<D>::SS, TS = SegLds<D>::TS;
    static constexpr int o_Kt = 0;
    static constexpr int o_T = o_Kt + SC * SS;
    static constexpr int o_G = o_T + TRI_FRAG_HALFS;
    static constexpr int G_KD = 68;
    static constexpr int SET = o_G + 2 * 132;
    static constexpr int o_Kd = 2 * SET;               // Kd^T [group][chunk parity][d_k][TS]
    static constexpr int n_half = o_Kd + 4 * D * TS;
    static constexpr int o_Qt = 0, o_P = 0, o_Out = 0; // not present
    static_assert(n_half <= SegLds<D>::n_half, "inside the kernel's LDS");
    static_assert(SET % 8 == 0, "sets stay 16-byte aligned");
};

// Block roles (uniform per block)
enum SegRole { ROLE_OUT = 0, ROLE_ACC_S = 1, ROLE_ACC_E = 2 };

template <int D>
struct SegArgs {
    const bf16_t *Q, *K, *V;
    const half_t *TF, *PF;
    const float *gamv, *kdv, *gamC;
    const float* S0;          // [BH][D][D] initial state or nullptr
    float* S_final;           // [BH][D][D] or nullptr
    float* S_start;           // [BH][n_seg][D][D] start state of every segment (slot 0 unused)
    float* Nbuf;              // [BH][n_seg][D][D] end state of a middle segment run from zero
    float* MTbuf;             // [BH][n_seg][D][D] transposed transition of a middle segment: MT[j][i] = M[i][j]
    half_t* O_la_h;           // fp16 linear-branch output, for the merge in the softmax kernel
    float* O_la_f32;          // optional fp32 copy of the linear-branch output
    int L, BH, n_seg, seg_len, pass, gated;   // BH counts output heads
    int G;                    // output heads per linear head (head grouping): K, Q, T'', P and the gates are the
                              // linear head's (index bh / G), V, the state and the outputs the output head's
    float la_scale;
};

// 8 consecutive bf16 -> 8 fp16.  Truncating conversion: a bf16 value has 8 significant bits, so it is exact
// inside the fp16 range, and beyond the range it saturates instead of overflowing to infinity.
__device__ __forceinline__ half8 cvt_bf16x8(u32x4 u) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    half8 h;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const h2 p = __builtin_bit_cast(h2, __builtin_amdgcn_cvt_pkrtz(__uint_as_float(u[i] << 16),
                                                                       __uint_as_float(u[i] & 0xffff0000u)));
        h[2 * i] = p[0];
        h[2 * i + 1] = p[1];
    }
    return h;
}

// two accumulator tiles (rows 4 lq + j of each) -> the 8 contraction slots of one operand fragment
__device__ __forceinline__ half8 pack_tiles(f32x4 lo, f32x4 hi) {
    half8 h;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        h[j] = (half_t)lo[j];
        h[4 + j] = (half_t)hi[j];
    }
    return h;
}

// ------------------------------------------------------------------------------------------------------------
// STATE wavefronts.  ROLE and F32OUT are compile-time: the chunk loop is straight-line code.
// Index conventions of a lane (l16 = lane % 16, lq = lane / 16):
//   accumulator tile      : rows 4 lq + j (j < 4), column l16
//   operand fragment      : row / column l16, contraction slots s < 8 of step ks:
//                           index 32 ks + 16 (s / 4) + 4 lq + s % 4   (d_k, or token)
// ------------------------------------------------------------------------------------------------------------
// PAIR: the block runs the two output-free roles of a segment side by side, wavefronts 0-3 one, 4-7 the other, and
// has no staging group: the 512 threads bring in the operand set themselves (K tile, T'', gates: 2-3 loads of 16
// bytes per thread and chunk, asked for two chunks ahead at the top of a step and written into the set of the
// next chunk at the top of the following step).  Kd^T (one for both groups at d = 128, each group's own at
// d = 64) has a buffer per chunk parity:
// with the sets and Kd^T both double-buffered the barrier in the middle of a step is the only one (what a
// wavefront writes before it in step c + 1 was last read before that barrier in step c, or in step c - 1).
template <int D, int ROLE, bool F32OUT>
__device__ __forceinline__ void seg_state_waves(const SegArgs<D>& a, const int bh, const int seg, half_t* lds) {
    constexpr bool PAIR = ROLE != ROLE_OUT;   // the output-free roles always run as a pair
    using Lds = typename std::conditional<PAIR, PairLds<D>, SegLds<D>>::type;
    constexpr int SS = Lds::SS, TS = Lds::TS;
    constexpr int KS_D = D / 32;      // contraction steps over d_k
    constexpr int NDT = D / 16;       // 16-row d_k tiles of S^T
    constexpr int NVT = D / 64;       // 16-wide d_v tiles of one wavefront (a quarter of d_v)
    constexpr bool HAS_OUT = ROLE == ROLE_OUT, HAS_V = ROLE != ROLE_ACC_E;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);   // 0..3 inside the group
    const int l16 = lane & 15, lq = lane >> 4;
    const int vbase = wave * (D / 4);
    const int n_chunks = a.L / SC;
    const int c_begin = seg * a.seg_len, c_end = min(c_begin + a.seg_len, n_chunks);
    const size_t seg_slot = (size_t)bh * a.n_seg + seg;
    const float* init = nullptr;           // state the segment starts from (nullptr: zero, or the unit rows)
    float* dest = nullptr;                 // where its end state goes
    if (ROLE == ROLE_OUT) {
        init = seg == 0 ? (a.S0 ? a.S0 + (size_t)bh * D * D : nullptr) : a.S_start + seg_slot * D * D;
        if (seg == a.n_seg - 1) dest = a.S_final ? a.S_final + (size_t)bh * D * D : nullptr;
        else if (seg == 0) dest = a.S_start + (seg_slot + 1) * D * D;   // the later start states come from the fix-up
    } else if (ROLE == ROLE_ACC_S) {
        dest = a.Nbuf + seg_slot * D * D;
    } else {
        dest = a.MTbuf + seg_slot * D * D;
    }

    // ---- state: S^T tiles (rows d_k, cols v) as fp32 accumulators, and its fp16 operand form ----
    f32x4 accS[NDT][NVT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) {
            const int dk = 16 * dt + 4 * lq, v = vbase + 16 * vt + l16;
            if (ROLE == ROLE_ACC_E) {   // unit rows: "v" counts the rows e of the identity
                accS[dt][vt] = f32x4{v == dk ? 1.f : 0.f, v == dk + 1 ? 1.f : 0.f, v == dk + 2 ? 1.f : 0.f,
                                     v == dk + 3 ? 1.f : 0.f};
            } else if (init != nullptr) {
                const float4 x = *reinterpret_cast<const float4*>(init + (size_t)v * D + dk);
                accS[dt][vt] = f32x4{x.x, x.y, x.z, x.w};
            } else {
                accS[dt][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        }
    half8 sfrag[NVT][KS_D];   // S[v = l16][d_k slots]: B operand of K S0^T, A operand of S0 Q^T
#pragma unroll
    for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) sfrag[vt][ks] = pack_tiles(accS[2 * ks][vt], accS[2 * ks + 1][vt]);

    // 0/1 selector fragments: B operand whose column n picks slot n (lo) or 16 + n (hi) of a row-major fragment
    // (there the slots of a lane are the 8 consecutive indices 8 lq + j)
    half8 isel[2];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int j = 0; j < 8; ++j) isel[hf][j] = (8 * lq + j == 16 * hf + l16) ? (half_t)1.f : (half_t)0.f;

    // V rows of the four token tiles, the 32 columns that hold this wavefront's slice: row-major fragments
    // straight from global memory, one chunk ahead
    const int vb32 = vbase & ~31, vhf = (vbase & 31) >> 4;   // d = 64: two wavefronts share a 32-column group
    u32x4 vraw[4];
    const size_t tokb = (size_t)bh * a.L;
    const uint32_t v_off = (uint32_t)(l16 * D + vb32 + 8 * lq);
    auto load_v = [&](int c) __attribute__((always_inline)) {
        if (!HAS_V) return;
        const bf16_t* Vc = a.V + (tokb + (size_t)c * SC) * D;
#pragma unroll
        for (int tt = 0; tt < 4; ++tt) vraw[tt] = *reinterpret_cast<const u32x4*>(Vc + v_off + (uint32_t)(16 * tt * D));
    };
    const float gated_off = a.gated ? 0.f : 1.f;   // without the delta rule the state does not enter R
    half_t* OutT = lds + Lds::o_Out;
    // Kd^T[d_k][token slots] = kd_tok K[tok][d_k] is made here too, from the K tile: a product with a 0/1 selector
    // hands 16 d_k columns of a token tile's K fragment back as an accumulator tile (rows tok 4 lq + j, col d_k),
    // exactly; those are 4 consecutive slots of a Kd^T row.  The (contraction step, column half) pairs are dealt
    // to the four wavefronts: d = 128: step = wavefront, both halves; d = 64: step = wavefront % 2, half = wavefront / 2.
    // In a paired block at d = 128 the two groups make one Kd^T together: step = wavefront, half = group.
    constexpr bool SHARE_KD = PAIR && KS_D == 4;
    constexpr int NTR = SHARE_KD ? 1 : KS_D / 2;    // pairs per wavefront and token tile
    const int tr_ks = KS_D == 4 ? wave : (wave & 1);
    half8 iselp[NTR];                               // selector for a fragment in slot order: column n <- d_k 16 hf + n
    int tr_hf[NTR];
#pragma unroll
    for (int i = 0; i < NTR; ++i) {
        tr_hf[i] = SHARE_KD ? (tid >> 8) : KS_D == 4 ? i : (wave >> 1);
#pragma unroll
        for (int s8 = 0; s8 < 8; ++s8)
            iselp[i][s8] = (lq == (l16 >> 2) && s8 == 4 * tr_hf[i] + (l16 & 3)) ? (half_t)1.f : (half_t)0.f;
    }

    // ---- PAIR: this thread's share of the operand set ----
    constexpr int NPC8 = SC * D / 8 / SEG_THREADS;   // 16-byte pieces of the K tile per thread
    constexpr int NTP8 = TRI_FRAG_HALFS / 8;         // pieces of T'': threads below this number take one
    static_assert(!PAIR || (NPC8 >= 1 && NTP8 <= SEG_THREADS), "shares of the operand set");
    u32x4 skp[NPC8 > 0 ? NPC8 : 1];
    half8 stp;
    float sg0 = 0.f, sg1 = 0.f;
    const size_t tokl = (size_t)(bh / a.G) * a.L, chb = (size_t)(bh / a.G) * n_chunks;   // the linear head's rows, chunks
    auto stage_load = [&](int c) __attribute__((always_inline)) {
        if (!PAIR) return;
        const u32x4* Kp = reinterpret_cast<const u32x4*>(a.K + (tokl + (size_t)c * SC) * D);
#pragma unroll
        for (int i = 0; i < NPC8; ++i) skp[i] = Kp[tid + SEG_THREADS * i];
        if (tid < NTP8) stp = reinterpret_cast<const half8*>(a.TF + (chb + c) * (size_t)TRI_FRAG_HALFS)[tid];   // wavefronts 0-5
        if (tid <= SC) sg0 = tid < SC ? a.gamv[(chb + c) * SC + tid] : a.gamC[chb + c];
        if (tid < SC) sg1 = a.kdv[(chb + c) * SC + tid];
    };
    auto stage_write = [&](half_t* set) __attribute__((always_inline)) {
        if (!PAIR) return;
#pragma unroll
        for (int i = 0; i < NPC8; ++i) {   // the K tile in slot order (see the staging group)
            const int e = tid + SEG_THREADS * i, row = e / (D / 8), c8 = e % (D / 8);
            const int pos = 32 * (c8 >> 2) + 16 * (c8 & 1) + 4 * ((c8 >> 1) & 1);
            const half8 hk = cvt_bf16x8(skp[i]);
            *reinterpret_cast<half4*>(set + Lds::o_Kt + row * SS + pos) = half4{hk[0], hk[1], hk[2], hk[3]};
            *reinterpret_cast<half4*>(set + Lds::o_Kt + row * SS + pos + 8) = half4{hk[4], hk[5], hk[6], hk[7]};
        }
        if (tid < NTP8) reinterpret_cast<half8*>(set + Lds::o_T)[tid] = stp;
        float* G = reinterpret_cast<float*>(set + Lds::o_G);
        if (tid <= SC) G[tid] = sg0;
        if (tid < SC) G[Lds::G_KD + tid] = sg1;
    };
    if (PAIR) {
        stage_load(c_begin);
        stage_write(lds);
        stage_load(min(c_begin + 1, c_end - 1));
    }

    load_v(c_begin);
    __syncthreads();   // the first operand set is complete

    for (int c = c_begin; c < c_end; ++c) {
        const int cn = min(c + 1, c_end - 1);   // the tail re-loads the last chunk: loads stay unconditional
        const half_t* set = lds + ((c - c_begin) & 1) * Lds::SET;
        if (PAIR) {
            // chunk c + 1 (asked for a step ago) into the set that the previous step has finished with, then the
            // request for chunk c + 2
            stage_write(lds + (((c - c_begin) & 1) ^ 1) * Lds::SET);
            stage_load(min(c + 2, c_end - 1));
        }
        half_t* Kd = lds + Lds::o_Kd + (PAIR ? ((SHARE_KD ? 0 : 2 * (tid >> 8)) + ((c - c_begin) & 1)) * (D * TS) : 0);
        const half_t* Kt = set + Lds::o_Kt;
        const half_t* Qt = set + Lds::o_Qt;
        const half8* Tt = reinterpret_cast<const half8*>(set + Lds::o_T);
        const half8* Pt = reinterpret_cast<const half8*>(set + Lds::o_P);
        const float* Gt = reinterpret_cast<const float*>(set + Lds::o_G);

        half8 vf[4];
        if (HAS_V) {
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) vf[tt] = cvt_bf16x8(vraw[tt]);
        }
        load_v(cn);

        // ---- K S0^T -> R, and S0 Q^T, two token tiles (one contraction step of the next product) at a time ----
        f32x4 accO[NVT][4];
        half8 rfrag[2][NVT];      // R[token slots][v = l16]: B operand of T'' R
        // Without outputs there are registers to spare: the K fragments of the next token tile are read while the
        // current tile's products run (the write of Kd^T below keeps the compiler from moving those reads up by
        // itself: it cannot tell the two LDS regions apart).
        half8 kf_next[KS_D], kt_next;
        if (!HAS_OUT) {
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks) kf_next[ks] = lds_read8(Kt + l16 * SS + 32 * ks + 8 * lq);
            kt_next = lds_read8(Kt + l16 * SS + 32 * tr_ks + 8 * lq);
        }
#pragma unroll
        for (int kp = 0; kp < 2; ++kp) {
            f32x4 accR[2][NVT];
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
                const int tt = 2 * kp + t2;
                half8 kf[KS_D], qf[KS_D];
                half8 kt;
                if (!HAS_OUT) {
#pragma unroll
                    for (int ks = 0; ks < KS_D; ++ks) kf[ks] = kf_next[ks];
                    kt = kt_next;
                    if (tt < 3) {
#pragma unroll
                        for (int ks = 0; ks < KS_D; ++ks)
                            kf_next[ks] = lds_read8(Kt + (16 * (tt + 1) + l16) * SS + 32 * ks + 8 * lq);
                        kt_next = lds_read8(Kt + (16 * (tt + 1) + l16) * SS + 32 * tr_ks + 8 * lq);
                    }
                } else {
#pragma unroll
                    for (int ks = 0; ks < KS_D; ++ks) kf[ks] = lds_read8(Kt + (16 * tt + l16) * SS + 32 * ks + 8 * lq);
                    kt = lds_read8(Kt + (16 * tt + l16) * SS + 32 * tr_ks + 8 * lq);
                }
                if (HAS_OUT) {
#pragma unroll
                    for (int ks = 0; ks < KS_D; ++ks) qf[ks] = lds_read8(Qt + (16 * tt + l16) * SS + 32 * ks + 8 * lq);
                }
#pragma unroll
                for (int vt = 0; vt < NVT; ++vt) {
                    accR[t2][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
                    if (HAS_OUT) accO[vt][tt] = f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
                for (int ks = 0; ks < KS_D; ++ks)
#pragma unroll
                    for (int vt = 0; vt < NVT; ++vt) {
                        accR[t2][vt] = mfma16(kf[ks], sfrag[vt][ks], accR[t2][vt]);                 // rows tok, col v
                        if (HAS_OUT) accO[vt][tt] = mfma16(sfrag[vt][ks], qf[ks], accO[vt][tt]);   // rows v, col tok
                    }
                {   // this wavefront's share of Kd^T for token tile tt
                    const float4 k4 = *reinterpret_cast<const float4*>(Gt + Lds::G_KD + 16 * tt + 4 * lq);
                    const float kk[4] = {k4.x, k4.y, k4.z, k4.w};
#pragma unroll
                    for (int i = 0; i < NTR; ++i) {
                        f32x4 t = mfma16(kt, iselp[i], f32x4{0.f, 0.f, 0.f, 0.f});   // col d_k = 32 tr_ks + 16 hf + l16
#pragma unroll
                        for (int j = 0; j < 4; ++j) t[j] *= kk[j];
                        *reinterpret_cast<half4*>(Kd + (32 * tr_ks + 16 * tr_hf[i] + l16) * TS + 32 * kp + 8 * lq + 4 * t2) =
                            to_half4_hw(t);
                    }
                }
                // R = V - gam (K S0^T): the gate per row, then V added by the selector product (exactly)
                const float4 g4 = *reinterpret_cast<const float4*>(Gt + 16 * tt + 4 * lq);
                const float gg[4] = {g4.x * gated_off, g4.y * gated_off, g4.z * gated_off, g4.w * gated_off};
#pragma unroll
                for (int vt = 0; vt < NVT; ++vt) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) accR[t2][vt][j] *= -gg[j];
                    if (HAS_V) accR[t2][vt] = mfma16(vf[tt], isel[vhf + vt], accR[t2][vt]);
                }
            }
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt) rfrag[kp][vt] = pack_tiles(accR[0][vt], accR[1][vt]);
        }

        // ---- U = T'' R (T'' lower triangular: token tiles 0, 1 need the first contraction step only) ----
        half8 ufrag[2][NVT];      // U[token slots][v = l16]: B operand of Kd^T U, A operand of U^T P^T
#pragma unroll
        for (int kp = 0; kp < 2; ++kp) {
            f32x4 accU[2][NVT];
#pragma unroll
            for (int t2 = 0; t2 < 2; ++t2) {
                const int tt = 2 * kp + t2;
#pragma unroll
                for (int vt = 0; vt < NVT; ++vt) accU[t2][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks <= kp; ++ks) {
                    const half8 tf = Tt[tri_frag(tt, ks) * 64 + lane];
#pragma unroll
                    for (int vt = 0; vt < NVT; ++vt) accU[t2][vt] = mfma16(tf, rfrag[ks][vt], accU[t2][vt]);   // rows r, col v
                }
            }
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt) ufrag[kp][vt] = pack_tiles(accU[0][vt], accU[1][vt]);
        }

        // ---- output rows: gam (S0 Q^T) + U^T P^T, into the LDS tile (la_scale rides on the gate and on P) ----
        if (HAS_OUT) {
#pragma unroll
            for (int tt = 0; tt < 4; ++tt) {
                const float go = Gt[16 * tt + l16] * a.la_scale;
#pragma unroll
                for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
                    for (int j = 0; j < 4; ++j) accO[vt][tt][j] *= go;
#pragma unroll
                for (int ks = 0; ks <= tt / 2; ++ks) {
                    const half8 pf = Pt[tri_frag(tt, ks) * 64 + lane];
#pragma unroll
                    for (int vt = 0; vt < NVT; ++vt) accO[vt][tt] = mfma16(ufrag[ks][vt], pf, accO[vt][tt]);   // rows v, col r
                }
            }
        }
        const float gC = Gt[64];   // (read before the barrier: in a paired block the set may be rewritten after it)
        __syncthreads();   // the staging group has taken the previous chunk's rows out of the output tile; Kd^T complete
        if (HAS_OUT) {
#pragma unroll
            for (int tt = 0; tt < 4; ++tt)
#pragma unroll
                for (int vt = 0; vt < NVT; ++vt) {
                    // this lane: token 16 tt + l16, d_v vbase + 16 vt + 4 lq + j
                    *reinterpret_cast<half4*>(OutT + (16 * tt + l16) * SS + vbase + 16 * vt + 4 * lq) = to_half4_hw(accO[vt][tt]);
                    if (F32OUT)
                        *reinterpret_cast<float4*>(a.O_la_f32 + (tokb + (size_t)c * SC + 16 * tt + l16) * D + vbase + 16 * vt + 4 * lq) =
                            make_float4(accO[vt][tt][0], accO[vt][tt][1], accO[vt][tt][2], accO[vt][tt][3]);
                }
        }

        // ---- S1^T = gam_C S0^T + Kd^T U, and its operand form for the next chunk ----
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) {
            half8 af[2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) af[ks] = lds_read8(Kd + (16 * dt + l16) * TS + 32 * ks + 8 * lq);
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt) {
#pragma unroll
                for (int j = 0; j < 4; ++j) accS[dt][vt][j] *= gC;
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) accS[dt][vt] = mfma16(af[ks], ufrag[ks][vt], accS[dt][vt]);   // rows d_k, col v
            }
        }
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks) sfrag[vt][ks] = pack_tiles(accS[2 * ks][vt], accS[2 * ks + 1][vt]);
        if (!PAIR) __syncthreads();   // the next operand set and this chunk's output tile are complete
    }

    // ---- end state ----
    if (dest != nullptr) {
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt) {
                const int dk = 16 * dt + 4 * lq, v = vbase + 16 * vt + l16;
                if (ROLE == ROLE_ACC_E) {
                    // M[i = unit row][j = d_k] as the fp16 pair the fix-up multiplies with (a plane of leading
                    // halves, then a plane of remainders), each plane in the order its wavefronts load it:
                    // [j / 16][i / 32][lane = 16 ((i % 32) / 8) + j % 16][i % 8]
                    half_t* mh = reinterpret_cast<half_t*>(dest);
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const float x = accS[dt][vt][j];
                        const half_t hi = f32_to_half_sat(x);
                        const int jj = dk + j;
                        const size_t o = ((size_t)((jj >> 4) * KS_D + (v >> 5)) * 64 + 16 * ((v & 31) >> 3) + (jj & 15)) * 8 +
                                         (v & 7);
                        mh[o] = hi;
                        mh[(size_t)D * D + o] = (half_t)(x - (float)hi);
                    }
                } else {
                    *reinterpret_cast<float4*>(dest + (size_t)v * D + dk) =
                        make_float4(accS[dt][vt][0], accS[dt][vt][1], accS[dt][vt][2], accS[dt][vt][3]);
                }
            }
    }
}

// ------------------------------------------------------------------------------------------------------------
// STAGING wavefronts (blocks with outputs only): the operand set of the next chunk, and the previous chunk's
// output rows.
// ------------------------------------------------------------------------------------------------------------
// what a staging thread carries from memory to the next operand set
template <int D>
struct StageRegs {
    static constexpr int NPC = SC * D / 8 / SEG_GROUP;     // 16-byte pieces of a [64][D] tile per thread
    static constexpr int NTP = (TRI_FRAG_HALFS / 8 + SEG_GROUP - 1) / SEG_GROUP;   // ... of a chunk's T'' or P
    // (6 fragments of 64 pieces: the second piece exists for the first half of the group only)
    static __device__ __forceinline__ bool has_tp(int i, int pt) { return pt + SEG_GROUP * i < TRI_FRAG_HALFS / 8; }
    u32x4 kp[NPC], qp[NPC];        // pieces of the K and Q tiles (contiguous)
    half8 tp[NTP], pp[NTP];        // pieces of T'' and P (already in fragment order)
    float g0, g1;                  // thread t < 64: gam and kd of token t; thread 64: gam_C
    static constexpr int N_LOADS = 2 * NPC + 2 * NTP + 2;
    // load number i of chunk c (one at a time, so that a step can spread them between its other work: issued
    // in a burst they queue in the CU's vector-memory path and the wavefront stalls until all are accepted)
    __device__ __forceinline__ void load_piece(int i, const SegArgs<D>& a, size_t cb, size_t ch, int pt) {
        if (i < NPC) { kp[i] = reinterpret_cast<const u32x4*>(a.K + cb)[pt + SEG_GROUP * i]; return; }
        i -= NPC;
        if (i < NPC) { qp[i] = reinterpret_cast<const u32x4*>(a.Q + cb)[pt + SEG_GROUP * i]; return; }
        i -= NPC;
        if (i < NTP) {
            if (has_tp(i, pt)) tp[i] = reinterpret_cast<const half8*>(a.TF + ch * (size_t)TRI_FRAG_HALFS)[pt + SEG_GROUP * i];
            return;
        }
        i -= NTP;
        if (i < NTP) {
            if (has_tp(i, pt)) pp[i] = reinterpret_cast<const half8*>(a.PF + ch * (size_t)TRI_FRAG_HALFS)[pt + SEG_GROUP * i];
            return;
        }
        i -= NTP;
        if (i == 0) g0 = pt < SC ? a.gamv[ch * SC + pt] : a.gamC[ch];
        else g1 = a.kdv[ch * SC + (pt & (SC - 1))];
    }
};

// ------------------------------------------------------------------------------------------------------------
// STAGING wavefronts: the operand set of the next chunk, and the current chunk's output rows (fp16).
// ------------------------------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ void seg_staging_waves(const SegArgs<D>& a, const int bh, const int seg, half_t* lds) {
    using Lds = SegLds<D>;
    constexpr int SS = Lds::SS;
    using Regs = StageRegs<D>;
    constexpr int NPC = Regs::NPC, NTP = Regs::NTP;
    const int pt = threadIdx.x - SEG_GROUP;
    const int n_chunks = a.L / SC;
    const int c_begin = seg * a.seg_len, c_end = min(c_begin + a.seg_len, n_chunks);
    const size_t tokb = (size_t)bh * a.L;                  // output rows (and the softmax branch's)
    const size_t tokl = (size_t)(bh / a.G) * a.L;          // K, Q rows: the linear head's
    const size_t chb = (size_t)(bh / a.G) * n_chunks;      // its per-chunk operands
    const half_t lah = (half_t)a.la_scale;
    const half8 la8 = {lah, lah, lah, lah, lah, lah, lah, lah};
    half_t* OutT = lds + Lds::o_Out;

    // The operand set is written in N_WRITE pieces and the loads of the following chunk go out between them:
    // issued in one burst, the loads queue in the CU's vector-memory path (a KiB takes it 16 cycles) and the
    // wavefront stands still until all are accepted, although nothing it does next depends on them.
    constexpr int N_WRITE = NPC + 1;
    auto write_piece = [&](int i, const Regs& r, half_t* set) __attribute__((always_inline)) {
        if (i < NPC) {
            // K, Q tiles: fp16, the 32 columns of a contraction step permuted into slot order: column 8 q + j of
            // the step goes to position 16 (q % 2) + 8 (j / 4) + 4 (q / 2) + j % 4, i.e. a piece is stored as two halves
            const int e = pt + SEG_GROUP * i, row = e / (D / 8), c8 = e % (D / 8);
            const int pos = 32 * (c8 >> 2) + 16 * (c8 & 1) + 4 * ((c8 >> 1) & 1);
            const half8 hk = cvt_bf16x8(r.kp[i]);
            *reinterpret_cast<half4*>(set + Lds::o_Kt + row * SS + pos) = half4{hk[0], hk[1], hk[2], hk[3]};
            *reinterpret_cast<half4*>(set + Lds::o_Kt + row * SS + pos + 8) = half4{hk[4], hk[5], hk[6], hk[7]};
            const half8 hq = cvt_bf16x8(r.qp[i]);
            *reinterpret_cast<half4*>(set + Lds::o_Qt + row * SS + pos) = half4{hq[0], hq[1], hq[2], hq[3]};
            *reinterpret_cast<half4*>(set + Lds::o_Qt + row * SS + pos + 8) = half4{hq[4], hq[5], hq[6], hq[7]};
            return;
        }
#pragma unroll
        for (int k = 0; k < NTP; ++k) {
            if (!Regs::has_tp(k, pt)) continue;   // uniform per wavefront
            reinterpret_cast<half8*>(set + Lds::o_T)[pt + SEG_GROUP * k] = r.tp[k];
            reinterpret_cast<half8*>(set + Lds::o_P)[pt + SEG_GROUP * k] = r.pp[k] * la8;
        }
        float* G = reinterpret_cast<float*>(set + Lds::o_G);
        if (pt <= SC) G[pt] = r.g0;
        if (pt < SC) G[Lds::G_KD + pt] = r.g1;
    };
    auto write_set = [&](const Regs& r, half_t* set) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < N_WRITE; ++i) write_piece(i, r, set);
    };
    // rows of chunk c out of the output tile, as fp16 for the softmax kernel's merge epilogue: 16 bytes per lane,
    // whole rows contiguous
    auto store_rows = [&](int c) __attribute__((always_inline)) {
        const size_t ob = (tokb + (size_t)c * SC) * D;
#pragma unroll
        for (int i = 0; i < NPC; ++i) {
            const int e = pt + SEG_GROUP * i, row = e / (D / 8), c8 = e % (D / 8);
            reinterpret_cast<half8*>(a.O_la_h + ob)[e] = lds_read8(OutT + row * SS + 8 * c8);
        }
    };
    auto load_all = [&](Regs& r, int c) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < Regs::N_LOADS; ++i) r.load_piece(i, a, (tokl + (size_t)c * SC) * D, chb + c, pt);
    };

    // One step: the registers `cur` hold chunk c + 1; it goes into the LDS set the state group reads next, while
    // chunk c + 2 is asked for into `nxt`.
    auto step = [&](int c, const Regs& cur, Regs& nxt) __attribute__((always_inline)) {
        half_t* set = lds + (((c - c_begin) & 1) ^ 1) * Lds::SET;
        const int c2 = min(c + 2, c_end - 1);
        constexpr int PER = (Regs::N_LOADS + N_WRITE - 1) / N_WRITE;   // loads per written piece
        int li = 0;
#pragma unroll
        for (int i = 0; i < N_WRITE; ++i) {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < PER; ++k, ++li)
                if (li < Regs::N_LOADS) nxt.load_piece(li, a, (tokl + (size_t)c2 * SC) * D, chb + c2, pt);
            __builtin_amdgcn_sched_barrier(0);
            write_piece(i, cur, set);
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();   // (the state group overwrites the output tile after this)
        __syncthreads();   // the output tile of chunk c is complete
        store_rows(c);
    };

    Regs ra, rb;
    load_all(ra, c_begin);
    load_all(rb, min(c_begin + 1, c_end - 1));
    write_set(ra, lds);
    __syncthreads();   // the first operand set is complete
    // two steps per trip: the two register sets swap roles without a copy
    int c = c_begin;
    for (; c + 2 <= c_end; c += 2) {
        step(c, rb, ra);
        step(c + 1, ra, rb);
    }
    if (c < c_end) step(c, rb, ra);
}

template <int D, bool F32OUT>
__global__ __launch_bounds__(SEG_THREADS) void gdn_seg_scan_kernel(const SegArgs<D> a) {
    extern __shared__ __align__(16) unsigned char seg_smem[];
    half_t* lds = reinterpret_cast<half_t*>(seg_smem);
    fp16_saturate_on();   // conversions to fp16 clamp to the fp16 range (see to_half4_hw)
    // ---- block -> (batch*head, role, segment).  Blocks with ids congruent modulo 8 share an XCD and its L2:
    //      the blocks of one (batch, head) are given such ids (the two blocks of a middle segment read the
    //      same K and T'').
    const int n_mid = a.n_seg > 2 ? a.n_seg - 2 : 0;
    const int per_bh = a.pass == 1 ? 1 + n_mid : a.n_seg - 1;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    // (with head grouping the G output heads of a linear head, which read the same K, Q, T'', P, share it too)
    const int hq = slot / per_bh, grp = (hq / a.G) * 8 + xcd;
    if (grp >= a.BH / a.G) return;
    const int bh = grp * a.G + hq % a.G;
    const int sub = slot % per_bh;
    const bool staging = threadIdx.x >= SEG_GROUP;   // uniform per wavefront
    // pass 2: every later segment with outputs; pass 1: segment 0 with outputs, then one block per middle segment
    // that runs it from the zero state (wavefronts 0-3) and on the unit rows (wavefronts 4-7)
    const bool with_out = a.pass == 2 || sub == 0;
    const int seg = a.pass == 2 ? 1 + sub : sub;
    if (with_out) {
        if (staging) seg_staging_waves<D>(a, bh, seg, lds);
        else seg_state_waves<D, ROLE_OUT, F32OUT>(a, bh, seg, lds);
    } else {
        if (staging) seg_state_waves<D, ROLE_ACC_E, false>(a, bh, seg, lds);
        else seg_state_waves<D, ROLE_ACC_S, false>(a, bh, seg, lds);
    }
}

// ---- fix-up between the passes: S_start[s + 1] = S_start[s] M_s + N_s, s = 1 .. n_seg - 2 --------------------
// One block = 16 state rows of one (batch, head), 4 wavefronts, each owning d / 64 column tiles of 16.  The
// product runs on fp16 MFMA with both operands split into two fp16 terms (hi + lo, three products): the error
// is about 2^-21 relative, so the carried state keeps fp32-level accuracy.
constexpr int FIX_THREADS = 512;   // four multiplying wavefronts and four that only pull the operands into L2

template <int D>
__global__ __launch_bounds__(FIX_THREADS) void gdn_seg_fix_kernel(float* __restrict__ S_start,
                                                                 const float* __restrict__ Nbuf,
                                                                 const float* __restrict__ MTbuf, int BH, int n_seg) {
    constexpr int KS_D = D / 32, NT = D / 64;   // contraction steps; column tiles per wavefront
    constexpr int RS = D + 8;                   // fp16 row stride of the carried rows in LDS
    // the 16 carried rows as an fp16 pair (leading half, remainder): the A operand of the next step as it is
    __shared__ __align__(16) half_t Shi[16 * RS], Slo[16 * RS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    // The D/16 blocks of one (batch, head) read the same M and N: consecutive block indices go to different
    // XCDs, so the blocks are renumbered to put them behind one L2 (grid = 8 x ceil(blocks / 8)).
    const int vid = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    const int bh = vid / (D / 16), v0 = (vid % (D / 16)) * 16;
    if (bh >= BH) return;
    const size_t base = (size_t)bh * n_seg;
    const int last = n_seg - 2;   // steps s = 1 .. last
    if (last < 1) return;
    if (wave >= 4) {
        // The operands of every step were written by blocks behind other L2s, so a first read comes from memory
        // and a step that waits for it costs a full memory latency.  These wavefronts read, once and all at the
        // start, the block's share of every later step's M (a (D/16)-th: the blocks of this (batch, head) sit
        // behind the same L2) and its own rows of N, so that the multiplying wavefronts find them in L2.
        constexpr int SHARE = D * D * 4 / (D / 16);   // bytes of M (and of N) per block and step
        constexpr int PIECES = SHARE / 16 / 256;      // 16-byte pieces per thread
        const int t = tid - 256, part = vid % (D / 16);
        unsigned seen = 0;
        for (int sg = 2; sg <= last; ++sg) {
            const uint4* m = reinterpret_cast<const uint4*>(MTbuf + (base + sg) * D * D) + (size_t)part * (SHARE / 16);
            const uint4* n = reinterpret_cast<const uint4*>(Nbuf + (base + sg) * D * D) + (size_t)part * (SHARE / 16);
#pragma unroll
            for (int i = 0; i < PIECES; ++i) {
                const uint4 a = m[t + 256 * i], b = n[t + 256 * i];
                seen |= a.x | b.x;
            }
        }
        if (seen == 0xffffffffu && n_seg < 0) S_start[0] = 0.f;   // never true: keeps the reads alive
        for (int sg = 1; sg <= last; ++sg) {
            __syncthreads();
            __syncthreads();
        }
        __syncthreads();
        return;
    }
    // What a step takes from memory (its M and N) does not depend on the carried rows: it is fetched one step
    // ahead, so that the dependent chain along the segments holds no memory latency.  Two register sets take
    // turns (two steps per loop trip): with one set the compiler would copy the fresh values into the registers
    // the loop carries, and wait for them, inside the same step.
    struct Fetch {
        half8 mh[NT][KS_D], ml[NT][KS_D];   // A operand: row j0 + l16 of M^T, slots i = 32 ks + 8 lq + s
        float4 n[NT];                       // N[v0 + l16][j0 + 4 lq ..]
    };
    auto load_step = [&](Fetch& f, int sg) __attribute__((always_inline)) {
        const half_t* MT = reinterpret_cast<const half_t*>(MTbuf + (base + sg) * D * D);
        const float* Nn = Nbuf + (base + sg) * D * D;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int jt = wave * NT + nt;
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks) {
                const half_t* mp = MT + ((size_t)(jt * KS_D + ks) * 64 + lane) * 8;
                f.mh[nt][ks] = *reinterpret_cast<const half8*>(mp);
                f.ml[nt][ks] = *reinterpret_cast<const half8*>(mp + D * D);
            }
            f.n[nt] = *reinterpret_cast<const float4*>(Nn + (size_t)(v0 + l16) * D + 16 * jt + 4 * lq);
        }
    };
    auto step = [&](int sg, const Fetch& cur, Fetch& nxt) __attribute__((always_inline)) {
        load_step(nxt, min(sg + 1, last));
        __builtin_amdgcn_sched_barrier(0);   // the fetch leads the step
        // B operand: the carried rows, col v0 + l16, slots i = 32 ks + 8 lq + s
        half8 bhi[KS_D], blo[KS_D];
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) {
            bhi[ks] = *reinterpret_cast<const half8*>(Shi + l16 * RS + 32 * ks + 8 * lq);
            blo[ks] = *reinterpret_cast<const half8*>(Slo + l16 * RS + 32 * ks + 8 * lq);
        }
        f32x4 acc[NT];   // transposed product: rows j0 + 4 lq + jj, col v0 + l16
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks) {
                acc[nt] = mfma16(cur.mh[nt][ks], blo[ks], acc[nt]);
                acc[nt] = mfma16(cur.ml[nt][ks], bhi[ks], acc[nt]);
                acc[nt] = mfma16(cur.mh[nt][ks], bhi[ks], acc[nt]);
            }
        }
        __syncthreads();   // every wavefront has read the old rows
        float* out = S_start + (base + sg + 1) * D * D;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int j = 16 * (wave * NT + nt) + 4 * lq;
            const float y[4] = {acc[nt][0] + cur.n[nt].x, acc[nt][1] + cur.n[nt].y, acc[nt][2] + cur.n[nt].z,
                                acc[nt][3] + cur.n[nt].w};
            half4 hi, lo;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
                hi[jj] = f32_to_half_sat(y[jj]);
                lo[jj] = (half_t)(y[jj] - (float)hi[jj]);
            }
            *reinterpret_cast<half4*>(Shi + l16 * RS + j) = hi;
            *reinterpret_cast<half4*>(Slo + l16 * RS + j) = lo;
            *reinterpret_cast<float4*>(out + (size_t)(v0 + l16) * D + j) = make_float4(y[0], y[1], y[2], y[3]);
        }
        __syncthreads();
    };
    Fetch fa, fb;
    load_step(fa, 1);
    for (int e = tid; e < 16 * D / 4; e += 256) {
        const int r = e / (D / 4), c4 = (e % (D / 4)) * 4;
        const float4 x4 = *reinterpret_cast<const float4*>(S_start + ((base + 1) * D + v0 + r) * D + c4);
        const float x[4] = {x4.x, x4.y, x4.z, x4.w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const half_t hi = f32_to_half_sat(x[j]);
            Shi[r * RS + c4 + j] = hi;
            Slo[r * RS + c4 + j] = (half_t)(x[j] - (float)hi);
        }
    }
    __syncthreads();
    int sg = 1;
    for (; sg + 1 <= last; sg += 2) {
        step(sg, fa, fb);
        step(sg + 1, fb, fa);
    }
    if (sg <= last) step(sg, fa, fb);
}

// number of segments a (batch, head) is cut into: enough blocks to fill the chip, at least 4 chunks each
int gdn_segments(const FwdPlan& pl) {
    const int n_chunks = pl.L / SC;
    int n = pl.gdn_segments > 0 ? pl.gdn_segments : std::max(1, 256 / pl.BHG);
    n = std::min(n, std::max(1, n_chunks / 4));
    return std::max(1, std::min(n, 64));
}

template <int D, bool F32OUT>
static nats_status launch_seg_k(const FwdPlan& pl, SegArgs<D> a, hipStream_t st) {
    static bool attr_done[64] = {};
    int dev = 0;
    (void)hipGetDevice(&dev);
    dev = (dev >= 0 && dev < 64) ? dev : 0;
    auto kern = gdn_seg_scan_kernel<D, F32OUT>;
    if (!attr_done[dev]) {   // the LDS-size attribute is per function and device
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                SegLds<D>::bytes) != hipSuccess)
            return check_launch("gdn_seg_scan (LDS attribute)");
        attr_done[dev] = true;
    }
    const int n_chunks = pl.L / SC;
    a.n_seg = gdn_segments(pl);
    a.seg_len = (n_chunks + a.n_seg - 1) / a.n_seg;
    a.n_seg = (n_chunks + a.seg_len - 1) / a.seg_len;   // no empty segment
    const int bh8 = 8 * ((pl.BH + 7) / 8) * pl.G;   // linear heads padded to the XCD count, times the group size
    const int n_mid = a.n_seg > 2 ? a.n_seg - 2 : 0;
    {
        ProfScope ps("gdn_seg_pass1", st);
        a.pass = 1;
        hipLaunchKernelGGL(kern, dim3(bh8 * (1 + n_mid)), dim3(SEG_THREADS), SegLds<D>::bytes, st, a);
    }
    nats_status s = check_launch("gdn_seg_scan (pass 1)");
    if (s != NATS_OK || a.n_seg == 1) return s;
    if (n_mid > 0) {
        ProfScope ps("gdn_seg_fix", st);
        hipLaunchKernelGGL(gdn_seg_fix_kernel<D>, dim3(8 * ((pl.BHG * (D / 16) + 7) / 8)), dim3(FIX_THREADS), 0, st, a.S_start, a.Nbuf,
                           a.MTbuf, pl.BHG, a.n_seg);
        s = check_launch("gdn_seg_fix");
        if (s != NATS_OK) return s;
    }
    {
        ProfScope ps("gdn_seg_pass2", st);
        a.pass = 2;
        hipLaunchKernelGGL(kern, dim3(bh8 * (a.n_seg - 1)), dim3(SEG_THREADS), SegLds<D>::bytes, st, a);
    }
    return check_launch("gdn_seg_scan (pass 2)");
}

template <int D>
static nats_status launch_seg_t(const FwdPlan& pl, const SegArgs<D>& a, hipStream_t st) {
    return a.O_la_f32 != nullptr ? launch_seg_k<D, true>(pl, a, st) : launch_seg_k<D, false>(pl, a, st);
}

// Writes O_la_h (fp16) for the softmax kernel to merge, and O_la_f32 if given.
// seg_ws: 3 * BH * n_seg * d * d floats (start states, N, M^T).
nats_status launch_gdn_seg_scan(const FwdPlan& pl, const void* Q, const void* K, const void* V, const void* TF,
                                const void* PF, const float* gamv, const float* kdv, const float* gamC,
                                const float* S0, float* S_final, float* seg_ws, void* O_la_h, float* O_la_f32,
                                hipStream_t st) {
    const size_t per = (size_t)pl.BHG * gdn_segments(pl) * pl.d * pl.d;
    if (pl.d == 64) {
        SegArgs<64> a{(const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const half_t*)TF, (const half_t*)PF,
                      gamv, kdv, gamC, S0, S_final, seg_ws, seg_ws + per, seg_ws + 2 * per, (half_t*)O_la_h,
                      O_la_f32, pl.L, pl.BHG, 0, 0, 0,
                      pl.linear_op == NATS_LINEAR_GATED, pl.G, pl.la_scale};
        return launch_seg_t<64>(pl, a, st);
    }
    SegArgs<128> a{(const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const half_t*)TF, (const half_t*)PF,
                   gamv, kdv, gamC, S0, S_final, seg_ws, seg_ws + per, seg_ws + 2 * per, (half_t*)O_la_h,
                   O_la_f32, pl.L, pl.BHG, 0, 0, 0,
                   pl.linear_op == NATS_LINEAR_GATED, pl.G, pl.la_scale};
    return launch_seg_t<128>(pl, a, st);
}

}  // namespace nats
