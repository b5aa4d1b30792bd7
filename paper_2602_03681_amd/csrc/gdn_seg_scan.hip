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
//            segment two blocks run the same recurrence without outputs: one from the zero state (its end
//            state is the segment's N), one on the d_k unit rows with V = 0 (its end state is the segment's M);
//   fix-up   (gdn_seg_fix) S_start[s + 1] = S_start[s] M_s + N_s along the few segments of a (batch, head);
//   pass 2   every later segment runs the recurrence from its start state, outputs included.
// A (batch, head) with L / 64 chunks then costs about 2 L / (64 n_seg) dependent steps instead of L / 64, for
// 2 (n_seg - 2) / n_seg more state products.
//
// One block = one (batch, head, segment), 8 wavefronts, all d_v rows: wavefront (tw, vh) owns token tile tw
// (16 tokens) and half vh of the d_v columns in the products over d_k and over tokens, and a quarter of d_k
// by half of d_v of the state.  The state lives transposed, S^T [d_k x d_v], as fp32 MFMA accumulators and
// never leaves registers in fp32; an fp16 copy S[v][d_k] in LDS is the operand of the products that read it.
// Every operand that comes from memory (K, Q, V rows, T'', P) is loaded as the MFMA fragment of the
// wavefront that uses it, straight from global memory, one chunk ahead; LDS carries the exchanged copies
// S, R, U and the transposed K.  Transpositions run on the matrix cores: a product with a 0/1 selector
// matrix hands a row-major fragment back in the accumulator layout, exactly (K^T for the state update, V
// added onto - gam K S0^T).  The output is computed transposed (S0 Q^T, U^T P^T): an accumulator then holds
// four consecutive d_v of one token, which is the layout O is stored in.
// Per chunk: three block barriers (R ready, U ready, S ready).
#include <algorithm>

#include "mfma_util.h"
#include "nats_common.h"

namespace nats {

constexpr int SEG_THREADS = 512;
constexpr int SC = 64;   // chunk size

template <int D>
struct SegLds {
    static constexpr int SS = D + LDS_PAD;     // halves per row of the state copy   S [d_v][SS]
    static constexpr int TS = SC + LDS_PAD;    // halves per row of a token-contraction copy: R, U [d_v][TS], Kd^T [d_k][TS]
    static constexpr int o_S = 0;
    static constexpr int o_R = o_S + D * SS;
    static constexpr int o_U = o_R + D * TS;
    static constexpr int o_K = o_U + D * TS;
    static constexpr int n_half = o_K + D * TS;
    static constexpr int bytes = n_half * 2;
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
    half_t* O_la_h;           // fp16 linear-branch output (for the merge in the softmax kernel) or nullptr
    float* O_la_f32;          // optional fp32 copy of the linear-branch output
    const half_t* O_nla_h;    // fp16 softmax-branch output to add (plain-sum merge) or nullptr
    bf16_t* O;                // merged output (with O_nla_h)
    int L, BH, n_seg, seg_len, pass, gated;
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

template <int D>
__global__ __launch_bounds__(SEG_THREADS) void gdn_seg_scan_kernel(const SegArgs<D> a) {
    using Lds = SegLds<D>;
    constexpr int SS = Lds::SS, TS = Lds::TS;
    constexpr int KS_D = D / 32;      // contraction steps over d_k
    constexpr int NVT = D / 32;       // 16-wide d_v tiles of one wavefront (half of d_v)
    constexpr int KS_V = D / 64;      // 32-wide steps over this wavefront's d_v half, for the V fragments
    constexpr int MS = D / 64;        // 16-row d_k tiles of S^T owned by one wavefront
    extern __shared__ __align__(16) unsigned char seg_smem[];
    half_t* Ss = reinterpret_cast<half_t*>(seg_smem) + Lds::o_S;
    half_t* Rs = reinterpret_cast<half_t*>(seg_smem) + Lds::o_R;
    half_t* Us = reinterpret_cast<half_t*>(seg_smem) + Lds::o_U;
    half_t* Kds = reinterpret_cast<half_t*>(seg_smem) + Lds::o_K;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tw = wave & 3, vh = wave >> 2;
    const int l16 = lane & 15, lq = lane >> 4;
    const int vbase = vh * (D / 2);
    const int n_chunks = a.L / SC;

    // ---- block -> (batch*head, role, segment).  Blocks with ids congruent modulo 8 share an XCD and its L2:
    //      the blocks of one (batch, head) are given such ids (the two blocks of a middle segment read the
    //      same K and T'').
    const int n_mid = a.n_seg > 2 ? a.n_seg - 2 : 0;
    const int per_bh = a.pass == 1 ? 1 + 2 * n_mid : a.n_seg - 1;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int bh = (slot / per_bh) * 8 + xcd;
    if (bh >= a.BH) return;
    const int sub = slot % per_bh;
    int role, seg;
    if (a.pass == 1) {
        role = sub == 0 ? ROLE_OUT : (((sub - 1) & 1) ? ROLE_ACC_E : ROLE_ACC_S);
        seg = sub == 0 ? 0 : 1 + ((sub - 1) >> 1);
    } else {
        role = ROLE_OUT;
        seg = 1 + sub;
    }
    const bool has_out = role == ROLE_OUT, has_v = role != ROLE_ACC_E;
    const int c_begin = seg * a.seg_len, c_end = min(c_begin + a.seg_len, n_chunks);
    const size_t seg_slot = (size_t)bh * a.n_seg + seg;
    const float* init = nullptr;           // state the segment starts from (nullptr: zero, or the unit rows)
    float* dest = nullptr;                 // where its end state goes
    if (role == ROLE_OUT) {
        init = seg == 0 ? (a.S0 ? a.S0 + (size_t)bh * D * D : nullptr) : a.S_start + seg_slot * D * D;
        if (seg == a.n_seg - 1) dest = a.S_final ? a.S_final + (size_t)bh * D * D : nullptr;
        else if (seg == 0) dest = a.S_start + (seg_slot + 1) * D * D;   // the later start states come from the fix-up
    } else if (role == ROLE_ACC_S) {
        dest = a.Nbuf + seg_slot * D * D;
    } else {
        dest = a.MTbuf + seg_slot * D * D;
    }

    // ---- state: S^T tiles (rows d_k, cols v) as fp32 accumulators; fp16 copy S[v][d_k] in LDS -----
    const int dq = tw;   // this wavefront's quarter of d_k in the state update
    f32x4 accS[MS][NVT];
#pragma unroll
    for (int m = 0; m < MS; ++m)
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) {
            const int dk = (D / 4) * dq + 16 * m + 4 * lq, v = vbase + 16 * vt + l16;
            if (init != nullptr) {
                const float4 x = *reinterpret_cast<const float4*>(init + (size_t)v * D + dk);
                accS[m][vt] = f32x4{x.x, x.y, x.z, x.w};
            } else if (role == ROLE_ACC_E) {   // unit rows: "v" counts the rows e of the identity
                accS[m][vt] = f32x4{v == dk ? 1.f : 0.f, v == dk + 1 ? 1.f : 0.f, v == dk + 2 ? 1.f : 0.f,
                                    v == dk + 3 ? 1.f : 0.f};
            } else {
                accS[m][vt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            *reinterpret_cast<half4*>(Ss + v * SS + dk) = to_half4(accS[m][vt]);
        }

    // 0/1 selector fragments: B operand whose column n picks contraction slot n (lo) or 16 + n (hi) of a 32-slot step
    half8 isel[2];
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int j = 0; j < 8; ++j) isel[hf][j] = (8 * lq + j == 16 * hf + l16) ? (half_t)1.f : (half_t)0.f;

    // ---- operands of one chunk, as this wavefront's MFMA fragments (raw bf16 words for K, Q, V) ----
    // contraction slot (lq, j) of step ks stands for d_k (or token, or d_v) index 32 ks + 8 lq + j
    u32x4 kraw[KS_D], qraw[KS_D], vraw[KS_V];
    half8 tfr[2], pfr[2];
    uint2 onla[NVT];
    float4 gam4, kd4;      // gates of rows 4 lq + j of token tile tw
    float gam_t, gC;       // gate of token 16 tw + l16; decay of the whole chunk
    const size_t tokb = (size_t)bh * a.L;
    const size_t chb = (size_t)bh * n_chunks;
    auto load_kqv = [&](int c) __attribute__((always_inline)) {
        const size_t row = (tokb + (size_t)c * SC + 16 * tw + l16) * D;
        const bf16_t* Kr = a.K + row + 8 * lq;
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) kraw[ks] = *reinterpret_cast<const u32x4*>(Kr + 32 * ks);
        if (has_out) {
            const bf16_t* Qr = a.Q + row + 8 * lq;
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks) qraw[ks] = *reinterpret_cast<const u32x4*>(Qr + 32 * ks);
        }
        if (has_v) {
            const bf16_t* Vr = a.V + row + vbase + 8 * lq;
#pragma unroll
            for (int ks = 0; ks < KS_V; ++ks) vraw[ks] = *reinterpret_cast<const u32x4*>(Vr + 32 * ks);
        }
        const size_t gv = (chb + c) * SC + 16 * tw;
        gam4 = *reinterpret_cast<const float4*>(a.gamv + gv + 4 * lq);
        kd4 = *reinterpret_cast<const float4*>(a.kdv + gv + 4 * lq);
        gam_t = a.gamv[gv + l16];
        gC = a.gamC[chb + c];
    };
    auto load_t = [&](int c) __attribute__((always_inline)) {
        const half8* Tc = reinterpret_cast<const half8*>(a.TF + (chb + c) * (size_t)(SC * SC)) + (tw * 2) * 64 + lane;
        tfr[0] = Tc[0];
        if (tw >= 2) tfr[1] = Tc[64];
    };
    auto load_p = [&](int c) __attribute__((always_inline)) {
        if (!has_out) return;
        const half8* Pc = reinterpret_cast<const half8*>(a.PF + (chb + c) * (size_t)(SC * SC)) + (tw * 2) * 64 + lane;
        pfr[0] = Pc[0];
        if (tw >= 2) pfr[1] = Pc[64];
        if (a.O_nla_h != nullptr) {
            const half_t* Or = a.O_nla_h + (tokb + (size_t)c * SC + 16 * tw + l16) * D + vbase + 4 * lq;
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt) onla[vt] = *reinterpret_cast<const uint2*>(Or + 16 * vt);
        }
    };
    // One word of every 128 bytes of a later chunk's K, Q, V (and of the softmax branch's rows), so that the
    // fragment loads one step ahead find them in L2; the value is not used.
    // (The word of one step is folded into a sink one step later, so that nothing waits for it where it is issued.)
    uint32_t sink = 0, touched = 0;
    auto touch = [&](int c) __attribute__((always_inline)) {
        sink ^= touched;
        if (c >= c_end) return;
        constexpr int LINES = SC * D * 2 / 128;          // 128-byte lines of one [64][D] bf16 tile
        const size_t off = (tokb + (size_t)c * SC) * D;
        const int t = tid;
        if (t < LINES) touched = *reinterpret_cast<const uint32_t*>(a.K + off + (size_t)t * 64);
        else if (t < 2 * LINES && has_v)
            touched = *reinterpret_cast<const uint32_t*>(a.V + off + (size_t)(t - LINES) * 64);
        else if (t < 3 * LINES && has_out)
            touched = *reinterpret_cast<const uint32_t*>(a.Q + off + (size_t)(t - 2 * LINES) * 64);
        else if (t < 4 * LINES && has_out && a.O_nla_h != nullptr)
            touched = *reinterpret_cast<const uint32_t*>(a.O_nla_h + off + (size_t)(t - 3 * LINES) * 64);
    };

    load_kqv(c_begin);
    load_t(c_begin);
    load_p(c_begin);
    touch(c_begin + 1);
    __syncthreads();   // initial state copy visible

    for (int c = c_begin; c < c_end; ++c) {
        const int cn = min(c + 1, c_end - 1);   // the tail re-loads the last chunk: loads stay unconditional
        touch(c + 2);
        // ================= phase a: R = V - gam K S0^T,  O^T = S0 Q^T,  Kd^T ==================
        half8 kf[KS_D], qf[KS_D];
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) kf[ks] = cvt_bf16x8(kraw[ks]);
        if (has_out) {
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks) qf[ks] = cvt_bf16x8(qraw[ks]);
        }
        f32x4 accR[NVT], accO[NVT];
#pragma unroll
        for (int vt = 0; vt < NVT; ++vt) {
            half8 fs[KS_D];
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks) fs[ks] = lds_read8(Ss + (vbase + 16 * vt + l16) * SS + 32 * ks + 8 * lq);
            accR[vt] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (!a.gated) {
#pragma unroll
                for (int ks = 0; ks < KS_D; ++ks) accR[vt] = mfma16(kf[ks], fs[ks], accR[vt]);   // rows tok, col v
            }
            if (has_out) {
                accO[vt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS_D; ++ks) accO[vt] = mfma16(fs[ks], qf[ks], accO[vt]);   // rows v, col tok
            }
        }
        {
            const float g4[4] = {gam4.x, gam4.y, gam4.z, gam4.w};
            half8 vf[KS_V];
            if (has_v) {
#pragma unroll
                for (int ks = 0; ks < KS_V; ++ks) vf[ks] = cvt_bf16x8(vraw[ks]);
            }
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt) {
                f32x4 r;
#pragma unroll
                for (int j = 0; j < 4; ++j) r[j] = -g4[j] * accR[vt][j];
                if (has_v) r = mfma16(vf[vt >> 1], isel[vt & 1], r);    // + V[tok][v], exactly
                *reinterpret_cast<half4*>(Rs + (vbase + 16 * vt + l16) * TS + 16 * tw + 4 * lq) = to_half4(r);
            }
        }
        {   // Kd^T[d_k][tok] = kd_tok K[tok][d_k]: this wavefront's share of the d_k steps of token tile tw
            const float k4[4] = {kd4.x, kd4.y, kd4.z, kd4.w};
#pragma unroll
            for (int kk = 0; kk < KS_D / 2; ++kk) {
                const int ks = vh * (KS_D / 2) + kk;
#pragma unroll
                for (int hf = 0; hf < 2; ++hf) {
                    f32x4 t = mfma16(kf[ks], isel[hf], f32x4{0.f, 0.f, 0.f, 0.f});   // rows tok, col d_k = 32 ks + 16 hf + l16
#pragma unroll
                    for (int j = 0; j < 4; ++j) t[j] *= k4[j];
                    *reinterpret_cast<half4*>(Kds + (32 * ks + 16 * hf + l16) * TS + 16 * tw + 4 * lq) = to_half4(t);
                }
            }
        }
        const float gC_cur = gC, gam_t_cur = gam_t;
        load_kqv(cn);      // next chunk's rows and gates: their registers are free from here on
        __syncthreads();   // R and Kd^T complete; every wavefront has read the old state copy

        // ================= phase b: U = T'' R ==================
        {
            f32x4 accU[NVT];
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt) {
                accU[vt] = f32x4{0.f, 0.f, 0.f, 0.f};
                const half_t* Rr = Rs + (vbase + 16 * vt + l16) * TS + 8 * lq;
                accU[vt] = mfma16(tfr[0], lds_read8(Rr), accU[vt]);
                if (tw >= 2) accU[vt] = mfma16(tfr[1], lds_read8(Rr + 32), accU[vt]);   // T'' is lower triangular
                *reinterpret_cast<half4*>(Us + (vbase + 16 * vt + l16) * TS + 16 * tw + 4 * lq) = to_half4(accU[vt]);
            }
        }
        load_t(cn);
        __syncthreads();   // U complete

        // ================= phase c: S1^T = gam_C S0^T + Kd^T U,  O^T += U^T P^T ==================
        {
            half8 fu[NVT][2];
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt)
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) fu[vt][ks] = lds_read8(Us + (vbase + 16 * vt + l16) * TS + 32 * ks + 8 * lq);
#pragma unroll
            for (int m = 0; m < MS; ++m) {
                const int dk0 = (D / 4) * dq + 16 * m;
                half8 fa[2];
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) fa[ks] = lds_read8(Kds + (dk0 + l16) * TS + 32 * ks + 8 * lq);
#pragma unroll
                for (int vt = 0; vt < NVT; ++vt) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) accS[m][vt][j] *= gC_cur;
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) accS[m][vt] = mfma16(fa[ks], fu[vt][ks], accS[m][vt]);
                    *reinterpret_cast<half4*>(Ss + (vbase + 16 * vt + l16) * SS + dk0 + 4 * lq) = to_half4(accS[m][vt]);
                }
            }
            if (has_out) {
                const size_t orow = (tokb + (size_t)c * SC + 16 * tw + l16) * D + vbase + 4 * lq;
#pragma unroll
                for (int vt = 0; vt < NVT; ++vt) {
                    f32x4 o;
#pragma unroll
                    for (int j = 0; j < 4; ++j) o[j] = gam_t_cur * accO[vt][j];
                    o = mfma16(fu[vt][0], pfr[0], o);                       // rows v, col r = 16 tw + l16
                    if (tw >= 2) o = mfma16(fu[vt][1], pfr[1], o);          // P is lower triangular
#pragma unroll
                    for (int j = 0; j < 4; ++j) o[j] *= a.la_scale;
                    if (a.O_la_f32 != nullptr)
                        *reinterpret_cast<float4*>(a.O_la_f32 + orow + 16 * vt) = make_float4(o[0], o[1], o[2], o[3]);
                    if (a.O_nla_h != nullptr) {   // plain-sum merge (Section 4.1): add the softmax branch's row piece, store bf16
                        const half4 h = __builtin_bit_cast(half4, onla[vt]);
                        *reinterpret_cast<uint2*>(a.O + orow + 16 * vt) =
                            make_uint2(pack_bf16x2(o[0] + (float)h[0], o[1] + (float)h[1]),
                                       pack_bf16x2(o[2] + (float)h[2], o[3] + (float)h[3]));
                    } else {                      // the linear branch's rows as fp16 for the softmax kernel's merge epilogue
                        *reinterpret_cast<half4*>(a.O_la_h + orow + 16 * vt) = to_half4(o);
                    }
                }
            }
        }
        load_p(cn);
        __syncthreads();   // new state copy visible; R, U and Kd^T free again
    }
    sink ^= touched;
    asm volatile("" ::"v"(sink));   // keeps the touching loads alive

    // ---- end state ----
    if (dest != nullptr) {
#pragma unroll
        for (int m = 0; m < MS; ++m)
#pragma unroll
            for (int vt = 0; vt < NVT; ++vt) {
                const int dk = (D / 4) * dq + 16 * m + 4 * lq, v = vbase + 16 * vt + l16;
                if (role == ROLE_ACC_E) {   // transposed: MT[j = d_k][i = unit row]
#pragma unroll
                    for (int j = 0; j < 4; ++j) dest[(size_t)(dk + j) * D + v] = accS[m][vt][j];
                } else {
                    *reinterpret_cast<float4*>(dest + (size_t)v * D + dk) =
                        make_float4(accS[m][vt][0], accS[m][vt][1], accS[m][vt][2], accS[m][vt][3]);
                }
            }
    }
}

// ---- fix-up between the passes: S_start[s + 1] = S_start[s] M_s + N_s, s = 1 .. n_seg - 2 --------------------
// One block = 16 state rows of one (batch, head), 4 wavefronts, each owning d / 64 column tiles of 16.  The
// product runs on fp16 MFMA with both operands split into two fp16 terms (hi + lo, three products): the error
// is about 2^-21 relative, so the carried state keeps fp32-level accuracy.
constexpr int FIX_THREADS = 256;

__device__ __forceinline__ void split8(const float* x, half8& hi, half8& lo) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        hi[j] = f32_to_half_sat(x[j]);
        lo[j] = (half_t)(x[j] - (float)hi[j]);
    }
}

template <int D>
__global__ __launch_bounds__(FIX_THREADS) void gdn_seg_fix_kernel(float* __restrict__ S_start,
                                                                 const float* __restrict__ Nbuf,
                                                                 const float* __restrict__ MTbuf, int BH, int n_seg) {
    constexpr int KS_D = D / 32, NT = D / 64;   // contraction steps; column tiles per wavefront
    constexpr int RS = D + 4;                   // fp32 row stride of the state rows in LDS
    __shared__ __align__(16) float Srow[16 * RS];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    const int bh = blockIdx.x / (D / 16), v0 = (blockIdx.x % (D / 16)) * 16;
    if (bh >= BH) return;
    const size_t base = (size_t)bh * n_seg;
    for (int e = tid; e < 16 * D / 4; e += FIX_THREADS) {
        const int r = e / (D / 4), c4 = (e % (D / 4)) * 4;
        *reinterpret_cast<float4*>(Srow + r * RS + c4) =
            *reinterpret_cast<const float4*>(S_start + ((base + 1) * D + v0 + r) * D + c4);
    }
    __syncthreads();
    for (int s = 1; s + 1 < n_seg; ++s) {
        const float* MT = MTbuf + (base + s) * D * D;
        const float* Nn = Nbuf + (base + s) * D * D;
        // A operand: rows v0 + l16, slots i = 32 ks + 8 lq + j
        half8 ahi[KS_D], alo[KS_D];
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) {
            float x[8];
            const float4 x0 = *reinterpret_cast<const float4*>(Srow + l16 * RS + 32 * ks + 8 * lq);
            const float4 x1 = *reinterpret_cast<const float4*>(Srow + l16 * RS + 32 * ks + 8 * lq + 4);
            x[0] = x0.x; x[1] = x0.y; x[2] = x0.z; x[3] = x0.w; x[4] = x1.x; x[5] = x1.y; x[6] = x1.z; x[7] = x1.w;
            split8(x, ahi[ks], alo[ks]);
        }
        f32x4 acc[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int j0 = 16 * (wave * NT + nt);
            acc[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KS_D; ++ks) {   // B operand: col j0 + l16, slots i: row j of MT is contiguous in i
                float x[8];
                const float* mp = MT + (size_t)(j0 + l16) * D + 32 * ks + 8 * lq;
                const float4 x0 = *reinterpret_cast<const float4*>(mp);
                const float4 x1 = *reinterpret_cast<const float4*>(mp + 4);
                x[0] = x0.x; x[1] = x0.y; x[2] = x0.z; x[3] = x0.w; x[4] = x1.x; x[5] = x1.y; x[6] = x1.z; x[7] = x1.w;
                half8 bhi, blo;
                split8(x, bhi, blo);
                acc[nt] = mfma16(alo[ks], bhi, acc[nt]);
                acc[nt] = mfma16(ahi[ks], blo, acc[nt]);
                acc[nt] = mfma16(ahi[ks], bhi, acc[nt]);
            }
        }
        __syncthreads();   // every wavefront has read the old rows
        float* out = S_start + (base + s + 1) * D * D;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int j = 16 * (wave * NT + nt) + l16;
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {   // rows v0 + 4 lq + jj, col j
                const int r = 4 * lq + jj;
                const float y = acc[nt][jj] + Nn[(size_t)(v0 + r) * D + j];
                Srow[r * RS + j] = y;
                out[(size_t)(v0 + r) * D + j] = y;
            }
        }
        __syncthreads();
    }
}

// number of segments a (batch, head) is cut into: enough blocks to fill the chip, at least 4 chunks each
int gdn_segments(const FwdPlan& pl) {
    const int n_chunks = pl.L / SC;
    int n = pl.gdn_segments > 0 ? pl.gdn_segments : std::max(1, 256 / pl.BH);
    n = std::min(n, std::max(1, n_chunks / 4));
    return std::max(1, std::min(n, 64));
}

template <int D>
static nats_status launch_seg_t(const FwdPlan& pl, SegArgs<D> a, hipStream_t st) {
    static bool attr_done[64] = {};
    int dev = 0;
    (void)hipGetDevice(&dev);
    dev = (dev >= 0 && dev < 64) ? dev : 0;
    auto kern = gdn_seg_scan_kernel<D>;
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
    const int bh8 = 8 * ((pl.BH + 7) / 8);
    const int n_mid = a.n_seg > 2 ? a.n_seg - 2 : 0;
    {
        ProfScope ps("gdn_seg_scan", st);
        a.pass = 1;
        hipLaunchKernelGGL(kern, dim3(bh8 * (1 + 2 * n_mid)), dim3(SEG_THREADS), SegLds<D>::bytes, st, a);
    }
    nats_status s = check_launch("gdn_seg_scan (pass 1)");
    if (s != NATS_OK || a.n_seg == 1) return s;
    if (n_mid > 0) {
        ProfScope ps("gdn_seg_fix", st);
        hipLaunchKernelGGL(gdn_seg_fix_kernel<D>, dim3(pl.BH * (D / 16)), dim3(FIX_THREADS), 0, st, a.S_start, a.Nbuf,
                           a.MTbuf, pl.BH, a.n_seg);
        s = check_launch("gdn_seg_fix");
        if (s != NATS_OK) return s;
    }
    {
        ProfScope ps("gdn_seg_scan", st);
        a.pass = 2;
        hipLaunchKernelGGL(kern, dim3(bh8 * (a.n_seg - 1)), dim3(SEG_THREADS), SegLds<D>::bytes, st, a);
    }
    return check_launch("gdn_seg_scan (pass 2)");
}

// O_nla_h == nullptr: writes O_la_h (fp16) for the softmax kernel to merge.  Otherwise merges (plain sum)
// with O_nla_h and writes O.  seg_ws: 3 * BH * n_seg * d * d floats (start states, N, M^T).
nats_status launch_gdn_seg_scan(const FwdPlan& pl, const void* Q, const void* K, const void* V, const void* TF,
                                const void* PF, const float* gamv, const float* kdv, const float* gamC,
                                const float* S0, float* S_final, float* seg_ws, void* O_la_h, float* O_la_f32,
                                const void* O_nla_h, void* O, hipStream_t st) {
    const size_t per = (size_t)pl.BH * gdn_segments(pl) * pl.d * pl.d;
    if (pl.d == 64) {
        SegArgs<64> a{(const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const half_t*)TF, (const half_t*)PF,
                      gamv, kdv, gamC, S0, S_final, seg_ws, seg_ws + per, seg_ws + 2 * per, (half_t*)O_la_h,
                      O_la_f32, (const half_t*)O_nla_h, (bf16_t*)O, pl.L, pl.BH, 0, 0, 0,
                      pl.linear_op == NATS_LINEAR_GATED, pl.la_scale};
        return launch_seg_t<64>(pl, a, st);
    }
    SegArgs<128> a{(const bf16_t*)Q, (const bf16_t*)K, (const bf16_t*)V, (const half_t*)TF, (const half_t*)PF,
                   gamv, kdv, gamC, S0, S_final, seg_ws, seg_ws + per, seg_ws + 2 * per, (half_t*)O_la_h,
                   O_la_f32, (const half_t*)O_nla_h, (bf16_t*)O, pl.L, pl.BH, 0, 0, 0,
                   pl.linear_op == NATS_LINEAR_GATED, pl.la_scale};
    return launch_seg_t<128>(pl, a, st);
}

}  // namespace nats
