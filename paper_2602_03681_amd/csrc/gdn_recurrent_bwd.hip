// Backward of the linear branch in fp32 arithmetic (Section 4.2): the reverse sweep of
//     Sd = a_t S_{t-1};   linear token:  r = v_t - Sd k_t,  S_t = Sd + b_t r k_t^T   (Eq. 19, delta rule; the
//     gated operation has r = v_t);   softmax token: S_t = Sd (Eq. 14);   o_t = la_scale S_t q_t
// with dS the gradient of the state after token t (from the tokens behind it) and do_t given:
//     dq_t  = la_scale S_t^T do_t ;              dS += la_scale do_t q_t^T
//     linear token:  A = dS k_t ;  dbeta_t = r . A ;  dr = b_t A ;  dv_t = dr ;
//                    dk_t = b_t dS^T r - Sd^T dr ;  dS -= dr k_t^T          (the last two terms: delta rule only)
//     dalpha_t = <dS, S_{t-1}> = <dS, Sd> / a_t ;  dS <- a_t dS
// Rows of S (index d_v) never mix: 16 adjacent lanes own one row (a sixteenth of its d_k columns each): of dS
// in registers across the whole sweep, and of Sd for the token at hand.  The states are not kept by the forward
// pass: it leaves one checkpoint per chunk of 64 tokens, and a block walks the chunks from the back, first
// re-running the chunk forwards from its checkpoint and parking its rows Sd in a scratch area (0.5 MB per
// block for d = 128, written and read once, laid out so that a wavefront's accesses are contiguous), then
// sweeping it backwards.  dq_t, dk_t (vectors over d_k) and dalpha_t, dbeta_t add up over all rows: a block
// (16 rows, 4 wavefronts) reduces its share in a fixed order (the 4 rows of a wavefront by recursive halving
// over lane exchanges, the wavefronts through LDS; one barrier per token) and writes one partial per block; a small
// kernel adds the partials (d / 16 of them) and finishes the outputs.  No floating-point atomics.
//
// VALU- and latency-bound (d / 16 blocks of four wavefronts per (batch, head): the arithmetic of a token is the
// same however many lanes share a row, so what helps is more CUs): this is the path for
// checking gradients and for small problems, the counterpart of the fp32 forward path.
#include "nats_common.h"

namespace nats {

constexpr int RB_TT = 16;         // tokens staged per tile (a multiple of 4)
constexpr int RB_CH = 64;         // tokens between checkpoints

// One step of a sum over the rows of a wavefront by recursive halving.  In the step for lane bit b a lane keeps
// the half of its N values that its bit selects, hands the other half to its partner and adds what the partner
// hands over: N values of one row become N / 2 values of two rows.
template <int N, int BIT>
__device__ __forceinline__ void halve_step(float* v, int lane);   // defined below the lane exchanges

constexpr int RBW_ROWS = BWD_SWEEP_ROWS;         // state rows per block of the reverse sweep
// 16 lanes per state row: a row is then one 16-lane row of the wavefront, inside which sums run on DPP moves;
// sums across the four rows of a wavefront run on gfx950's row swaps.  (Through __shfl_xor every step of these
// sums was an LDS round trip of its own, about thirty of them in a row per token.)
constexpr int rbw_lpr(int d) { return d / 4; }                       // 4 columns per lane
constexpr int rbw_threads(int d) { return RBW_ROWS * rbw_lpr(d); }   // 512 for d = 128, 256 for d = 64

template <int N, int BIT>
__device__ __forceinline__ void halve_step(float* v, int lane) {
    static_assert(BIT == 4 || BIT == 5, "rows of a wavefront differ in lane bits 4 and 5");
    const bool up = ((lane >> BIT) & 1) != 0;
#pragma unroll
    for (int c = 0; c < N / 2; ++c) {
        const float keep = up ? v[c + N / 2] : v[c];
        const float send = up ? v[c] : v[c + N / 2];
        v[c] = keep + (BIT == 4 ? lane_xor16(send, lane) : lane_xor32(send, lane));
    }
}

// CHUNK: routing per chunk (mask holds one byte per chunk of 64 tokens).  Inside a chunk every token is written
// (both operations compute every chunk's inner part) from the carried state at the chunk's start, which is what
// the checkpoint holds; a linear chunk hands its last state on, a softmax chunk hands on decay x (state at its
// start).  In reverse: a linear chunk's sweep starts from the gradient of the state carried out of it; a softmax
// chunk's sweep starts from zero (its provisional states end with the chunk), and when it reaches the chunk's start
// the gradient of the carried state joins it, times the chunk's decay, whose own gradient <dS_next, S_start> goes
// to the alphas of the chunk's tokens.  ds_la_part [d/16][BH][L/64] (optional): Eq. 17 for a linear chunk, this
// block's rows' share of <dS_next, S_end - decay S_start>.
template <typename T, int D, bool CHUNK>
__global__ __launch_bounds__(rbw_threads(D)) void gdn_recurrent_bwd_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V, const T* __restrict__ dO,
    const float* __restrict__ alpha, const float* __restrict__ beta, const uint8_t* __restrict__ mask,
    const float* __restrict__ ckpt, float* __restrict__ scratch, float* __restrict__ dq_part,
    float* __restrict__ dk_part, float* __restrict__ dalpha_part, float* __restrict__ dbeta_part,
    float* __restrict__ dV, float* __restrict__ dS0, float* __restrict__ ds_la_part, int L, int BH, float la_scale,
    int linear_op, int freeze_on_softmax) {
    constexpr int EPL = Vec16<T>::N;
    constexpr int LPR = rbw_lpr(D), RBW_THREADS = rbw_threads(D), NW = RBW_THREADS / 64;
    constexpr int RPW = 64 / LPR;   // rows of a wavefront: 2 or 4
    constexpr int DP = D / LPR;     // columns of a row per lane
    constexpr int KQ = 2 * DP + 4;  // a lane's columns of k, then of q, then padding: the 16 lanes of a row read
                                    // their 16-byte pieces from different banks
    constexpr int NF = DP / RPW;    // values of a lane that are left after the sum over its wavefront's rows
    static_assert(DP % 4 == 0 && (RPW == 2 || RPW == 4), "16-byte pieces; one or two halving steps");
    __shared__ __align__(16) float s_kq[RB_TT][LPR * KQ];
    __shared__ float s_v[RB_TT][RBW_ROWS], s_do[RB_TT][RBW_ROWS];
    __shared__ float s_a[RB_TT], s_b[RB_TT];
    __shared__ uint8_t s_dec[RB_TT];           // 1: the decay acts at this token
    __shared__ uint8_t s_lin[RB_TT];           // 1: linear token (the state is written)
    __shared__ float s_part[2][2][NW][D];      // [token parity][dq, dk][wavefront][column]
    __shared__ float s_sc[2][2][NW];           // [token parity][dalpha, dbeta][wavefront]
    __shared__ float s_blk[NW];                // a sum over the block's rows, once per chunk (routing per chunk)

    const int bh = blockIdx.y, slice = blockIdx.x, tid = threadIdx.x;
    const int r = tid / LPR, part = tid % LPR, lane = tid & 63, wave = tid >> 6;
    const int row = slice * RBW_ROWS + r;
    const size_t base = (size_t)bh * L;
    const int n_chunks = L / RB_CH;
    const size_t n_tok = (size_t)BH * L;
    // this block's scratch: [token of the chunk][group of 4 columns of a lane][thread][4], so that the threads of
    // the block, in order, touch consecutive 16 bytes
    float* my_scr = scratch + ((size_t)bh * gridDim.x + slice) * (size_t)(RB_CH * D * RBW_ROWS);
    float* dq_p = dq_part + (size_t)slice * n_tok * D;
    float* dk_p = dk_part + (size_t)slice * n_tok * D;
    float* da_p = dalpha_part + (size_t)slice * n_tok;
    float* db_p = dbeta_part + (size_t)slice * n_tok;

    // stages tokens [t0, t0 + RB_TT): k, v and the gates always, q and do for the backward sweep
    auto stage = [&](int t0, bool with_q) {
        __syncthreads();
        for (int e = tid * EPL; e < RB_TT * D; e += RBW_THREADS * EPL) {
            const int i = e / D, c = e % D;
            float tmp[EPL];
            Vec16<T>::load(K + (base + t0 + i) * D + c, tmp);
#pragma unroll
            for (int j = 0; j < EPL; ++j) s_kq[i][((c + j) / DP) * KQ + (c + j) % DP] = tmp[j];
            if (with_q) {
                Vec16<T>::load(Q + (base + t0 + i) * D + c, tmp);
#pragma unroll
                for (int j = 0; j < EPL; ++j) s_kq[i][((c + j) / DP) * KQ + DP + (c + j) % DP] = tmp[j];
            }
        }
        for (int e = tid * EPL; e < RB_TT * RBW_ROWS; e += RBW_THREADS * EPL) {
            const int i = e / RBW_ROWS, c = e % RBW_ROWS;
            float tmp[EPL];
            Vec16<T>::load(V + (base + t0 + i) * D + slice * RBW_ROWS + c, tmp);
#pragma unroll
            for (int j = 0; j < EPL; ++j) s_v[i][c + j] = tmp[j];
            if (with_q) {
                Vec16<T>::load(dO + (base + t0 + i) * D + slice * RBW_ROWS + c, tmp);
#pragma unroll
                for (int j = 0; j < EPL; ++j) s_do[i][c + j] = tmp[j];
            }
        }
        if (tid < RB_TT) {
            const bool soft = CHUNK ? false : mask[base + t0 + tid] != 0;   // CHUNK: every token of a chunk is written
            const bool dec = !(soft && freeze_on_softmax);
            s_dec[tid] = dec ? 1 : 0;
            s_lin[tid] = soft ? 0 : 1;
            s_a[tid] = dec ? alpha[base + t0 + tid] : 1.f;
            s_b[tid] = soft ? 0.f : beta[base + t0 + tid];
        }
        __syncthreads();
    };
    auto row_sum = [](float x) { return lane_group_sum<LPR>(x); };   // over a row's lanes
    // sum over the block's rows of a value every lane of a row holds: rows of a wavefront by lane exchanges, the
    // wavefronts in order through LDS (two barriers; called by every thread)
    auto block_sum = [&](float x) -> float {
        float y = part == 0 ? x : 0.f;
        if (RPW == 4) y += lane_xor16(y, lane);
        y += lane_xor32(y, lane);
        __syncthreads();
        if (lane == 0) s_blk[wave] = y;
        __syncthreads();
        float tot = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) tot += s_blk[w];
        return tot;
    };
    const uint8_t* mask_c = mask + (size_t)bh * (L / RB_CH);   // CHUNK only

    float dS[DP];
#pragma unroll
    for (int c = 0; c < DP; ++c) dS[c] = 0.f;

    for (int chunk = n_chunks - 1; chunk >= 0; --chunk) {
        const int tc0 = chunk * RB_CH;
        // ---- forwards through the chunk from its checkpoint: park Sd of every token ----------------
        const bool soft_chunk = CHUNK && mask_c[chunk] != 0;   // uniform
        float dS_next[DP];          // CHUNK, softmax chunk: gradient of the state carried out of the chunk
        float carry_dd = 0.f;       // ... and this block's share of <dS_next, S_start> x decay (to the alphas)
        float carry_scale = 1.f;    // decay of the chunk (1 in the variant without decay on softmax chunks)
        {
            float S[DP], S_start[DP];
            float decay = 1.f;
            const float* src = ckpt + (((size_t)bh * n_chunks + chunk) * D + row) * D + part * DP;
#pragma unroll
            for (int c = 0; c < DP; c += 4) {
                const float4 x = *reinterpret_cast<const float4*>(src + c);
                S[c] = x.x; S[c + 1] = x.y; S[c + 2] = x.z; S[c + 3] = x.w;
            }
#pragma unroll
            for (int c = 0; c < DP; ++c) S_start[c] = S[c];
#pragma unroll 1
            for (int tt = 0; tt < RB_CH; tt += RB_TT) {
                stage(tc0 + tt, false);
#pragma unroll 1
                for (int i = 0; i < RB_TT; ++i) {
                    const float a = s_a[i], b = s_b[i];
                    decay *= a;
                    const float* kr = &s_kq[i][part * KQ];
                    float* dst = my_scr + (size_t)(tt + i) * (D * RBW_ROWS) + tid * 4;
                    float pred = 0.f;
#pragma unroll
                    for (int c = 0; c < DP; c += 4) {
                        const float4 k4 = *reinterpret_cast<const float4*>(kr + c);
                        S[c] *= a; S[c + 1] *= a; S[c + 2] *= a; S[c + 3] *= a;
                        *reinterpret_cast<float4*>(dst + (c / 4) * (RBW_THREADS * 4)) = make_float4(S[c], S[c + 1], S[c + 2], S[c + 3]);
                        pred += S[c] * k4.x + S[c + 1] * k4.y + S[c + 2] * k4.z + S[c + 3] * k4.w;
                    }
                    if (s_lin[i]) {   // uniform across the block
                        pred = row_sum(pred);
                        const float delta = b * (s_v[i][r] - (linear_op == 0 ? pred : 0.f));
#pragma unroll
                        for (int c = 0; c < DP; c += 4) {
                            const float4 k4 = *reinterpret_cast<const float4*>(kr + c);
                            S[c] += delta * k4.x; S[c + 1] += delta * k4.y; S[c + 2] += delta * k4.z; S[c + 3] += delta * k4.w;
                        }
                    }
                }
            }
            if (CHUNK) {
                if (soft_chunk) {
                    float dd = 0.f;
#pragma unroll
                    for (int c = 0; c < DP; ++c) { dS_next[c] = dS[c]; dd += dS[c] * S_start[c]; dS[c] = 0.f; }
                    carry_scale = freeze_on_softmax ? 1.f : decay;
                    carry_dd = freeze_on_softmax ? 0.f : block_sum(row_sum(dd)) * decay;
                } else if (ds_la_part != nullptr) {   // Eq. 17: <dS_next, what the chunk added to the carried state>
                    float x = 0.f;
#pragma unroll
                    for (int c = 0; c < DP; ++c) x += dS[c] * (S[c] - decay * S_start[c]);
                    x = block_sum(row_sum(x));
                    if (tid == 0) ds_la_part[((size_t)slice * BH + bh) * n_chunks + chunk] = x;
                }
                if (soft_chunk && ds_la_part != nullptr && tid == 0)
                    ds_la_part[((size_t)slice * BH + bh) * n_chunks + chunk] = 0.f;
            }
        }
        // ---- backwards through the chunk ------------------------------------------------------------
        // The parked rows come back PFR tokens ahead of use, through a ring of registers (token tok in slot
        // tok % PFR; the token loop is unrolled PFR times, so the slots are fixed at compile time): read at the
        // token that needs them, or only one token ahead, their latency (a trip past L2: the scratch of all
        // blocks is 134 MB) is paid at every token.
        constexpr int PFR = 4;
        float Sn[PFR][DP];
        auto fetch_rows = [&](int tok, float* dst) {   // this thread's own stores of token tok of the chunk
            const float* src = my_scr + (size_t)tok * (D * RBW_ROWS) + tid * 4;
#pragma unroll
            for (int c = 0; c < DP; c += 4) {
                const float4 x = *reinterpret_cast<const float4*>(src + (c / 4) * (RBW_THREADS * 4));
                dst[c] = x.x; dst[c + 1] = x.y; dst[c + 2] = x.z; dst[c + 3] = x.w;
            }
        };
#pragma unroll
        for (int u = 0; u < PFR; ++u) fetch_rows(RB_CH - 1 - u, Sn[(RB_CH - 1 - u) % PFR]);
#pragma unroll 1
        for (int tt = RB_CH - RB_TT; tt >= 0; tt -= RB_TT) {
            stage(tc0 + tt, true);
#pragma unroll 1
            for (int i4 = RB_TT - PFR; i4 >= 0; i4 -= PFR)
#pragma unroll
            for (int u = PFR - 1; u >= 0; --u) {
                const int i = i4 + u;
                const int t = tc0 + tt + i;
                const float a = s_a[i], b = s_b[i], go = la_scale * s_do[i][r];
                const bool lin = s_lin[i] != 0;   // uniform across the block
                const float* kr = &s_kq[i][part * KQ];
                const float* qr = kr + DP;
                float Sd[DP], kk[DP], qq[DP];
#pragma unroll
                for (int c = 0; c < DP; c += 4) {
                    const float4 k4 = *reinterpret_cast<const float4*>(kr + c);
                    const float4 q4 = *reinterpret_cast<const float4*>(qr + c);
                    kk[c] = k4.x; kk[c + 1] = k4.y; kk[c + 2] = k4.z; kk[c + 3] = k4.w;
                    qq[c] = q4.x; qq[c + 1] = q4.y; qq[c + 2] = q4.z; qq[c + 3] = q4.w;
                }
#pragma unroll
                for (int c = 0; c < DP; ++c) Sd[c] = Sn[u][c];   // (tt + i) % PFR == u: tt and i4 are multiples of PFR
                fetch_rows(max(tt + i - PFR, 0), Sn[u]);   // unconditional (the last four re-read token 0): see below
                float pred = 0.f;
#pragma unroll
                for (int c = 0; c < DP; ++c) pred += Sd[c] * kk[c];
                pred = row_sum(pred);
                const float rv = lin ? s_v[i][r] - (linear_op == 0 ? pred : 0.f) : 0.f;
                // dq_t: this row's share la_scale do S_t, S_t = Sd + b r k;   dS += la_scale do q^T;   A = dS k
                float A = 0.f;
                const float br = b * rv;
                float xq[DP], xk[DP];
#pragma unroll
                for (int c = 0; c < DP; ++c) {
                    xq[c] = go * (Sd[c] + br * kk[c]);
                    dS[c] += go * qq[c];
                    A += dS[c] * kk[c];
                }
                A = row_sum(A);
                float dbeta_p = 0.f, dr = 0.f;
                if (lin) {
                    dbeta_p = rv * A;
                    dr = b * A;
                    const float drd = linear_op == 0 ? dr : 0.f;
#pragma unroll
                    for (int c = 0; c < DP; ++c) {
                        xk[c] = br * dS[c] - drd * Sd[c];
                        dS[c] -= drd * kk[c];
                    }
                } else {
#pragma unroll
                    for (int c = 0; c < DP; ++c) xk[c] = 0.f;
                }
                // Every memory operation of the token body is issued by every wavefront on every path: the loads of
                // the ring and the stores share one in-order counter, and only with a fixed number of operations
                // between a load and its use can the compiler wait for that load alone; with a store under a
                // condition it waits for the newest stores as well, at every token.  So lanes that hold a copy
                // of a value store it too (same value, same address).
                dV[(base + t) * D + row] = dr;   // all lanes of the row hold dr
                float dalpha_p = 0.f;
                if (s_dec[i]) {   // uniform
#pragma unroll
                    for (int c = 0; c < DP; ++c) { dalpha_p += dS[c] * Sd[c]; dS[c] *= a; }
                    dalpha_p = row_sum(dalpha_p) / fmaxf(a, 1e-30f);   // S_{t-1} = Sd / a
                }
                // sums over the rows of the block: the rows of a wavefront by recursive halving, which leaves a
                // lane with NF columns: the halves its row bits selected ...
                int col = part * DP;
                if (RPW == 4) {   // rows differ in lane bits 4 and 5
                    halve_step<DP, 4>(xq, lane);     halve_step<DP, 4>(xk, lane);
                    halve_step<DP / 2, 5>(xq, lane); halve_step<DP / 2, 5>(xk, lane);
                    col += (DP / 2) * ((lane >> 4) & 1) + (DP / 4) * ((lane >> 5) & 1);
                } else {          // in lane bit 5
                    halve_step<DP, 5>(xq, lane);     halve_step<DP, 5>(xk, lane);
                    col += (DP / 2) * ((lane >> 5) & 1);
                }
                const int buf = t & 1;
#pragma unroll
                for (int j = 0; j < NF; ++j) {
                    s_part[buf][0][wave][col + j] = xq[j];
                    s_part[buf][1][wave][col + j] = xk[j];
                }
                // the two scalars: one value per row (its lane 0), rows of a wavefront, then the wavefronts in order
                float xa = part == 0 ? dalpha_p : 0.f, xb = part == 0 ? dbeta_p : 0.f;
                if (RPW == 4) { xa += lane_xor16(xa, lane); xb += lane_xor16(xb, lane); }   // only the rows' lanes 0 hold
                xa += lane_xor32(xa, lane); xb += lane_xor32(xb, lane);   // values: lane 0 ends up with the sum over the rows
                if (lane == 0) { s_sc[buf][0][wave] = xa; s_sc[buf][1][wave] = xb; }
                // ... then the wavefronts, in order.  One barrier per token: the next token writes the other half
                // of the buffers, and the barrier after it separates these reads from the writes that follow.
                __syncthreads();
                {   // threads beyond 2 D repeat the first ones
                    const int e = tid % (2 * D), which = e / D, c = e % D;
                    float sum = 0.f;
#pragma unroll
                    for (int w = 0; w < NW; ++w) sum += s_part[buf][which][w][c];
                    (which == 0 ? dq_p : dk_p)[(base + t) * D + c] = sum;
                    float sa = 0.f, sb = 0.f;
#pragma unroll
                    for (int w = 0; w < NW; ++w) { sa += s_sc[buf][0][w]; sb += s_sc[buf][1][w]; }
                    // (softmax chunk: the decay handed on with the carried state is a product of the chunk's alphas)
                    da_p[base + t] = (CHUNK && soft_chunk) ? sa + carry_dd / fmaxf(a, 1e-30f) : sa;
                    db_p[base + t] = sb;
                }
            }
        }
        if (CHUNK && soft_chunk) {   // the gradient of the state carried over the chunk joins at the chunk's start
#pragma unroll
            for (int c = 0; c < DP; ++c) dS[c] += carry_scale * dS_next[c];
        }
    }
    if (dS0 != nullptr) {
        float* dst = dS0 + ((size_t)bh * D + row) * D + part * DP;
#pragma unroll
        for (int c = 0; c < DP; c += 4) *reinterpret_cast<float4*>(dst + c) = make_float4(dS[c], dS[c + 1], dS[c + 2], dS[c + 3]);
    }
}

// The forward recurrence once more, only to leave the checkpoints the reverse sweep starts from: the row of the
// state before every chunk of 64 tokens, ckpt[bh][chunk][row][d_k].  Same thread layout as the kernel above
// (16 rows per block, 16 lanes per row).
template <typename T, int D, bool CHUNK>
__global__ __launch_bounds__(rbw_threads(D)) void gdn_checkpoint_kernel(
    const T* __restrict__ K, const T* __restrict__ V, const float* __restrict__ alpha, const float* __restrict__ beta,
    const uint8_t* __restrict__ mask, const float* __restrict__ S0, float* __restrict__ ckpt, int L, int linear_op,
    int freeze_on_softmax) {
    constexpr int EPL = Vec16<T>::N;
    constexpr int LPR = rbw_lpr(D), RBW_THREADS = rbw_threads(D), DP = D / LPR, DPP = DP + 4;
    constexpr int TT = 32;
    __shared__ __align__(16) float s_k[TT][LPR * DPP];
    __shared__ float s_v[TT][RBW_ROWS];
    __shared__ float s_a[TT], s_b[TT];
    __shared__ uint8_t s_lin[TT];
    const int bh = blockIdx.y, slice = blockIdx.x, tid = threadIdx.x;
    const int r = tid / LPR, part = tid % LPR;
    const int row = slice * RBW_ROWS + r;
    const size_t base = (size_t)bh * L;
    const int n_chunks = L / RB_CH;
    float S[DP];
    if (S0 != nullptr) {
        const float* src = S0 + ((size_t)bh * D + row) * D + part * DP;
#pragma unroll
        for (int c = 0; c < DP; c += 4) {
            const float4 x = *reinterpret_cast<const float4*>(src + c);
            S[c] = x.x; S[c + 1] = x.y; S[c + 2] = x.z; S[c + 3] = x.w;
        }
    } else {
#pragma unroll
        for (int c = 0; c < DP; ++c) S[c] = 0.f;
    }
    // routing per chunk: the carried state; a softmax chunk hands on decay x (its start state), see the sweep kernel
    float S_start[DP], decay = 1.f;
    const uint8_t* mask_c = mask + (size_t)bh * (L / RB_CH);
    for (int t0 = 0; t0 < L; t0 += TT) {
        __syncthreads();
        for (int e = tid * EPL; e < TT * D; e += RBW_THREADS * EPL) {
            const int i = e / D, c = e % D;
            float tmp[EPL];
            Vec16<T>::load(K + (base + t0 + i) * D + c, tmp);
#pragma unroll
            for (int j = 0; j < EPL; ++j) s_k[i][((c + j) / DP) * DPP + (c + j) % DP] = tmp[j];
        }
        for (int e = tid * EPL; e < TT * RBW_ROWS; e += RBW_THREADS * EPL) {
            const int i = e / RBW_ROWS, c = e % RBW_ROWS;
            float tmp[EPL];
            Vec16<T>::load(V + (base + t0 + i) * D + slice * RBW_ROWS + c, tmp);
#pragma unroll
            for (int j = 0; j < EPL; ++j) s_v[i][c + j] = tmp[j];
        }
        if (tid < TT) {
            const bool soft = CHUNK ? false : mask[base + t0 + tid] != 0;
            s_lin[tid] = soft ? 0 : 1;
            s_a[tid] = (soft && freeze_on_softmax) ? 1.f : alpha[base + t0 + tid];
            s_b[tid] = soft ? 0.f : beta[base + t0 + tid];
        }
        __syncthreads();
#pragma unroll 1
        for (int i = 0; i < TT; ++i) {
            if (((t0 + i) & (RB_CH - 1)) == 0) {
                float* dst = ckpt + (((size_t)bh * n_chunks + (t0 + i) / RB_CH) * D + row) * D + part * DP;
#pragma unroll
                for (int c = 0; c < DP; c += 4) *reinterpret_cast<float4*>(dst + c) = make_float4(S[c], S[c + 1], S[c + 2], S[c + 3]);
                if (CHUNK) {
                    decay = 1.f;
#pragma unroll
                    for (int c = 0; c < DP; ++c) S_start[c] = S[c];
                }
            }
            const float a = s_a[i];
            decay *= a;
            const float* kr = &s_k[i][part * DPP];
            float kk[DP];
            float pred = 0.f;
#pragma unroll
            for (int c = 0; c < DP; c += 4) {
                const float4 k4 = *reinterpret_cast<const float4*>(kr + c);
                kk[c] = k4.x; kk[c + 1] = k4.y; kk[c + 2] = k4.z; kk[c + 3] = k4.w;
            }
#pragma unroll
            for (int c = 0; c < DP; ++c) { S[c] *= a; pred += S[c] * kk[c]; }
            if (s_lin[i]) {   // uniform across the block
                pred = lane_group_sum<LPR>(pred);
                const float delta = s_b[i] * (s_v[i][r] - (linear_op == 0 ? pred : 0.f));
#pragma unroll
                for (int c = 0; c < DP; ++c) S[c] += delta * kk[c];
            }
            if (CHUNK && ((t0 + i) & (RB_CH - 1)) == RB_CH - 1 && mask_c[(t0 + i) / RB_CH]) {   // end of a softmax chunk
                const float f = freeze_on_softmax ? 1.f : decay;
#pragma unroll
                for (int c = 0; c < DP; ++c) S[c] = f * S_start[c];
            }
        }
    }
}

// dQ += sum of the blocks' partials (it already holds the softmax branch's share); dK, dalpha, dbeta = the sums;
// g_nla (optional) is cleared for the kernel that fills in the softmax tokens' entries afterwards.
template <int D>
__global__ __launch_bounds__(256) void bwd_combine_kernel(
    const float* __restrict__ dq_part, const float* __restrict__ dk_part, const float* __restrict__ dalpha_part,
    const float* __restrict__ dbeta_part, float* __restrict__ dQ, float* __restrict__ dK,
    float* __restrict__ dalpha, float* __restrict__ dbeta, float* __restrict__ g_nla, size_t n_tok) {
    constexpr int NS = D / RBW_ROWS;
    const size_t n4 = n_tok * D / 4;
    for (size_t e = (size_t)blockIdx.x * 256 + threadIdx.x; e < n4; e += (size_t)gridDim.x * 256) {
        float4 q = reinterpret_cast<const float4*>(dQ)[e];
        float4 k = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            const float4 a = reinterpret_cast<const float4*>(dq_part + (size_t)s * n_tok * D)[e];
            const float4 b = reinterpret_cast<const float4*>(dk_part + (size_t)s * n_tok * D)[e];
            q.x += a.x; q.y += a.y; q.z += a.z; q.w += a.w;
            k.x += b.x; k.y += b.y; k.z += b.z; k.w += b.w;
        }
        reinterpret_cast<float4*>(dQ)[e] = q;
        reinterpret_cast<float4*>(dK)[e] = k;
    }
    for (size_t t = (size_t)blockIdx.x * 256 + threadIdx.x; t < n_tok; t += (size_t)gridDim.x * 256) {
        float a = 0.f, b = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s) { a += dalpha_part[(size_t)s * n_tok + t]; b += dbeta_part[(size_t)s * n_tok + t]; }
        dalpha[t] = a;
        dbeta[t] = b;
        if (g_nla != nullptr) g_nla[t] = 0.f;
    }
}

template <typename T>
static void launch_rb(const FwdPlan& pl, const void* Q, const void* K, const void* V, const void* dO, const float* alpha,
                      const float* beta, const uint8_t* mask, const float* ckpt, float* scratch, float* dq_part,
                      float* dk_part, float* dalpha_part, float* dbeta_part, float* dV, float* dS0, float* ds_la_part,
                      hipStream_t st) {
    dim3 grid(pl.d / RBW_ROWS, pl.BH);
#define NATS_RB_LAUNCH(DD, CH)                                                                                                   \
    hipLaunchKernelGGL((gdn_recurrent_bwd_kernel<T, DD, CH>), grid, dim3(rbw_threads(DD)), 0, st, (const T*)Q, (const T*)K,      \
                       (const T*)V, (const T*)dO, alpha, beta, mask, ckpt, scratch, dq_part, dk_part, dalpha_part, dbeta_part,  \
                       dV, dS0, ds_la_part, pl.L, pl.BH, pl.la_scale, pl.linear_op, pl.freeze_on_softmax)
    const bool chunk = pl.routing == NATS_ROUTE_CHUNK;
    if (pl.d == 64) { if (chunk) NATS_RB_LAUNCH(64, true); else NATS_RB_LAUNCH(64, false); }
    else { if (chunk) NATS_RB_LAUNCH(128, true); else NATS_RB_LAUNCH(128, false); }
#undef NATS_RB_LAUNCH
}

// scratch: BH * d * d * 64 floats;  dq_part, dk_part: (d / 16) * BH * L * d floats;
// dalpha_part, dbeta_part: (d / 16) * BH * L floats;  dV [B,H,L,d] f32 is written for every token
nats_status launch_gdn_recurrent_bwd(const FwdPlan& pl, const void* Q, const void* K, const void* V, const void* dO,
                                     const float* alpha, const float* beta, const uint8_t* mask, const float* ckpt,
                                     float* scratch, float* dq_part, float* dk_part, float* dalpha_part,
                                     float* dbeta_part, float* dV, float* dS0, float* ds_la_part, hipStream_t st) {
    if (pl.dtype == NATS_BF16)
        launch_rb<bf16_t>(pl, Q, K, V, dO, alpha, beta, mask, ckpt, scratch, dq_part, dk_part, dalpha_part, dbeta_part,
                          dV, dS0, ds_la_part, st);
    else
        launch_rb<float>(pl, Q, K, V, dO, alpha, beta, mask, ckpt, scratch, dq_part, dk_part, dalpha_part, dbeta_part,
                         dV, dS0, ds_la_part, st);
    return check_launch("gdn_recurrent_bwd");
}

// ckpt [BH][L/64][d][d] f32: the state before every chunk of 64 tokens (S0 may be NULL: zero)
nats_status launch_gdn_checkpoints(const FwdPlan& pl, const void* K, const void* V, const float* alpha, const float* beta,
                                   const uint8_t* mask, const float* S0, float* ckpt, hipStream_t st) {
    dim3 grid(pl.d / RBW_ROWS, pl.BH);
#define NATS_CK_LAUNCH(TT, DD)                                                                                        \
    do {                                                                                                              \
        if (pl.routing == NATS_ROUTE_CHUNK)                                                                           \
            hipLaunchKernelGGL((gdn_checkpoint_kernel<TT, DD, true>), grid, dim3(rbw_threads(DD)), 0, st, (const TT*)K, \
                               (const TT*)V, alpha, beta, mask, S0, ckpt, pl.L, pl.linear_op, pl.freeze_on_softmax);   \
        else                                                                                                          \
            hipLaunchKernelGGL((gdn_checkpoint_kernel<TT, DD, false>), grid, dim3(rbw_threads(DD)), 0, st, (const TT*)K, \
                               (const TT*)V, alpha, beta, mask, S0, ckpt, pl.L, pl.linear_op, pl.freeze_on_softmax);   \
    } while (0)
    if (pl.dtype == NATS_BF16) { if (pl.d == 64) NATS_CK_LAUNCH(bf16_t, 64); else NATS_CK_LAUNCH(bf16_t, 128); }
    else { if (pl.d == 64) NATS_CK_LAUNCH(float, 64); else NATS_CK_LAUNCH(float, 128); }
#undef NATS_CK_LAUNCH
    return check_launch("gdn_checkpoints");
}

nats_status launch_bwd_combine(const FwdPlan& pl, const float* dq_part, const float* dk_part, const float* dalpha_part,
                               const float* dbeta_part, float* dQ, float* dK, float* dalpha, float* dbeta,
                               float* g_nla, hipStream_t st) {
    const size_t n_tok = (size_t)pl.BH * pl.L;
    const unsigned blocks = (unsigned)((n_tok * pl.d / 4 + 255) / 256 < 4096 ? (n_tok * pl.d / 4 + 255) / 256 : 4096);
    if (pl.d == 64)
        hipLaunchKernelGGL(bwd_combine_kernel<64>, dim3(blocks), dim3(256), 0, st, dq_part, dk_part, dalpha_part,
                           dbeta_part, dQ, dK, dalpha, dbeta, g_nla, n_tok);
    else
        hipLaunchKernelGGL(bwd_combine_kernel<128>, dim3(blocks), dim3(256), 0, st, dq_part, dk_part, dalpha_part,
                           dbeta_part, dQ, dK, dalpha, dbeta, g_nla, n_tok);
    return check_launch("bwd_combine");
}

// Score gradients with routing per token (Section 4.2).  Eq. 17 for one token: the sum over the state's entries
// of (gradient w.r.t. the state after the token's write) x (what the token wrote) = beta_t (r_t . dS_t k_t), which is
// beta_t times the gradient of beta_t that the reverse sweep has already reduced; zero for softmax tokens.  Eq. 16
// and Eq. 17 per chunk of 64 tokens: the sums over the chunk.  One wavefront per (chunk, batch*head).
__global__ __launch_bounds__(64) void score_gradients_kernel(const float* __restrict__ beta, const uint8_t* __restrict__ mask,
                                                            const float* __restrict__ dbeta, const float* __restrict__ g_nla,
                                                            float* __restrict__ g_la, float* __restrict__ dscore_nla,
                                                            float* __restrict__ dscore_la, int L) {
    const size_t t = (size_t)blockIdx.y * L + (size_t)blockIdx.x * 64 + threadIdx.x;
    const float gl = mask[t] ? 0.f : beta[t] * dbeta[t];
    if (g_la != nullptr) g_la[t] = gl;
    const size_t c = (size_t)blockIdx.y * (L / 64) + blockIdx.x;
    if (dscore_la != nullptr) {
        const float s = lane_group_sum<64>(gl);
        if (threadIdx.x == 0) dscore_la[c] = s;
    }
    if (dscore_nla != nullptr) {
        const float s = lane_group_sum<64>(g_nla[t]);
        if (threadIdx.x == 0) dscore_nla[c] = s;
    }
}

nats_status launch_score_gradients(const FwdPlan& pl, const float* beta, const uint8_t* mask, const float* dbeta,
                                   const float* g_nla, float* g_la, float* dscore_nla, float* dscore_la, hipStream_t st) {
    hipLaunchKernelGGL(score_gradients_kernel, dim3(pl.L / 64, pl.BH), dim3(64), 0, st, beta, mask, dbeta, g_nla, g_la,
                       dscore_nla, dscore_la, pl.L);
    return check_launch("score_gradients");
}

// Score gradients with routing per chunk: Eq. 16 = the column sums of the mask gradient over the chunk's tokens
// (only columns of earlier softmax chunks stand behind the mask, and only they are in g_nla); Eq. 17 = the sum of
// the reverse sweep's d / 16 partials of <dS_next, what the chunk added> (zero for softmax chunks).
__global__ __launch_bounds__(64) void score_gradients_chunk_kernel(const float* __restrict__ g_nla,
                                                                  const float* __restrict__ ds_la_part,
                                                                  float* __restrict__ dscore_nla,
                                                                  float* __restrict__ dscore_la, int L, int n_part,
                                                                  size_t n_chunks_all) {
    const size_t c = (size_t)blockIdx.y * (L / 64) + blockIdx.x;
    if (dscore_nla != nullptr) {
        const float s = lane_group_sum<64>(g_nla[(size_t)blockIdx.y * L + (size_t)blockIdx.x * 64 + threadIdx.x]);
        if (threadIdx.x == 0) dscore_nla[c] = s;
    }
    if (dscore_la != nullptr && ds_la_part != nullptr && threadIdx.x == 0) {
        float s = 0.f;
        for (int p = 0; p < n_part; ++p) s += ds_la_part[(size_t)p * n_chunks_all + c];
        dscore_la[c] = s;
    }
}

nats_status launch_score_gradients_chunk(const FwdPlan& pl, const float* g_nla, const float* ds_la_part, float* dscore_nla,
                                         float* dscore_la, hipStream_t st) {
    hipLaunchKernelGGL(score_gradients_chunk_kernel, dim3(pl.L / 64, pl.BH), dim3(64), 0, st, g_nla, ds_la_part, dscore_nla,
                       dscore_la, pl.L, pl.d / RBW_ROWS, (size_t)pl.BH * (pl.L / 64));
    return check_launch("score_gradients (routing per chunk)");
}

}  // namespace nats
