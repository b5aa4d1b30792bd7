// Single-token decode step (Section 4.1, per-token generation; per-token routing):
//   S <- alpha S ;  linear token: S <- S + beta (v - S k) k^T  (Eq. 19, Eq. 20)
//   softmax token: (k, v) appended to the KV cache of softmax tokens, and attended (Eq. 12, i >= j)
//   o = merge( la_scale * S q ,  softmax(scale * q . Kcache^T) Vcache )     (Section 4.1 / Eq. 21)
// One block per (batch, head).  HBM-bound: the fp32 state is streamed once (read +
// write, 8 d^2 bytes) and the live cache rows once (4 d len bytes for bf16).
//
//  phase A  state: LPR = D/4 lanes hold one row of S as a float4 each; all row passes of a
//           thread are loaded up front so the loads overlap; S k and S q are reduced across
//           the LPR lanes with xor shuffles.
//  phase B  cache: LPK = D/(16/sizeof T) lanes share one key row (16 bytes per lane); the
//           256 threads form NSG key groups that stride over the cache with their own
//           running max / sum / accumulator, merged through LDS at the end.  The new
//           token is folded in from registers (no read-back of the row just written).
#include <math.h>

#include "nats_common.h"

namespace nats {

constexpr int DEC_THREADS = 256;

// CHUNK = false: routing per token (mask: the token's type).
// CHUNK = true : routing per chunk, known only after the chunk (Section 4.1, per-token generation): every
//   token is written into the state and appended to the cache provisionally (row cache_len +
//   chunk_pos); at a chunk's first token the state is copied to state_start; chunk_decay collects the
//   chunk's decay; cache_len stays, chunk_pos advances.  decode_commit_kernel settles the chunk.
template <typename T, int D, bool CHUNK>
__global__ __launch_bounds__(DEC_THREADS) void decode_kernel(
    float* __restrict__ state, float* __restrict__ state_start, float* __restrict__ chunk_decay,
    int32_t* __restrict__ chunk_pos, T* __restrict__ k_cache, T* __restrict__ v_cache,
    int32_t* __restrict__ cache_len, const T* __restrict__ q, const T* __restrict__ k,
    const T* __restrict__ v, const float* __restrict__ alpha, const float* __restrict__ beta,
    const uint8_t* __restrict__ mask, const float* __restrict__ w_nla, const float* __restrict__ w_la,
    T* __restrict__ o, int32_t* __restrict__ err_flags, int cap, float scale, float la_scale,
    int combine_mode, float eps, int linear_op, int freeze_on_softmax, const T* __restrict__ q_nla,
    const T* __restrict__ k_nla) {
    constexpr int LPR = D / 4;                    // lanes per state row
    constexpr int ROWS_PER_PASS = DEC_THREADS / LPR;
    constexpr int PASSES = D / ROWS_PER_PASS;     // 16 (D=128) or 4 (D=64)
    constexpr int EPL = Vec16<T>::N;              // elements per lane of a cache row
    constexpr int LPK = D / EPL;                  // lanes per key
    constexpr int NSG = DEC_THREADS / LPK;        // key groups in the block
    constexpr int UNROLL = 4;

    __shared__ float s_q[D], s_k[D], s_v[D], s_ola[D];
    __shared__ float s_qn[D], s_kn[D];            // query and key of the softmax branch (q, k unless given apart)
    __shared__ float s_m[NSG], s_l[NSG];
    __shared__ float s_acc[NSG][D];

    const int bh = blockIdx.x, tid = threadIdx.x;
    for (int c = tid; c < D; c += DEC_THREADS) {
        s_q[c] = to_float(q[(size_t)bh * D + c]);
        s_k[c] = to_float(k[(size_t)bh * D + c]);
        s_qn[c] = to_float((q_nla != nullptr ? q_nla : q)[(size_t)bh * D + c]);
        s_kn[c] = to_float((k_nla != nullptr ? k_nla : k)[(size_t)bh * D + c]);
        s_v[c] = to_float(v[(size_t)bh * D + c]);
    }
    const int pos = CHUNK ? chunk_pos[bh] : 0;
    const bool is_softmax = CHUNK ? true : mask[bh] != 0;     // CHUNK: every token goes to the cache ...
    // variant without decay on softmax tokens: alpha counts as 1 there (routing per chunk: the commit decides)
    const float a = (!CHUNK && is_softmax && freeze_on_softmax) ? 1.f : alpha[bh];
    const float b = (!CHUNK && is_softmax) ? 0.f : beta[bh];  // ... and into the state
    // Rows present, provisional ones included.  Never beyond the cache: once an open chunk has filled it, or when
    // the caller's cache_len exceeds cap, the rows that exist are [0, cap) and later tokens are not stored.
    const int n_want = cache_len[bh] + pos;
    const int n_old = min(max(n_want, 0), cap);
    const bool append = is_softmax && n_want >= 0 && n_want < cap;
    __syncthreads();

    // ---- phase A: state update and o_la = la_scale * S q --------------------------------
    {
        const int lr = tid % LPR, r0 = tid / LPR;
        float* Sb = state + (size_t)bh * D * D;
        float4 S4[PASSES];
#pragma unroll
        for (int p = 0; p < PASSES; ++p)
            S4[p] = *reinterpret_cast<const float4*>(Sb + (size_t)(p * ROWS_PER_PASS + r0) * D + lr * 4);
        const float4 k4 = *reinterpret_cast<const float4*>(&s_k[lr * 4]);
        const float4 q4 = *reinterpret_cast<const float4*>(&s_q[lr * 4]);
        if (CHUNK && pos == 0) {   // first token of a chunk: keep the state it starts from
            float* Sst = state_start + (size_t)bh * D * D;
#pragma unroll
            for (int p = 0; p < PASSES; ++p)
                *reinterpret_cast<float4*>(Sst + (size_t)(p * ROWS_PER_PASS + r0) * D + lr * 4) = S4[p];
        }
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int row = p * ROWS_PER_PASS + r0;
            float4 s = S4[p];
            s.x *= a; s.y *= a; s.z *= a; s.w *= a;
            if (b != 0.f) {
                const float pred = lane_group_sum<LPR>(s.x * k4.x + s.y * k4.y + s.z * k4.z + s.w * k4.w);
                const float delta = b * (s_v[row] - (linear_op == 0 ? pred : 0.f));   // no correction without the delta rule
                s.x += delta * k4.x; s.y += delta * k4.y; s.z += delta * k4.z; s.w += delta * k4.w;
            }
            const float oq = lane_group_sum<LPR>(s.x * q4.x + s.y * q4.y + s.z * q4.z + s.w * q4.w);
            if (lr == 0) s_ola[row] = la_scale * oq;
            *reinterpret_cast<float4*>(Sb + (size_t)row * D + lr * 4) = s;
        }
    }

    // ---- phase B: softmax over the cache (+ the new token) ---------------------------------
    const int lk = tid % LPK, sg = tid / LPK;
    float qf[EPL], acc[EPL];
#pragma unroll
    for (int j = 0; j < EPL; ++j) { qf[j] = s_qn[lk * EPL + j] * scale; acc[j] = 0.f; }
    float m_run = -INFINITY, l_run = 0.f;
    const T* Kb = k_cache + (size_t)bh * cap * D + lk * EPL;
    const T* Vb = v_cache + (size_t)bh * cap * D + lk * EPL;

    for (int c0 = sg; c0 < n_old; c0 += NSG * UNROLL) {
        float kf[UNROLL][EPL], vf[UNROLL][EPL], s[UNROLL];
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int c = c0 + u * NSG;
            if (c < n_old) {
                Vec16<T>::load(Kb + (size_t)c * D, kf[u]);
                Vec16<T>::load(Vb + (size_t)c * D, vf[u]);
            } else {
#pragma unroll
                for (int j = 0; j < EPL; ++j) { kf[u][j] = 0.f; vf[u][j] = 0.f; }
            }
        }
        float bm = -INFINITY;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float dot = 0.f;
#pragma unroll
            for (int j = 0; j < EPL; ++j) dot += qf[j] * kf[u][j];
            dot = lane_group_sum<LPK>(dot);
            s[u] = (c0 + u * NSG < n_old) ? dot : -INFINITY;
            bm = fmaxf(bm, s[u]);
        }
        const float m_new = fmaxf(m_run, bm);   // finite: key c0 is live
        const float corr = expf(m_run - m_new);
        l_run *= corr;
#pragma unroll
        for (int j = 0; j < EPL; ++j) acc[j] *= corr;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const float p = expf(s[u] - m_new);
            l_run += p;
#pragma unroll
            for (int j = 0; j < EPL; ++j) acc[j] += p * vf[u][j];
        }
        m_run = m_new;
    }
    if (append && sg == 0) {   // the new softmax token attends to itself
        float dot = 0.f;
#pragma unroll
        for (int j = 0; j < EPL; ++j) dot += qf[j] * s_kn[lk * EPL + j];
        dot = lane_group_sum<LPK>(dot);
        const float m_new = fmaxf(m_run, dot);
        const float corr = expf(m_run - m_new);
        const float p = expf(dot - m_new);
        l_run = l_run * corr + p;
#pragma unroll
        for (int j = 0; j < EPL; ++j) acc[j] = acc[j] * corr + p * s_v[lk * EPL + j];
        m_run = m_new;
    }
    if (lk == 0) { s_m[sg] = m_run; s_l[sg] = l_run; }
#pragma unroll
    for (int j = 0; j < EPL; ++j) s_acc[sg][lk * EPL + j] = acc[j];
    __syncthreads();

    // ---- append the new token to the cache -------------------------------------------------
    if (append) {
        for (int c = tid; c < D; c += DEC_THREADS) {
            k_cache[((size_t)bh * cap + n_old) * D + c] = (k_nla != nullptr ? k_nla : k)[(size_t)bh * D + c];
            v_cache[((size_t)bh * cap + n_old) * D + c] = v[(size_t)bh * D + c];
        }
        if (tid == 0 && !CHUNK) cache_len[bh] = n_old + 1;
    }
    if (CHUNK && tid == 0) {
        chunk_pos[bh] = pos + 1;
        chunk_decay[bh] = (pos == 0 ? 1.f : chunk_decay[bh]) * a;
    }
    if (tid == 0 && err_flags != nullptr) err_flags[bh] = (is_softmax && !append) ? 1 : 0;

    // ---- merge the key groups, then the two branches (threads 0..D-1, one output each) --------
    // D <= 128 <= 2 wavefronts; row statistics for Eq. 21 go through LDS.
    __shared__ float s_red[4];
    float o_nla = 0.f, o_la = 0.f;
    if (tid < D) {
        float M = -INFINITY;
#pragma unroll
        for (int g = 0; g < NSG; ++g) M = fmaxf(M, s_m[g]);
        float num = 0.f, den = 0.f;
        if (M > -INFINITY) {
#pragma unroll
            for (int g = 0; g < NSG; ++g) {
                const float wgt = expf(s_m[g] - M);   // groups that saw no key have m = -inf -> 0
                num += wgt * s_acc[g][tid];
                den += wgt * s_l[g];
            }
            o_nla = num / den;
        }
        o_la = s_ola[tid];
    }
    if (combine_mode == 0) {
        if (tid < D) o[(size_t)bh * D + tid] = from_float<T>(o_la + o_nla);
    } else if (combine_mode == 2) {   // one normalisation of the (weighted) sum
        const float sum = (w_nla ? w_nla[bh] : 1.f) * o_nla + (w_la ? w_la[bh] : 1.f) * o_la;
        float x = (tid < D) ? sum * sum : 0.f;
        x = lane_group_sum<64>(x);
        if ((tid & 63) == 0 && tid < 128) s_red[tid >> 6] = x;
        __syncthreads();
        if (tid < D) {
            const float ss = s_red[0] + (D > 64 ? s_red[1] : 0.f);
            o[(size_t)bh * D + tid] = from_float<T>(sum / sqrtf(ss / D + eps));
        }
    } else {
        float x = (tid < D) ? o_la * o_la : 0.f, y = (tid < D) ? o_nla * o_nla : 0.f;
        x = lane_group_sum<64>(x); y = lane_group_sum<64>(y);
        if ((tid & 63) == 0 && tid < 128) { s_red[(tid >> 6) * 2] = x; s_red[(tid >> 6) * 2 + 1] = y; }
        __syncthreads();
        if (tid < D) {
            const float ss_la = s_red[0] + (D > 64 ? s_red[2] : 0.f);
            const float ss_nla = s_red[1] + (D > 64 ? s_red[3] : 0.f);
            const float wn = (w_nla ? w_nla[bh] : 0.5f) / sqrtf(ss_nla / D + eps);
            const float wl = (w_la ? w_la[bh] : 0.5f) / sqrtf(ss_la / D + eps);
            o[(size_t)bh * D + tid] = from_float<T>(wn * o_nla + wl * o_la);
        }
    }
}

// ------------------------------------------------------------------------------------------------------------
// The same step (routing per token) as many small blocks of equal size, for batches whose caches differ in
// length: with one block per (batch, head) the longest caches set the time of the step while most CUs idle.
//   decode_split_kernel   grid (D / DSP_SROWS + n_split, B*H): the first D / DSP_SROWS blocks of a (batch, head)
//                         each update DSP_SROWS rows of the state (rows are independent) and leave their part
//                         of o_la in the workspace; block D / DSP_SROWS + s runs the online softmax over cache
//                         rows [s DSP_ROWS, (s + 1) DSP_ROWS) (exits at once if the cache ends before them) and
//                         leaves (acc[D], max, sum) in the workspace;
//   decode_combine_kernel one block per (batch, head): merges the partial softmax results and the new token
//                         (from registers), merges the branches, appends the token, stores o.
// Workspace per (batch, head): n_split x (D + 4) floats of partial results, then D floats of o_la.
// ------------------------------------------------------------------------------------------------------------
constexpr int DSP_ROWS = 256;    // cache rows per block
constexpr int DSP_SROWS = 32;    // state rows per block

template <typename T, int D>
__global__ __launch_bounds__(DEC_THREADS) void decode_split_kernel(
    float* __restrict__ state, const T* __restrict__ k_cache, const T* __restrict__ v_cache,
    const int32_t* __restrict__ cache_len, const T* __restrict__ q, const T* __restrict__ k,
    const T* __restrict__ v, const float* __restrict__ alpha, const float* __restrict__ beta,
    const uint8_t* __restrict__ mask, float* __restrict__ ws, int cap, int n_split, float scale, float la_scale,
    int linear_op, int freeze_on_softmax, const T* __restrict__ q_nla) {
    constexpr int NSP = D / DSP_SROWS;            // state blocks per (batch, head)
    constexpr int LPR = D / 4;                    // lanes per state row
    constexpr int ROWS_PER_PASS = DEC_THREADS / LPR;
    constexpr int PASSES = DSP_SROWS / ROWS_PER_PASS;
    constexpr int EPL = Vec16<T>::N;
    constexpr int LPK = D / EPL;
    constexpr int NSG = DEC_THREADS / LPK;
    constexpr int UNROLL = 4;
    const int bh = blockIdx.y, tid = threadIdx.x;
    float* wsb = ws + (size_t)bh * ((size_t)n_split * (D + 4) + D);

    if (blockIdx.x < NSP) {   // ---- state rows [part * DSP_SROWS, + DSP_SROWS) ----
        const int lr = tid % LPR, r0 = tid / LPR, row0 = blockIdx.x * DSP_SROWS;
        float* Sb = state + (size_t)bh * D * D;
        float4 S4[PASSES];
#pragma unroll
        for (int p = 0; p < PASSES; ++p)
            S4[p] = *reinterpret_cast<const float4*>(Sb + (size_t)(row0 + p * ROWS_PER_PASS + r0) * D + lr * 4);
        const bool is_softmax = mask[bh] != 0;
        const float a = (is_softmax && freeze_on_softmax) ? 1.f : alpha[bh];
        const float b = is_softmax ? 0.f : beta[bh];
        float kk[4], qq[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            kk[j] = to_float(k[(size_t)bh * D + lr * 4 + j]);
            qq[j] = to_float(q[(size_t)bh * D + lr * 4 + j]);
        }
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            const int row = row0 + p * ROWS_PER_PASS + r0;
            float4 s = S4[p];
            s.x *= a; s.y *= a; s.z *= a; s.w *= a;
            if (b != 0.f) {
                const float pred = lane_group_sum<LPR>(s.x * kk[0] + s.y * kk[1] + s.z * kk[2] + s.w * kk[3]);
                const float delta = b * (to_float(v[(size_t)bh * D + row]) - (linear_op == 0 ? pred : 0.f));
                s.x += delta * kk[0]; s.y += delta * kk[1]; s.z += delta * kk[2]; s.w += delta * kk[3];
            }
            const float oq = lane_group_sum<LPR>(s.x * qq[0] + s.y * qq[1] + s.z * qq[2] + s.w * qq[3]);
            if (lr == 0) wsb[(size_t)n_split * (D + 4) + row] = la_scale * oq;
            *reinterpret_cast<float4*>(Sb + (size_t)row * D + lr * 4) = s;
        }
        return;
    }

    // ---- cache rows [split * DSP_ROWS, ...) of the rows present ----
    const int split = blockIdx.x - NSP;
    const int n_old = min(max(cache_len[bh], 0), cap);
    const int c_lo = split * DSP_ROWS, c_hi = min(c_lo + DSP_ROWS, n_old);
    if (c_lo >= c_hi) return;   // uniform: the combine kernel knows which parts exist from the same length
    __shared__ float s_m[NSG], s_l[NSG];
    __shared__ float s_acc[NSG][D];
    const int lk = tid % LPK, sg = tid / LPK;
    float qf[EPL], acc[EPL];
    {
        const T* qs = (q_nla != nullptr ? q_nla : q) + (size_t)bh * D + lk * EPL;
#pragma unroll
        for (int j = 0; j < EPL; ++j) { qf[j] = to_float(qs[j]) * scale; acc[j] = 0.f; }
    }
    float m_run = -INFINITY, l_run = 0.f;
    const T* Kb = k_cache + (size_t)bh * cap * D + lk * EPL;
    const T* Vb = v_cache + (size_t)bh * cap * D + lk * EPL;
    // Rows as they come from memory (16 bytes of a row per lane); the next group of rows is asked for before the
    // current one is used, so that a wavefront always has loads in flight.
    typedef uint4 raw_t;
    static_assert(sizeof(T) * EPL == 16, "one 16-byte word per lane and row");
    auto load_rows = [&](int c0, raw_t (&kr)[UNROLL], raw_t (&vr)[UNROLL]) {
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const int c = min(c0 + u * NSG, c_hi - 1);   // rows past the end repeat the last one; masked below
            kr[u] = *reinterpret_cast<const raw_t*>(Kb + (size_t)c * D);
            vr[u] = *reinterpret_cast<const raw_t*>(Vb + (size_t)c * D);
        }
    };
    auto use_rows = [&](int c0, const raw_t (&kr)[UNROLL], const raw_t (&vr)[UNROLL]) {
        float sc[UNROLL], bm = -INFINITY;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            float kf[EPL];
            Vec16<T>::unpack(kr[u], kf);
            float dot = 0.f;
#pragma unroll
            for (int j = 0; j < EPL; ++j) dot += qf[j] * kf[j];
            dot = lane_group_sum<LPK>(dot);
            sc[u] = (c0 + u * NSG < c_hi) ? dot : -INFINITY;
            bm = fmaxf(bm, sc[u]);
        }
        const float m_new = fmaxf(m_run, bm);   // finite: row c0 exists
        const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * 1.44269504088896341f);   // exp2(-inf) = 0
        l_run *= corr;
#pragma unroll
        for (int j = 0; j < EPL; ++j) acc[j] *= corr;
#pragma unroll
        for (int u = 0; u < UNROLL; ++u) {
            const float pw = __builtin_amdgcn_exp2f((sc[u] - m_new) * 1.44269504088896341f);
            l_run += pw;
            float vf[EPL];
            Vec16<T>::unpack(vr[u], vf);
#pragma unroll
            for (int j = 0; j < EPL; ++j) acc[j] += pw * vf[j];
        }
        m_run = m_new;
    };
    {
        raw_t ka[UNROLL], va[UNROLL], kb2[UNROLL], vb2[UNROLL];
        constexpr int STEP = NSG * UNROLL;
        int c0 = c_lo + sg;
        if (c0 < c_hi) load_rows(c0, ka, va);
        while (c0 < c_hi) {
            if (c0 + STEP < c_hi) load_rows(c0 + STEP, kb2, vb2);
            use_rows(c0, ka, va);
            c0 += STEP;
            if (c0 >= c_hi) break;
            if (c0 + STEP < c_hi) load_rows(c0 + STEP, ka, va);
            use_rows(c0, kb2, vb2);
            c0 += STEP;
        }
    }
    if (lk == 0) { s_m[sg] = m_run; s_l[sg] = l_run; }
#pragma unroll
    for (int j = 0; j < EPL; ++j) s_acc[sg][lk * EPL + j] = acc[j];
    __syncthreads();
    if (tid < D) {   // the block's key groups into one partial result, relative to the block's maximum
        float M = -INFINITY;
#pragma unroll
        for (int g = 0; g < NSG; ++g) M = fmaxf(M, s_m[g]);
        float num = 0.f, den = 0.f;
#pragma unroll
        for (int g = 0; g < NSG; ++g) {
            const float wgt = expf(s_m[g] - M);   // groups that saw no row have m = -inf -> 0
            num += wgt * s_acc[g][tid];
            den += wgt * s_l[g];
        }
        float* part = wsb + (size_t)split * (D + 4);
        part[tid] = num;
        if (tid == 0) { part[D] = M; part[D + 1] = den; }
    }
}

template <typename T, int D>
__global__ __launch_bounds__(128) void decode_combine_kernel(
    const float* __restrict__ ws, T* __restrict__ k_cache, T* __restrict__ v_cache, int32_t* __restrict__ cache_len,
    const T* __restrict__ q, const T* __restrict__ k, const T* __restrict__ v, const uint8_t* __restrict__ mask,
    const float* __restrict__ w_nla, const float* __restrict__ w_la, T* __restrict__ o,
    int32_t* __restrict__ err_flags, int cap, int n_split, float scale, int combine_mode, float eps,
    const T* __restrict__ q_nla, const T* __restrict__ k_nla) {
    const int bh = blockIdx.x, tid = threadIdx.x;
    const float* wsb = ws + (size_t)bh * ((size_t)n_split * (D + 4) + D);
    __shared__ float s_red[4];
    const bool is_softmax = mask[bh] != 0;
    const int n_want = cache_len[bh];
    const int n_old = min(max(n_want, 0), cap);
    const bool append = is_softmax && n_want >= 0 && n_want < cap;
    const int n_parts = (n_old + DSP_ROWS - 1) / DSP_ROWS;
    const bool live = tid < D;
    const T* qs = q_nla != nullptr ? q_nla : q;
    const T* ks = k_nla != nullptr ? k_nla : k;
    // logit of the new token (it attends to itself, Eq. 12 i >= j)
    float dot = 0.f;
    if (append) {
        float x = live ? to_float(qs[(size_t)bh * D + tid]) * scale * to_float(ks[(size_t)bh * D + tid]) : 0.f;
        x = lane_group_sum<64>(x);
        if ((tid & 63) == 0) s_red[tid >> 6] = x;
        __syncthreads();
        dot = s_red[0] + (D > 64 ? s_red[1] : 0.f);
        __syncthreads();
    }
    // maxima and sums of the parts: loaded side by side (one per thread), then shared
    __shared__ float s_pm[128], s_pl[128];
    if (tid < n_parts) {
        s_pm[tid] = wsb[(size_t)tid * (D + 4) + D];
        s_pl[tid] = wsb[(size_t)tid * (D + 4) + D + 1];
    }
    __syncthreads();
    float M = append ? dot : -INFINITY;
    for (int sp = 0; sp < n_parts; ++sp) M = fmaxf(M, s_pm[sp]);
    float o_nla = 0.f, o_la = 0.f;
    if (live) {
        o_la = wsb[(size_t)n_split * (D + 4) + tid];
        if (M > -INFINITY) {
            float num = 0.f, den = 0.f;
#pragma unroll 4
            for (int sp = 0; sp < n_parts; ++sp) {   // the loads do not depend on each other
                const float wgt = expf(s_pm[sp] - M);
                num += wgt * wsb[(size_t)sp * (D + 4) + tid];
                den += wgt * s_pl[sp];
            }
            if (append) {
                const float pw = expf(dot - M);
                num += pw * to_float(v[(size_t)bh * D + tid]);
                den += pw;
            }
            o_nla = num / den;
        }
    }
    // ---- append the new token, bookkeeping ----
    if (append && live) {
        k_cache[((size_t)bh * cap + n_old) * D + tid] = ks[(size_t)bh * D + tid];
        v_cache[((size_t)bh * cap + n_old) * D + tid] = v[(size_t)bh * D + tid];
    }
    if (tid == 0) {
        if (append) cache_len[bh] = n_old + 1;
        if (err_flags != nullptr) err_flags[bh] = (is_softmax && !append) ? 1 : 0;
    }
    // ---- merge of the branches ----
    if (combine_mode == 0) {
        if (live) o[(size_t)bh * D + tid] = from_float<T>(o_la + o_nla);
    } else if (combine_mode == 2) {   // one normalisation of the (weighted) sum
        const float sum = (w_nla ? w_nla[bh] : 1.f) * o_nla + (w_la ? w_la[bh] : 1.f) * o_la;
        float x = live ? sum * sum : 0.f;
        x = lane_group_sum<64>(x);
        if ((tid & 63) == 0) s_red[tid >> 6] = x;
        __syncthreads();
        if (live) {
            const float ss = s_red[0] + (D > 64 ? s_red[1] : 0.f);
            o[(size_t)bh * D + tid] = from_float<T>(sum / sqrtf(ss / D + eps));
        }
    } else {
        float x = live ? o_la * o_la : 0.f, y = live ? o_nla * o_nla : 0.f;
        x = lane_group_sum<64>(x); y = lane_group_sum<64>(y);
        if ((tid & 63) == 0) { s_red[(tid >> 6) * 2] = x; s_red[(tid >> 6) * 2 + 1] = y; }
        __syncthreads();
        if (live) {
            const float ss_la = s_red[0] + (D > 64 ? s_red[2] : 0.f);
            const float ss_nla = s_red[1] + (D > 64 ? s_red[3] : 0.f);
            const float wn = (w_nla ? w_nla[bh] : 0.5f) / sqrtf(ss_nla / D + eps);
            const float wl = (w_la ? w_la[bh] : 0.5f) / sqrtf(ss_la / D + eps);
            o[(size_t)bh * D + tid] = from_float<T>(wn * o_nla + wl * o_la);
        }
    }
}

// After a chunk has been seen and its type decided (mask_c[b,h] != 0: softmax chunk): a softmax chunk keeps
// its provisional cache rows and gives the state back as (chunk decay) x (chunk-start state); a linear
// chunk keeps the state and drops the rows.  chunk_pos returns to 0.  err_flags (optional) is set where
// rows of a softmax chunk did not fit into the cache (they were never stored).
template <int D>
__global__ __launch_bounds__(DEC_THREADS) void decode_commit_kernel(
    float* __restrict__ state, const float* __restrict__ state_start, const float* __restrict__ chunk_decay,
    int32_t* __restrict__ chunk_pos, int32_t* __restrict__ cache_len, const uint8_t* __restrict__ mask_c,
    int32_t* __restrict__ err_flags, int cap, int freeze_on_softmax) {
    const int bh = blockIdx.x, tid = threadIdx.x;
    const int pos = chunk_pos[bh];
    const bool soft = mask_c[bh] != 0;
    const int n = cache_len[bh];
    if (soft && pos > 0) {
        const float dec = freeze_on_softmax ? 1.f : chunk_decay[bh];   // variant: the state as the chunk found it
        float4* S = reinterpret_cast<float4*>(state + (size_t)bh * D * D);
        const float4* S0 = reinterpret_cast<const float4*>(state_start + (size_t)bh * D * D);
        for (int i = tid; i < D * D / 4; i += DEC_THREADS) {
            const float4 x = S0[i];
            S[i] = make_float4(dec * x.x, dec * x.y, dec * x.z, dec * x.w);
        }
    }
    __syncthreads();   // every thread has read pos and n
    if (tid == 0) {
        if (soft) cache_len[bh] = min(n + pos, cap);
        if (err_flags != nullptr) err_flags[bh] = (soft && n + pos > cap) ? 1 : 0;
        chunk_pos[bh] = 0;
    }
}

template <typename T, bool CHUNK>
static void launch_dec(const nats_dec_params& p, float scale, float la_scale, float eps, float* state,
                       float* state_start, float* chunk_decay, int32_t* chunk_pos,
                       void* k_cache, void* v_cache, int32_t* cache_len, const void* q, const void* k,
                       const void* v, const float* alpha, const float* beta, const uint8_t* mask,
                       const float* w_nla, const float* w_la, void* o, int32_t* err_flags, hipStream_t st) {
    dim3 grid(p.B * p.H);
    if (p.d == 64)
        hipLaunchKernelGGL((decode_kernel<T, 64, CHUNK>), grid, dim3(DEC_THREADS), 0, st, state, state_start,
                           chunk_decay, chunk_pos, (T*)k_cache,
                           (T*)v_cache, cache_len, (const T*)q, (const T*)k, (const T*)v, alpha, beta, mask,
                           w_nla, w_la, (T*)o, err_flags, p.cap, scale, la_scale, p.combine_mode, eps,
                           p.linear_op, p.freeze_on_softmax, (const T*)p.q_nla, (const T*)p.k_nla);
    else
        hipLaunchKernelGGL((decode_kernel<T, 128, CHUNK>), grid, dim3(DEC_THREADS), 0, st, state, state_start,
                           chunk_decay, chunk_pos, (T*)k_cache,
                           (T*)v_cache, cache_len, (const T*)q, (const T*)k, (const T*)v, alpha, beta, mask,
                           w_nla, w_la, (T*)o, err_flags, p.cap, scale, la_scale, p.combine_mode, eps,
                           p.linear_op, p.freeze_on_softmax, (const T*)p.q_nla, (const T*)p.k_nla);
}

nats_status launch_decode(const nats_dec_params& p, float softmax_scale, float la_scale, float eps,
                          float* state, void* k_cache, void* v_cache, int32_t* cache_len, const void* q,
                          const void* k, const void* v, const float* alpha, const float* beta,
                          const uint8_t* mask, const float* w_nla, const float* w_la, void* o,
                          int32_t* err_flags, hipStream_t st) {
    if (p.dtype == NATS_BF16)
        launch_dec<bf16_t, false>(p, softmax_scale, la_scale, eps, state, nullptr, nullptr, nullptr, k_cache, v_cache,
                                  cache_len, q, k, v, alpha, beta, mask, w_nla, w_la, o, err_flags, st);
    else
        launch_dec<float, false>(p, softmax_scale, la_scale, eps, state, nullptr, nullptr, nullptr, k_cache, v_cache,
                                 cache_len, q, k, v, alpha, beta, mask, w_nla, w_la, o, err_flags, st);
    return check_launch("decode");
}

size_t decode_split_workspace_bytes(const nats_dec_params& p) {
    const size_t n_split = ((size_t)p.cap + DSP_ROWS - 1) / DSP_ROWS;
    return (size_t)p.B * p.H * (n_split * (p.d + 4) + p.d) * sizeof(float);
}

template <typename T, int D>
static void launch_dec_split(const nats_dec_params& p, float scale, float la_scale, float eps, float* state,
                             void* k_cache, void* v_cache, int32_t* cache_len, const void* q, const void* k,
                             const void* v, const float* alpha, const float* beta, const uint8_t* mask,
                             const float* w_nla, const float* w_la, void* o, int32_t* err_flags, float* ws,
                             hipStream_t st) {
    const int n_split = (p.cap + DSP_ROWS - 1) / DSP_ROWS;
    {
        ProfScope ps("decode_split", st);
        hipLaunchKernelGGL((decode_split_kernel<T, D>), dim3(D / DSP_SROWS + n_split, p.B * p.H), dim3(DEC_THREADS), 0, st,
                           state, (const T*)k_cache, (const T*)v_cache, cache_len, (const T*)q, (const T*)k, (const T*)v,
                           alpha, beta, mask, ws, p.cap, n_split, scale, la_scale, p.linear_op, p.freeze_on_softmax,
                           (const T*)p.q_nla);
    }
    ProfScope ps("decode_combine", st);
    hipLaunchKernelGGL((decode_combine_kernel<T, D>), dim3(p.B * p.H), dim3(128), 0, st, ws, (T*)k_cache, (T*)v_cache,
                       cache_len, (const T*)q, (const T*)k, (const T*)v, mask, w_nla, w_la, (T*)o, err_flags, p.cap,
                       n_split, scale, p.combine_mode, eps, (const T*)p.q_nla, (const T*)p.k_nla);
}

nats_status launch_decode_split(const nats_dec_params& p, float softmax_scale, float la_scale, float eps,
                                float* state, void* k_cache, void* v_cache, int32_t* cache_len, const void* q,
                                const void* k, const void* v, const float* alpha, const float* beta,
                                const uint8_t* mask, const float* w_nla, const float* w_la, void* o,
                                int32_t* err_flags, float* ws, hipStream_t st) {
#define NATS_DEC_SPLIT(T, D) launch_dec_split<T, D>(p, softmax_scale, la_scale, eps, state, k_cache, v_cache, cache_len, q, k, \
                                                    v, alpha, beta, mask, w_nla, w_la, o, err_flags, ws, st)
    if (p.dtype == NATS_BF16) { if (p.d == 64) NATS_DEC_SPLIT(bf16_t, 64); else NATS_DEC_SPLIT(bf16_t, 128); }
    else { if (p.d == 64) NATS_DEC_SPLIT(float, 64); else NATS_DEC_SPLIT(float, 128); }
#undef NATS_DEC_SPLIT
    return check_launch("decode (split)");
}

nats_status launch_decode_chunk(const nats_dec_params& p, float softmax_scale, float la_scale, float eps,
                                float* state, float* state_start, float* chunk_decay, int32_t* chunk_pos,
                                void* k_cache, void* v_cache, int32_t* cache_len, const void* q, const void* k,
                                const void* v, const float* alpha, const float* beta, const float* w_nla,
                                const float* w_la, void* o, int32_t* err_flags, hipStream_t st) {
    if (p.dtype == NATS_BF16)
        launch_dec<bf16_t, true>(p, softmax_scale, la_scale, eps, state, state_start, chunk_decay, chunk_pos, k_cache,
                                 v_cache, cache_len, q, k, v, alpha, beta, nullptr, w_nla, w_la, o, err_flags, st);
    else
        launch_dec<float, true>(p, softmax_scale, la_scale, eps, state, state_start, chunk_decay, chunk_pos, k_cache,
                                v_cache, cache_len, q, k, v, alpha, beta, nullptr, w_nla, w_la, o, err_flags, st);
    return check_launch("decode (routing per chunk)");
}

nats_status launch_decode_commit(const nats_dec_params& p, float* state, const float* state_start,
                                 const float* chunk_decay, int32_t* chunk_pos, int32_t* cache_len,
                                 const uint8_t* mask_c, int32_t* err_flags, hipStream_t st) {
    dim3 grid(p.B * p.H);
    if (p.d == 64)
        hipLaunchKernelGGL(decode_commit_kernel<64>, grid, dim3(DEC_THREADS), 0, st, state, state_start, chunk_decay,
                           chunk_pos, cache_len, mask_c, err_flags, p.cap, p.freeze_on_softmax);
    else
        hipLaunchKernelGGL(decode_commit_kernel<128>, grid, dim3(DEC_THREADS), 0, st, state, state_start, chunk_decay,
                           chunk_pos, cache_len, mask_c, err_flags, p.cap, p.freeze_on_softmax);
    return check_launch("decode_commit");
}

}  // namespace nats
