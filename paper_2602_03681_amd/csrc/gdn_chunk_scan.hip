// Chunkwise Gated DeltaNet, step 2 of 2: the recurrence over chunks (Section 3, Eq. 6-7;
// update rule Eq. 19 with Eq. 14 / Eq. 20 folded into the per-chunk operands).
// With the per-chunk operands of the preparation kernel (W negated, U~ and Kd transposed):
//   U  = U~ - W S0^T                          [C x d_v]
//   O  = la_scale (diag(gam) Q S0^T + P U)    [C x d_v]   (linear-branch output, Eq. 7 / Eq. 10)
//   S1 = gam_C S0 + U^T Kd                    [d_v x d_k]
// The rows of S (index d_v) never mix, so a block owns a slice of BV values of d_v for one
// (batch, head) and walks the chunks in order; the grid is (d / BV) x (B*H) blocks.
//
// The state lives transposed, S^T [d_k x BV], as fp32 MFMA accumulators spread over the 4
// wavefronts (each owns d_k/4 rows) and never leaves registers in fp32; an fp16 copy
// S[v][d_k] in LDS is the B operand of the two products that read it.  Every operand is laid
// out so that fragments are 16-byte LDS reads along the contraction index and results are
// written back as 4 consecutive fp16.  Per chunk: two block barriers on the dependent chain
// (U ready, S ready).  Operands are software-pipelined: chunk c is read from one of two LDS
// buffers while chunk c+1 moves from registers to the other and chunk c+2 is being loaded.
//
// MFMA work per chunk and block: (2 d + 2 d + 2 C + 2 d) C BV FLOP; the path is bound by the
// length of the dependent chain (L / C steps), not by MFMA throughput.
#include "mfma_util.h"
#include "nats_common.h"

namespace nats {

constexpr int SCAN_THREADS_G = 256;
constexpr int CS = 64;  // chunk size

template <int D, int BV>
struct ScanLds {
    static constexpr int RS = D + LDS_PAD;   // [tok][d] rows
    static constexpr int TS = CS + LDS_PAD;  // [x][tok] rows
    // per-chunk operands, double buffered
    static constexpr int o_W = 0;                       // [64][RS]  -W
    static constexpr int o_Q = o_W + CS * RS;           // [64][RS]  Q (fp16)
    static constexpr int o_Kd = o_Q + CS * RS;          // [D][TS]   Kd^T
    static constexpr int o_P = o_Kd + D * TS;           // [64][TS]  P
    static constexpr int o_Ut = o_P + CS * TS;          // [BV][TS]  U~^T slice
    static constexpr int n_stage = o_Ut + BV * TS;      // halves per buffer
    // carried between the phases of a step
    static constexpr int o_S = 2 * n_stage;             // [BV][RS]  state copy, fp16
    static constexpr int o_U = o_S + BV * RS;           // [BV][TS]  U^T, fp16
    static constexpr int n_half = o_U + BV * TS;
    static constexpr size_t bytes = (size_t)n_half * sizeof(half_t) + 2 * CS * sizeof(float);
};

// One chunk's operands on their way from global memory to LDS, held in registers so that the
// loads of chunk c+2 are in flight while chunk c is computed.
template <int D, int BV>
struct ScanStage {
    static constexpr int NW = CS * D / 8 / SCAN_THREADS_G;   // 16-byte pieces per thread of a [64][D] tile
    static constexpr int NP = CS * CS / 8 / SCAN_THREADS_G;  // ... of the [64][64] tile
    static constexpr int NU = BV * CS / 8;                   // pieces of the U~^T slice (<= 256)
    uint4 w[NW], q[NW], kd[NW], p[NP], ut;
    float g;

    __device__ __forceinline__ void load(const bf16_t* __restrict__ Q, const half_t* __restrict__ Wneg,
                                         const half_t* __restrict__ KdT, const half_t* __restrict__ UtT,
                                         const half_t* __restrict__ P, const float* __restrict__ gam,
                                         size_t gc, size_t tok0, int v0, int tid) {
        const uint4* Wc = reinterpret_cast<const uint4*>(Wneg + gc * (size_t)(CS * D));
        const uint4* Qc = reinterpret_cast<const uint4*>(Q + tok0 * D);
        const uint4* Kc = reinterpret_cast<const uint4*>(KdT + gc * (size_t)(D * CS));
        const uint4* Pc = reinterpret_cast<const uint4*>(P + gc * (size_t)(CS * CS));
        const uint4* Uc = reinterpret_cast<const uint4*>(UtT + gc * (size_t)(D * CS) + (size_t)v0 * CS);
#pragma unroll
        for (int i = 0; i < NW; ++i) {   // the tiles are contiguous in global memory: piece e = tid + 256 i
            w[i] = Wc[tid + SCAN_THREADS_G * i];
            q[i] = Qc[tid + SCAN_THREADS_G * i];
            kd[i] = Kc[tid + SCAN_THREADS_G * i];
        }
#pragma unroll
        for (int i = 0; i < NP; ++i) p[i] = Pc[tid + SCAN_THREADS_G * i];
        if (tid < NU) ut = Uc[tid];
        if (tid < CS) g = gam[gc * CS + tid];
    }

    __device__ __forceinline__ void store(half_t* buf, float* s_gam, int tid) const {
        using Lds = ScanLds<D, BV>;
        constexpr int RS = Lds::RS, TS = Lds::TS;
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const int e = tid + SCAN_THREADS_G * i;
            const int row = e / (D / 8), c8 = e % (D / 8);
            *reinterpret_cast<uint4*>(buf + Lds::o_W + row * RS + c8 * 8) = w[i];
            *reinterpret_cast<half8*>(buf + Lds::o_Q + row * RS + c8 * 8) = bf16x8_to_half8(q[i]);
            *reinterpret_cast<uint4*>(buf + Lds::o_Kd + (e >> 3) * TS + (e & 7) * 8) = kd[i];
        }
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int e = tid + SCAN_THREADS_G * i;
            *reinterpret_cast<uint4*>(buf + Lds::o_P + (e >> 3) * TS + (e & 7) * 8) = p[i];
        }
        if (tid < NU) *reinterpret_cast<uint4*>(buf + Lds::o_Ut + (tid >> 3) * TS + (tid & 7) * 8) = ut;
        if (tid < CS) s_gam[tid] = g;
    }
};

template <int D, int BV>
__global__ __launch_bounds__(SCAN_THREADS_G) void gdn_chunk_scan_kernel(
    const bf16_t* __restrict__ Q, const half_t* __restrict__ Wneg, const half_t* __restrict__ KdT,
    const half_t* __restrict__ UtT, const half_t* __restrict__ P, const float* __restrict__ gam,
    const float* __restrict__ S0, float* __restrict__ S_final, float* __restrict__ O_la, int L,
    float la_scale) {
    using Lds = ScanLds<D, BV>;
    constexpr int RS = Lds::RS, TS = Lds::TS;
    constexpr int NT = BV / 16;       // 16-wide tiles along the d_v slice
    constexpr int MS = D / 64;        // 16-row d_k tiles of S^T owned by one wavefront
    constexpr int KS_D = D / 32;      // contraction steps over d_k
    extern __shared__ __align__(16) unsigned char smem[];
    half_t* sh = reinterpret_cast<half_t*>(smem);
    half_t* Ss = sh + Lds::o_S;
    half_t* Us = sh + Lds::o_U;
    float* s_gam_all = reinterpret_cast<float*>(sh + Lds::n_half);   // [2][64]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    const int bh = blockIdx.y;
    const int v0 = blockIdx.x * BV;
    const int n_chunks = L / CS;
    const size_t gc0 = (size_t)bh * n_chunks;
    const size_t tokb = (size_t)bh * L;

    // ---- state: S^T tiles (rows d_k, cols v) as accumulators ---------------------------------
    f32x4 accS[MS][NT];
#pragma unroll
    for (int ms = 0; ms < MS; ++ms)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int dk = 16 * (MS * wave + ms) + 4 * lq, v = v0 + 16 * nt + l16;
            if (S0 != nullptr) {
                const float4 x = *reinterpret_cast<const float4*>(S0 + ((size_t)bh * D + v) * D + dk);
                accS[ms][nt] = f32x4{x.x, x.y, x.z, x.w};
            } else {
                accS[ms][nt] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
            *reinterpret_cast<half4*>(Ss + (16 * nt + l16) * RS + dk) = to_half4(accS[ms][nt]);
        }

    // ---- software pipeline: chunk c in LDS buffer c&1, chunks c+1 and c+2 in registers ----------
    ScanStage<D, BV> st[2];
    st[0].load(Q, Wneg, KdT, UtT, P, gam, gc0, tokb, v0, tid);
    if (n_chunks > 1) st[1].load(Q, Wneg, KdT, UtT, P, gam, gc0 + 1, tokb + CS, v0, tid);
    st[0].store(sh, s_gam_all, tid);
    __syncthreads();

    auto step = [&](int c, ScanStage<D, BV>& st_far, const ScanStage<D, BV>& st_near) {
        half_t* buf = sh + (c & 1) * Lds::n_stage;
        const half_t* Ws = buf + Lds::o_W;
        const half_t* Qs = buf + Lds::o_Q;
        const half_t* Kds = buf + Lds::o_Kd;
        const half_t* Ps = buf + Lds::o_P;
        const half_t* Uts = buf + Lds::o_Ut;
        const float* s_gam = s_gam_all + (c & 1) * CS;
        const size_t tok0 = tokb + (size_t)c * CS;
        // chunk c+2: global -> registers (its previous content, chunk c, is already in LDS)
        if (c + 2 < n_chunks) st_far.load(Q, Wneg, KdT, UtT, P, gam, gc0 + c + 2, tok0 + 2 * CS, v0, tid);

        // ---- phase 1: this wavefront's 16 tokens: U = U~ - W S0^T and O1 = Q S0^T -------------
        const int mt = wave;
        f32x4 accU[NT], accO[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const half4 u = lds_read4(Uts + (16 * nt + l16) * TS + 16 * mt + 4 * lq);
            accU[nt] = f32x4{(float)u[0], (float)u[1], (float)u[2], (float)u[3]};
            accO[nt] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int ks = 0; ks < KS_D; ++ks) {
            const int ko = 32 * ks + 8 * lq;
            const half8 fw = lds_read8(Ws + (16 * mt + l16) * RS + ko);
            const half8 fq = lds_read8(Qs + (16 * mt + l16) * RS + ko);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const half8 fs = lds_read8(Ss + (16 * nt + l16) * RS + ko);
                accU[nt] = mfma16(fw, fs, accU[nt]);
                accO[nt] = mfma16(fq, fs, accO[nt]);
            }
        }
        {
            const float4 g4 = *reinterpret_cast<const float4*>(s_gam + 16 * mt + 4 * lq);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                accO[nt][0] *= g4.x; accO[nt][1] *= g4.y; accO[nt][2] *= g4.z; accO[nt][3] *= g4.w;
                *reinterpret_cast<half4*>(Us + (16 * nt + l16) * TS + 16 * mt + 4 * lq) = to_half4(accU[nt]);
            }
        }
        const float gam_C = s_gam[CS - 1];
        // chunk c+1: registers -> the other LDS buffer (last read in step c-1, before its final barrier)
        if (c + 1 < n_chunks) st_near.store(sh + ((c + 1) & 1) * Lds::n_stage, s_gam_all + ((c + 1) & 1) * CS, tid);
        __syncthreads();   // U complete; every wavefront has read the old state copy

        // ---- phase 2: O += P U ; S^T = gam_C S^T + Kd^T U ---------------------------------------
        half8 fu[2][NT];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) fu[ks][nt] = lds_read8(Us + (16 * nt + l16) * TS + 32 * ks + 8 * lq);
#pragma unroll
        for (int ms = 0; ms < MS; ++ms) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                accS[ms][nt][0] *= gam_C; accS[ms][nt][1] *= gam_C;
                accS[ms][nt][2] *= gam_C; accS[ms][nt][3] *= gam_C;
            }
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const half8 fk = lds_read8(Kds + (16 * (MS * wave + ms) + l16) * TS + 32 * ks + 8 * lq);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) accS[ms][nt] = mfma16(fk, fu[ks][nt], accS[ms][nt]);
            }
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                *reinterpret_cast<half4*>(Ss + (16 * nt + l16) * RS + 16 * (MS * wave + ms) + 4 * lq) =
                    to_half4(accS[ms][nt]);
        }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            if (ks <= mt / 2) {   // P is lower triangular: tokens beyond this tile's rows contribute nothing
                const half8 fp = lds_read8(Ps + (16 * mt + l16) * TS + 32 * ks + 8 * lq);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) accO[nt] = mfma16(fp, fu[ks][nt], accO[nt]);
            }
        }
        // linear-branch output rows of this wavefront's tokens, columns of this block's slice
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                O_la[(tok0 + 16 * mt + 4 * lq + j) * D + v0 + 16 * nt + l16] = la_scale * accO[nt][j];
        __syncthreads();   // new state copy visible; this step's operand buffer is free again
    };

    for (int c = 0; c < n_chunks; c += 2) {
        step(c, st[0], st[1]);
        if (c + 1 < n_chunks) step(c + 1, st[1], st[0]);
    }

    if (S_final != nullptr) {
#pragma unroll
        for (int ms = 0; ms < MS; ++ms)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int dk = 16 * (MS * wave + ms) + 4 * lq, v = v0 + 16 * nt + l16;
                *reinterpret_cast<float4*>(S_final + ((size_t)bh * D + v) * D + dk) =
                    make_float4(accS[ms][nt][0], accS[ms][nt][1], accS[ms][nt][2], accS[ms][nt][3]);
            }
    }
}

template <int D, int BV>
static nats_status launch_scan_t(const FwdPlan& pl, const void* Q, const void* Wneg, const void* KdT,
                                 const void* UtT, const void* P, const float* gam, const float* S0,
                                 float* S_final, float* O_la, hipStream_t st) {
    auto kern = gdn_chunk_scan_kernel<D, BV>;
    constexpr size_t lds = ScanLds<D, BV>::bytes;
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess)
        return check_launch("gdn_chunk_scan (LDS attribute)");
    dim3 grid(D / BV, pl.BH);
    hipLaunchKernelGGL(kern, grid, dim3(SCAN_THREADS_G), lds, st, (const bf16_t*)Q, (const half_t*)Wneg,
                       (const half_t*)KdT, (const half_t*)UtT, (const half_t*)P, gam, S0, S_final, O_la, pl.L,
                       pl.la_scale);
    return check_launch("gdn_chunk_scan");
}

nats_status launch_gdn_chunk_scan(const FwdPlan& pl, const void* Q, const void* Wneg, const void* KdT,
                                  const void* UtT, const void* P, const float* gam, const float* S0,
                                  float* S_final, float* O_la, hipStream_t st) {
    if (pl.d == 64) return launch_scan_t<64, 16>(pl, Q, Wneg, KdT, UtT, P, gam, S0, S_final, O_la, st);
    return launch_scan_t<128, 32>(pl, Q, Wneg, KdT, UtT, P, gam, S0, S_final, O_la, st);
}

}  // namespace nats
