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
// (U ready, S ready) and one for the staged operands.
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
    static constexpr int o_W = 0;                       // [64][RS]  -W
    static constexpr int o_Q = o_W + CS * RS;           // [64][RS]  Q (fp16)
    static constexpr int o_Kd = o_Q + CS * RS;          // [D][TS]   Kd^T
    static constexpr int o_P = o_Kd + D * TS;           // [64][TS]  P
    static constexpr int o_Ut = o_P + CS * TS;          // [BV][TS]  U~^T slice
    static constexpr int o_S = o_Ut + BV * TS;          // [BV][RS]  state copy, fp16
    static constexpr int o_U = o_S + BV * RS;           // [BV][TS]  U^T, fp16
    static constexpr int n_half = o_U + BV * TS;
    static constexpr size_t bytes = (size_t)n_half * sizeof(half_t) + CS * sizeof(float);
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
    half_t* Ws = sh + Lds::o_W;
    half_t* Qs = sh + Lds::o_Q;
    half_t* Kds = sh + Lds::o_Kd;
    half_t* Ps = sh + Lds::o_P;
    half_t* Uts = sh + Lds::o_Ut;
    half_t* Ss = sh + Lds::o_S;
    half_t* Us = sh + Lds::o_U;
    float* s_gam = reinterpret_cast<float*>(sh + Lds::n_half);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l16 = lane & 15, lq = lane >> 4;
    const int bh = blockIdx.y;
    const int v0 = blockIdx.x * BV;
    const int n_chunks = L / CS;

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

    for (int c = 0; c < n_chunks; ++c) {
        const size_t gc = (size_t)bh * n_chunks + c;
        const size_t tok0 = (size_t)bh * L + (size_t)c * CS;
        // ---- stage this chunk's operands into LDS ------------------------------------------
        {
            const half_t* Wc = Wneg + gc * (size_t)(CS * D);
            const bf16_t* Qc = Q + tok0 * D;
            for (int e = tid; e < CS * D / 8; e += SCAN_THREADS_G) {
                const int row = e / (D / 8), c8 = e % (D / 8);
                *reinterpret_cast<uint4*>(Ws + row * RS + c8 * 8) =
                    *reinterpret_cast<const uint4*>(Wc + row * D + c8 * 8);
                *reinterpret_cast<half8*>(Qs + row * RS + c8 * 8) =
                    bf16x8_to_half8(*reinterpret_cast<const uint4*>(Qc + row * D + c8 * 8));
            }
            const half_t* Kc = KdT + gc * (size_t)(D * CS);
            for (int e = tid; e < D * CS / 8; e += SCAN_THREADS_G) {
                const int row = e >> 3, c8 = e & 7;
                *reinterpret_cast<uint4*>(Kds + row * TS + c8 * 8) =
                    *reinterpret_cast<const uint4*>(Kc + row * CS + c8 * 8);
            }
            const half_t* Pc = P + gc * (size_t)(CS * CS);
            for (int e = tid; e < CS * CS / 8; e += SCAN_THREADS_G) {
                const int row = e >> 3, c8 = e & 7;
                *reinterpret_cast<uint4*>(Ps + row * TS + c8 * 8) =
                    *reinterpret_cast<const uint4*>(Pc + row * CS + c8 * 8);
            }
            const half_t* Uc = UtT + gc * (size_t)(D * CS) + (size_t)v0 * CS;
            for (int e = tid; e < BV * CS / 8; e += SCAN_THREADS_G) {
                const int row = e >> 3, c8 = e & 7;
                *reinterpret_cast<uint4*>(Uts + row * TS + c8 * 8) =
                    *reinterpret_cast<const uint4*>(Uc + row * CS + c8 * 8);
            }
            if (tid < CS) s_gam[tid] = gam[gc * CS + tid];
        }
        __syncthreads();

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
        __syncthreads();   // U complete; every wavefront has read the old state copy

        // ---- phase 2: O += P U ; S^T = gam_C S^T + Kd^T U ---------------------------------------
        half8 fu[2][NT];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) fu[ks][nt] = lds_read8(Us + (16 * nt + l16) * TS + 32 * ks + 8 * lq);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            if (ks <= mt / 2) {   // P is lower triangular: tokens beyond this tile's rows contribute nothing
                const half8 fp = lds_read8(Ps + (16 * mt + l16) * TS + 32 * ks + 8 * lq);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) accO[nt] = mfma16(fp, fu[ks][nt], accO[nt]);
            }
        }
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
        // linear-branch output rows of this wavefront's tokens, columns of this block's slice
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                O_la[(tok0 + 16 * mt + 4 * lq + j) * D + v0 + 16 * nt + l16] = la_scale * accO[nt][j];
        __syncthreads();   // new state copy visible; staged operands free to be overwritten
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
