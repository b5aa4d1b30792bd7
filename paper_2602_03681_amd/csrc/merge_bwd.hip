// Adjoint of the normalised, weighted merges of the two branches' output rows (Eq. 21; Section 5, ablation (iii)).
//   mode 1:  O = w_nla RMSNorm(o_nla) + w_la RMSNorm(o_la)        mode 2:  O = RMSNorm(w_nla o_nla + w_la o_la)
// with RMSNorm(x) = x r, r = (mean(x^2) + eps)^(-1/2), no gain.  For y = x r and a gradient dy of y:
//   dx = r (dy - y (y . dy) / d).
// The merge acts row by row, so the kernel turns dO into one gradient per branch (each branch's backward then runs on
// its own, as for the plain sum) and gives the gradients of the two weights.  fp32 throughout; a row is held by d / 4
// adjacent lanes, four columns each.  Streams three rows in and two out: HBM-bound.
// Also here: the widening copy bf16 -> fp32 that the backward pass with these merges runs on its inputs (the
// branches then receive fp32 gradients of their outputs, which the kernels for bf16 tensors do not take).
#include "nats_common.h"

namespace nats {

constexpr int MB_THREADS = 256;

template <int D>
__global__ __launch_bounds__(MB_THREADS) void merge_bwd_kernel(
    const float* __restrict__ O_la, const float* __restrict__ O_nla, const float* __restrict__ dO,
    const float* __restrict__ w_nla, const float* __restrict__ w_la, float* __restrict__ dO_la,
    float* __restrict__ dO_nla, float* __restrict__ dw_nla, float* __restrict__ dw_la, size_t n_rows, int mode,
    float eps) {
    constexpr int W = D / 4;                   // lanes per row
    constexpr int ROWS = MB_THREADS / W;       // rows per block and trip
    const int sub = threadIdx.x % W, r_in = threadIdx.x / W;
    const float inv_d = 1.0f / (float)D;
    const float w_default = mode == 2 ? 1.0f : 0.5f;
    // every lane of a row's group runs every trip (the sums below are over the group): a row index past the end
    // is clamped for the loads and its stores are skipped
    const size_t trips = (n_rows + (size_t)gridDim.x * ROWS - 1) / ((size_t)gridDim.x * ROWS);
    for (size_t t = 0; t < trips; ++t) {
        const size_t row_raw = (t * gridDim.x + blockIdx.x) * ROWS + r_in;
        const bool live = row_raw < n_rows;
        const size_t row = live ? row_raw : n_rows - 1;
        const size_t off = row * D + 4 * sub;
        const float4 xl4 = *reinterpret_cast<const float4*>(O_la + off);
        const float4 xn4 = *reinterpret_cast<const float4*>(O_nla + off);
        const float4 g4 = *reinterpret_cast<const float4*>(dO + off);
        const float wn = w_nla ? w_nla[row] : w_default, wl = w_la ? w_la[row] : w_default;
        const float xl[4] = {xl4.x, xl4.y, xl4.z, xl4.w}, xn[4] = {xn4.x, xn4.y, xn4.z, xn4.w};
        const float g[4] = {g4.x, g4.y, g4.z, g4.w};
        float dl[4], dn[4], gwn, gwl;
        if (mode == 2) {
            float z[4], ss = 0.f, zg = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                z[j] = wn * xn[j] + wl * xl[j];
                ss += z[j] * z[j];
                zg += z[j] * g[j];
            }
            ss = lane_group_sum<W>(ss);
            zg = lane_group_sum<W>(zg);
            const float r = 1.0f / sqrtf(ss * inv_d + eps);
            const float c = r * r * zg * inv_d;          // (y . dO) / d  times r, folded: y = z r
            float sn = 0.f, sl = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const float dz = r * (g[j] - z[j] * c);  // r (dO - y (y . dO) / d)
                dn[j] = wn * dz;
                dl[j] = wl * dz;
                sn += dz * xn[j];
                sl += dz * xl[j];
            }
            gwn = lane_group_sum<W>(sn);
            gwl = lane_group_sum<W>(sl);
        } else {
            float ssn = 0.f, ssl = 0.f, ng = 0.f, lg = 0.f;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                ssn += xn[j] * xn[j];
                ssl += xl[j] * xl[j];
                ng += xn[j] * g[j];
                lg += xl[j] * g[j];
            }
            ssn = lane_group_sum<W>(ssn);
            ssl = lane_group_sum<W>(ssl);
            ng = lane_group_sum<W>(ng);
            lg = lane_group_sum<W>(lg);
            const float rn = 1.0f / sqrtf(ssn * inv_d + eps), rl = 1.0f / sqrtf(ssl * inv_d + eps);
            gwn = rn * ng;                               // dO . RMSNorm(o_nla)
            gwl = rl * lg;
            const float cn = rn * gwn * inv_d, cl = rl * gwl * inv_d;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                dn[j] = wn * rn * (g[j] - xn[j] * cn);
                dl[j] = wl * rl * (g[j] - xl[j] * cl);
            }
        }
        if (live) {
            *reinterpret_cast<float4*>(dO_la + off) = make_float4(dl[0], dl[1], dl[2], dl[3]);
            *reinterpret_cast<float4*>(dO_nla + off) = make_float4(dn[0], dn[1], dn[2], dn[3]);
            if (sub == 0) {
                if (dw_nla) dw_nla[row] = gwn;
                if (dw_la) dw_la[row] = gwl;
            }
        }
    }
}

// dst[i] = (float) src[i], eight elements per thread and trip; n8 = n / 8
__global__ __launch_bounds__(MB_THREADS) void widen_bf16_kernel(const bf16_t* __restrict__ src, float* __restrict__ dst,
                                                               size_t n8) {
    for (size_t e = (size_t)blockIdx.x * MB_THREADS + threadIdx.x; e < n8; e += (size_t)gridDim.x * MB_THREADS) {
        float x[8];
        Vec16<bf16_t>::load(src + 8 * e, x);
        *reinterpret_cast<float4*>(dst + 8 * e) = make_float4(x[0], x[1], x[2], x[3]);
        *reinterpret_cast<float4*>(dst + 8 * e + 4) = make_float4(x[4], x[5], x[6], x[7]);
    }
}

static int mb_grid(size_t units) {
    const size_t blocks = (units + MB_THREADS - 1) / MB_THREADS;
    return (int)(blocks < 1 ? 1 : (blocks > 4096 ? 4096 : blocks));
}

// rows: B x H x L rows of pl.d columns (pl.d is 64 or 128).  dw_nla, dw_la may be NULL (not wanted).
nats_status launch_merge_bwd(const FwdPlan& pl, int mode, float eps, const float* O_la, const float* O_nla,
                             const float* dO, const float* w_nla, const float* w_la, float* dO_la, float* dO_nla,
                             float* dw_nla, float* dw_la, hipStream_t st) {
    const size_t n_rows = (size_t)pl.BH * pl.L;
    if (n_rows == 0) return NATS_OK;
    if (pl.d == 64)
        hipLaunchKernelGGL(merge_bwd_kernel<64>, dim3(mb_grid(n_rows * 16)), dim3(MB_THREADS), 0, st, O_la, O_nla, dO,
                           w_nla, w_la, dO_la, dO_nla, dw_nla, dw_la, n_rows, mode, eps);
    else
        hipLaunchKernelGGL(merge_bwd_kernel<128>, dim3(mb_grid(n_rows * 32)), dim3(MB_THREADS), 0, st, O_la, O_nla, dO,
                           w_nla, w_la, dO_la, dO_nla, dw_nla, dw_la, n_rows, mode, eps);
    return check_launch("merge_bwd");
}

// n: a multiple of 8 (whole rows of 64 or 128 columns)
nats_status launch_widen_bf16(const void* src, float* dst, size_t n, hipStream_t st) {
    if (n == 0) return NATS_OK;
    hipLaunchKernelGGL(widen_bf16_kernel, dim3(mb_grid(n / 8)), dim3(MB_THREADS), 0, st, (const bf16_t*)src, dst, n / 8);
    return check_launch("widen_bf16");
}

}  // namespace nats
