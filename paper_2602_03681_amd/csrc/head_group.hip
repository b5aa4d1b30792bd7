// Head grouping (Section 4.3) in the backward pass: G output heads (own V, own state) share the Q, K, alpha, beta
// and mask of one linear head, so the gradient of a shared input is the sum of what each of the G heads sends back.
// The backward pass runs once per member of the groups on that member's heads, gathered into contiguous tensors;
// the two kernels here move a member's rows in and out of the [B, H G, ...] tensors and add a member's share onto
// the sums.  Both only stream memory.  (Also here: the zero fill the pass needs when the softmax branch has queries
// and keys of its own, whose gradients are then tensors of their own.)
#include "nats_common.h"

namespace nats {

constexpr int HG_THREADS = 256;

// dst row r <- src row r (rows of row_vec 16-byte pieces, row strides in pieces)
__global__ __launch_bounds__(HG_THREADS) void copy_rows_kernel(const uint4* __restrict__ src, size_t src_stride,
                                                              uint4* __restrict__ dst, size_t dst_stride,
                                                              size_t row_vec, size_t n_rows) {
    const size_t n = row_vec * n_rows;
    for (size_t e = (size_t)blockIdx.x * HG_THREADS + threadIdx.x; e < n; e += (size_t)gridDim.x * HG_THREADS) {
        const size_t r = e / row_vec, c = e % row_vec;
        dst[r * dst_stride + c] = src[r * src_stride + c];
    }
}

// dst += src, n4 pieces of four floats
__global__ __launch_bounds__(HG_THREADS) void add_f32_kernel(float4* __restrict__ dst, const float4* __restrict__ src,
                                                            size_t n4) {
    for (size_t e = (size_t)blockIdx.x * HG_THREADS + threadIdx.x; e < n4; e += (size_t)gridDim.x * HG_THREADS) {
        float4 a = dst[e];
        const float4 b = src[e];
        a.x += b.x;
        a.y += b.y;
        a.z += b.z;
        a.w += b.w;
        dst[e] = a;
    }
}

// the same for any length and alignment
__global__ __launch_bounds__(HG_THREADS) void add_f32_scalar_kernel(float* __restrict__ dst, const float* __restrict__ src,
                                                                   size_t n) {
    for (size_t e = (size_t)blockIdx.x * HG_THREADS + threadIdx.x; e < n; e += (size_t)gridDim.x * HG_THREADS)
        dst[e] += src[e];
}

// dst[i] = 0 (a kernel, not a memset: the call may be part of a captured graph)
__global__ __launch_bounds__(HG_THREADS) void zero_f32_kernel(float* __restrict__ dst, size_t n) {
    for (size_t e = (size_t)blockIdx.x * HG_THREADS + threadIdx.x; e < n; e += (size_t)gridDim.x * HG_THREADS) dst[e] = 0.f;
}

static int hg_grid(size_t n) {
    const size_t blocks = (n + HG_THREADS - 1) / HG_THREADS;
    return (int)(blocks < 1 ? 1 : (blocks > 4096 ? 4096 : blocks));
}

// n_rows rows of row_bytes bytes (a multiple of 16; both buffers 16-byte aligned, strides in bytes, multiples of 16)
nats_status launch_copy_rows(const void* src, size_t src_stride_bytes, void* dst, size_t dst_stride_bytes,
                             size_t row_bytes, size_t n_rows, hipStream_t st) {
    if (row_bytes % 16 || src_stride_bytes % 16 || dst_stride_bytes % 16) {
        set_error("copy_rows: row size and strides must be multiples of 16 bytes");
        return NATS_ERR_SHAPE;
    }
    if (n_rows == 0 || row_bytes == 0) return NATS_OK;
    hipLaunchKernelGGL(copy_rows_kernel, dim3(hg_grid(row_bytes / 16 * n_rows)), dim3(HG_THREADS), 0, st,
                       (const uint4*)src, src_stride_bytes / 16, (uint4*)dst, dst_stride_bytes / 16, row_bytes / 16, n_rows);
    return check_launch("copy_rows");
}

// dst[i] += src[i], i < n
nats_status launch_add_f32(float* dst, const float* src, size_t n, hipStream_t st) {
    if (n == 0) return NATS_OK;
    const bool vec = n % 4 == 0 && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0 && (reinterpret_cast<uintptr_t>(src) & 15u) == 0;
    if (vec)
        hipLaunchKernelGGL(add_f32_kernel, dim3(hg_grid(n / 4)), dim3(HG_THREADS), 0, st, (float4*)dst, (const float4*)src, n / 4);
    else
        hipLaunchKernelGGL(add_f32_scalar_kernel, dim3(hg_grid(n)), dim3(HG_THREADS), 0, st, dst, src, n);
    return check_launch("add_f32");
}

nats_status launch_zero_f32(float* dst, size_t n, hipStream_t st) {
    if (n == 0) return NATS_OK;
    hipLaunchKernelGGL(zero_f32_kernel, dim3(hg_grid(n)), dim3(HG_THREADS), 0, st, dst, n);
    return check_launch("zero_f32");
}

}  // namespace nats
