// Shared device/host helpers for the NAtS-L gfx950 kernels (internal header).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "nats.h"

namespace nats {

// ---- element types ------------------------------------------------------------------
// bf16 is carried as its raw 16 bits; conversions are written out so that the rounding
// (round-to-nearest-even) is the same everywhere and independent of library headers.
struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float to_float(float x) { return x; }
__device__ __forceinline__ float to_float(bf16_t x) { return __uint_as_float(((uint32_t)x.bits) << 16); }

__device__ __forceinline__ uint16_t f32_to_bf16_bits(float f) {
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// two floats -> two bf16 (round to nearest even) in one word, low half first: one instruction on gfx950
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}

// ---- sums across lanes without LDS ------------------------------------------------------------------------
// __shfl_xor compiles to an LDS permute with a wait behind it; a reduction of n steps is n LDS round trips in
// a row.  Inside a 16-lane row the steps below are DPP moves (a modifier of an ordinary vector instruction);
// across rows they are gfx950's row swaps.  Blocks are one-dimensional and a multiple of 64 threads wide.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {   // x of the lane that the DPP control CTRL names
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}
// x of lane ^ 16 / lane ^ 32.  v_permlane16_swap exchanges the odd rows of its first operand with the even rows of
// its second, v_permlane32_swap the upper half of the first with the lower half of the second; given the same
// value twice, one of the two results holds the partner's value, which one depends on the lane's own row / half.
__device__ __forceinline__ float lane_xor16(float x, int lane) {
    const auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(((lane >> 4) & 1) ? r[0] : r[1]);
}
__device__ __forceinline__ float lane_xor32(float x, int lane) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(((lane >> 5) & 1) ? r[0] : r[1]);
}
// sum over aligned groups of W lanes (a power of two), in every lane of the group; fixed order
template <int W>
__device__ __forceinline__ float lane_group_sum(float x) {
    static_assert(W == 1 || W == 2 || W == 4 || W == 8 || W == 16 || W == 32 || W == 64, "group width");
    if (W >= 2) x += dpp_move<0xB1>(x);    // quad_perm [1, 0, 3, 2]
    if (W >= 4) x += dpp_move<0x4E>(x);    // quad_perm [2, 3, 0, 1]
    if (W >= 8) x += dpp_move<0x141>(x);   // row_half_mirror: lane i of 8 <- lane 7 - i (the other quad's sum)
    if (W >= 16) x += dpp_move<0x140>(x);  // row_mirror: lane i of 16 <- lane 15 - i (the other half's sum)
    if (W >= 32) x += lane_xor16(x, (int)(threadIdx.x & 63));
    if (W >= 64) x += lane_xor32(x, (int)(threadIdx.x & 63));
    return x;
}

// maximum / minimum of an int over the 64 lanes of a wavefront, in every lane (same steps as lane_group_sum<64>)
template <bool MAX>
__device__ __forceinline__ int wave_extreme_i32(int x) {
    auto pick = [](int a, int b) { return MAX ? max(a, b) : min(a, b); };
    const int lane = (int)(threadIdx.x & 63);
    x = pick(x, __builtin_amdgcn_update_dpp(x, x, 0xB1, 0xF, 0xF, false));
    x = pick(x, __builtin_amdgcn_update_dpp(x, x, 0x4E, 0xF, 0xF, false));
    x = pick(x, __builtin_amdgcn_update_dpp(x, x, 0x141, 0xF, 0xF, false));
    x = pick(x, __builtin_amdgcn_update_dpp(x, x, 0x140, 0xF, 0xF, false));
    x = pick(x, __float_as_int(lane_xor16(__int_as_float(x), lane)));
    x = pick(x, __float_as_int(lane_xor32(__int_as_float(x), lane)));
    return x;
}

// sum of an int over the 64 lanes of a wavefront, in every lane; inclusive prefix sum over the lanes
__device__ __forceinline__ int wave_sum_i32(int x) {
    const int lane = (int)(threadIdx.x & 63);
    x += __builtin_amdgcn_update_dpp(0, x, 0xB1, 0xF, 0xF, false);
    x += __builtin_amdgcn_update_dpp(0, x, 0x4E, 0xF, 0xF, false);
    x += __builtin_amdgcn_update_dpp(0, x, 0x141, 0xF, 0xF, false);
    x += __builtin_amdgcn_update_dpp(0, x, 0x140, 0xF, 0xF, false);
    x += __float_as_int(lane_xor16(__int_as_float(x), lane));
    x += __float_as_int(lane_xor32(__int_as_float(x), lane));
    return x;
}
__device__ __forceinline__ int wave_inclusive_scan_i32(int x) {
    x += __builtin_amdgcn_update_dpp(0, x, 0x111, 0xF, 0xF, false);   // row_shr 1, 2, 4, 8: a lane without a source adds 0
    x += __builtin_amdgcn_update_dpp(0, x, 0x112, 0xF, 0xF, false);
    x += __builtin_amdgcn_update_dpp(0, x, 0x114, 0xF, 0xF, false);
    x += __builtin_amdgcn_update_dpp(0, x, 0x118, 0xF, 0xF, false);
    x += __builtin_amdgcn_update_dpp(0, x, 0x142, 0xA, 0xF, false);   // lane 15 of rows 0 and 2 into rows 1 and 3
    x += __builtin_amdgcn_update_dpp(0, x, 0x143, 0xC, 0xF, false);   // lane 31 into the upper half
    return x;
}

template <typename T>
__device__ __forceinline__ T from_float(float f);
template <>
__device__ __forceinline__ float from_float<float>(float f) { return f; }
template <>
__device__ __forceinline__ bf16_t from_float<bf16_t>(float f) { return bf16_t{f32_to_bf16_bits(f)}; }

// 16-byte global load of consecutive elements, widened to float.  N = 16 / sizeof(T).
template <typename T>
struct Vec16;
template <>
struct Vec16<float> {
    static constexpr int N = 4;
    __device__ __forceinline__ static void unpack(const uint4 v, float* out) {
        out[0] = __uint_as_float(v.x); out[1] = __uint_as_float(v.y); out[2] = __uint_as_float(v.z); out[3] = __uint_as_float(v.w);
    }
    __device__ __forceinline__ static void load(const float* p, float* out) {
        float4 v = *reinterpret_cast<const float4*>(p);
        out[0] = v.x; out[1] = v.y; out[2] = v.z; out[3] = v.w;
    }
    __device__ __forceinline__ static void store(float* p, const float* in) {
        *reinterpret_cast<float4*>(p) = make_float4(in[0], in[1], in[2], in[3]);
    }
};
template <>
struct Vec16<bf16_t> {
    static constexpr int N = 8;
    // a 16-byte word as it came from memory -> floats (for loads that are used later than they are issued)
    __device__ __forceinline__ static void unpack(const uint4 v, float* out) {
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ __forceinline__ static void load(const bf16_t* p, float* out) {
        uint4 v = *reinterpret_cast<const uint4*>(p);
        uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            out[2 * i] = __uint_as_float(w[i] << 16);
            out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    __device__ __forceinline__ static void store(bf16_t* p, const float* in) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
            w[i] = pack_bf16x2(in[2 * i], in[2 * i + 1]);
        *reinterpret_cast<uint4*>(p) = make_uint4(w[0], w[1], w[2], w[3]);
    }
};

// Column of compacted row c inside its V^T tile of 64 keys.  Within each group of 32 keys the columns
// are stored in the order in which the softmax kernel's second MFMA consumes them: a lane quad lq holds
// keys {4 lq + j} of the first 16-key result tile and {16 + 4 lq + j} of the second in its 8
// contraction slots, so those 8 keys are made contiguous (one 16-byte LDS read per fragment).
__device__ __forceinline__ int vht_col(int c) {
    const int k32 = c & 31;
    return (c & 32) + 8 * ((k32 & 15) >> 2) + 4 * (k32 >> 4) + (k32 & 3);
}

// number of non-zero bytes in a 32-bit word
__device__ __forceinline__ int nonzero_bytes(uint32_t w) {
    uint32_t t = ((w & 0x7f7f7f7fu) + 0x7f7f7f7fu) | w;
    return __popc(t & 0x80808080u);
}

// ---- host side ------------------------------------------------------------------------
void set_error(const char* fmt, ...);
nats_status check_launch(const char* what);

// Brackets one kernel launch with a hipEvent pair while nats_profile_begin/end recording is on.
struct ProfScope {
    ProfScope(const char* name, hipStream_t st);
    ~ProfScope();
    int slot;
    hipStream_t stream;
};

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

constexpr int BWD_DKV_SEGMENTS = 8;   // blocks that share the queries of one key tile in the softmax branch's dK / dV kernel
// The lower triangular 64 x 64 fp16 operands of the forward's linear branch (T'' and P of a chunk) travel from the
// inversion kernel to the state-carrying kernel as matrix-instruction fragments of 16 rows x 32 columns (1 KiB each).
// Of the 8 fragments of a matrix the two that lie wholly above the diagonal (rows 0..31, columns 32..63) are
// neither written nor read: a chunk's matrix is 6 fragments, in this order.
constexpr int TRI_FRAGS = 6;
constexpr int TRI_FRAG_HALFS = TRI_FRAGS * 64 * 8;   // fp16 elements per chunk and matrix
// fragment number of row tile tw (16 rows) and contraction step ks (32 columns); (0, 1) and (1, 1) do not exist
__host__ __device__ constexpr int tri_frag(int tw, int ks) { return tw < 2 ? tw : 2 * tw - 2 + ks; }

constexpr int BWD_SWEEP_ROWS = 16;   // state rows per block of the reverse sweep: d / 16 blocks and partial sums per (batch, head)

// Resolved forward problem handed to the kernel launchers.
struct FwdPlan {
    int B, H, L, d, C, BH;   // C: the kernels' own chunk (64)
    int RC;                  // tokens per routing decision with routing per chunk (64 or 128; p->C)
    // head grouping (Section 4.3): G output heads (own V, own softmax branch, own state rows) per linear head (own
    // Q, K, alpha, beta, mask).  BHG = BH * G output heads; qk_per_out_head: the softmax branch's queries and keys
    // are given per output head (otherwise it uses the linear head's)
    int G, BHG, qk_per_out_head;
    int inner_chunk;   // routing per chunk: 0 both operations compute a chunk's inner part, 1 softmax attention only, 2 the linear operation only
    int dtype;
    int math;
    float softmax_scale, la_scale, rms_eps;
    int combine_mode;
    int routing;   // nats_routing
    int linear_op, freeze_on_softmax;   // variants of the linear branch, see nats_fwd_params
    int weight_act;                     // nats_weight_act
    int gdn_segments;                   // requested number of sequence segments of the chunkwise linear branch (0: automatic)
    // workspace carve-up (byte offsets)
    size_t off_cnt, off_idx, off_ns, off_kc, off_vc, off_ola, total;
    // chunkwise (MFMA) linear branch: per-chunk operands
    size_t off_tf, off_p, off_gamv, off_kdv, off_gam, off_seg, off_vht, off_olah, off_snap, off_wout;
};

// kernel launchers (one per .hip file); every pointer is a device pointer
nats_status launch_scan_compact(const FwdPlan& pl, const uint8_t* mask, const void* K, const void* V,
                                int32_t* cnt, int32_t* idx, int32_t* n_s, void* Kc, void* Vc,
                                void* Kc_user, void* Vc_user, int cap_user, void* VhT, hipStream_t st);
nats_status launch_gdn_recurrent(const FwdPlan& pl, const void* Q, const void* K, const void* V,
                                 const float* alpha, const float* beta, const uint8_t* mask,
                                 const float* S0, float* S_final, float* O_la, float* snap, hipStream_t st);
nats_status launch_gdn_chunk_inv(const FwdPlan& pl, const void* Q, const void* K, const float* alpha,
                                 const float* beta, const uint8_t* mask, void* TF, void* PF, float* gamv,
                                 float* kdv, float* gamC, const void* K_sm, const void* V, int32_t* cnt, int32_t* idx,
                                 int32_t* n_s, void* Kc, void* Vc, void* Kc_user, void* Vc_user, int cap_user, void* VhT,
                                 hipStream_t st);
int gdn_segments(const FwdPlan& pl);   // segments per (batch, head) the chunkwise linear branch will use
nats_status launch_gdn_seg_scan(const FwdPlan& pl, const void* Q, const void* K, const void* V, const void* TF,
                                const void* PF, const float* gamv, const float* kdv, const float* gamC,
                                const float* S0, float* S_final, float* seg_ws, void* O_la_h, float* O_la_f32,
                                hipStream_t st);
nats_status launch_softmax_fp32(const FwdPlan& pl, const void* Q, const void* Kc, const void* Vc,
                                const void* K, const void* V,
                                const int32_t* cnt, const float* O_la, const float* w_nla,
                                const float* w_la, void* O, float* O_nla_out, float* lse_out,
                                hipStream_t st);
nats_status launch_flash_softmax(const FwdPlan& pl, const void* Q, const void* Kc, const void* VhT,
                                 const void* K, const void* V,
                                 const int32_t* cnt, const void* O_la, const float* w_nla,
                                 const float* w_la, void* O, float* O_nla_out, float* lse_out, hipStream_t st,
                                 const float* W_out = nullptr);   // W_out: Eq. 22 inside the kernel (see the launcher)
nats_status launch_decode(const nats_dec_params& p, float softmax_scale, float la_scale, float eps,
                          float* state, void* k_cache, void* v_cache, int32_t* cache_len, const void* q,
                          const void* k, const void* v, const float* alpha, const float* beta,
                          const uint8_t* mask, const float* w_nla, const float* w_la, void* o,
                          int32_t* err_flags, hipStream_t st);
size_t decode_split_workspace_bytes(const nats_dec_params& p);
nats_status launch_decode_split(const nats_dec_params& p, float softmax_scale, float la_scale, float eps,
                                float* state, void* k_cache, void* v_cache, int32_t* cache_len, const void* q,
                                const void* k, const void* v, const float* alpha, const float* beta,
                                const uint8_t* mask, const float* w_nla, const float* w_la, void* o,
                                int32_t* err_flags, float* ws, hipStream_t st);
nats_status launch_decode_chunk(const nats_dec_params& p, float softmax_scale, float la_scale, float eps,
                                float* state, float* state_start, float* chunk_decay, int32_t* chunk_pos,
                                void* k_cache, void* v_cache, int32_t* cache_len, const void* q, const void* k,
                                const void* v, const float* alpha, const float* beta, const float* w_nla,
                                const float* w_la, void* o, int32_t* err_flags, hipStream_t st);
nats_status launch_route_chunks(int B, int L, int C, int d_model, int H, int dtype, const void* X, const float* W_s,
                                float* scores, uint8_t* mask_c, float* w_nla, float* w_la, int act, hipStream_t st);
nats_status launch_merge_weights(int B, int H, int L, int d, int dtype, const void* Q, const float* W_out,
                                 float* w_nla, float* w_la, int act, int G, hipStream_t st);
nats_status launch_decode_commit(const nats_dec_params& p, float* state, const float* state_start,
                                 const float* chunk_decay, int32_t* chunk_pos, int32_t* cache_len,
                                 const uint8_t* mask_c, int32_t* err_flags, hipStream_t st);

// ---- backward pass (fp32 arithmetic) ----
nats_status launch_softmax_bwd_dq(const FwdPlan& pl, const void* Q, const void* Kc, const void* Vc, const void* dO,
                                  const int32_t* cnt, const float* O_nla, const float* lse, float* Dvec, float* dQ,
                                  hipStream_t st);
nats_status launch_softmax_bwd_dkv(const FwdPlan& pl, const void* Q, const void* Kc, const void* Vc, const void* dO,
                                   const int32_t* cnt, const int32_t* idx, const int32_t* n_s, const float* lse,
                                   const float* Dvec, float* dK, float* dV, float* g_nla, float* dk_part, float* dv_part, float* g_part,
                                   hipStream_t st);
nats_status launch_gdn_recurrent_bwd(const FwdPlan& pl, const void* Q, const void* K, const void* V, const void* dO,
                                     const float* alpha, const float* beta, const uint8_t* mask, const float* ckpt,
                                     float* scratch, float* dq_part, float* dk_part, float* dalpha_part,
                                     float* dbeta_part, float* dV, float* dS0, float* ds_la_part, hipStream_t st);
nats_status launch_gdn_checkpoints(const FwdPlan& pl, const void* K, const void* V, const float* alpha, const float* beta,
                                   const uint8_t* mask, const float* S0, float* ckpt, hipStream_t st);
// chunkwise backward of the linear branch (fp32 matrix instructions), routing per token
size_t chunk_ops_floats(const FwdPlan& pl);
nats_status launch_gdn_bwd_prep(const FwdPlan& pl, const void* Q, const void* K, const float* alpha, const float* beta,
                                const uint8_t* mask, float* ops, hipStream_t st);
nats_status launch_gdn_chunk_states(const FwdPlan& pl, const void* K, const void* V, float* ops, const float* S_init,
                                    float* ck, float* Ug, float* Uh, hipStream_t st);
nats_status launch_gdn_chunk_state_grads(const FwdPlan& pl, const void* Q, const void* K, const void* dO,
                                         const uint8_t* mask, float* ops, float* dck, float* Uh, float* dV,
                                         float* dbeta_part, float* dS0, hipStream_t st);
nats_status launch_gdn_chunk_grads(const FwdPlan& pl, const void* Q, const void* K, const void* dO, const float* alpha,
                                   const uint8_t* mask, float* ops, const float* ck, const float* dck, const float* Ug,
                                   const float* dR, const float* dbeta_part, float* dQ, float* dK, float* dalpha,
                                   float* dbeta, float* g_nla, float* dscore_la, hipStream_t st);
nats_status launch_visible_rows(const FwdPlan& pl, const int32_t* cnt, int32_t* vis, hipStream_t st);
nats_status launch_softmax_bwd_own_chunk(const FwdPlan& pl, const void* Q, const void* K, const void* V, const void* dO,
                                         const float* lse, const float* Dvec, float* dQ, float* dK, float* dV,
                                         hipStream_t st);
// head grouping in the backward pass (head_group.hip)
nats_status launch_copy_rows(const void* src, size_t src_stride_bytes, void* dst, size_t dst_stride_bytes,
                             size_t row_bytes, size_t n_rows, hipStream_t st);
nats_status launch_add_f32(float* dst, const float* src, size_t n, hipStream_t st);
nats_status launch_zero_f32(float* dst, size_t n, hipStream_t st);
nats_status launch_merge_bwd(const FwdPlan& pl, int mode, float eps, const float* O_la, const float* O_nla,
                             const float* dO, const float* w_nla, const float* w_la, float* dO_la, float* dO_nla,
                             float* dw_nla, float* dw_la, hipStream_t st);
nats_status launch_gdn_chunk_out(const FwdPlan& pl, const void* Q, float* ops, const float* ck, const float* Ug,
                                 float* O_la, hipStream_t st);
nats_status launch_widen_bf16(const void* src, float* dst, size_t n, hipStream_t st);
nats_status launch_score_gradients_chunk(const FwdPlan& pl, const float* g_nla, const float* ds_la_part, float* dscore_nla,
                                         float* dscore_la, hipStream_t st);   // ds_la_part NULL: dscore_la is left as it is
nats_status launch_score_gradients(const FwdPlan& pl, const float* beta, const uint8_t* mask, const float* dbeta,
                                   const float* g_nla, float* g_la, float* dscore_nla, float* dscore_la, hipStream_t st);
nats_status launch_bwd_combine(const FwdPlan& pl, const float* dq_part, const float* dk_part, const float* dalpha_part,
                               const float* dbeta_part, float* dQ, float* dK, float* dalpha, float* dbeta,
                               float* g_nla, hipStream_t st);

}  // namespace nats
