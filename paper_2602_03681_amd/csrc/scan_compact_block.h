// Mask scan + K/V compaction: the work of one block (see scan_compact.hip), as a device function, so that the
// compaction's few, latency-bound blocks can also ride along in another kernel's grid.
#ifndef NATS_SCAN_COMPACT_BLOCK_H
#define NATS_SCAN_COMPACT_BLOCK_H

#include "mfma_util.h"
#include "nats_common.h"

namespace nats {

// fp16 value of one stored element (the MFMA softmax kernel's V^T operand)
__device__ __forceinline__ half_t elem_to_half(bf16_t x) { return f32_to_half_sat(to_float(x)); }
__device__ __forceinline__ half_t elem_to_half(float x) { return f32_to_half_sat(x); }

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_SEG = SCAN_THREADS * 4;  // tokens per block, 4 per thread

// what a block of the compaction takes (one struct, so that another kernel can carry these blocks along)
template <typename T>
struct ScanArgs {
    const uint8_t* mask;
    const T *K, *V;
    int L, d;
    int32_t *cnt, *idx, *n_s;
    T *Kc, *Vc, *Kc_user, *Vc_user;
    int cap_user;
    half_t* VhT;
    int chunk_mask;   // 0: one mask byte per token; otherwise log2 of the routing chunk (6 or 7): one byte per chunk
    int G, k_per_out_head;
};

// One block: SCAN_SEG tokens (segment number seg_no) of output head bo.  SCAN_THREADS threads.
// lds: SCAN_LDS_INTS ints of the block's shared memory (the caller's: a kernel that carries other kinds of block
// too gives every kind the same bytes).
constexpr int SCAN_LDS_INTS = SCAN_THREADS / 64 + SCAN_SEG;
template <typename T>
__device__ __forceinline__ void scan_compact_block(const ScanArgs<T>& a, const int seg_no, const int bo, int* lds) {
    const uint8_t* __restrict__ mask = a.mask;
    const T* __restrict__ K = a.K;
    const T* __restrict__ V = a.V;
    const int L = a.L, d = a.d, cap_user = a.cap_user, chunk_mask = a.chunk_mask, G = a.G, k_per_out_head = a.k_per_out_head;
    int32_t* __restrict__ cnt = a.cnt;
    int32_t* __restrict__ idx = a.idx;
    int32_t* __restrict__ n_s = a.n_s;
    T* __restrict__ Kc = a.Kc;
    T* __restrict__ Vc = a.Vc;
    T* __restrict__ Kc_user = a.Kc_user;
    T* __restrict__ Vc_user = a.Vc_user;
    half_t* __restrict__ VhT = a.VhT;
    int* s_wave = lds;                        // [SCAN_THREADS / 64]
    int* s_pos = lds + SCAN_THREADS / 64;     // [SCAN_SEG]
    // Head grouping (Section 4.3): G output heads share the mask of linear head bh.  Every output head gathers
    // its own value rows (and its own key rows, if the softmax heads have keys of their own); the integers are
    // the group's and are stored by its first head.
    const int bh = bo / G;               // linear head: mask, cnt, idx, n_s (bo: output head)
    const bool first = bo % G == 0;
    const int bk = k_per_out_head ? bo : bh;
    const int seg0 = seg_no * SCAN_SEG;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // chunk_mask: one mask byte per chunk of 2^chunk_mask tokens (routing per chunk: every token of a softmax
    // chunk is a softmax token); otherwise one byte per token
    const uint8_t* m = mask + (size_t)bh * (chunk_mask ? L >> chunk_mask : L);

    // ---- 1. softmax tokens in front of this segment -----------------------------------
    int before = 0;
    {
        if (chunk_mask) {   // a few hundred bytes at most, at no particular alignment
            for (int i = tid; i < (seg0 >> chunk_mask); i += SCAN_THREADS) before += m[i] ? (1 << chunk_mask) : 0;
        } else {
            const uint4* m16 = reinterpret_cast<const uint4*>(m);  // seg0 is a multiple of 1024
            for (int i = tid; i < seg0 / 16; i += SCAN_THREADS) {
                uint4 w = m16[i];
                before += nonzero_bytes(w.x) + nonzero_bytes(w.y) + nonzero_bytes(w.z) + nonzero_bytes(w.w);
            }
        }
        before = wave_sum_i32(before);
        if (lane == 0) s_wave[wave] = before;
        __syncthreads();
        before = s_wave[0] + s_wave[1] + s_wave[2] + s_wave[3];
        __syncthreads();
    }

    // ---- 2. scan of the segment: 4 tokens per thread ------------------------------------
    const int t0 = seg0 + tid * 4;
    uint32_t w = 0;
    if (t0 < L)   // L % 4 == 0: a word is all in or all out; its 4 tokens lie in one chunk
        w = chunk_mask ? (m[t0 >> chunk_mask] ? 0x01010101u : 0u) : *reinterpret_cast<const uint32_t*>(m + t0);
    const int mine = nonzero_bytes(w);
    const int incl = wave_inclusive_scan_i32(mine);
    if (lane == 63) s_wave[wave] = incl;
    __syncthreads();
    int wave_base = 0, seg_total = 0;
#pragma unroll
    for (int i = 0; i < SCAN_THREADS / 64; ++i) {
        if (i < wave) wave_base += s_wave[i];
        seg_total += s_wave[i];
    }
    int local = wave_base + incl - mine;  // softmax tokens of this segment before t0
    if (t0 < L) {
        int c[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if ((w >> (8 * j)) & 0xffu) {
                s_pos[local] = t0 + j;
                if (first) idx[(size_t)bh * L + before + local] = t0 + j;
                ++local;
            }
            c[j] = before + local;
        }
        if (first) *reinterpret_cast<int4*>(cnt + (size_t)bh * L + t0) = make_int4(c[0], c[1], c[2], c[3]);
    }
    if (seg0 + SCAN_SEG >= L && tid == 0 && first) n_s[bh] = before + seg_total;
    __syncthreads();

    // ---- 3. gather the K / V rows of this segment's softmax tokens ------------------------
    constexpr int EPL = 16 / (int)sizeof(T);  // elements per 16-byte lane access
    const int lpr = d / EPL;                  // lanes per row (8..32, divides 256)
    const int rows_per_pass = SCAN_THREADS / lpr;
    const int part = tid % lpr;
    for (int r = tid / lpr; r < seg_total; r += rows_per_pass) {
        const int t = s_pos[r];
        const int c = before + r;
        const uint4 kv = *reinterpret_cast<const uint4*>(K + ((size_t)bk * L + t) * d + part * EPL);
        const uint4 vv = *reinterpret_cast<const uint4*>(V + ((size_t)bo * L + t) * d + part * EPL);
        const size_t dst = ((size_t)bo * L + c) * d + part * EPL;
        *reinterpret_cast<uint4*>(Kc + dst) = kv;
        *reinterpret_cast<uint4*>(Vc + dst) = vv;
        if (Kc_user != nullptr && c < cap_user) {
            const size_t du = ((size_t)bo * cap_user + c) * d + part * EPL;
            *reinterpret_cast<uint4*>(Kc_user + du) = kv;
            *reinterpret_cast<uint4*>(Vc_user + du) = vv;
        }
        if (VhT != nullptr) {   // fp16 copy, transposed inside tiles of 64 compacted rows: [tile][d][64]
            const T* ve = reinterpret_cast<const T*>(&vv);
            half_t* tile = VhT + ((size_t)bo * L + (size_t)(c >> 6) * 64) * d;
#pragma unroll
            for (int j = 0; j < EPL; ++j) tile[(size_t)(part * EPL + j) * 64 + vht_col(c)] = elem_to_half(ve[j]);
        }
    }
    // the tail of the last V^T tile is multiplied by zero weights downstream: make it finite
    if (VhT != nullptr && seg0 + SCAN_SEG >= L) {
        const int n_total = before + seg_total;
        const int pad = ((n_total + 63) & ~63) - n_total;
        half_t* tile = VhT + ((size_t)bo * L + (size_t)(n_total >> 6) * 64) * d;
        for (int e = tid; e < pad * d; e += SCAN_THREADS) {
            const int dv = e / pad, cc = (n_total & 63) + e % pad;
            tile[(size_t)dv * 64 + vht_col(cc)] = (half_t)0.f;
        }
    }
}

}  // namespace nats

#endif
