// C ABI of the NAtS-L hybrid attention library: host-side validation, workspace
// carve-up and kernel sequencing.  Declarations and argument semantics: nats.h.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "nats_common.h"
#include "nats_measure.h"

namespace nats {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

nats_status check_launch(const char* what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) {
        set_error("%s: HIP launch failed: %s", what, hipGetErrorString(e));
        return NATS_ERR_HIP;
    }
    return NATS_OK;
}

// ---- optional per-kernel timing -----------------------------------------------------------
// Inside one call that launches several kernels back to back on one stream (a ProfChain is alive), the stop
// event of a scope also serves as the start event of the next one: 5 events per forward instead of 8 (every
// recorded event costs the stream a few microseconds).
struct ProfRecord { const char* name; hipEvent_t start, stop; int start_from; };   // start_from: slot whose stop is this start, or -1
static std::mutex g_prof_mu;
static std::vector<ProfRecord> g_prof;
static int g_prof_used = 0;
static bool g_prof_on = false;
static thread_local int g_chain_prev = -2;            // -2: no chain; -1: chain open, no scope yet; else the last scope's slot
static thread_local hipStream_t g_chain_stream = nullptr;
struct ProfChain {
    ProfChain() { g_chain_prev = -1; }
    ~ProfChain() { g_chain_prev = -2; }
};

ProfScope::ProfScope(const char* name, hipStream_t st) : slot(-1), stream(st) {
    if (!g_prof_on) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (!g_prof_on || g_prof_used >= (int)g_prof.size()) return;
    slot = g_prof_used++;
    g_prof[slot].name = name;
    if (g_chain_prev >= 0 && g_chain_stream == stream) {
        g_prof[slot].start_from = g_chain_prev;
    } else {
        g_prof[slot].start_from = -1;
        (void)hipEventRecord(g_prof[slot].start, stream);
    }
}
ProfScope::~ProfScope() {
    if (slot < 0) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (slot >= (int)g_prof.size()) return;   // recording was ended in between
    (void)hipEventRecord(g_prof[slot].stop, stream);
    if (g_chain_prev != -2) { g_chain_prev = slot; g_chain_stream = stream; }
}

// bf16 tensors take the chunkwise MFMA kernels unless fp32 arithmetic is asked for
// (routing chunks of 128 tokens run on the token-by-token kernels: the matrix-core path hands a chunk's provisional
// state on inside its own chunk of 64 only)
static bool uses_chunk_path(const FwdPlan& pl) {
    return pl.dtype == NATS_BF16 && pl.math == NATS_MATH_AUTO && !(pl.routing == NATS_ROUTE_CHUNK && pl.RC != 64);
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static nats_status validate_fwd_params(const nats_fwd_params* p, FwdPlan* pl) {
    if (p == nullptr) { set_error("params is NULL"); return NATS_ERR_NULL; }
    if (p->dtype != NATS_F32 && p->dtype != NATS_BF16) {
        set_error("dtype %d is neither NATS_F32 nor NATS_BF16", p->dtype);
        return NATS_ERR_DTYPE;
    }
    if (p->B <= 0 || p->H <= 0 || p->L <= 0 || p->C <= 0) {
        set_error("B, H, L, C must be positive (got %d, %d, %d, %d)", p->B, p->H, p->L, p->C);
        return NATS_ERR_SHAPE;
    }
    if (p->d != 64 && p->d != 128) { set_error("d must be 64 or 128 (got %d)", p->d); return NATS_ERR_SHAPE; }
    if (p->L % p->C != 0) { set_error("L (%d) must be a multiple of C (%d)", p->L, p->C); return NATS_ERR_SHAPE; }
    if ((long long)p->B * p->H > 65535) { set_error("B*H must not exceed 65535"); return NATS_ERR_SHAPE; }
    if ((long long)p->B * p->H * p->L > (1ll << 31) - 1) {
        set_error("B*H*L must fit in 31 bits");
        return NATS_ERR_SHAPE;
    }
    // C: with routing per token the result does not depend on it (the chunkwise form is exact for any chunk, and the
    // kernels use their own of 64); with routing per chunk it is the number of tokens per routing decision
    if (p->C != 64 && p->C != 128) { set_error("chunk size C=%d has no kernel in this build (64 or 128)", p->C); return NATS_ERR_UNSUPPORTED; }
    if (p->combine_mode < 0 || p->combine_mode > 2) {
        set_error("combine_mode must be 0, 1 or 2 (got %d)", p->combine_mode);
        return NATS_ERR_SHAPE;
    }
    if (p->math != NATS_MATH_AUTO && p->math != NATS_MATH_FP32) {
        set_error("math must be NATS_MATH_AUTO or NATS_MATH_FP32 (got %d)", p->math);
        return NATS_ERR_SHAPE;
    }
    if (p->routing != NATS_ROUTE_TOKEN && p->routing != NATS_ROUTE_CHUNK) {
        set_error("routing must be NATS_ROUTE_TOKEN or NATS_ROUTE_CHUNK (got %d)", p->routing);
        return NATS_ERR_SHAPE;
    }
    if (p->linear_op != NATS_LINEAR_GDN && p->linear_op != NATS_LINEAR_GATED) {
        set_error("linear_op must be NATS_LINEAR_GDN or NATS_LINEAR_GATED (got %d)", p->linear_op);
        return NATS_ERR_SHAPE;
    }
    if (p->freeze_on_softmax != 0 && p->freeze_on_softmax != 1) {
        set_error("freeze_on_softmax must be 0 or 1 (got %d)", p->freeze_on_softmax);
        return NATS_ERR_SHAPE;
    }
    pl->routing = p->routing;
    pl->linear_op = p->linear_op;
    pl->freeze_on_softmax = p->freeze_on_softmax;
    if (p->weight_act < NATS_WEIGHTS_SOFTMAX || p->weight_act > NATS_WEIGHTS_LINEAR) {
        set_error("weight_act must be a nats_weight_act (got %d)", p->weight_act);
        return NATS_ERR_SHAPE;
    }
    pl->weight_act = p->weight_act;
    if (p->gdn_segments < 0 || p->gdn_segments > 64) {
        set_error("gdn_segments must be between 0 (automatic) and 64 (got %d)", p->gdn_segments);
        return NATS_ERR_SHAPE;
    }
    pl->gdn_segments = p->gdn_segments;
    if (p->group < 0 || p->group > 8) { set_error("group must be between 1 and 8 (0 counts as 1; got %d)", p->group); return NATS_ERR_SHAPE; }
    pl->G = p->group > 0 ? p->group : 1;
    if ((long long)p->B * p->H * pl->G > 65535 || (long long)p->B * p->H * pl->G * p->L > (1ll << 31) - 1) {
        set_error("B*H*group must not exceed 65535 and B*H*group*L must fit in 31 bits");
        return NATS_ERR_SHAPE;
    }
    if (p->inner_chunk < 0 || p->inner_chunk > 2 || (p->inner_chunk != 0 && p->routing != NATS_ROUTE_CHUNK)) {
        set_error("inner_chunk must be 0, or 1 / 2 with routing per chunk (got %d)", p->inner_chunk);
        return NATS_ERR_SHAPE;
    }
    pl->inner_chunk = p->inner_chunk;
    pl->qk_per_out_head = 0;   // set by the call: whether the softmax heads have queries and keys of their own
    pl->B = p->B; pl->H = p->H; pl->L = p->L; pl->d = p->d; pl->C = 64; pl->RC = p->C; pl->BH = p->B * p->H;
    pl->BHG = pl->BH * pl->G;
    pl->dtype = p->dtype;
    pl->math = p->math;
    pl->softmax_scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->d);
    pl->la_scale = p->la_scale > 0.f ? p->la_scale : 1.0f;
    pl->rms_eps = p->rms_eps > 0.f ? p->rms_eps : 1e-6f;
    pl->combine_mode = p->combine_mode;

    const size_t esz = p->dtype == NATS_BF16 ? 2 : 4;
    const size_t n_tok = (size_t)pl->BH * pl->L;     // per linear head: the integers and the per-chunk operands
    const size_t n_out = (size_t)pl->BHG * pl->L;    // per output head: rows of the cache, of the outputs, weights
    size_t off = 0;
    pl->off_cnt = off; off = align_up(off + n_tok * 4, 256);
    pl->off_idx = off; off = align_up(off + n_tok * 4, 256);
    pl->off_ns = off;  off = align_up(off + (size_t)pl->BH * 4, 256);
    pl->off_kc = off;  off = align_up(off + n_out * pl->d * esz, 256);
    pl->off_vc = off;  off = align_up(off + n_out * pl->d * esz, 256);
    pl->off_ola = off; off = align_up(off + n_out * pl->d * 4, 256);
    pl->off_tf = pl->off_p = pl->off_gamv = pl->off_kdv = pl->off_gam = pl->off_seg = pl->off_vht = pl->off_olah = 0;
    pl->off_snap = 0;
    pl->off_wout = off; off = align_up(off + 2 * n_out * 4, 256);   // weights of Eq. 21 when computed by Eq. 22
    if (!uses_chunk_path(*pl) && pl->routing == NATS_ROUTE_CHUNK) {   // chunk-start state of the fp32 recurrence
        pl->off_snap = off; off = align_up(off + (size_t)pl->BHG * pl->d * pl->d * 4, 256);
    }
    if (uses_chunk_path(*pl)) {   // per-chunk operands of the chunkwise linear branch
        const size_t tri = n_tok / pl->C * TRI_FRAG_HALFS * 2;               // lower triangular, fp16, per chunk
        pl->off_tf = off;   off = align_up(off + tri, 256);                  // T''
        pl->off_p = off;    off = align_up(off + tri, 256);                  // P
        pl->off_gamv = off; off = align_up(off + n_tok * 4, 256);
        pl->off_kdv = off;  off = align_up(off + n_tok * 4, 256);
        pl->off_gam = off;  off = align_up(off + (n_tok / pl->C) * 4, 256);
        // start state, zero-run end state and transposed transition of every segment
        pl->off_seg = off;  off = align_up(off + 3 * (size_t)pl->BHG * gdn_segments(*pl) * pl->d * pl->d * 4, 256);
        pl->off_vht = off;  off = align_up(off + n_out * pl->d * 2, 256);   // fp16 V^T tiles of the softmax branch
        pl->off_olah = off; off = align_up(off + n_out * pl->d * 2, 256);   // fp16 hand-off between the branches
    }
    pl->total = off;
    return NATS_OK;
}

// Workspace of the backward pass, behind the forward's integer bookkeeping and compacted cache (the same
// offsets): branch output and lse of the softmax branch, D_i, checkpoints of the state, the scratch rows of
// the reverse sweep and the partial sums of its blocks.
struct BwdPlan {
    size_t off_onla, off_lse, off_dvec, off_ckpt, off_scratch, off_dqp, off_dkp, off_dap, off_dbp, off_skp, off_svp, off_sgp,
        off_gnla, off_vis, off_dslap, off_ops, off_ug, off_uh, off_dck, off_vht, total;
    // head grouping: the pass runs once per member of the groups on `total` bytes; behind them, one member's heads
    // of V, dO, the initial state (gathered) and the member's gradients before they are added or scattered
    int G;
    size_t off_gv, off_gdo, off_gdv, off_gdq, off_gdk, off_gda, off_gdb, off_gs0, off_gds0, off_ggn, off_ggl, off_gsn,
        off_gsl, off_gqn, off_gkn, off_gdqn, off_gdkn, total_grouped;
    // the merges of Eq. 21 and its ablation (merge_mode 1, 2; 0: the plain sum): the linear branch's output rows, the
    // two branches' gradients of their rows, the snapshot rows of the token-by-token forward (routing per chunk), a
    // member's weights and their gradients (head grouping), and fp32 copies of bf16 tensors (the pass then runs on fp32
    // tensors: pl.dtype is NATS_F32 whatever src_dtype is)
    int merge_mode, src_dtype;
    size_t off_mola, off_mdol, off_mdon, off_msnap, off_mwn, off_mwl, off_mdwn, off_mdwl, off_cq, off_ck, off_cv, off_cdo,
        off_cqn, off_ckn;
};
static void plan_bwd(const FwdPlan& pl, BwdPlan* bp) {
    const size_t n_tok = (size_t)pl.BH * pl.L, ns = (size_t)pl.d / BWD_SWEEP_ROWS;
    size_t off = align_up(pl.off_ola, 256);   // first byte behind cnt, idx, n_s, Kc, Vc
    bp->off_onla = off;    off = align_up(off + n_tok * pl.d * 4, 256);
    bp->off_lse = off;     off = align_up(off + n_tok * 4, 256);
    bp->off_dvec = off;    off = align_up(off + n_tok * 4, 256);
    bp->off_ckpt = off;    off = align_up(off + (size_t)pl.BH * (pl.L / 64) * pl.d * pl.d * 4, 256);
    // the token-by-token adjoint of the linear branch (math = NATS_MATH_FP32): the parked rows of a chunk and the
    // d/16 partial sums per (batch, head); by chunks only the partials of dbeta are used
    const size_t tk = pl.math == NATS_MATH_FP32 ? 1 : 0;
    bp->off_scratch = off; off = align_up(off + tk * pl.BH * pl.d * 64 * pl.d * 4, 256);   // 64 tokens of every row
    bp->off_dqp = off;     off = align_up(off + tk * ns * n_tok * pl.d * 4, 256);
    bp->off_dkp = off;     off = align_up(off + tk * ns * n_tok * pl.d * 4, 256);
    bp->off_dap = off;     off = align_up(off + tk * ns * n_tok * 4, 256);
    bp->off_dbp = off;     off = align_up(off + ns * n_tok * 4, 256);
    // partial dK, dV and column sums of the softmax branch, one per query segment and compacted key
    bp->off_skp = off;     off = align_up(off + (size_t)BWD_DKV_SEGMENTS * n_tok * pl.d * 4, 256);
    bp->off_svp = off;     off = align_up(off + (size_t)BWD_DKV_SEGMENTS * n_tok * pl.d * 4, 256);
    bp->off_sgp = off;     off = align_up(off + (size_t)BWD_DKV_SEGMENTS * n_tok * 4, 256);
    bp->off_gnla = off;    off = align_up(off + n_tok * 4, 256);   // column sums of Eq. 15 when only their chunk sums are asked for
    bp->off_vis = off;     off = align_up(off + n_tok * 4, 256);   // routing per chunk: compacted rows visible to a query
    bp->off_dslap = off;   off = align_up(off + ns * (n_tok / 64) * 4, 256);   // ... and the sweep's partials of Eq. 17
    // chunkwise backward of the linear branch: operands of every chunk, U and the residuals, state gradients per chunk
    const size_t ch = (pl.routing == NATS_ROUTE_CHUNK && tk) ? 0 : 1;   // (token by token with routing per chunk: own checkpoint kernel)
    bp->off_ops = off;     off = align_up(off + ch * chunk_ops_floats(pl) * 4, 256);
    bp->off_ug = off;      off = align_up(off + ch * n_tok * pl.d * 4, 256);
    bp->off_uh = off;      off = align_up(off + ch * n_tok * pl.d * 4, 256);
    bp->off_dck = off;     off = align_up(off + ch * (1 - tk) * pl.BH * (pl.L / 64) * pl.d * pl.d * 4, 256);
    bp->off_vht = off;     off = align_up(off + n_tok * pl.d * 2, 256);   // fp16 V^T tiles of the compacted values (bf16 tensors)
    bp->total = off;
    bp->G = 1;
    bp->total_grouped = off;
}

// the buffers of one member of the groups, behind the workspace of the pass itself (pl: the plan of one member, G = 1)
static void plan_bwd_group(const FwdPlan& pl, int G, BwdPlan* bp) {
    const size_t n_tok = (size_t)pl.BH * pl.L, esz = pl.dtype == NATS_BF16 ? 2 : 4;
    const size_t nd = n_tok * pl.d, st = (size_t)pl.BH * pl.d * pl.d;
    size_t off = bp->total;
    bp->G = G;
    bp->off_gv = off;   off = align_up(off + nd * esz, 256);
    bp->off_gdo = off;  off = align_up(off + nd * esz, 256);
    bp->off_gdv = off;  off = align_up(off + nd * 4, 256);
    bp->off_gdq = off;  off = align_up(off + nd * 4, 256);
    bp->off_gdk = off;  off = align_up(off + nd * 4, 256);
    bp->off_gda = off;  off = align_up(off + n_tok * 4, 256);
    bp->off_gdb = off;  off = align_up(off + n_tok * 4, 256);
    bp->off_gs0 = off;  off = align_up(off + st * 4, 256);
    bp->off_gds0 = off; off = align_up(off + st * 4, 256);
    bp->off_ggn = off;  off = align_up(off + n_tok * 4, 256);
    bp->off_ggl = off;  off = align_up(off + n_tok * 4, 256);
    bp->off_gsn = off;  off = align_up(off + (n_tok / pl.C) * 4, 256);
    bp->off_gsl = off;  off = align_up(off + (n_tok / pl.C) * 4, 256);
    // the member's own queries and keys of the softmax branch and their gradients (used if Q_nla, K_nla are given)
    bp->off_gqn = off;  off = align_up(off + nd * esz, 256);
    bp->off_gkn = off;  off = align_up(off + nd * esz, 256);
    bp->off_gdqn = off; off = align_up(off + nd * 4, 256);
    bp->off_gdkn = off; off = align_up(off + nd * 4, 256);
    bp->total_grouped = off;
}

// the buffers of the backward through Eq. 21's merge, behind everything else (pl: the fp32 plan of one member)
static void plan_bwd_merge(const FwdPlan& pl, int G, BwdPlan* bp) {
    const size_t n_tok = (size_t)pl.BH * pl.L, nd = n_tok * pl.d;
    size_t off = bp->total_grouped;
    bp->off_mola = off;  off = align_up(off + nd * 4, 256);
    bp->off_mdol = off;  off = align_up(off + nd * 4, 256);
    bp->off_mdon = off;  off = align_up(off + nd * 4, 256);
    bp->off_msnap = off; off = align_up(off + (size_t)pl.BH * pl.d * pl.d * 4, 256);
    bp->off_mwn = off;   off = align_up(off + n_tok * 4, 256);
    bp->off_mwl = off;   off = align_up(off + n_tok * 4, 256);
    bp->off_mdwn = off;  off = align_up(off + n_tok * 4, 256);
    bp->off_mdwl = off;  off = align_up(off + n_tok * 4, 256);
    const size_t cv = bp->src_dtype == NATS_BF16 ? 1 : 0;
    bp->off_cq = off;    off = align_up(off + cv * nd * 4, 256);
    bp->off_ck = off;    off = align_up(off + cv * nd * 4, 256);
    bp->off_cv = off;    off = align_up(off + cv * nd * G * 4, 256);
    bp->off_cdo = off;   off = align_up(off + cv * nd * G * 4, 256);
    bp->off_cqn = off;   off = align_up(off + cv * nd * G * 4, 256);
    bp->off_ckn = off;   off = align_up(off + cv * nd * G * 4, 256);
    bp->total_grouped = off;
}

// pl: the plan of the pass itself.  With head grouping (p->group = G > 1) that is the plan of one member of the groups,
// B x H heads with G = 1, and bp->G = G.
static nats_status validate_bwd_params(const nats_fwd_params* p, FwdPlan* pl, BwdPlan* bp) {
    if (p == nullptr) { set_error("params is NULL"); return NATS_ERR_NULL; }
    nats_fwd_params one = *p;
    const int G = p->group > 1 ? p->group : 1;
    if (G > 8) { set_error("group must be at most 8 (got %d)", p->group); return NATS_ERR_SHAPE; }
    one.group = 1;
    // Eq. 21's merge (and its ablation): each branch's backward runs as for the plain sum, on its own gradient of its
    // output rows; these gradients are fp32, so the pass runs on fp32 tensors (bf16 ones are widened first)
    bp->merge_mode = p->combine_mode;
    bp->src_dtype = p->dtype;
    if (p->combine_mode < 0 || p->combine_mode > 2) { set_error("combine_mode must be 0, 1 or 2 (got %d)", p->combine_mode); return NATS_ERR_SHAPE; }
    if (p->combine_mode != 0) {
        if (p->dtype != NATS_BF16 && p->dtype != NATS_F32) { set_error("dtype must be NATS_BF16 or NATS_F32"); return NATS_ERR_SHAPE; }
        one.combine_mode = 0;
        one.dtype = NATS_F32;
    }
    nats_status st = validate_fwd_params(&one, pl);
    if (st != NATS_OK) return st;
    if (pl->inner_chunk != 0) { set_error("the backward pass covers inner_chunk 0 only (got %d)", pl->inner_chunk); return NATS_ERR_UNSUPPORTED; }
    if (pl->routing == NATS_ROUTE_CHUNK && pl->RC != 64) {
        set_error("the backward pass with routing per chunk covers chunks of 64 tokens (C=%d given)", pl->RC);
        return NATS_ERR_UNSUPPORTED;
    }
    plan_bwd(*pl, bp);
    if (G > 1) plan_bwd_group(*pl, G, bp);
    if (bp->merge_mode != 0) plan_bwd_merge(*pl, G, bp);
    return NATS_OK;
}

}  // namespace nats

using namespace nats;

// Scratch memory of nats_hybrid_attn_fwd_noalloc: one array per GPU, part of the loaded code object, so that the
// call needs no allocation.  Host code never passes the array's name to a kernel (on the host it is only a
// stand-in for the symbol): the device address is looked up once per device and kept.
static __device__ __align__(256) unsigned char scratch[NATS_NOALLOC_SCRATCH_BYTES];
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[64] = {};

static nats_status noalloc_scratch(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        set_error("nats_hybrid_attn_fwd_noalloc: no current device (or device index beyond 63)");
        return NATS_ERR_HIP;
    }
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || ptr == nullptr) {
            set_error("nats_hybrid_attn_fwd_noalloc: hipGetSymbolAddress failed: %s", hipGetErrorString(e));
            return NATS_ERR_HIP;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return NATS_OK;
}

extern "C" {

const char* nats_last_error(void) { return g_err; }

int nats_abi_version(void) { return 113; }

nats_status nats_profile_begin(int max_records) {
    if (max_records <= 0 || max_records > (1 << 20)) { set_error("max_records out of range"); return NATS_ERR_SHAPE; }
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (!g_prof.empty()) { set_error("profiling is already on"); return NATS_ERR_UNSUPPORTED; }
    g_prof.resize(max_records);
    for (auto& r : g_prof) { r.start = nullptr; r.stop = nullptr; }
    for (auto& r : g_prof) {
        if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) {
            set_error("hipEventCreate failed");
            for (auto& q : g_prof) {   // give back what was created
                if (q.start) (void)hipEventDestroy(q.start);
                if (q.stop) (void)hipEventDestroy(q.stop);
            }
            g_prof.clear();
            return NATS_ERR_HIP;
        }
    }
    g_prof_used = 0;
    g_prof_on = true;
    return NATS_OK;
}

int nats_profile_end(char* names, float* total_ms, int32_t* launches, int max_kernels) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_on = false;
    int n = 0;
    if (names && total_ms && launches) {
        for (int i = 0; i < g_prof_used; ++i) {
            float ms = 0.f;
            const hipEvent_t start = g_prof[i].start_from >= 0 ? g_prof[g_prof[i].start_from].stop : g_prof[i].start;
            if (hipEventSynchronize(g_prof[i].stop) != hipSuccess ||
                hipEventElapsedTime(&ms, start, g_prof[i].stop) != hipSuccess)
                continue;
            int k = 0;
            while (k < n && strncmp(names + 32 * k, g_prof[i].name, 31) != 0) ++k;
            if (k == n) {
                if (n >= max_kernels) continue;
                strncpy(names + 32 * n, g_prof[i].name, 31);
                names[32 * n + 31] = 0;
                total_ms[n] = 0.f;
                launches[n] = 0;
                ++n;
            }
            total_ms[k] += ms;
            launches[k] += 1;
        }
    }
    for (auto& r : g_prof) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
    g_prof.clear();
    g_prof_used = 0;
    return n;
}

size_t nats_hybrid_attn_fwd_workspace_bytes(const nats_fwd_params* p) {
    FwdPlan pl;
    if (validate_fwd_params(p, &pl) != NATS_OK) return 0;
    return pl.total;
}

nats_status nats_hybrid_attn_fwd_ex(const nats_fwd_params* p, const void* Q, const void* K, const void* V,
                                    const float* alpha, const float* beta, const uint8_t* mask, void* O,
                                    const nats_fwd_extra* extra, void* workspace, size_t workspace_bytes,
                                    void* hip_stream) {
    FwdPlan pl;
    nats_status st = validate_fwd_params(p, &pl);
    if (st != NATS_OK) return st;
    if (!Q || !K || !V || !alpha || !beta || !mask || !O) {
        set_error("Q, K, V, alpha, beta, mask and O must all be non-NULL");
        return NATS_ERR_NULL;
    }
    if (workspace == nullptr || workspace_bytes < pl.total) {
        set_error("workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : (size_t)0, pl.total);
        return NATS_ERR_WORKSPACE;
    }
    nats_fwd_extra ex;
    memset(&ex, 0, sizeof(ex));
    if (extra) ex = *extra;
    if ((ex.Kc == nullptr) != (ex.Vc == nullptr)) { set_error("extra.Kc and extra.Vc must be given together"); return NATS_ERR_NULL; }
    if (ex.Kc != nullptr && ex.cap <= 0) { set_error("extra.cap must be positive when Kc/Vc are given"); return NATS_ERR_SHAPE; }
    if (ex.W_out != nullptr && (ex.w_nla != nullptr || ex.w_la != nullptr)) {
        set_error("extra.W_out (weights by Eq. 22) and extra.w_nla / w_la (given weights) exclude each other");
        return NATS_ERR_SHAPE;
    }
    if ((ex.Q_nla == nullptr) != (ex.K_nla == nullptr)) { set_error("extra.Q_nla and extra.K_nla must be given together"); return NATS_ERR_NULL; }
    const void* ptrs[] = {Q, K, V, alpha, beta, mask, O, workspace, ex.w_nla, ex.w_la, ex.initial_state,
                          ex.final_state, ex.Kc, ex.Vc, ex.n_s, ex.idx, ex.cnt, ex.O_la, ex.O_nla, ex.lse, ex.W_out,
                          ex.Q_nla, ex.K_nla};
    for (const void* ptr : ptrs)
        if (ptr != nullptr && !aligned16(ptr)) { set_error("pointer %p is not 16-byte aligned", ptr); return NATS_ERR_ALIGN; }
    if (O == Q || O == K || O == V || O == ex.Q_nla || O == ex.K_nla) { set_error("O must not alias Q, K or V"); return NATS_ERR_SHAPE; }
    // queries and keys of the softmax branch (the linear branch always takes Q, K)
    const void* Qs = ex.Q_nla != nullptr ? ex.Q_nla : Q;
    const void* Ks = ex.K_nla != nullptr ? ex.K_nla : K;
    pl.qk_per_out_head = ex.Q_nla != nullptr;   // [B,H*group,L,d]; otherwise the softmax heads of a group share Q, K

    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    int32_t* cnt = reinterpret_cast<int32_t*>(ws + pl.off_cnt);
    int32_t* idx = reinterpret_cast<int32_t*>(ws + pl.off_idx);
    int32_t* n_s = reinterpret_cast<int32_t*>(ws + pl.off_ns);
    void* Kc = ws + pl.off_kc;
    void* Vc = ws + pl.off_vc;
    // the per-branch fp32 output lives in the caller's buffer when one is given
    float* O_la = ex.O_la ? ex.O_la : reinterpret_cast<float*>(ws + pl.off_ola);
    // integer bookkeeping goes straight to the caller's arrays when given
    if (ex.cnt) cnt = ex.cnt;
    if (ex.idx) idx = ex.idx;
    if (ex.n_s) n_s = ex.n_s;

    ProfChain prof_chain;   // the kernels below follow each other on one stream
    // Eq. 22: the merge weights from Q.  On the matrix-core path the softmax kernel makes them itself from the query rows
    // it holds (when those are Q, not queries of the softmax branch's own, and no fp32 side output takes the kernel's
    // other epilogue); otherwise a kernel of its own writes them to the workspace.
    const float* W_fused = nullptr;
    if (ex.W_out != nullptr && pl.combine_mode != 0 && uses_chunk_path(pl) && ex.Q_nla == nullptr && ex.O_nla == nullptr)
        W_fused = ex.W_out;
    else if (ex.W_out != nullptr && pl.combine_mode != 0) {
        float* w = reinterpret_cast<float*>(ws + pl.off_wout);
        ProfScope ps("merge_weights", stream);
        st = launch_merge_weights(pl.B, pl.H * pl.G, pl.L, pl.d, pl.dtype, Q, ex.W_out, w, w + (size_t)pl.BHG * pl.L,
                                  pl.weight_act, pl.G, stream);
        if (st != NATS_OK) return st;
        ex.w_nla = w;
        ex.w_la = w + (size_t)pl.BHG * pl.L;
    }
    // The kernels run one after the other on the caller's stream.  (The softmax branch depends on nothing
    // the preparation of the linear branch computes, but the preparation kernel fills every CU by itself:
    // beside it on a second stream the softmax branch only waited for free slots, and nothing was gained.)
    if (!uses_chunk_path(pl)) {
        ProfScope ps("scan_compact", stream);
        st = launch_scan_compact(pl, mask, Ks, V, cnt, idx, n_s, Kc, Vc, ex.Kc, ex.Vc, ex.cap, nullptr, stream);
    }
    if (st != NATS_OK) return st;
    if (uses_chunk_path(pl)) {
        void* TF = ws + pl.off_tf;
        void* PF = ws + pl.off_p;
        float* gamv = reinterpret_cast<float*>(ws + pl.off_gamv);
        float* kdv = reinterpret_cast<float*>(ws + pl.off_kdv);
        float* gamC = reinterpret_cast<float*>(ws + pl.off_gam);
        float* seg_ws = reinterpret_cast<float*>(ws + pl.off_seg);
        void* VhT = ws + pl.off_vht;
        void* Oh = ws + pl.off_olah;   // fp16 hand-off between the two branches
        // The linear branch first, leaving its rows as fp16; the softmax kernel runs last and merges where its own
        // rows are in registers (the plain sum of Section 4.1 as well as Eq. 21, which needs whole rows of both
        // branches).  With the merge inside the scan instead, its second pass, which runs at the rate its bytes
        // stream at, read the softmax branch's rows on top of its operands and took longer than the softmax
        // kernel saved.
        {
            ProfScope ps("gdn_chunk_inv", stream);
            // (this launch also carries the blocks of the mask scan and compaction)
            st = launch_gdn_chunk_inv(pl, Q, K, alpha, beta, mask, TF, PF, gamv, kdv, gamC, Ks, V, cnt, idx, n_s, Kc, Vc,
                                      ex.Kc, ex.Vc, ex.cap, VhT, stream);
        }
        if (st != NATS_OK) return st;
        st = launch_gdn_seg_scan(pl, Q, K, V, TF, PF, gamv, kdv, gamC, ex.initial_state, ex.final_state, seg_ws, Oh,
                                 ex.O_la, stream);
        if (st != NATS_OK) return st;
        {
            ProfScope ps("flash_softmax", stream);
            st = launch_flash_softmax(pl, Qs, Kc, VhT, Ks, V, cnt, Oh, ex.w_nla, ex.w_la, O, ex.O_nla, ex.lse, stream, W_fused);
        }
    } else {
        {
            ProfScope ps("gdn_recurrent", stream);
            st = launch_gdn_recurrent(pl, Q, K, V, alpha, beta, mask, ex.initial_state, ex.final_state, O_la,
                                      pl.routing == NATS_ROUTE_CHUNK ? reinterpret_cast<float*>(ws + pl.off_snap) : nullptr,
                                      stream);
        }
        if (st != NATS_OK) return st;
        ProfScope ps("softmax_fp32", stream);
        st = launch_softmax_fp32(pl, Qs, Kc, Vc, Ks, V, cnt, O_la, ex.w_nla, ex.w_la, O, ex.O_nla, ex.lse, stream);
    }
    return st;
}

size_t nats_hybrid_attn_bwd_workspace_bytes(const nats_fwd_params* p) {
    FwdPlan pl;
    BwdPlan bp;
    if (validate_bwd_params(p, &pl, &bp) != NATS_OK) return 0;
    return bp.total_grouped;
}

// The backward pass on B x H heads without grouping (pl.G = 1).  ex by value: the optional outputs may be redirected.
static nats_status bwd_core(const FwdPlan& pl, const BwdPlan& bp, const void* Q, const void* K, const void* V,
                            const float* alpha, const float* beta, const uint8_t* mask, const void* dO, float* dQ,
                            float* dK, float* dV, float* dalpha, float* dbeta, nats_bwd_extra ex, char* ws,
                            hipStream_t stream) {
    nats_status st = NATS_OK;
    int32_t* cnt = reinterpret_cast<int32_t*>(ws + pl.off_cnt);
    int32_t* idx = reinterpret_cast<int32_t*>(ws + pl.off_idx);
    int32_t* n_s = reinterpret_cast<int32_t*>(ws + pl.off_ns);
    void* Kc = ws + pl.off_kc;
    void* Vc = ws + pl.off_vc;
    float* O_nla = reinterpret_cast<float*>(ws + bp.off_onla);
    float* lse = reinterpret_cast<float*>(ws + bp.off_lse);
    float* Dvec = reinterpret_cast<float*>(ws + bp.off_dvec);
    float* ckpt = reinterpret_cast<float*>(ws + bp.off_ckpt);
    float* scratch = reinterpret_cast<float*>(ws + bp.off_scratch);
    float* dqp = reinterpret_cast<float*>(ws + bp.off_dqp);
    float* dkp = reinterpret_cast<float*>(ws + bp.off_dkp);
    float* dap = reinterpret_cast<float*>(ws + bp.off_dap);
    float* dbp = reinterpret_cast<float*>(ws + bp.off_dbp);
    const bool chunk = pl.routing == NATS_ROUTE_CHUNK;
    if (chunk && ex.g_la != nullptr) {
        set_error("g_la (the linear score gradient per token) exists with routing per token only; ask for dscore_la");
        return NATS_ERR_UNSUPPORTED;
    }
    if (ex.dscore_nla != nullptr && ex.g_nla == nullptr) ex.g_nla = reinterpret_cast<float*>(ws + bp.off_gnla);
    // routing per chunk, token by token: the sweep's partials of Eq. 17 (by chunks the gradient kernel writes dscore_la)
    float* dslap = (chunk && ex.dscore_la != nullptr && pl.math == NATS_MATH_FP32)
                       ? reinterpret_cast<float*>(ws + bp.off_dslap) : nullptr;
    // The softmax branch's queries and keys, and where their gradients go: with tensors of their own (Section 4.3:
    // the two operations normalise the shared projections differently) dQs / dKs are separate outputs, start from zero,
    // and dQ, dK hold the linear branch's gradients alone.
    const bool own_qk = ex.Q_nla != nullptr;
    const void* Qs = own_qk ? ex.Q_nla : Q;
    const void* Ks = own_qk ? ex.K_nla : K;
    float* dQs = own_qk ? ex.dQ_nla : dQ;
    float* dKs = own_qk ? ex.dK_nla : dK;
    const size_t n_qk = (size_t)pl.BH * pl.L * pl.d;
    ProfChain prof_chain;   // the kernels below follow each other on one stream
    const bool mfma_stats = pl.dtype == NATS_BF16;   // the softmax branch's forward on the matrix cores
    void* VhT = mfma_stats ? ws + bp.off_vht : nullptr;
    {   // what the softmax branch's backward needs from its forward: the compacted cache, lse, the branch output
        ProfScope ps("scan_compact", stream);
        st = launch_scan_compact(pl, mask, Ks, V, cnt, idx, n_s, Kc, Vc, nullptr, nullptr, 0, VhT, stream);
        if (st != NATS_OK) return st;
    }
    if (mfma_stats) {
        ProfScope ps("flash_softmax", stream);
        st = launch_flash_softmax(pl, Qs, Kc, VhT, Ks, V, cnt, nullptr, nullptr, nullptr, nullptr, O_nla, lse, stream);
        if (st != NATS_OK) return st;
    } else {
        ProfScope ps("softmax_fp32", stream);
        st = launch_softmax_fp32(pl, Qs, Kc, Vc, Ks, V, cnt, nullptr, nullptr, nullptr, nullptr, O_nla, lse, stream);
        if (st != NATS_OK) return st;
    }
    float* ops = reinterpret_cast<float*>(ws + bp.off_ops);
    float* Ug = reinterpret_cast<float*>(ws + bp.off_ug);
    float* Uh = reinterpret_cast<float*>(ws + bp.off_uh);
    float* dck = reinterpret_cast<float*>(ws + bp.off_dck);
    const bool by_chunks = pl.math != NATS_MATH_FP32;   // the linear branch's backward by chunks of 64 tokens
    if (by_chunks || !chunk) {   // the linear branch forwards once more by chunks, leaving the state at the start of every chunk
        {
            ProfScope ps("gdn_bwd_prep", stream);
            st = launch_gdn_bwd_prep(pl, Q, K, alpha, beta, mask, ops, stream);
            if (st != NATS_OK) return st;
        }
        ProfScope ps("gdn_chunk_states", stream);
        st = launch_gdn_chunk_states(pl, K, V, ops, ex.initial_state, ckpt, Ug, Uh, stream);
        if (st != NATS_OK) return st;
    } else {   // ... token by token
        ProfScope ps("gdn_checkpoints", stream);
        st = launch_gdn_checkpoints(pl, K, V, alpha, beta, mask, ex.initial_state, ckpt, stream);
        if (st != NATS_OK) return st;
    }
    // The merges of Eq. 21 and its ablation: the linear branch's rows once more in fp32 (from the chunk-start states and
    // U just made, or token by token where the states were made token by token), then the merge's adjoint turns dO into
    // one gradient per branch; from here on each branch runs as for the plain sum.
    const void* dO_s = dO;   // gradient of the softmax branch's rows
    const void* dO_l = dO;   // ... of the linear branch's
    if (bp.merge_mode != 0) {
        float* O_la = reinterpret_cast<float*>(ws + bp.off_mola);
        if (by_chunks || !chunk) {
            ProfScope ps("gdn_chunk_out", stream);
            st = launch_gdn_chunk_out(pl, Q, ops, ckpt, Ug, O_la, stream);
            if (st != NATS_OK) return st;
        } else {
            ProfScope ps("gdn_recurrent", stream);
            st = launch_gdn_recurrent(pl, Q, K, V, alpha, beta, mask, ex.initial_state, nullptr, O_la,
                                      reinterpret_cast<float*>(ws + bp.off_msnap), stream);
            if (st != NATS_OK) return st;
        }
        ProfScope ps("merge_bwd", stream);
        float* dol = reinterpret_cast<float*>(ws + bp.off_mdol);
        float* don = reinterpret_cast<float*>(ws + bp.off_mdon);
        st = launch_merge_bwd(pl, bp.merge_mode, pl.rms_eps, O_la, O_nla, static_cast<const float*>(dO), ex.w_nla,
                              ex.w_la, dol, don, ex.dw_nla, ex.dw_la, stream);
        if (st != NATS_OK) return st;
        dO_s = don;
        dO_l = dol;
    }
    const int32_t* vis = cnt;   // compacted rows visible to a query
    if (chunk) {
        ProfScope ps("visible_rows", stream);
        int32_t* v = reinterpret_cast<int32_t*>(ws + bp.off_vis);
        st = launch_visible_rows(pl, cnt, v, stream);
        if (st != NATS_OK) return st;
        vis = v;
    }
    {   // dQ = the softmax branch's share over the compacted rows (written); also D_i
        ProfScope ps("softmax_bwd_dq", stream);
        st = launch_softmax_bwd_dq(pl, Qs, Kc, Vc, dO_s, vis, O_nla, lse, Dvec, dQs, stream);
        if (st != NATS_OK) return st;
    }
    if (own_qk) {   // the linear branch adds onto dQ, the softmax branch's key gradients scatter into dKs
        ProfScope ps("zero_fill", stream);
        st = launch_zero_f32(dQ, n_qk, stream);
        if (st == NATS_OK) st = launch_zero_f32(dKs, n_qk, stream);
        if (st != NATS_OK) return st;
    }
    if (by_chunks) {
        {   // backwards along the sequence: the state gradient behind every chunk, dV, the partials of dbeta
            ProfScope ps("gdn_chunk_state_grads", stream);
            st = launch_gdn_chunk_state_grads(pl, Q, K, dO_l, mask, ops, dck, Uh, dV, dbp, ex.d_initial_state, stream);
            if (st != NATS_OK) return st;
        }
        // dQ += linear share; dK, dalpha, dbeta = linear share; g_nla cleared
        ProfScope ps("gdn_chunk_grads", stream);
        st = launch_gdn_chunk_grads(pl, Q, K, dO_l, alpha, mask, ops, ckpt, dck, Ug, dV, dbp, dQ, dK, dalpha, dbeta, ex.g_nla,
                                    chunk ? ex.dscore_la : nullptr, stream);
        if (st != NATS_OK) return st;
    } else {
        {
            ProfScope ps("gdn_recurrent_bwd", stream);
            st = launch_gdn_recurrent_bwd(pl, Q, K, V, dO_l, alpha, beta, mask, ckpt, scratch, dqp, dkp, dap, dbp, dV,
                                          ex.d_initial_state, dslap, stream);
            if (st != NATS_OK) return st;
        }
        // dQ += linear share; dK, dalpha, dbeta = linear share; g_nla cleared
        ProfScope ps("bwd_combine", stream);
        st = launch_bwd_combine(pl, dqp, dkp, dap, dbp, dQ, dK, dalpha, dbeta, ex.g_nla, stream);
        if (st != NATS_OK) return st;
    }
    if (chunk) {   // every chunk's inner part of the softmax branch: added to dQ, dK, dV
        ProfScope ps("softmax_bwd_own_chunk", stream);
        st = launch_softmax_bwd_own_chunk(pl, Qs, Ks, V, dO_s, lse, Dvec, dQs, dKs, dV, stream);
        if (st != NATS_OK) return st;
    }
    {   // rows of the softmax tokens in dK, dV (routing per token: their linear share is zero; per chunk: added) and g_nla
        ProfScope ps("softmax_bwd_dkv", stream);
        st = launch_softmax_bwd_dkv(pl, Qs, Kc, Vc, dO_s, vis, idx, n_s, lse, Dvec, dKs, dV, ex.g_nla,
                                    reinterpret_cast<float*>(ws + bp.off_skp), reinterpret_cast<float*>(ws + bp.off_svp),
                                    reinterpret_cast<float*>(ws + bp.off_sgp), stream);
        if (st != NATS_OK) return st;
    }
    if (ex.g_la != nullptr || ex.dscore_nla != nullptr || ex.dscore_la != nullptr) {   // Eq. 16, Eq. 17
        ProfScope ps("score_gradients", stream);
        st = chunk ? launch_score_gradients_chunk(pl, ex.g_nla, dslap, ex.dscore_nla, ex.dscore_la, stream)
                   : launch_score_gradients(pl, beta, mask, dbeta, ex.g_nla, ex.g_la, ex.dscore_nla, ex.dscore_la, stream);
    }
    return st;
}


nats_status nats_hybrid_attn_bwd(const nats_fwd_params* p, const void* Q, const void* K, const void* V,
                                 const float* alpha, const float* beta, const uint8_t* mask, const void* dO,
                                 float* dQ, float* dK, float* dV, float* dalpha, float* dbeta,
                                 const nats_bwd_extra* extra, void* workspace, size_t workspace_bytes,
                                 void* hip_stream) {
    FwdPlan pl;
    BwdPlan bp;
    nats_status st = validate_bwd_params(p, &pl, &bp);
    if (st != NATS_OK) return st;
    if (!Q || !K || !V || !alpha || !beta || !mask || !dO || !dQ || !dK || !dV || !dalpha || !dbeta) {
        set_error("Q, K, V, alpha, beta, mask, dO, dQ, dK, dV, dalpha and dbeta must all be non-NULL");
        return NATS_ERR_NULL;
    }
    if (workspace == nullptr || workspace_bytes < bp.total_grouped) {
        set_error("workspace of %zu bytes given, %zu needed", workspace ? workspace_bytes : (size_t)0, bp.total_grouped);
        return NATS_ERR_WORKSPACE;
    }
    nats_bwd_extra ex;
    memset(&ex, 0, sizeof(ex));
    if (extra) ex = *extra;
    if ((ex.Q_nla == nullptr) != (ex.K_nla == nullptr)) { set_error("Q_nla and K_nla: both or neither"); return NATS_ERR_NULL; }
    if (ex.Q_nla != nullptr && (ex.dQ_nla == nullptr || ex.dK_nla == nullptr)) {
        set_error("with Q_nla and K_nla the gradients dQ_nla and dK_nla must be given");
        return NATS_ERR_NULL;
    }
    if (bp.merge_mode == 0 && (ex.w_nla || ex.w_la || ex.dw_nla || ex.dw_la)) {
        set_error("w_nla, w_la, dw_nla, dw_la belong to combine_mode 1 and 2 (the plain sum has no weights)");
        return NATS_ERR_SHAPE;
    }
    const void* ptrs[] = {Q, K, V, alpha, beta, mask, dO, dQ, dK, dV, dalpha, dbeta, workspace, ex.initial_state,
                          ex.d_initial_state, ex.g_nla, ex.g_la, ex.dscore_nla, ex.dscore_la, ex.Q_nla, ex.K_nla,
                          ex.dQ_nla, ex.dK_nla, ex.w_nla, ex.w_la, ex.dw_nla, ex.dw_la};
    for (const void* ptr : ptrs)
        if (ptr != nullptr && !aligned16(ptr)) { set_error("pointer %p is not 16-byte aligned", ptr); return NATS_ERR_ALIGN; }
    const void* outs[] = {dQ, dK, dV, dalpha, dbeta};
    for (const void* o : outs)
        if (o == Q || o == K || o == V || o == dO || o == alpha || o == beta) {
            set_error("a gradient output must not alias an input");
            return NATS_ERR_SHAPE;
        }

    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    if (bp.merge_mode != 0 && bp.src_dtype == NATS_BF16) {   // the pass runs on fp32 copies (pl.dtype is NATS_F32)
        ProfScope ps("widen_bf16", stream);
        const size_t nd = (size_t)pl.BH * pl.L * pl.d;
        struct { const void** src; size_t off, n; } conv[] = {
            {&Q, bp.off_cq, nd}, {&K, bp.off_ck, nd}, {&V, bp.off_cv, nd * bp.G}, {&dO, bp.off_cdo, nd * bp.G},
            {&ex.Q_nla, bp.off_cqn, nd * bp.G}, {&ex.K_nla, bp.off_ckn, nd * bp.G}};
        for (const auto& c : conv) {
            if (*c.src == nullptr) continue;
            float* dst = reinterpret_cast<float*>(ws + c.off);
            st = launch_widen_bf16(*c.src, dst, c.n, stream);
            if (st != NATS_OK) return st;
            *c.src = dst;
        }
    }
    if (bp.G == 1) return bwd_core(pl, bp, Q, K, V, alpha, beta, mask, dO, dQ, dK, dV, dalpha, dbeta, ex, ws, stream);

    // Head grouping (Section 4.3): member g of every group, i.e. the output heads bh G + g, is a problem of B x H heads
    // with the linear heads' Q, K, alpha, beta and mask.  Its V, dO and initial state are gathered, the pass runs on
    // them, its dV and state gradient go back to its heads, and what it sends to the shared inputs (dQ, dK, dalpha,
    // dbeta, the score gradients) is added up over the members.
    const int G = bp.G;
    const size_t n_tok = (size_t)pl.BH * pl.L, nd = n_tok * pl.d, esz = pl.dtype == NATS_BF16 ? 2 : 4;
    const size_t row = (size_t)pl.L * pl.d, srow = (size_t)pl.d * pl.d;
    void* Vg = ws + bp.off_gv;
    void* dOg = ws + bp.off_gdo;
    float* dVg = reinterpret_cast<float*>(ws + bp.off_gdv);
    float* S0g = reinterpret_cast<float*>(ws + bp.off_gs0);
    float* dS0g = reinterpret_cast<float*>(ws + bp.off_gds0);
    for (int g = 0; g < G; ++g) {
        const bool first = g == 0;
        st = launch_copy_rows(static_cast<const char*>(V) + g * row * esz, G * row * esz, Vg, row * esz, row * esz, pl.BH, stream);
        if (st != NATS_OK) return st;
        st = launch_copy_rows(static_cast<const char*>(dO) + g * row * esz, G * row * esz, dOg, row * esz, row * esz, pl.BH, stream);
        if (st != NATS_OK) return st;
        nats_bwd_extra e1;
        memset(&e1, 0, sizeof(e1));
        if (ex.initial_state) {
            st = launch_copy_rows(ex.initial_state + g * srow, G * srow * 4, S0g, srow * 4, srow * 4, pl.BH, stream);
            if (st != NATS_OK) return st;
            e1.initial_state = S0g;
        }
        if (ex.d_initial_state) e1.d_initial_state = dS0g;
        if (ex.Q_nla) {   // the member's own queries and keys of the softmax branch; its gradients go straight back
            st = launch_copy_rows(static_cast<const char*>(ex.Q_nla) + g * row * esz, G * row * esz, ws + bp.off_gqn, row * esz,
                                  row * esz, pl.BH, stream);
            if (st == NATS_OK)
                st = launch_copy_rows(static_cast<const char*>(ex.K_nla) + g * row * esz, G * row * esz, ws + bp.off_gkn,
                                      row * esz, row * esz, pl.BH, stream);
            if (st != NATS_OK) return st;
            e1.Q_nla = ws + bp.off_gqn;
            e1.K_nla = ws + bp.off_gkn;
            e1.dQ_nla = reinterpret_cast<float*>(ws + bp.off_gdqn);
            e1.dK_nla = reinterpret_cast<float*>(ws + bp.off_gdkn);
        }
        if (bp.merge_mode != 0) {   // the member's weights of the merge (per output head) and their gradients
            const size_t lrow = (size_t)pl.L * 4;
            float* wn = reinterpret_cast<float*>(ws + bp.off_mwn);
            float* wl = reinterpret_cast<float*>(ws + bp.off_mwl);
            if (ex.w_nla) {
                st = launch_copy_rows(ex.w_nla + g * pl.L, G * lrow, wn, lrow, lrow, pl.BH, stream);
                if (st != NATS_OK) return st;
                e1.w_nla = wn;
            }
            if (ex.w_la) {
                st = launch_copy_rows(ex.w_la + g * pl.L, G * lrow, wl, lrow, lrow, pl.BH, stream);
                if (st != NATS_OK) return st;
                e1.w_la = wl;
            }
            if (ex.dw_nla) e1.dw_nla = reinterpret_cast<float*>(ws + bp.off_mdwn);
            if (ex.dw_la) e1.dw_la = reinterpret_cast<float*>(ws + bp.off_mdwl);
        }
        // the first member writes the sums' buffers themselves, the others a buffer of their own that is then added
        if (ex.g_nla) e1.g_nla = first ? ex.g_nla : reinterpret_cast<float*>(ws + bp.off_ggn);
        if (ex.g_la) e1.g_la = first ? ex.g_la : reinterpret_cast<float*>(ws + bp.off_ggl);
        if (ex.dscore_nla) e1.dscore_nla = first ? ex.dscore_nla : reinterpret_cast<float*>(ws + bp.off_gsn);
        if (ex.dscore_la) e1.dscore_la = first ? ex.dscore_la : reinterpret_cast<float*>(ws + bp.off_gsl);
        float* dQg = first ? dQ : reinterpret_cast<float*>(ws + bp.off_gdq);
        float* dKg = first ? dK : reinterpret_cast<float*>(ws + bp.off_gdk);
        float* dag = first ? dalpha : reinterpret_cast<float*>(ws + bp.off_gda);
        float* dbg = first ? dbeta : reinterpret_cast<float*>(ws + bp.off_gdb);
        st = bwd_core(pl, bp, Q, K, Vg, alpha, beta, mask, dOg, dQg, dKg, dVg, dag, dbg, e1, ws, stream);
        if (st != NATS_OK) return st;
        st = launch_copy_rows(dVg, row * 4, dV + g * row, G * row * 4, row * 4, pl.BH, stream);
        if (st != NATS_OK) return st;
        if (ex.d_initial_state) {
            st = launch_copy_rows(dS0g, srow * 4, ex.d_initial_state + g * srow, G * srow * 4, srow * 4, pl.BH, stream);
            if (st != NATS_OK) return st;
        }
        if (e1.dw_nla) {
            st = launch_copy_rows(e1.dw_nla, (size_t)pl.L * 4, ex.dw_nla + g * pl.L, (size_t)G * pl.L * 4, (size_t)pl.L * 4, pl.BH, stream);
            if (st != NATS_OK) return st;
        }
        if (e1.dw_la) {
            st = launch_copy_rows(e1.dw_la, (size_t)pl.L * 4, ex.dw_la + g * pl.L, (size_t)G * pl.L * 4, (size_t)pl.L * 4, pl.BH, stream);
            if (st != NATS_OK) return st;
        }
        if (ex.Q_nla) {
            st = launch_copy_rows(e1.dQ_nla, row * 4, ex.dQ_nla + g * row, G * row * 4, row * 4, pl.BH, stream);
            if (st == NATS_OK) st = launch_copy_rows(e1.dK_nla, row * 4, ex.dK_nla + g * row, G * row * 4, row * 4, pl.BH, stream);
            if (st != NATS_OK) return st;
        }
        if (first) continue;
        struct { float* sum; const float* part; size_t n; } adds[] = {
            {dQ, dQg, nd}, {dK, dKg, nd}, {dalpha, dag, n_tok}, {dbeta, dbg, n_tok},
            {ex.g_nla, e1.g_nla, n_tok}, {ex.g_la, e1.g_la, n_tok},
            {ex.dscore_nla, e1.dscore_nla, n_tok / pl.C}, {ex.dscore_la, e1.dscore_la, n_tok / pl.C}};
        for (const auto& a : adds) {
            if (a.sum == nullptr) continue;
            st = launch_add_f32(a.sum, a.part, a.n, stream);
            if (st != NATS_OK) return st;
        }
    }
    return st;
}

nats_status nats_hybrid_attn_fwd(const nats_fwd_params* p, const void* Q, const void* K, const void* V,
                                 const float* alpha, const float* beta, const uint8_t* mask, void* O,
                                 void* workspace, size_t workspace_bytes, void* hip_stream) {
    return nats_hybrid_attn_fwd_ex(p, Q, K, V, alpha, beta, mask, O, nullptr, workspace, workspace_bytes,
                                   hip_stream);
}

nats_status nats_hybrid_attn_fwd_noalloc(const nats_fwd_params* p, const void* Q, const void* K, const void* V,
                                         const float* alpha, const float* beta, const uint8_t* mask, void* O,
                                         void* hip_stream) {
    FwdPlan pl;
    nats_status st = validate_fwd_params(p, &pl);
    if (st != NATS_OK) return st;
    if (pl.total > (size_t)NATS_NOALLOC_SCRATCH_BYTES) {
        set_error("nats_hybrid_attn_fwd_noalloc: this problem needs %zu bytes of scratch memory, the built-in buffer "
                  "holds %zu; use nats_hybrid_attn_fwd with a workspace", pl.total, (size_t)NATS_NOALLOC_SCRATCH_BYTES);
        return NATS_ERR_WORKSPACE;
    }
    void* ws = nullptr;
    st = noalloc_scratch(&ws);
    if (st != NATS_OK) return st;
    // nothing in the workspace has to start at zero: every kernel writes what it later reads
    return nats_hybrid_attn_fwd_ex(p, Q, K, V, alpha, beta, mask, O, nullptr, ws, (size_t)NATS_NOALLOC_SCRATCH_BYTES,
                                   hip_stream);
}

static nats_status validate_dec_params(const nats_dec_params* p);

nats_status nats_hybrid_attn_decode(const nats_dec_params* p, float* state, void* k_cache, void* v_cache,
                                    int32_t* cache_len, const void* q, const void* k, const void* v,
                                    const float* alpha, const float* beta, const uint8_t* mask,
                                    const float* w_nla, const float* w_la, void* o, int32_t* err_flags,
                                    void* hip_stream) {
    const nats_status vst = validate_dec_params(p);
    if (vst != NATS_OK) return vst;
    if (!state || !k_cache || !v_cache || !cache_len || !q || !k || !v || !alpha || !beta || !mask || !o) {
        set_error("state, caches, cache_len, q, k, v, alpha, beta, mask and o must all be non-NULL");
        return NATS_ERR_NULL;
    }
    const void* ptrs[] = {state, k_cache, v_cache, q, k, v, o};
    for (const void* ptr : ptrs)
        if (!aligned16(ptr)) { set_error("pointer %p is not 16-byte aligned", ptr); return NATS_ERR_ALIGN; }
    const float scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->d);
    const float la_scale = p->la_scale > 0.f ? p->la_scale : 1.0f;
    const float eps = p->rms_eps > 0.f ? p->rms_eps : 1e-6f;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    if (p->workspace != nullptr) {
        const size_t need = decode_split_workspace_bytes(*p);
        if (p->cap > 32768) { set_error("the decode step on a workspace covers caches of at most 32768 rows (cap %d)", p->cap); return NATS_ERR_UNSUPPORTED; }
        if (p->workspace_bytes < need) {
            set_error("decode workspace of %zu bytes given, %zu needed", p->workspace_bytes, need);
            return NATS_ERR_WORKSPACE;
        }
        if (!aligned16(p->workspace)) { set_error("the decode workspace is not 16-byte aligned"); return NATS_ERR_ALIGN; }
        ProfChain prof_chain;
        return launch_decode_split(*p, scale, la_scale, eps, state, k_cache, v_cache, cache_len, q, k, v, alpha, beta,
                                   mask, w_nla, w_la, o, err_flags, static_cast<float*>(p->workspace), stream);
    }
    ProfScope ps("decode", stream);
    return launch_decode(*p, scale, la_scale, eps, state, k_cache, v_cache, cache_len, q, k, v, alpha, beta,
                         mask, w_nla, w_la, o, err_flags, stream);
}

size_t nats_hybrid_attn_decode_workspace_bytes(const nats_dec_params* p) {
    if (validate_dec_params(p) != NATS_OK) return 0;
    return decode_split_workspace_bytes(*p);
}

nats_status nats_merge_weights(const nats_fwd_params* p, const void* Q, const float* W_out, float* w_nla,
                               float* w_la, void* hip_stream) {
    if (p == nullptr) { set_error("params is NULL"); return NATS_ERR_NULL; }
    if (p->dtype != NATS_F32 && p->dtype != NATS_BF16) {
        set_error("dtype %d is neither NATS_F32 nor NATS_BF16", p->dtype);
        return NATS_ERR_DTYPE;
    }
    if (p->B <= 0 || p->H <= 0 || p->L <= 0) {
        set_error("B, H, L must be positive (got %d, %d, %d)", p->B, p->H, p->L);
        return NATS_ERR_SHAPE;
    }
    if (p->d != 64 && p->d != 128) { set_error("d must be 64 or 128 (got %d)", p->d); return NATS_ERR_SHAPE; }
    if (p->weight_act < NATS_WEIGHTS_SOFTMAX || p->weight_act > NATS_WEIGHTS_LINEAR) {
        set_error("weight_act must be a nats_weight_act (got %d)", p->weight_act);
        return NATS_ERR_SHAPE;
    }
    if (!Q || !W_out || !w_nla || !w_la) { set_error("Q, W_out, w_nla and w_la must be non-NULL"); return NATS_ERR_NULL; }
    if (!aligned16(Q) || !aligned16(W_out)) { set_error("Q and W_out must be 16-byte aligned"); return NATS_ERR_ALIGN; }
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    ProfScope ps("merge_weights", stream);
    const int G = p->group > 0 ? p->group : 1;
    if (G > 8) { set_error("group must be between 1 and 8 (got %d)", p->group); return NATS_ERR_SHAPE; }
    return launch_merge_weights(p->B, p->H * G, p->L, p->d, p->dtype, Q, W_out, w_nla, w_la, p->weight_act, G, stream);
}

nats_status nats_route_chunks(int32_t B, int32_t L, int32_t C, int32_t d_model, int32_t H, int32_t dtype,
                              const void* X, const float* W_s, float* scores, uint8_t* mask_c, void* hip_stream) {
    if (dtype != NATS_F32 && dtype != NATS_BF16) { set_error("dtype %d is neither NATS_F32 nor NATS_BF16", dtype); return NATS_ERR_DTYPE; }
    if (B <= 0 || L <= 0 || C <= 0 || H <= 0 || d_model <= 0) {
        set_error("B, L, C, H, d_model must be positive (got %d, %d, %d, %d, %d)", B, L, C, H, d_model);
        return NATS_ERR_SHAPE;
    }
    if (L % C != 0) { set_error("L (%d) must be a multiple of C (%d)", L, C); return NATS_ERR_SHAPE; }
    if (H > 32) { set_error("H must not exceed 32 (got %d)", H); return NATS_ERR_SHAPE; }
    if (d_model % 8 != 0 || d_model > 65536) {
        set_error("d_model must be a multiple of 8 and at most 65536 (got %d)", d_model);
        return NATS_ERR_SHAPE;
    }
    if ((long long)B * (L / C) > (1ll << 31) - 1) { set_error("B * L / C must fit in 31 bits"); return NATS_ERR_SHAPE; }
    if (!X || !W_s || !mask_c) { set_error("X, W_s and mask_c must be non-NULL"); return NATS_ERR_NULL; }
    if (!aligned16(X) || !aligned16(W_s)) { set_error("X and W_s must be 16-byte aligned"); return NATS_ERR_ALIGN; }
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    ProfScope ps("route_chunks", stream);
    return launch_route_chunks(B, L, C, d_model, H, dtype, X, W_s, scores, mask_c, nullptr, nullptr, 0, stream);
}

nats_status nats_merge_weights_from_x(int32_t B, int32_t L, int32_t d_model, int32_t H, int32_t dtype, const void* X,
                                      const float* W_x, int32_t weight_act, float* w_nla, float* w_la, void* hip_stream) {
    if (dtype != NATS_F32 && dtype != NATS_BF16) { set_error("dtype %d is neither NATS_F32 nor NATS_BF16", dtype); return NATS_ERR_DTYPE; }
    if (B <= 0 || L <= 0 || H <= 0 || d_model <= 0) {
        set_error("B, L, H, d_model must be positive (got %d, %d, %d, %d)", B, L, H, d_model);
        return NATS_ERR_SHAPE;
    }
    if (H > 32) { set_error("H must not exceed 32 (got %d)", H); return NATS_ERR_SHAPE; }
    if (d_model % 8 != 0 || d_model > 65536) {
        set_error("d_model must be a multiple of 8 and at most 65536 (got %d)", d_model);
        return NATS_ERR_SHAPE;
    }
    if ((long long)B * L > (1ll << 31) - 1) { set_error("B * L must fit in 31 bits"); return NATS_ERR_SHAPE; }
    if (weight_act < NATS_WEIGHTS_SOFTMAX || weight_act > NATS_WEIGHTS_LINEAR) {
        set_error("weight_act must be a nats_weight_act (got %d)", weight_act);
        return NATS_ERR_SHAPE;
    }
    if (!X || !W_x || !w_nla || !w_la) { set_error("X, W_x, w_nla and w_la must be non-NULL"); return NATS_ERR_NULL; }
    if (!aligned16(X) || !aligned16(W_x)) { set_error("X and W_x must be 16-byte aligned"); return NATS_ERR_ALIGN; }
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    ProfScope ps("merge_weights_from_x", stream);
    // the score layer's kernel with chunks of one token: the same mean (of one row) and linear map
    return launch_route_chunks(B, L, 1, d_model, H, dtype, X, W_x, nullptr, nullptr, w_nla, w_la, weight_act, stream);
}

static nats_status validate_dec_params(const nats_dec_params* p) {
    if (p == nullptr) { set_error("params is NULL"); return NATS_ERR_NULL; }
    if (p->dtype != NATS_F32 && p->dtype != NATS_BF16) {
        set_error("dtype %d is neither NATS_F32 nor NATS_BF16", p->dtype);
        return NATS_ERR_DTYPE;
    }
    if (p->B <= 0 || p->H <= 0 || p->cap <= 0) {
        set_error("B, H, cap must be positive (got %d, %d, %d)", p->B, p->H, p->cap);
        return NATS_ERR_SHAPE;
    }
    if (p->d != 64 && p->d != 128) { set_error("d must be 64 or 128 (got %d)", p->d); return NATS_ERR_SHAPE; }
    if (p->combine_mode < 0 || p->combine_mode > 2) {
        set_error("combine_mode must be 0, 1 or 2 (got %d)", p->combine_mode);
        return NATS_ERR_SHAPE;
    }
    if ((p->linear_op != NATS_LINEAR_GDN && p->linear_op != NATS_LINEAR_GATED) ||
        (p->freeze_on_softmax != 0 && p->freeze_on_softmax != 1)) {
        set_error("linear_op must be a nats_linear_op and freeze_on_softmax 0 or 1 (got %d, %d)", p->linear_op,
                  p->freeze_on_softmax);
        return NATS_ERR_SHAPE;
    }
    if ((p->q_nla == nullptr) != (p->k_nla == nullptr)) { set_error("q_nla and k_nla must be given together"); return NATS_ERR_NULL; }
    if (!aligned16(p->q_nla) || !aligned16(p->k_nla)) { set_error("q_nla and k_nla must be 16-byte aligned"); return NATS_ERR_ALIGN; }
    return NATS_OK;
}

static nats_status validate_chunk_state(const nats_dec_chunk_state* s) {
    if (s == nullptr) { set_error("chunk state is NULL"); return NATS_ERR_NULL; }
    if (!s->state || !s->state_start || !s->chunk_decay || !s->chunk_pos || !s->k_cache || !s->v_cache ||
        !s->cache_len) {
        set_error("every pointer of the chunk state must be non-NULL");
        return NATS_ERR_NULL;
    }
    const void* ptrs[] = {s->state, s->state_start, s->k_cache, s->v_cache};
    for (const void* ptr : ptrs)
        if (!aligned16(ptr)) { set_error("pointer %p is not 16-byte aligned", ptr); return NATS_ERR_ALIGN; }
    return NATS_OK;
}

nats_status nats_hybrid_attn_decode_chunk(const nats_dec_params* p, const nats_dec_chunk_state* s, const void* q,
                                          const void* k, const void* v, const float* alpha, const float* beta,
                                          const float* w_nla, const float* w_la, void* o, int32_t* err_flags,
                                          void* hip_stream) {
    nats_status st = validate_dec_params(p);
    if (st != NATS_OK) return st;
    st = validate_chunk_state(s);
    if (st != NATS_OK) return st;
    if (!q || !k || !v || !alpha || !beta || !o) {
        set_error("q, k, v, alpha, beta and o must all be non-NULL");
        return NATS_ERR_NULL;
    }
    const void* ptrs[] = {q, k, v, o};
    for (const void* ptr : ptrs)
        if (!aligned16(ptr)) { set_error("pointer %p is not 16-byte aligned", ptr); return NATS_ERR_ALIGN; }
    const float scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->d);
    const float la_scale = p->la_scale > 0.f ? p->la_scale : 1.0f;
    const float eps = p->rms_eps > 0.f ? p->rms_eps : 1e-6f;
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    ProfScope ps("decode_chunk", stream);
    return launch_decode_chunk(*p, scale, la_scale, eps, s->state, s->state_start, s->chunk_decay, s->chunk_pos,
                               s->k_cache, s->v_cache, s->cache_len, q, k, v, alpha, beta, w_nla, w_la, o, err_flags,
                               stream);
}

nats_status nats_hybrid_attn_decode_commit(const nats_dec_params* p, const nats_dec_chunk_state* s,
                                           const uint8_t* mask_c, int32_t* err_flags, void* hip_stream) {
    nats_status st = validate_dec_params(p);
    if (st != NATS_OK) return st;
    st = validate_chunk_state(s);
    if (st != NATS_OK) return st;
    if (!mask_c) { set_error("mask_c is NULL"); return NATS_ERR_NULL; }
    hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
    ProfScope ps("decode_commit", stream);
    return launch_decode_commit(*p, s->state, s->state_start, s->chunk_decay, s->chunk_pos, s->cache_len, mask_c,
                                err_flags, stream);
}

}  // extern "C"
