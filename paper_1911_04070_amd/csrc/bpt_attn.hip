// Graph self-attention with tree relative positions (paper Sec. 3.1 eq. (6),
// Sec. 3.4 eq. (8)) forward and backward for gfx950: the host side.  Chooses per call
// between the gather kernels (attn_gather.h: fp32 tensors, fallback) and the matrix-core
// kernels over dense tiles (attn_token_tiles.h, attn_span_tiles.h, attn_key_tiles.h: bf16),
// lays out the workspace, launches, and exports the C entry points of bpt.h.
#include <algorithm>
#include <cmath>
#include <mutex>

#include "attn_device.h"
#include "attn_gather.h"
#include "attn_token_tiles.h"
#include "attn_span_tiles.h"
#include "attn_key_tiles.h"

// Scratch of bpt_attn_fwd_static: device memory that belongs to the library's code object, so that the call
// needs no allocation.  Every device the library is loaded on holds its own copy at its own address; the name
// below is only the host-side handle of the symbol -- device code and HIP calls get the address that
// hipGetSymbolAddress returns for the current device (static_scratch()).
constexpr size_t kStaticScratchBytes = (size_t)BPT_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace bpt {
namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];      // per device: address of that device's copy of `scratch`
std::mutex g_scratch_mutex;
}  // namespace

// Address of the current device's copy of the static scratch (resolved once per device; `device` must be current).
int static_scratch(int device, void** out) {
    if (device < 0 || device >= kMaxDevices) return BPT_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[device]) {
        void* ptr = nullptr;
        BPT_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) return BPT_ERR_LAUNCH;
        g_scratch_ptr[device] = ptr;
    }
    *out = g_scratch_ptr[device];
    return BPT_OK;
}

namespace {

// ---- host side --------------------------------------------------------------------
constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct DeviceLimits {
    int cus = 0;
    size_t lds = 0;     // LDS one workgroup may use
    size_t lds_cu = 0;  // LDS of one compute unit, shared by its resident workgroups
};

int device_limits(const bpt_graph* g, DeviceLimits* out) {
    int lds = 0, lds_cu = 0;
    BPT_HIP(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, g->device));
    if (hipDeviceGetAttribute(&lds_cu, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, g->device) != hipSuccess) {
        (void)hipGetLastError();
        lds_cu = 0;
    }
    out->cus = g->num_cus > 0 ? g->num_cus : 256;
    out->lds = lds > 0 ? (size_t)lds : 65536;
    out->lds_cu = std::max<size_t>(out->lds, lds_cu > 0 ? (size_t)lds_cu : 0);
    return BPT_OK;
}

int check_shape(const bpt_graph* g, const bpt_shape_t* s) {
    if (!g || !s) return BPT_ERR_INVALID_ARG;
    if (s->B < 1 || s->H < 1) return BPT_ERR_INVALID_ARG;
    if (s->D != kD) return BPT_ERR_UNSUPPORTED;
    if (s->dtype != BPT_F32 && s->dtype != BPT_BF16) return BPT_ERR_UNSUPPORTED;
    if (s->stride_n < kD || (s->stride_n % 8) || (s->stride_h % 8) || (s->stride_b % 8)) return BPT_ERR_INVALID_ARG;
    if (s->stride_h < 0 || s->stride_b < 0) return BPT_ERR_INVALID_ARG;
    if (!(s->dropout_p >= 0.f && s->dropout_p < 1.f)) return BPT_ERR_INVALID_ARG;
    // gradients rounded to bf16 are for bf16 tensors
    if (s->grad_dtype != BPT_F32 && !(s->grad_dtype == BPT_BF16 && s->dtype == BPT_BF16)) return BPT_ERR_INVALID_ARG;
    // a batch graph carries the lengths itself; dropout masks are defined on the nodes of one tree
    if (g->batch > 0 && s->seq_len) return BPT_ERR_INVALID_ARG;
    if (g->batch > 0 && s->dropout_p > 0.f) return BPT_ERR_UNSUPPORTED;
    if ((int64_t)s->B * s->H > (int64_t)INT32_MAX / std::max(1, std::max(g->fwd.num_tiles, g->tr.num_tiles)))
        return BPT_ERR_UNSUPPORTED;
    if ((int64_t)s->B * s->H * g->num_nodes > (int64_t)1 << 40) return BPT_ERR_UNSUPPORTED;
    if (g->num_edges >= ((int64_t)1 << 29)) return BPT_ERR_UNSUPPORTED;  // 32-bit byte offsets into the edge arrays
    // the gathers address one (batch, head) slab with 32-bit byte offsets
    const int64_t es = s->dtype == BPT_BF16 ? 2 : 4;
    if (s->stride_n * es >= (1 << 24) || (int64_t)g->num_nodes * s->stride_n * es >= ((int64_t)1 << 31))
        return BPT_ERR_UNSUPPORTED;
    return BPT_OK;
}

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Workgroups of `kernel` one compute unit holds at once: the larger of the runtime's
// occupancy figure and an estimate from the kernel's registers (512 per SIMD lane,
// shared by at most 8 resident wavefronts per SIMD, 4 SIMDs) and the LDS of the whole
// compute unit.  Over-estimating is harmless for a persistent launch: surplus
// workgroups start when others finish and still take only their own share of the work.
template <typename K>
int resident_blocks(K kernel, int threads, size_t dyn_lds, const DeviceLimits& lim) {
    int api = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&api, kernel, threads, dyn_lds) != hipSuccess) {
        (void)hipGetLastError();
        api = 0;
    }
    int est = 0;
    hipFuncAttributes fa;
    if (hipFuncGetAttributes(&fa, reinterpret_cast<const void*>(kernel)) == hipSuccess) {
        const int regs = std::max(8, (fa.numRegs + 7) / 8 * 8);
        const int waves_per_simd = std::min(8, 512 / regs);
        const int wg_waves_per_simd = (threads / 64 + 3) / 4;
        const size_t lds = dyn_lds + fa.sharedSizeBytes;
        est = waves_per_simd / wg_waves_per_simd;
        if (lds > 0) est = std::min<int>(est, (int)(lim.lds_cu / lds));
        est = std::min(est, 2048 / threads);
    } else {
        (void)hipGetLastError();
    }
    return std::max(1, std::max(api, est));
}

// Grid of a persistent launch: resident workgroups per compute unit times their number,
// rounded down to a multiple of 8 (one share of the tile space per XCD).
template <typename K>
int persistent_grid(K kernel, int threads, size_t lds, const DeviceLimits& lim, int* grid) {
    if (lds > 65536)
        BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    *grid = std::max(8, lim.cus * resident_blocks(kernel, threads, lds, lim) / 8 * 8);
    return BPT_OK;
}

template <typename K>
int launch(const char* name, K kernel, int grid, int threads, size_t lds, hipStream_t st, const AttnArgs& a) {
    BPT_LAUNCH(name, kernel, dim3(grid), dim3(threads), lds, st, a);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

void fill_common(AttnArgs& a, const bpt_graph* g, const bpt_shape_t* s) {
    a = AttnArgs();
    a.sb = s->stride_b;
    a.sh = s->stride_h;
    a.sn = s->stride_n;
    a.BH = s->B * s->H;
    a.H = s->H;
    a.N = g->num_nodes;
    a.n_tokens = g->n_tokens;
    a.scale = s->scale > 0.f ? s->scale : 0.125f;  // 1/sqrt(64)
    a.rel_rows = g->num_levels * g->rel_width;
    const int64_t es = s->dtype == BPT_BF16 ? 2 : 4;
    a.row_bytes = (int32_t)(s->stride_n * es);
    a.slab_bytes = (uint32_t)(((int64_t)(g->num_nodes - 1) * s->stride_n + kD) * es);
    a.idx_bytes = (uint32_t)(g->num_edges * 4);
    a.seq_len = s->seq_len;
    a.leave_unkept = s->seq_len && s->leave_unkept ? 1 : 0;
    a.grad_bf16 = s->grad_dtype == BPT_BF16 ? 1 : 0;
    a.delta = nullptr;
    a.lse_sb = (int64_t)s->H * g->num_nodes;
    a.lse_sh = g->num_nodes;
    a.lg = g->num_levels - 1;
    const double p = s->dropout_p > 0.f ? (double)s->dropout_p : 0.0;
    a.drop_thr = p > 0.0 ? (uint32_t)std::min(std::floor(p * 4294967296.0), 4294967295.0) : 0u;
    a.drop_seed = s->dropout_seed;
    a.drop_inv_keep = p > 0.0 ? (float)(1.0 / (1.0 - p)) : 1.f;
}

void use_schedule(AttnArgs& a, const Schedule& sc) {
    a.seg_row = sc.seg_row;
    a.seg_begin = sc.seg_begin;
    a.seg_part = sc.seg_part;
    a.tile_ptr = sc.tile_ptr;
    a.num_tiles = sc.num_tiles;
    a.num_part = sc.num_part;
}

// LDS of fwd_tile_kernel for this graph, or 0 if the tile path does not apply
struct TilePlan {
    bool ok = false;       // the token tile kernels apply
    bool rel_lds = false;  // with the compact relative-position table staged in LDS
    int cid_pad = 0, bias_stride = 0;
    size_t lds = 0;
};
// dense: the plan of bwd_q_tile_kernel<.., DENSE> -- ids padded to 32, two more [16][bias_stride] fp32
// tables per wavefront, and the relative-position table must be in LDS
TilePlan plan_tiles(const bpt_graph* g, const DeviceLimits& lim, bool dense = false) {
    TilePlan t;
    if (g->tiles.num_tiles == 0) return t;
    t.cid_pad = dense ? (g->tiles.num_cids + 31) & ~31 : (g->tiles.num_cids + 15) & ~15;
    t.bias_stride = t.cid_pad + ((4 - t.cid_pad % 32) + 32) % 32;  // = 4 mod 32: the 16 token rows hit different banks
    const size_t rel = (size_t)t.cid_pad * kRelStride * sizeof(bf16_t);
    const size_t rest = (size_t)kTileWaves * 16 * t.bias_stride * sizeof(float) +
                        (size_t)kTileWaves * 64 * kRowStride * sizeof(bf16_t) +
                        (size_t)t.cid_pad * sizeof(int32_t) +   // relative-position ids of the compact ids (dropout)
                        (dense ? (size_t)kTileWaves * 32 * t.bias_stride * sizeof(float) : 0);
    const size_t room = lim.lds - (kMaxLenBatch + 1) * sizeof(int32_t) - 16;   // the kernels' static LDS (prefix sums of a length mix)
    t.rel_lds = rel + rest <= room;
    t.lds = t.rel_lds ? rel + rest : rest;
    // (dense: dS of a tile, bf16 hi and lo with 16 bytes of padding per row, has to fit a wavefront's row buffers)
    t.ok = dense ? t.rel_lds && 64 * (t.cid_pad + 8) <= 64 * kRowStride * (int)sizeof(bf16_t) : t.lds <= room;
    return t;
}

void fill_tile_args(TileArgs& t, const bpt_graph* g, const AttnArgs& a, const TilePlan& tp);

// grid: workgroups to launch, or 0 for as many as the device holds at once
template <typename K>
int launch_tiles(const char* name, K kernel, const TileArgs& t, const DeviceLimits& lim, size_t lds, hipStream_t st,
                 int grid = 0) {
    if (lds > 65536)
        BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    if (grid <= 0) grid = std::max(8, lim.cus * resident_blocks(kernel, kTileThreads, lds, lim) / 8 * 8);
    BPT_LAUNCH(name, kernel, dim3(grid), dim3(kTileThreads), lds, st, t);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

// workgroups of bwd_q_tile_kernel<.., DENSE>: its LDS allows one per compute unit; fixed, because every
// workgroup leaves a copy of d_rel and the workspace is sized for them
int dense_grid(const DeviceLimits& lim) { return std::max(8, lim.cus / 8 * 8); }

// bf16 backward, query side of the token rows on dense tiles
int run_bwd_q_tiles(const bpt_graph* g, const AttnArgs& a, const DeviceLimits& lim, bool dense, hipStream_t st) {
    const TilePlan tp = plan_tiles(g, lim, dense);
    TileArgs t = {};
    fill_tile_args(t, g, a, tp);
    if (dense) {   // no (w, p) pairs: the kernel leaves one copy of d_rel per workgroup
        t.drel_part = a.drel_part;
        const int grid = dense_grid(lim);
        if (a.delta) return launch_tiles("bwd_q_tile_kernel", bwd_q_tile_kernel<true, false, true, true>, t, lim, tp.lds, st, grid);
        return a.drop_thr ? launch_tiles("bwd_q_tile_kernel", bwd_q_tile_kernel<true, true, true>, t, lim, tp.lds, st, grid)
                          : launch_tiles("bwd_q_tile_kernel", bwd_q_tile_kernel<true, false, true>, t, lim, tp.lds, st, grid);
    }
    if (a.delta)   // a packed batch (no dropout there)
        return tp.rel_lds ? launch_tiles("bwd_q_tile_kernel", bwd_q_tile_kernel<true, false, false, true>, t, lim, tp.lds, st)
                          : launch_tiles("bwd_q_tile_kernel", bwd_q_tile_kernel<false, false, false, true>, t, lim, tp.lds, st);
    if (a.drop_thr)
        return tp.rel_lds ? launch_tiles("bwd_q_tile_kernel", bwd_q_tile_kernel<true, true>, t, lim, tp.lds, st)
                          : launch_tiles("bwd_q_tile_kernel", bwd_q_tile_kernel<false, true>, t, lim, tp.lds, st);
    return tp.rel_lds ? launch_tiles("bwd_q_tile_kernel", bwd_q_tile_kernel<true, false>, t, lim, tp.lds, st)
                      : launch_tiles("bwd_q_tile_kernel", bwd_q_tile_kernel<false, false>, t, lim, tp.lds, st);
}

void fill_tile_args(TileArgs& t, const bpt_graph* g, const AttnArgs& a, const TilePlan& tp) {
    t.dout = static_cast<const bf16_t*>(a.dout);
    t.lse_r = a.lse_r;
    t.dQ = a.dQ;
    t.stat = a.stat;
    t.wp = a.wp;
    t.Q = static_cast<const bf16_t*>(a.Q);
    t.K = static_cast<const bf16_t*>(a.K);
    t.V = static_cast<const bf16_t*>(a.V);
    t.rel = static_cast<const bf16_t*>(a.rel);
    t.out = static_cast<bf16_t*>(a.out);
    t.lse = a.lse_w;
    t.sb = a.sb;
    t.sh = a.sh;
    t.sn = a.sn;
    t.BH = a.BH;
    t.H = a.H;
    t.N = a.N;
    t.scale = a.scale;
    t.chunk_ptr = g->tiles.chunk_ptr;
    t.cols = g->tiles.cols;
    t.cid_to_id = g->tiles.cid_to_id;
    t.map = g->tiles.map;
    t.num_tiles = g->tiles.num_tiles;
    t.num_chunks = g->tiles.num_chunks;
    t.num_cids = g->tiles.num_cids;
    t.cid_pad = tp.cid_pad;
    t.bias_stride = tp.bias_stride;
    t.row_bytes = a.row_bytes;
    t.slab_bytes = a.slab_bytes;
    t.seq_len = a.seq_len;
    t.leave_unkept = a.leave_unkept;
    t.grad_bf16 = a.grad_bf16;
    t.delta = a.delta;
    t.levels = g->num_levels;
    t.lg = g->num_levels - 1;
    t.lse_sb = a.lse_sb;
    t.lse_sh = a.lse_sh;
    t.id_to_cid = g->tiles.id_to_cid;
    t.n = g->n;
    t.k = g->k;
    t.W = g->rel_width;
    t.ctx_levels = g->ctx_levels;
    t.causal = g->causal;
    t.drop_thr = a.drop_thr;
    t.drop_seed = a.drop_seed;
    t.drop_inv_keep = a.drop_inv_keep;
}

// Span rows on blocks of 32 tokens (fwd_span_tile_kernel, bwd_q_span_tile_kernel): needs the token
// tiles (so that the gather kernels are not needed for token rows either), at least one block,
// and at most 16 levels above the blocks.
bool span_tiles_ok(const bpt_graph* g) {
    return g->tiles.num_tiles > 0 && g->n >= kSpanTok && g->num_levels - 1 - kSpanInLevels <= 16;
}
// partial rows per (batch, head): one per block and ancestor level
size_t span_partials(const bpt_graph* g) {
    const int L = g->num_levels - 1;
    return span_tiles_ok(g) && L > kSpanInLevels ? (size_t)(L - kSpanInLevels) * (g->n / kSpanTok) : 0;
}
void fill_span_args(SpanArgs& t, const bpt_graph* g, const AttnArgs& a) {
    t = SpanArgs();
    t.Q = static_cast<const bf16_t*>(a.Q);
    t.K = static_cast<const bf16_t*>(a.K);
    t.V = static_cast<const bf16_t*>(a.V);
    t.rel = static_cast<const bf16_t*>(a.rel);
    t.dout = static_cast<const bf16_t*>(a.dout);
    t.out = static_cast<bf16_t*>(a.out);
    t.lse = a.lse_w;
    t.lse_r = a.lse_r;
    t.dQ = a.dQ;
    t.stat = a.stat;
    t.part = a.part;
    t.sb = a.sb;
    t.sh = a.sh;
    t.sn = a.sn;
    t.BH = a.BH;
    t.H = a.H;
    t.N = a.N;
    t.n = g->n;
    t.L = g->num_levels - 1;
    t.W = g->rel_width;
    t.zero = g->k + 1;
    t.scale = a.scale;
    t.seq_len = a.seq_len;
    t.leave_unkept = a.leave_unkept;
    t.grad_bf16 = a.grad_bf16;
    t.delta = a.delta;
    t.lse_sb = a.lse_sb;
    t.lse_sh = a.lse_sh;
    t.drop_thr = a.drop_thr;
    t.drop_seed = a.drop_seed;
    t.drop_inv_keep = a.drop_inv_keep;
}
// forward == true: out and lse of all span rows; else delta, lse and dQ of all span rows
int run_span_tiles(const bpt_graph* g, const AttnArgs& a, bool forward, hipStream_t st) {
    SpanArgs t;
    fill_span_args(t, g, a);
    const int64_t items = (int64_t)a.BH * (g->n / kSpanTok);
    const unsigned grid = (unsigned)((items + kTileWaves - 1) / kTileWaves);
    const size_t lds = (size_t)kTileWaves * kSpanTok * kVStride * sizeof(bf16_t);
    if (t.delta && forward)
        BPT_LAUNCH("fwd_span_tile_kernel", (fwd_span_tile_kernel<false, true>), dim3(grid), dim3(kTileThreads), lds, st, t);
    else if (t.delta && t.grad_bf16)
        BPT_LAUNCH("bwd_q_span_tile_kernel", (bwd_q_span_tile_kernel<false, true, true>), dim3(grid), dim3(kTileThreads), lds, st, t);
    else if (t.delta)
        BPT_LAUNCH("bwd_q_span_tile_kernel", (bwd_q_span_tile_kernel<false, false, true>), dim3(grid), dim3(kTileThreads), lds, st, t);
    else if (forward && t.drop_thr)
        BPT_LAUNCH("fwd_span_tile_kernel", fwd_span_tile_kernel<true>, dim3(grid), dim3(kTileThreads), lds, st, t);
    else if (forward)
        BPT_LAUNCH("fwd_span_tile_kernel", fwd_span_tile_kernel<false>, dim3(grid), dim3(kTileThreads), lds, st, t);
    else if (t.drop_thr && t.grad_bf16)
        BPT_LAUNCH("bwd_q_span_tile_kernel", (bwd_q_span_tile_kernel<true, true>), dim3(grid), dim3(kTileThreads), lds, st, t);
    else if (t.drop_thr)
        BPT_LAUNCH("bwd_q_span_tile_kernel", (bwd_q_span_tile_kernel<true, false>), dim3(grid), dim3(kTileThreads), lds, st, t);
    else if (t.grad_bf16)
        BPT_LAUNCH("bwd_q_span_tile_kernel", (bwd_q_span_tile_kernel<false, true>), dim3(grid), dim3(kTileThreads), lds, st, t);
    else
        BPT_LAUNCH("bwd_q_span_tile_kernel", (bwd_q_span_tile_kernel<false, false>), dim3(grid), dim3(kTileThreads), lds, st, t);
    BPT_HIP(hipGetLastError());
    if (t.L > kSpanInLevels) {
        // rows of levels 6..9 (at most 16 partials each), then the longer rows
        const int first = 2 * g->n - ((2 * g->n) >> (kSpanInLevels + 1));
        const int big_level = kSpanInLevels + 1 + kSpanSmallLevels;
        const int first_big = t.L >= big_level ? 2 * g->n - ((2 * g->n) >> big_level) : g->num_nodes;
        const int rows_small = first_big - first, rows_big = g->num_nodes - first_big;
        const int per_block = kSpanBigThreads / 64;   // short rows per workgroup
        const int small_blocks = (int)(((int64_t)a.BH * rows_small + per_block - 1) / per_block);
        const unsigned mgrid = (unsigned)(small_blocks + (int64_t)a.BH * rows_big);
        if (forward && t.delta)
            BPT_LAUNCH("fwd_span_merge_kernel", fwd_span_merge_kernel<true>, dim3(mgrid), dim3(kSpanBigThreads), 0, st, t, first,
                       rows_small, first_big, rows_big, small_blocks);
        else if (forward)
            BPT_LAUNCH("fwd_span_merge_kernel", fwd_span_merge_kernel<false>, dim3(mgrid), dim3(kSpanBigThreads), 0, st, t, first,
                       rows_small, first_big, rows_big, small_blocks);
        else if (t.delta)
            BPT_LAUNCH("bwd_q_span_merge_kernel", bwd_q_span_merge_kernel<true>, dim3(mgrid), dim3(kSpanBigThreads), 0, st, t, first,
                       rows_small, first_big, rows_big, small_blocks);
        else
            BPT_LAUNCH("bwd_q_span_merge_kernel", bwd_q_span_merge_kernel<false>, dim3(mgrid), dim3(kSpanBigThreads), 0, st, t, first,
                       rows_small, first_big, rows_big, small_blocks);
        BPT_HIP(hipGetLastError());
    }
    return BPT_OK;
}

// bf16 forward: token rows as dense tiles on the matrix cores, span rows with the gather kernel
int run_fwd_tiles(const bpt_graph* g, AttnArgs& a, const DeviceLimits& lim, const TilePlan& tp, hipStream_t st) {
    TileArgs t = {};
    fill_tile_args(t, g, a, tp);
    if (a.delta)   // a packed batch (no dropout there)
        return tp.rel_lds ? launch_tiles("fwd_tile_kernel", fwd_tile_kernel<true, false, true>, t, lim, tp.lds, st)
                          : launch_tiles("fwd_tile_kernel", fwd_tile_kernel<false, false, true>, t, lim, tp.lds, st);
    if (a.drop_thr)
        return tp.rel_lds ? launch_tiles("fwd_tile_kernel", fwd_tile_kernel<true, true>, t, lim, tp.lds, st)
                          : launch_tiles("fwd_tile_kernel", fwd_tile_kernel<false, true>, t, lim, tp.lds, st);
    return tp.rel_lds ? launch_tiles("fwd_tile_kernel", fwd_tile_kernel<true, false>, t, lim, tp.lds, st)
                      : launch_tiles("fwd_tile_kernel", fwd_tile_kernel<false, false>, t, lim, tp.lds, st);
}

template <typename T>
int run_fwd(const bpt_graph* g, AttnArgs& a, hipStream_t st) {
    DeviceLimits lim;
    int rc = device_limits(g, &lim);
    if (rc) return rc;
    if (sizeof(T) == 2) {
        const TilePlan tp = plan_tiles(g, lim);
        if (tp.ok) {
            if ((rc = run_fwd_tiles(g, a, lim, tp, st))) return rc;
            if (span_tiles_ok(g)) return run_span_tiles(g, a, true, st);
            use_schedule(a, g->fwd_span);  // the gather kernel below only sees span rows
        }
    }
    const int ctx_rows = g->ctx_levels * g->rel_width;
    const size_t rel_b = (size_t)ctx_rows * kD * sizeof(T);
    const bool rel_lds = rel_b <= lim.lds;
    a.rel_rows_lds = rel_lds ? ctx_rows : 0;
    const size_t lds = rel_lds ? rel_b : 0;
    int grid = 8;
    if (rel_lds) {
        if ((rc = persistent_grid(fwd_kernel<T, true>, kThreads, lds, lim, &grid))) return rc;
        rc = launch("fwd_kernel", fwd_kernel<T, true>, grid, kThreads, lds, st, a);
    } else {
        if ((rc = persistent_grid(fwd_kernel<T, false>, kThreads, 0, lim, &grid))) return rc;
        rc = launch("fwd_kernel", fwd_kernel<T, false>, grid, kThreads, 0, st, a);
    }
    if (rc) return rc;
    const Schedule& sc = a.seg_row == g->fwd_span.seg_row ? g->fwd_span : g->fwd;
    if (sc.num_multi > 0) {
        const int items = a.BH * sc.num_multi;
        BPT_LAUNCH("fwd_merge_kernel", fwd_merge_kernel<T>, dim3((items + 3) / 4), dim3(256), 0, st, a, sc.multi_row, sc.multi_ptr,
                           sc.num_multi);
        BPT_HIP(hipGetLastError());
    }
    return BPT_OK;
}

// Workspace layout of the backward and the launch shape of rel_grad_kernel.
constexpr int kQueueInts = 8 * 16;   // one counter per XCD, 64 bytes apart
struct BwdPlan {
    int drel_rows = 0;        // d_rel rows token rows can touch
    bool drel_mfma = false;   // bf16 tensors: rel_grad_mfma_kernel; fp32: rel_grad_kernel
    bool drel_tile = false;   // bf16 tensors with token tiles and at most 256 ids in use: rel_grad_tile_kernel
    int drel_part_rows = 0;   // rows of one workgroup's copy of d_rel
    bool q_tiles = false;     // query side of token rows on dense tiles (bwd_q_tile_kernel)
    bool dense_ds = false;    // ... which also forms d_rel (one copy per wavefront): no (w, p) pairs, no d_rel kernel
    bool kv_tiles = false;    // key side on dense tiles of key nodes (bwd_kv_tile_kernel)
    bool kv_chain = false;    // ... with at most 32 ids per tile: bwd_kv_chain_kernel (tasks that walk several tiles)
    size_t kv_lds = 0;
    int drel_ipw = 32;        // ids per wavefront: 8, 16 or 32
    int drel_block = 32;      // token rows per block
    int drel_grid_x = 8, drel_grid_y = 1;
    size_t drel_lds = 0;
    size_t off_stat = 0, off_wp = 0, off_qpart = 0, off_kvpart = 0, off_drel = 0, off_queue = 0, total = 0;
};

int plan_bwd(const bpt_graph* g, const bpt_shape_t* s, BwdPlan* p) {
    DeviceLimits lim;
    int rc = device_limits(g, &lim);
    if (rc) return rc;
    p->drel_rows = g->ctx_levels * g->rel_width;
    int64_t blocks;
    if (s->dtype == BPT_BF16) {  // matrix-core kernel
        p->drel_mfma = true;
        const int nids = std::min(kRgIds, (p->drel_rows + 31) & ~31);
        p->drel_lds = ((size_t)2 * nids + kD) * kRgStride * sizeof(bf16_t);
        // dense tiles for the query side: when one workgroup of the d_rel kernel can hold all ids in use
        const int cids = (g->tiles.num_cids + 31) & ~31;
        const size_t rg_lds = ((size_t)2 * cids * kRgStride + kRgRows * kRowStride + (size_t)cids * kRelStride) * sizeof(bf16_t);
        if (plan_tiles(g, lim).ok && cids <= kRgTileMaxIds && rg_lds + 256 <= lim.lds) {
            p->q_tiles = true;
            p->drel_tile = true;
            p->drel_part_rows = cids;
            p->drel_lds = rg_lds;
            if (cids <= 16 * kDenseChunks && plan_tiles(g, lim, true).ok) p->dense_ds = true;
        }
        if (g->ktiles.num_tasks > 0 && g->ktiles.nb_pad <= 16 * kMaxBiasChunks) {
            const int parked = std::max(0, g->ktiles.nb_pad / 16 - kRegBiasChunks);   // table operands kept in LDS
            p->kv_lds = (size_t)kTileWaves * (32 * (g->ktiles.nb_pad + 1) * sizeof(float) + 64 * kRowStride * sizeof(bf16_t) +
                                              32 * sizeof(float2) + 32 * sizeof(uint32_t) + (size_t)parked * 64 * 32);
            p->kv_tiles = p->kv_lds <= lim.lds;
            const size_t chain_lds = (size_t)kTileWaves * (64 * kRowStride * sizeof(bf16_t) + 16 * kKvOutStride * sizeof(float) +
                                                            32 * sizeof(float2) + 32 * sizeof(uint32_t));
            if (g->ktiles.nb_pad <= 32 && chain_lds <= lim.lds) {
                p->kv_tiles = p->kv_chain = true;
                p->kv_lds = chain_lds;
            }
        }
        p->drel_grid_y = p->drel_tile ? 1 : (p->drel_rows + kRgIds - 1) / kRgIds;
        blocks = (int64_t)s->B * s->H * ((g->n_tokens + kRgRows - 1) / kRgRows);
    } else {
        p->drel_ipw = p->drel_rows <= 64 ? 8 : p->drel_rows <= 128 ? 16 : 32;
        const int chunk = p->drel_ipw * kWaves;
        p->drel_block = std::min(g->n_tokens, chunk > 128 ? 32 : 64);
        p->drel_lds = (size_t)p->drel_block * (chunk + kD) * sizeof(float);
        p->drel_grid_y = (p->drel_rows + chunk - 1) / chunk;
        blocks = (int64_t)s->B * s->H * ((g->n_tokens + p->drel_block - 1) / p->drel_block);
    }
    const int per_cu = (int)std::max<size_t>(1, std::min<size_t>(4, lim.lds_cu / p->drel_lds));
    p->drel_grid_x = (int)std::max<int64_t>(1, std::min<int64_t>(blocks, (int64_t)lim.cus * per_cu / p->drel_grid_y));
    if (p->dense_ds) p->drel_grid_x = dense_grid(lim);   // copies of d_rel: one per workgroup of bwd_q_tile_kernel
    const size_t bh = (size_t)s->B * s->H;
    size_t off = 0;
    p->off_stat = off;
    off += align_up(bh * g->num_nodes * sizeof(float2));
    p->off_wp = off;
    // (w, p) pairs: per edge of a token row in CSR order, or per slot of the token tiles
    // (none with dense_ds)
    off += align_up(p->dense_ds ? 0
                                : bh * (p->q_tiles ? (size_t)g->tiles.num_chunks * 256 : (size_t)g->num_token_edges) * sizeof(float2));
    p->off_qpart = off;
    off += align_up(bh * std::max<size_t>(std::max(g->fwd.num_part, g->fwd_span.num_part), span_partials(g)) *
                    kQPartStride * sizeof(float));
    p->off_kvpart = off;
    off += align_up(bh * std::max<size_t>(g->tr.num_part, p->kv_tiles ? (size_t)g->ktiles.num_part * 16 : 0) * 2 * kD *
                    sizeof(float));
    p->off_drel = off;
    if (!p->drel_tile) p->drel_part_rows = p->drel_rows;
    off += align_up((size_t)p->drel_grid_x * p->drel_part_rows * kD * sizeof(float));
    p->off_queue = off;
    off += align_up(kQueueInts * sizeof(int32_t));   // task counters of the key-tile kernel
    p->total = off;
    return BPT_OK;
}

template <typename T, int IPW>
int launch_rel_grad(const BwdPlan& p, hipStream_t st, const AttnArgs& a) {
    if (p.drel_lds > 65536)
        BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rel_grad_kernel<T, IPW>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.drel_lds));
    BPT_LAUNCH("rel_grad_kernel", (rel_grad_kernel<T, IPW>), dim3(p.drel_grid_x, p.drel_grid_y), dim3(kThreads), p.drel_lds, st,
                       a);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

// query side: delta, dQ, then d_rel
template <typename T>
int run_bwd_q(const bpt_graph* g, const BwdPlan& p, AttnArgs& a, hipStream_t st) {
    DeviceLimits lim;
    int rc = device_limits(g, &lim);
    if (rc) return rc;
    a.ptr = g->row_ptr;
    a.ia = g->col;
    a.ib = g->rel;
    use_schedule(a, g->fwd);
    const int ctx_rows = g->ctx_levels * g->rel_width;
    const size_t rel_b = (size_t)ctx_rows * kD * sizeof(T);
    const bool rel_lds = rel_b <= lim.lds;
    a.rel_rows_lds = rel_lds ? ctx_rows : 0;
    a.drel_rows = p.drel_rows;
    a.drel_block = p.drel_block;
    const Schedule* sc = &g->fwd;
    if (p.q_tiles) {  // token rows on the matrix cores; the gather kernel below only sees span rows
        if ((rc = run_bwd_q_tiles(g, a, lim, p.dense_ds, st))) return rc;
        use_schedule(a, g->fwd_span);
        sc = &g->fwd_span;
    }
    int grid = 8;
    if (p.q_tiles && span_tiles_ok(g)) {
        if ((rc = run_span_tiles(g, a, false, st))) return rc;
        sc = nullptr;
    } else if (rel_lds) {
        if ((rc = persistent_grid(bwd_q_kernel<T, true>, kThreads, rel_b, lim, &grid))) return rc;
        rc = launch("bwd_q_kernel", bwd_q_kernel<T, true>, grid, kThreads, rel_b, st, a);
    } else {
        if ((rc = persistent_grid(bwd_q_kernel<T, false>, kThreads, 0, lim, &grid))) return rc;
        rc = launch("bwd_q_kernel", bwd_q_kernel<T, false>, grid, kThreads, 0, st, a);
    }
    if (rc) return rc;
    if (sc && sc->num_multi > 0) {
        const int items = a.BH * sc->num_multi;
        BPT_LAUNCH("bwd_q_merge_kernel", bwd_q_merge_kernel, dim3((items + 3) / 4), dim3(256), 0, st, a, sc->multi_row,
                           sc->multi_ptr, sc->num_multi);
        BPT_HIP(hipGetLastError());
    }
    if (p.drel_tile) {
        RelGradArgs t = {};
        t.Q = static_cast<const bf16_t*>(a.Q);
        t.rel = static_cast<const bf16_t*>(a.rel);
        t.dQ = a.dQ;
        t.stat = a.stat;
        t.wp = a.wp;
        t.drel_part = a.drel_part;
        t.chunk_ptr = g->tiles.chunk_ptr;
        t.cid_to_id = g->tiles.cid_to_id;
        t.map = g->tiles.map;
        t.sb = a.sb;
        t.sh = a.sh;
        t.sn = a.sn;
        t.BH = a.BH;
        t.H = a.H;
        t.N = a.N;
        t.n = g->n;
        t.num_tiles = g->tiles.num_tiles;
        t.num_chunks = g->tiles.num_chunks;
        t.num_cids = g->tiles.num_cids;
        t.nids = p.drel_part_rows;
        t.scale = a.scale;
        t.seq_len = a.seq_len;
        t.grad_bf16 = a.grad_bf16;
        t.delta = a.delta;
        if (p.dense_ds) {
            // bwd_q_tile_kernel has left the copies of d_rel
        } else if (p.drel_part_rows <= 256 && t.delta) {
            if (p.drel_lds > 65536)
                BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rel_grad_tile_kernel<2, true>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.drel_lds));
            BPT_LAUNCH("rel_grad_tile_kernel", (rel_grad_tile_kernel<2, true>), dim3(p.drel_grid_x), dim3(kThreads), p.drel_lds, st, t);
        } else if (p.drel_part_rows <= 256) {
            if (p.drel_lds > 65536)
                BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rel_grad_tile_kernel<2>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.drel_lds));
            BPT_LAUNCH("rel_grad_tile_kernel", rel_grad_tile_kernel<2>, dim3(p.drel_grid_x), dim3(kThreads), p.drel_lds, st, t);
        } else if (t.delta) {
            if (p.drel_lds > 65536)
                BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rel_grad_tile_kernel<4, true>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.drel_lds));
            BPT_LAUNCH("rel_grad_tile_kernel", (rel_grad_tile_kernel<4, true>), dim3(p.drel_grid_x), dim3(kThreads), p.drel_lds, st, t);
        } else {
            if (p.drel_lds > 65536)
                BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rel_grad_tile_kernel<4>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.drel_lds));
            BPT_LAUNCH("rel_grad_tile_kernel", rel_grad_tile_kernel<4>, dim3(p.drel_grid_x), dim3(kThreads), p.drel_lds, st, t);
        }
        BPT_HIP(hipGetLastError());
        rc = BPT_OK;
    } else if (p.drel_mfma) {
        if (p.drel_lds > 65536)
            BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rel_grad_mfma_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.drel_lds));
        BPT_LAUNCH("rel_grad_mfma_kernel", rel_grad_mfma_kernel, dim3(p.drel_grid_x, p.drel_grid_y), dim3(kThreads), p.drel_lds,
                   st, a);
        BPT_HIP(hipGetLastError());
        rc = BPT_OK;
    } else {
        rc = p.drel_ipw == 8 ? launch_rel_grad<T, 8>(p, st, a)
                             : p.drel_ipw == 16 ? launch_rel_grad<T, 16>(p, st, a) : launch_rel_grad<T, 32>(p, st, a);
    }
    if (rc) return rc;
    BPT_LAUNCH("drel_reduce_kernel", drel_reduce_kernel, dim3(a.rel_rows), dim3(1024), 0, st, a.drel_part, p.drel_grid_x,
               p.drel_part_rows, p.drel_tile ? g->tiles.id_to_cid : nullptr, a.d_rel, a.queue, kQueueInts);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

template <int NBC, bool DROP, bool PACKED = false>
int launch_kv_tiles_as(const KeyArgs& t, const BwdPlan& p, const DeviceLimits& lim, hipStream_t st) {
    if (p.kv_lds > 65536)
        BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_kv_tile_kernel<NBC, DROP, PACKED>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.kv_lds));
    const int grid =
        std::max(8, lim.cus * resident_blocks(bwd_kv_tile_kernel<NBC, DROP, PACKED>, kTileThreads, p.kv_lds, lim) / 8 * 8);
    BPT_LAUNCH("bwd_kv_tile_kernel", (bwd_kv_tile_kernel<NBC, DROP, PACKED>), dim3(grid), dim3(kTileThreads), p.kv_lds, st, t);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}
template <int NBC>
int launch_kv_tiles(const KeyArgs& t, const BwdPlan& p, const DeviceLimits& lim, hipStream_t st) {
    if (t.delta) return launch_kv_tiles_as<NBC, false, true>(t, p, lim, st);   // a packed batch (no dropout there)
    return t.drop_thr ? launch_kv_tiles_as<NBC, true>(t, p, lim, st) : launch_kv_tiles_as<NBC, false>(t, p, lim, st);
}
template <int NBC, bool DROP, bool G16, bool PACKED = false>
int launch_kv_chain_as(const KeyArgs& t, const BwdPlan& p, const DeviceLimits& lim, hipStream_t st) {
    if (p.kv_lds > 65536)
        BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_kv_chain_kernel<NBC, DROP, G16, PACKED>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.kv_lds));
    const int grid =
        std::max(8, lim.cus * resident_blocks(bwd_kv_chain_kernel<NBC, DROP, G16, PACKED>, kTileThreads, p.kv_lds, lim) / 8 * 8);
    BPT_LAUNCH("bwd_kv_chain_kernel", (bwd_kv_chain_kernel<NBC, DROP, G16, PACKED>), dim3(grid), dim3(kTileThreads), p.kv_lds, st, t);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}
template <int NBC>
int launch_kv_chain(const KeyArgs& t, const BwdPlan& p, const DeviceLimits& lim, hipStream_t st) {
    if (t.delta)   // a packed batch (no dropout there)
        return t.grad_bf16 ? launch_kv_chain_as<NBC, false, true, true>(t, p, lim, st) : launch_kv_chain_as<NBC, false, false, true>(t, p, lim, st);
    if (t.grad_bf16)
        return t.drop_thr ? launch_kv_chain_as<NBC, true, true>(t, p, lim, st) : launch_kv_chain_as<NBC, false, true>(t, p, lim, st);
    return t.drop_thr ? launch_kv_chain_as<NBC, true, false>(t, p, lim, st) : launch_kv_chain_as<NBC, false, false>(t, p, lim, st);
}

// bf16 key side on dense tiles of key nodes
// queue_cleared: the query side ran in the same call and its last kernel has put the task counters to zero
int run_bwd_kv_tiles(const bpt_graph* g, const BwdPlan& p, const AttnArgs& a, const DeviceLimits& lim, bool queue_cleared,
                     hipStream_t st) {
    const KeyTiles& kt = g->ktiles;
    KeyArgs t = {};
    t.Q = static_cast<const bf16_t*>(a.Q);
    t.K = static_cast<const bf16_t*>(a.K);
    t.V = static_cast<const bf16_t*>(a.V);
    t.rel = static_cast<const bf16_t*>(a.rel);
    t.dout = static_cast<const bf16_t*>(a.dout);
    t.stat = a.stat;
    t.dK = a.dK;
    t.dV = a.dV;
    t.part = a.part;
    t.sb = a.sb;
    t.sh = a.sh;
    t.sn = a.sn;
    t.BH = a.BH;
    t.H = a.H;
    t.N = a.N;
    t.num_levels = g->num_levels;
    t.scale = a.scale;
    t.row_bytes = a.row_bytes;
    t.slab_bytes = a.slab_bytes;
    t.tile_node0 = kt.tile_node0;
    t.tile_info = kt.tile_info;
    t.cols = kt.cols;
    t.task_tile = kt.task_tile;
    t.task_c0 = kt.task_c0;
    t.task_nch = kt.task_nch;
    t.task_part = kt.task_part;
    t.task_ntiles = kt.task_ntiles;
    t.chunk_ptr = kt.chunk_ptr;
    t.map = kt.map;
    t.num_tasks = kt.num_tasks;
    t.num_part = kt.num_part;
    t.nb_pad = kt.nb_pad;
    t.W = g->rel_width;
    t.zero = g->k + 1;
    t.num_chunks = kt.num_chunks;
    t.seq_len = a.seq_len;
    t.leave_unkept = a.leave_unkept;
    t.grad_bf16 = a.grad_bf16;
    t.delta = a.delta;
    t.n = g->n;
    t.drop_thr = a.drop_thr;
    t.drop_seed = a.drop_seed;
    t.drop_inv_keep = a.drop_inv_keep;
    t.queue = a.queue;
    if ((int64_t)a.BH * kt.num_tasks > INT32_MAX) return BPT_ERR_UNSUPPORTED;
    if (!queue_cleared) {
        BPT_LAUNCH("zero_ints_kernel", zero_ints_kernel, dim3(1), dim3(kQueueInts), 0, st, t.queue, kQueueInts);
        BPT_HIP(hipGetLastError());
    }
    int rc = BPT_ERR_UNSUPPORTED;
    switch (kt.nb_pad / 16) {
        case 1: rc = p.kv_chain ? launch_kv_chain<1>(t, p, lim, st) : launch_kv_tiles<1>(t, p, lim, st); break;
        case 2: rc = p.kv_chain ? launch_kv_chain<2>(t, p, lim, st) : launch_kv_tiles<2>(t, p, lim, st); break;
        case 3: rc = launch_kv_tiles<3>(t, p, lim, st); break;
        case 4: rc = launch_kv_tiles<4>(t, p, lim, st); break;
        case 5: rc = launch_kv_tiles<5>(t, p, lim, st); break;
        case 6: rc = launch_kv_tiles<6>(t, p, lim, st); break;
        case 7: rc = launch_kv_tiles<7>(t, p, lim, st); break;
        case 8: rc = launch_kv_tiles<8>(t, p, lim, st); break;
        case 9: rc = launch_kv_tiles<9>(t, p, lim, st); break;
        case 10: rc = launch_kv_tiles<10>(t, p, lim, st); break;
        default: break;
    }
    if (rc) return rc;
    // threads of the zero pass of kv_tile_merge_kernel: one per node it has to look at, in wavefronts of 64 nodes
    const int zero_row0 = a.seq_len && !a.leave_unkept ? 0 : (kt.first_uncovered & ~63);
    const int64_t zero_elems = (int64_t)a.BH * ((a.N - zero_row0 + 63) / 64) * 64;
    const int64_t blocks = (int64_t)a.BH * kt.num_multi + (zero_elems + 255) / 256;
    if (blocks > 0) {
        if (t.delta)
            BPT_LAUNCH("kv_tile_merge_kernel", kv_tile_merge_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, t, kt.multi_tile,
                       kt.multi_ptr, kt.num_multi, kt.first_uncovered);
        else
            BPT_LAUNCH("kv_tile_merge_kernel", kv_tile_merge_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, t, kt.multi_tile,
                       kt.multi_ptr, kt.num_multi, kt.first_uncovered);
        BPT_HIP(hipGetLastError());
    }
    return BPT_OK;
}

template <typename T>
int run_bwd_kv(const bpt_graph* g, const BwdPlan& p, AttnArgs& a, bool queue_cleared, hipStream_t st) {
    DeviceLimits lim;
    int rc = device_limits(g, &lim);
    if (rc) return rc;
    if (p.kv_tiles) return run_bwd_kv_tiles(g, p, a, lim, queue_cleared, st);
    a.ptr = g->t_ptr;
    a.ia = g->t_src;
    a.ib = g->t_rel;
    use_schedule(a, g->tr);
    const int all_rows = g->num_levels * g->rel_width;  // queries that are spans carry r_anc of any level
    const size_t rel_b = (size_t)all_rows * kD * sizeof(T);
    const bool rel_lds = rel_b <= lim.lds;
    a.rel_rows_lds = rel_lds ? all_rows : 0;
    int grid = 8;
    if (rel_lds) {
        if ((rc = persistent_grid(bwd_kv_kernel<T, true>, kThreads, rel_b, lim, &grid))) return rc;
        rc = launch("bwd_kv_kernel", bwd_kv_kernel<T, true>, grid, kThreads, rel_b, st, a);
    } else {
        if ((rc = persistent_grid(bwd_kv_kernel<T, false>, kThreads, 0, lim, &grid))) return rc;
        rc = launch("bwd_kv_kernel", bwd_kv_kernel<T, false>, grid, kThreads, 0, st, a);
    }
    if (rc) return rc;
    if (g->tr.num_multi > 0) {
        const int items = a.BH * g->tr.num_multi;
        BPT_LAUNCH("bwd_kv_merge_kernel", bwd_kv_merge_kernel, dim3((items + 3) / 4), dim3(256), 0, st, a, g->tr.multi_row,
                           g->tr.multi_ptr, g->tr.num_multi);
        BPT_HIP(hipGetLastError());
    }
    return BPT_OK;
}

// A batch graph on the matrix-core kernels.  The kernels walk the tree of one sequence (g->tree: ids, tile
// metadata) once per sequence and head, with the lengths the graph was built for and with the rows of nodes that a
// sequence does not keep neither computed nor written -- exactly a call with seq_len and leave_unkept on the padded
// trees -- and move every row of a caller's tensor by the sequence's delta of the node's level (AttnArgs.delta).
// Applies to bf16 tensors with B = 1 when the tree has token tiles and span blocks; *view is then the shape the
// kernels see: one batch entry per sequence, all at the same base address.
bool packed_tiles(const bpt_graph* g, const bpt_shape_t* s, bpt_shape_t* view) {
    if (g->batch <= 0 || !g->tree || !g->d_delta || !g->d_lengths || s->dtype != BPT_BF16 || s->B != 1) return false;
    *view = *s;
    view->B = g->batch;
    view->stride_b = 0;
    view->seq_len = g->d_lengths;
    view->leave_unkept = 1;
    if (check_shape(g->tree, view) != BPT_OK) return false;
    DeviceLimits lim;
    if (device_limits(g->tree, &lim) != BPT_OK) return false;
    return plan_tiles(g->tree, lim).ok && span_tiles_ok(g->tree);
}
// the arguments of such a call: those of the view on the tree, with the extent of the packed tensors and their rows
void fill_packed(AttnArgs& a, const bpt_graph* g, const bpt_shape_t* s, const bpt_shape_t* view) {
    fill_common(a, g->tree, view);
    const int64_t es = 2;
    a.slab_bytes = (uint32_t)(((int64_t)(g->num_nodes - 1) * s->stride_n + kD) * es);
    a.delta = g->d_delta;
    a.lse_sb = 0;
    a.lse_sh = g->num_nodes;
}

// the same for the backward: all three of its tile kernels have to apply to the tree
bool packed_tiles_bwd(const bpt_graph* g, const bpt_shape_t* s, bpt_shape_t* view) {
    if (!packed_tiles(g, s, view)) return false;
    BwdPlan p;
    return plan_bwd(g->tree, view, &p) == BPT_OK && p.q_tiles && p.kv_tiles;
}

enum { kStageQ = 1, kStageKV = 2 };

int backward(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K, const void* V, const void* rel,
             const float* lse, const void* dout, void* dQ, void* dK, void* dV, float* d_rel, void* workspace,
             size_t workspace_bytes, void* stream, int stages) {
    int rc = check_shape(g, s);
    if (rc) return rc;
    if (!Q || !K || !V || !rel || !lse || !dout) return BPT_ERR_INVALID_ARG;
    if ((stages & kStageQ) && (!dQ || !d_rel)) return BPT_ERR_INVALID_ARG;
    if ((stages & kStageKV) && (!dK || !dV)) return BPT_ERR_INVALID_ARG;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(rel) || misaligned(dout) || misaligned(dQ) ||
        misaligned(dK) || misaligned(dV) || misaligned(d_rel) || misaligned(workspace))
        return BPT_ERR_INVALID_ARG;
    // a batch graph on the matrix-core kernels: from here on g and s are the tree of one sequence and the view of
    // the packed tensors as one batch entry per sequence
    bpt_shape_t view;
    AttnArgs a;
    if (packed_tiles_bwd(g, s, &view)) {
        fill_packed(a, g, s, &view);
        g = g->tree;
        s = &view;
    } else {
        if (!g->row_ptr) return BPT_ERR_UNSUPPORTED;   // a batch graph without its edge lists: matrix-core kernels only
        fill_common(a, g, s);
    }
    BwdPlan p;
    if ((rc = plan_bwd(g, s, &p))) return rc;
    if (!workspace || workspace_bytes < p.total) return BPT_ERR_INVALID_ARG;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    a.Q = Q;
    a.K = K;
    a.V = V;
    a.rel = rel;
    a.lse_r = lse;
    a.dout = dout;
    a.dQ = static_cast<float*>(dQ);   // bf16 elements with grad_dtype = BPT_BF16 (AttnArgs.grad_bf16)
    a.dK = static_cast<float*>(dK);
    a.dV = static_cast<float*>(dV);
    a.d_rel = d_rel;
    a.stat = reinterpret_cast<float2*>(ws + p.off_stat);
    a.wp = reinterpret_cast<float2*>(ws + p.off_wp);
    a.e_tok = g->num_token_edges;
    a.drel_part = reinterpret_cast<float*>(ws + p.off_drel);
    a.queue = reinterpret_cast<int32_t*>(ws + p.off_queue);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = s->dtype == BPT_BF16;
    if (stages & kStageQ) {
        a.part = reinterpret_cast<float*>(ws + p.off_qpart);
        if ((rc = bf ? run_bwd_q<bf16_t>(g, p, a, st) : run_bwd_q<float>(g, p, a, st))) return rc;
    }
    if (stages & kStageKV) {
        a.part = reinterpret_cast<float*>(ws + p.off_kvpart);
        const bool cleared = (stages & kStageQ) != 0;
        if ((rc = bf ? run_bwd_kv<bf16_t>(g, p, a, cleared, st) : run_bwd_kv<float>(g, p, a, cleared, st))) return rc;
    }
    return BPT_OK;
}

}  // namespace
}  // namespace bpt

extern "C" {

size_t bpt_attn_fwd_workspace(const bpt_graph_t* g, const bpt_shape_t* s) {
    if (bpt::check_shape(g, s) != BPT_OK) return SIZE_MAX;
    bpt_shape_t view;
    if (bpt::packed_tiles(g, s, &view)) return bpt_attn_fwd_workspace(g->tree, &view);
    if (!g->row_ptr) return SIZE_MAX;   // a batch graph without its edge lists runs the matrix-core kernels only
    return bpt::align_up((size_t)s->B * s->H *
                         std::max<size_t>(std::max(g->fwd.num_part, g->fwd_span.num_part), bpt::span_partials(g)) *
                         bpt::kPartStride * sizeof(float));
}

size_t bpt_attn_bwd_workspace(const bpt_graph_t* g, const bpt_shape_t* s) {
    if (bpt::check_shape(g, s) != BPT_OK) return SIZE_MAX;
    bpt_shape_t view;
    if (bpt::packed_tiles_bwd(g, s, &view)) return bpt_attn_bwd_workspace(g->tree, &view);
    if (!g->row_ptr) return SIZE_MAX;
    bpt::BwdPlan p;
    if (bpt::plan_bwd(g, s, &p) != BPT_OK) return SIZE_MAX;
    return p.total;
}

int bpt_attn_fwd(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K, const void* V,
                 const void* rel, void* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
    int rc = bpt::check_shape(g, s);
    if (rc) return rc;
    if (!Q || !K || !V || !rel || !out || !lse) return BPT_ERR_INVALID_ARG;
    if (bpt::misaligned(Q) || bpt::misaligned(K) || bpt::misaligned(V) || bpt::misaligned(rel) ||
        bpt::misaligned(out) || bpt::misaligned(workspace))
        return BPT_ERR_INVALID_ARG;
    const size_t need = bpt_attn_fwd_workspace(g, s);
    if (need == SIZE_MAX) return BPT_ERR_UNSUPPORTED;
    if (need > 0 && (!workspace || workspace_bytes < need)) return BPT_ERR_INVALID_ARG;
    bpt::AttnArgs a;
    bpt_shape_t view;
    const bool packed = bpt::packed_tiles(g, s, &view);
    if (packed) {
        bpt::fill_packed(a, g, s, &view);
        g = g->tree;
    } else {
        bpt::fill_common(a, g, s);
    }
    a.Q = Q;
    a.K = K;
    a.V = V;
    a.rel = rel;
    a.out = out;
    a.lse_w = lse;
    a.part = static_cast<float*>(workspace);
    a.ptr = g->row_ptr;
    a.ia = g->col;
    a.ib = g->rel;
    bpt::use_schedule(a, g->fwd);
    hipStream_t st = static_cast<hipStream_t>(stream);
    return s->dtype == BPT_BF16 ? bpt::run_fwd<bpt::bf16_t>(g, a, st) : bpt::run_fwd<float>(g, a, st);
}

int bpt_attn_fwd_static(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K, const void* V,
                        const void* rel, void* out, float* lse, void* stream) {
    int rc = bpt::check_shape(g, s);
    if (rc) return rc;
    const size_t need = bpt_attn_fwd_workspace(g, s);
    if (need == SIZE_MAX) return BPT_ERR_UNSUPPORTED;
    if (need > kStaticScratchBytes) return BPT_ERR_SCRATCH;
    int device = -1;
    BPT_HIP(hipGetDevice(&device));
    if (device != g->device) return BPT_ERR_INVALID_ARG;   // the scratch used is the current device's
    void* ws = nullptr;
    if ((rc = bpt::static_scratch(device, &ws))) return rc;
    // the forward's kernels write every partial they later read, so nothing has to be cleared between calls
    return bpt_attn_fwd(g, s, Q, K, V, rel, out, lse, ws, kStaticScratchBytes, stream);
}

int bpt_attn_bwd(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K, const void* V,
                 const void* rel, const float* lse, const void* dout, void* dQ, void* dK, void* dV, float* d_rel,
                 void* workspace, size_t workspace_bytes, void* stream) {
    return bpt::backward(g, s, Q, K, V, rel, lse, dout, dQ, dK, dV, d_rel, workspace, workspace_bytes, stream,
                         bpt::kStageQ | bpt::kStageKV);
}

int bpt_attn_bwd_query_side(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K, const void* V,
                            const void* rel, const float* lse, const void* dout, void* dQ, float* d_rel,
                            void* workspace, size_t workspace_bytes, void* stream) {
    return bpt::backward(g, s, Q, K, V, rel, lse, dout, dQ, nullptr, nullptr, d_rel, workspace, workspace_bytes,
                         stream, bpt::kStageQ);
}

int bpt_attn_bwd_key_side(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K, const void* V,
                          const void* rel, const float* lse, const void* dout, void* dK, void* dV, void* workspace,
                          size_t workspace_bytes, void* stream) {
    return bpt::backward(g, s, Q, K, V, rel, lse, dout, nullptr, dK, dV, nullptr, workspace, workspace_bytes, stream,
                         bpt::kStageKV);
}

}  // extern "C"
