// Matrix-core kernels for the span rows (bf16): blocks of 32 tokens serve all tree levels.
#pragma once

#include "attn_token_tiles.h"

namespace bpt {
namespace {

// ---- span rows on the matrix cores (bf16): blocks of 32 tokens -------------------------
// Span node (l, m) attends to exactly the 2^l tokens it contains (Sec. 3.2.2, affiliated
// edges), so all span rows over a block of 32 consecutive tokens share the block's K and
// V rows.  One wavefront takes a block: the 31 spans inside it (levels 1..5) and the
// block's ancestors at levels 6..L, one query per column of three 16-query groups:
//   group 0: the 16 level-1 spans; group 1: 8 + 4 + 2 + 1 spans of levels 2..5 (slot 15
//   unused); group 2: the ancestor at level 6 + slot.
//   S^T [32 tokens x 16 queries] = K_block (A, rows from memory) x Q^T (B),
//   out [16 queries x 64]        = P (A: the C layout of S^T, two token chunks interleaved)
//                                  x V_block (B, read transposed out of LDS).
// A span inside the block is finished here; an ancestor covers 2^(l-5) blocks, so the
// block contributes a partial (accumulators, running max, sum) that a merge kernel
// combines in block order.  K and V of the tokens are read once for all levels instead
// of once per level.  Every edge of a span row carries r_anc(l): the constant
// scale * q . r_anc(l) is added to the row's scores (it only moves lse).
constexpr int kSpanTok = 32;       // tokens per block
constexpr int kSpanInLevels = 5;   // levels whose spans lie inside one block
struct SpanArgs {
    const bf16_t *Q, *K, *V, *rel, *dout;
    bf16_t* out;
    float* lse;
    const float* lse_r;
    float* dQ;
    float2* stat;
    float* part;
    int64_t sb, sh, sn;
    int32_t BH, H, N, n, L, W, zero;
    float scale;
    const int32_t* seq_len;   // [B] tokens of every sequence, or null
    int32_t leave_unkept;     // rows of nodes a shorter sequence does not keep: left unwritten instead of zero-filled
    int32_t grad_bf16;        // dQ leaves rounded to bf16
    // packed batch: delta[level][sequence] (see attn_device.h) or null; lse of (bh, node u) is at
    // (bh / H) * lse_sb + (bh % H) * lse_sh + row of u
    const int32_t* delta;
    int64_t lse_sb, lse_sh;
    uint32_t drop_thr, drop_seed;   // dropout on the attention weights (DROP variants)
    float drop_inv_keep;
};
__device__ __forceinline__ int span_level_offset(int n, int level) { return 2 * n - ((2 * n) >> level); }
// query slot -> (level, index inside the block at that level); group is wave-uniform
__device__ __forceinline__ void span_slot(int group, int slot, int L, int& level, int& loc, bool& valid) {
    if (group == 0) {
        level = 1; loc = slot; valid = true;
    } else if (group == 1) {
        level = slot < 8 ? 2 : slot < 12 ? 3 : slot < 14 ? 4 : 5;
        loc = slot < 8 ? slot : slot < 12 ? slot - 8 : slot < 14 ? slot - 12 : 0;
        valid = slot < 15;
    } else {
        level = kSpanInLevels + 1 + slot; loc = 0; valid = level <= L;
    }
    valid = valid && level <= L;
    if (!valid) { level = L; loc = 0; }   // the root: a valid address, every score masked
}
__device__ __forceinline__ int span_slot_node(int group, int slot, int L, int n, int t0) {
    int level, loc;
    bool valid;
    span_slot(group, slot, L, level, loc, valid);
    return span_level_offset(n, level) + (t0 >> level) + loc;
}
// the same as a row of the caller's tensors: the node id, or in a packed batch (dvec: this lane's delta of the
// sequence) the node's packed row
template <bool PACKED>
__device__ __forceinline__ int span_slot_row(const SpanArgs& a, int group, int slot, int t0, int dvec) {
    int level, loc;
    bool valid;
    span_slot(group, slot, a.L, level, loc, valid);
    const int node = span_level_offset(a.n, level) + (t0 >> level) + loc;
    return PACKED ? node + __shfl(dvec, level) : node;
}
// whether a sequence of len tokens keeps the node of the slot (its first token exists)
__device__ __forceinline__ bool span_slot_kept(const SpanArgs& a, int group, int slot, int t0, int len) {
    int level, loc;
    bool valid;
    span_slot(group, slot, a.L, level, loc, valid);
    return valid && ((((t0 >> level) + loc) << level) < len);
}
template <bool PACKED>
__device__ __forceinline__ int64_t span_lse_at(const SpanArgs& a, int bh) {
    return PACKED ? (int64_t)(bh / a.H) * a.lse_sb + (int64_t)(bh % a.H) * a.lse_sh : (int64_t)bh * a.N;
}
// scale * log2(e) * q . r_anc(level) for the query of this lane's column: every lane holds 16
// features of its query (the B operand), the four lane groups hold the four quarters
__device__ __forceinline__ float span_shift(const SpanArgs& a, int level, int g, const bf16x8_t& q0, const bf16x8_t& q1,
                                            float qscale) {
    const bf16_t* rr = a.rel + ((int64_t)level * a.W + a.zero) * kD + 16 * g;
    const uint4 r0 = *reinterpret_cast<const uint4*>(rr), r1 = *reinterpret_cast<const uint4*>(rr + 8);
    const uint4 x0 = __builtin_bit_cast(uint4, q0), x1 = __builtin_bit_cast(uint4, q1);
    float d = 0.f;
    d = dot2_bf16(x0.x, r0.x, d); d = dot2_bf16(x0.y, r0.y, d); d = dot2_bf16(x0.z, r0.z, d); d = dot2_bf16(x0.w, r0.w, d);
    d = dot2_bf16(x1.x, r1.x, d); d = dot2_bf16(x1.y, r1.y, d); d = dot2_bf16(x1.z, r1.z, d); d = dot2_bf16(x1.w, r1.w, d);
    d += __shfl_xor(d, 16);
    d += __shfl_xor(d, 32);
    return d * qscale;
}

// A block of 32 tokens past the end of a shorter sequence: nothing is read; its spans inside the
// block get zero rows (forward: out, lse; backward: dQ) unless such rows are left unwritten, and in the
// backward a `stat` entry that switches the row off on the key side.  Its ancestors get nothing from
// it: the merge kernels only read the partials of the blocks that exist.
// The spans of a level are consecutive nodes, so the rows are written 16 bytes per lane.
__device__ __forceinline__ void span_block_gone(const SpanArgs& a, int bh, int t0, int64_t base, bool forward, int lane) {
    const int top = min(kSpanInLevels, a.L);
    for (int level = 1; level <= top; ++level) {
        const int node0 = span_level_offset(a.n, level) + (t0 >> level), cnt = kSpanTok >> level;
        if (forward) {
            if (a.leave_unkept) continue;
            for (int i = lane; i < cnt * 8; i += 64)     // 64 bf16 per row
                *reinterpret_cast<uint4*>(a.out + base + (int64_t)(node0 + (i >> 3)) * a.sn + (i & 7) * 8) = make_uint4(0u, 0u, 0u, 0u);
            if (lane < cnt) a.lse[(int64_t)bh * a.N + node0 + lane] = 0.f;   // (never with a packed batch: leave_unkept)
        } else {
            if (!a.leave_unkept)
                for (int i = lane; i < cnt * 16; i += 64)    // 64 floats per row
                    store_grad4(a.dQ, base + (int64_t)(node0 + (i >> 4)) * a.sn + (i & 15) * 4, make_float4(0.f, 0.f, 0.f, 0.f), a.grad_bf16);
            if (lane < cnt) a.stat[(int64_t)bh * a.N + node0 + lane] = make_float2(kLseGone, 0.f);
        }
    }
}

// PACKED: the rows of the caller's tensors are those of a packed batch (SpanArgs.delta; see attn_device.h)
template <bool DROP, bool PACKED = false>
__global__ void __launch_bounds__(kTileThreads) fwd_span_tile_kernel(const SpanArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, j = lane & 15;
    bf16_t* v_s = reinterpret_cast<bf16_t*>(smem) + (size_t)wave * kSpanTok * kVStride;   // [32 tokens][kVStride]
    const int nblk = a.n / kSpanTok;
    const int item = blockIdx.x * kTileWaves + wave;
    if (item >= a.BH * nblk) return;   // wave-uniform; the kernel has no workgroup barrier
    const int bh = item / nblk, blk = item - bh * nblk, t0 = blk * kSpanTok;
    const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
    const float qscale = a.scale * kLog2e;
    const int ngroups = a.L > kSpanInLevels ? 3 : 2;
    const int nanc = a.L - kSpanInLevels;
    const int len = seq_length(a.seq_len, bh / a.H, a.n);   // tokens from `len` on do not exist

    // the block's K rows as A operands (token j of chunk c, features 16g..16g+15); V rows into LDS
    if (t0 >= len) {   // wave-uniform: a block past the end of a shorter sequence
        span_block_gone(a, bh, t0, base, true, lane);
        return;
    }
    // packed batch: rows of the caller's tensors are the node ids moved by the sequence's delta of the node's level;
    // a node the sequence does not keep has no row, its loads go to the last kept node of its level instead (every
    // score of such a query, and of such a token, is masked) and nothing is stored for it
    const int dvec = PACKED ? load_delta(a.delta, a.BH / a.H, bh / a.H, lane, a.L + 1) : 0;
    // the query rows of all three groups are asked for together with the block's K and V: one round trip
    // to memory per block instead of four
    bf16x8_t qall[3][2];
#pragma unroll
    for (int grp = 0; grp < 3; ++grp) {
        int level, loc;
        bool valid;
        span_slot(min(grp, ngroups - 1), j, a.L, level, loc, valid);
        int idx = (t0 >> level) + loc, shift_row = 0;
        if (PACKED) {
            idx = min(idx, ((len + (1 << level) - 1) >> level) - 1);
            shift_row = __shfl(dvec, level);
        }
        const bf16_t* qrow = a.Q + base + (int64_t)(span_level_offset(a.n, level) + idx + shift_row) * a.sn + 16 * g;
        qall[grp][0] = *reinterpret_cast<const bf16x8_t*>(qrow);
        qall[grp][1] = *reinterpret_cast<const bf16x8_t*>(qrow + 8);
    }
    bf16x8_t ka[2][2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int tk = PACKED ? min(t0 + 16 * c + j, len - 1) + level_delta(dvec, 0) : t0 + 16 * c + j;
        const int64_t at = base + (int64_t)tk * a.sn + 16 * g;
        ka[c][0] = *reinterpret_cast<const bf16x8_t*>(a.K + at);
        ka[c][1] = *reinterpret_cast<const bf16x8_t*>(a.K + at + 8);
        const uint4 v0 = *reinterpret_cast<const uint4*>(a.V + at), v1 = *reinterpret_cast<const uint4*>(a.V + at + 8);
        uint2* d = reinterpret_cast<uint2*>(v_s + (16 * c + j) * kVStride + 16 * g);
        d[0] = make_uint2(v0.x, v0.y);
        d[1] = make_uint2(v0.z, v0.w);
        d[2] = make_uint2(v1.x, v1.y);
        d[3] = make_uint2(v1.z, v1.w);
    }
    wave_lds_sync();
    // V^T operands of all three groups; v_s is then free to carry the finished rows on their way out
    bf16x8_t vB[4];
#pragma unroll
    for (int f = 0; f < 4; ++f) vB[f] = lds_transposed_b(v_s, kVStride, f, g, j);
    const int r8 = lane >> 3, piece = lane & 7;

#pragma unroll
    for (int grp = 0; grp < 3; ++grp) {
        if (grp >= ngroups) break;   // wave-uniform
        int level, loc;
        bool valid;
        span_slot(grp, j, a.L, level, loc, valid);
        const int node = span_level_offset(a.n, level) + (t0 >> level) + loc;
        const bf16x8_t qb0 = qall[grp][0], qb1 = qall[grp][1];
        const float shift = span_shift(a, level, g, qb0, qb1, qscale);
        float p[2][4], m = kNegBig;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            f32x4_t s4 = {0.f, 0.f, 0.f, 0.f};
            s4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[c][0], qb0, s4, 0, 0, 0);
            s4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[c][1], qb1, s4, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int tt = 16 * c + 4 * g + r;   // token of the block
                const bool member = valid && (grp == 2 || (tt >> level) == loc) && t0 + tt < len;
                p[c][r] = member ? s4[r] * qscale + shift : kNegBig;
                m = fmaxf(m, p[c][r]);
            }
        }
        m = fmaxf(m, __shfl_xor(m, 16));
        m = fmaxf(m, __shfl_xor(m, 32));
        float l = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                p[c][r] = p[c][r] > 0.5f * kNegBig ? fast_exp2(p[c][r] - m) : 0.f;
                l += p[c][r];
            }
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        if (DROP) {   // the row sum keeps every edge; the weighted sum of values takes the mask of (span node, token)
            const uint32_t rowh = drop_row_hash(drop_bh_hash(a.drop_seed, bh), node);
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    p[c][r] *= drop_scale(rowh, drop_edge_x(false, 0, t0 + 16 * c + 4 * g + r), a.drop_thr, a.drop_inv_keep);
        }
        u32x4 pa;
        pa.x = pack_bf16(p[0][0], p[0][1]);
        pa.y = pack_bf16(p[0][2], p[0][3]);
        pa.z = pack_bf16(p[1][0], p[1][1]);
        pa.w = pack_bf16(p[1][2], p[1][3]);
        const bf16x8_t pA = __builtin_bit_cast(bf16x8_t, pa);
        f32x4_t o[4];
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            o[f] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            o[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vB[f], pA, o[f], 0, 0, 0);
        }
        // out^T = V^T P^T (the operands of P V changed places, the registers are the same), C[m = feature][n = query]:
        // this lane holds features 16f + 4g .. + 3 of query j
        if (grp < 2) {
            // l == 0: a span past the end of a shorter sequence, its row is zero
            constexpr bool guard = PACKED;
            const int lse_row = PACKED ? node + __shfl(dvec, level) : node;   // (all lanes take part in the exchange)
            if (g == 0 && valid && !(guard && l <= 0.f))
                a.lse[span_lse_at<PACKED>(a, bh) + lse_row] = l > 0.f ? (m + fast_log2(l)) * kLn2 : 0.f;
            // the rows go through v_s and leave whole, 16 bytes per lane: eight rows of 128 contiguous bytes per store
            const float inv = l > 0.f ? 1.f / l : 0.f;
            wave_lds_sync();   // the previous group's rows have been read
#pragma unroll
            for (int f = 0; f < 4; ++f)
                *reinterpret_cast<uint2*>(v_s + j * kVStride + 16 * f + 4 * g) =
                    make_uint2(pack_bf16(o[f][0] * inv, o[f][1] * inv), pack_bf16(o[f][2] * inv, o[f][3] * inv));
            wave_lds_sync();
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int slot = 8 * h + r8;
                const float lq = __shfl(l, slot);
                const int orow_at = span_slot_row<PACKED>(a, grp, slot, t0, dvec);
                if (grp == 1 && slot == 15) continue;
                if (guard && lq <= 0.f) continue;   // a span past the end of the sequence has no row
                const uint2* src = reinterpret_cast<const uint2*>(v_s + slot * kVStride + piece * 8);
                const uint2 x0 = src[0], x1 = src[1];
                store_once(reinterpret_cast<uint4*>(a.out + base + (int64_t)orow_at * a.sn + piece * 8), make_uint4(x0.x, x0.y, x1.x, x1.y));
            }
        } else {
            // partial of the ancestor at level 6 + slot: [bh][level][block][66]
            if (g == 0 && valid) {
                float* dst = a.part + (((int64_t)bh * nanc + j) * nblk + blk) * kPartStride;
                dst[64] = m;
                dst[65] = l;
            }
            if (j < nanc) {   // (a partial is 264 bytes: 8-byte stores)
                float* dst = a.part + (((int64_t)bh * nanc + j) * nblk + blk) * kPartStride + 4 * g;
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    *reinterpret_cast<float2*>(dst + 16 * f) = make_float2(o[f][0], o[f][1]);
                    *reinterpret_cast<float2*>(dst + 16 * f + 2) = make_float2(o[f][2], o[f][3]);
                }
            }
        }
    }
}

// level and index of span node v >= n
__device__ __forceinline__ void span_node_level(int n, int L, int v, int& level, int& m) {
    const int x = 2 * n - v;                                   // (n >> l) < x <= (2n >> l)
    level = L + 1 - (32 - __clz(x - 1));
    m = v - span_level_offset(n, level);
}

// Ancestors (levels 6..L): combine the per-block partials of a row in block order.  A row of
// level l has 2^(l-5) partials.  Rows with at most 16 (levels 6..9) take one wavefront each,
// lane = feature, all loads issued at once; longer rows take a workgroup of 1024 threads
// (thread = 4 features x one of 64 interleaved block lists) and a fixed-order sum of the 64
// lists, so the result does not depend on timing.
constexpr int kSpanSmallLevels = 4;                                  // levels 6..9
constexpr int kSpanSmallMax = 1 << kSpanSmallLevels;                 // 16 partials
constexpr int kSpanBigThreads = 1024;
struct SpanRow {
    int bh, v, cnt;   // cnt: partials of the row that exist -- its blocks that begin before the end of the sequence
    const float* src;
};
// rows [first, first + rows) of every (batch, head); stride = floats per partial
__device__ __forceinline__ bool span_merge_row(const SpanArgs& a, int item, int first, int rows, int stride, SpanRow& r) {
    if (item >= a.BH * rows) return false;
    r.bh = item / rows;
    r.v = first + (item - r.bh * rows);
    int level, mi;
    span_node_level(a.n, a.L, r.v, level, mi);
    const int nblk = a.n / kSpanTok, nanc = a.L - kSpanInLevels;
    const int all = 1 << (level - kSpanInLevels);
    const int live_blocks = (seq_length(a.seq_len, r.bh / a.H, a.n) + kSpanTok - 1) / kSpanTok;
    r.cnt = min(all, max(live_blocks - mi * all, 0));
    r.src = a.part + (((int64_t)r.bh * nanc + (level - kSpanInLevels - 1)) * nblk + (int64_t)mi * all) * stride;
    return true;
}

// the row of a merged node in the caller's tensors: its id, or its packed row (a merged row with partials is kept)
template <bool PACKED>
__device__ __forceinline__ int span_merged_row(const SpanArgs& a, const SpanRow& r) {
    if (!PACKED) return r.v;
    int level, mi;
    span_node_level(a.n, a.L, r.v, level, mi);
    return r.v + a.delta[level * (a.BH / a.H) + r.bh / a.H];
}

// lse * log2(e) of a merged row for the key side, kLseGone if the sequence does not keep the node
template <bool PACKED>
__device__ __forceinline__ float span_row_lse2(const SpanArgs& a, const SpanRow& r) {
    int level, mi;
    span_node_level(a.n, a.L, r.v, level, mi);
    return (mi << level) < seq_length(a.seq_len, r.bh / a.H, a.n) ? a.lse_r[span_lse_at<PACKED>(a, r.bh) + span_merged_row<PACKED>(a, r)] * kLog2e
                                                                   : kLseGone;
}

template <bool PACKED>
__device__ __forceinline__ void fwd_span_merge_small(const SpanArgs& a, int item, int first, int rows) {
    const int lane = threadIdx.x & 63;
    SpanRow r;
    if (!span_merge_row(a, item, first, rows, kPartStride, r)) return;
    if (r.cnt == 0 && a.leave_unkept) return;   // the sequence does not keep the node
    float o[kSpanSmallMax], m[kSpanSmallMax], l[kSpanSmallMax];
#pragma unroll
    for (int b = 0; b < kSpanSmallMax; ++b) {
        const float* pb = r.src + (int64_t)max(min(b, r.cnt - 1), 0) * kPartStride;
        o[b] = b < r.cnt ? pb[lane] : 0.f;
        m[b] = b < r.cnt ? pb[64] : kNegBig;
        l[b] = b < r.cnt ? pb[65] : 0.f;
    }
    float mx = kNegBig;
#pragma unroll
    for (int b = 0; b < kSpanSmallMax; ++b) mx = fmaxf(mx, m[b]);
    float acc = 0.f, ls = 0.f;
#pragma unroll
    for (int b = 0; b < kSpanSmallMax; ++b) {
        const float c = b < r.cnt ? fast_exp2(m[b] - mx) : 0.f;
        ls += l[b] * c;
        acc += o[b] * c;
    }
    const int64_t base = (int64_t)(r.bh / a.H) * a.sb + (int64_t)(r.bh % a.H) * a.sh;
    const int row = span_merged_row<PACKED>(a, r);
    store_once(&a.out[base + (int64_t)row * a.sn + lane], (bf16_t)to_bf16_bits(ls > 0.f ? acc / ls : 0.f));
    if (lane == 0) a.lse[span_lse_at<PACKED>(a, r.bh) + row] = ls > 0.f ? (mx + fast_log2(ls)) * kLn2 : 0.f;
}

// one kernel for both kinds of rows: the first workgroups take one long row each, the longest rows (the highest
// levels) of all (batch, head)s first, so that they run while the short rows are handed out; the `small_blocks`
// workgroups behind them take 16 short rows each (one per wavefront)
template <bool PACKED>
__global__ void __launch_bounds__(kSpanBigThreads) fwd_span_merge_kernel(const SpanArgs a, int first, int rows_small,
                                                                         int first_big, int rows_big, int small_blocks) {
    __shared__ float s_acc[64][kD + 4];
    __shared__ float s_l[64];
    __shared__ float s_m[kSpanBigThreads / 64];
    const int big_blocks = a.BH * rows_big;
    if ((int)blockIdx.x >= big_blocks) {   // uniform for the workgroup; this path has no barrier
        fwd_span_merge_small<PACKED>(a, (blockIdx.x - big_blocks) * (kSpanBigThreads / 64) + (threadIdx.x >> 6), first, rows_small);
        return;
    }
    SpanRow r;
    const int big_item = (blockIdx.x % a.BH) * rows_big + (rows_big - 1 - blockIdx.x / a.BH);
    if (!span_merge_row(a, big_item, first_big, rows_big, kPartStride, r)) return;   // uniform for the workgroup
    if (r.cnt == 0 && a.leave_unkept) return;
    const int t = threadIdx.x, fq = t & 15, pl = t >> 4;
    float mx = kNegBig;
    for (int b = t; b < r.cnt; b += kSpanBigThreads) mx = fmaxf(mx, r.src[(int64_t)b * kPartStride + 64]);
#pragma unroll
    for (int w = 1; w < 64; w <<= 1) mx = fmaxf(mx, __shfl_xor(mx, w));
    if ((t & 63) == 0) s_m[t >> 6] = mx;
    __syncthreads();
    mx = s_m[0];
#pragma unroll
    for (int w = 1; w < kSpanBigThreads / 64; ++w) mx = fmaxf(mx, s_m[w]);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float ls = 0.f;
#pragma unroll 4
    for (int b = pl; b < r.cnt; b += 64) {
        const float* pb = r.src + (int64_t)b * kPartStride;
        const float2 x0 = *reinterpret_cast<const float2*>(pb + 4 * fq), x1 = *reinterpret_cast<const float2*>(pb + 4 * fq + 2);
        const float c = fast_exp2(pb[64] - mx);
        ls += pb[65] * c;
        acc.x += x0.x * c;
        acc.y += x0.y * c;
        acc.z += x1.x * c;
        acc.w += x1.y * c;
    }
    *reinterpret_cast<float4*>(&s_acc[pl][4 * fq]) = acc;
    if (fq == 0) s_l[pl] = ls;
    __syncthreads();
    if (t < 64) {
        float sum = 0.f, lt = 0.f;
        for (int p = 0; p < 64; ++p) {
            sum += s_acc[p][t];
            lt += s_l[p];
        }
        const int64_t base = (int64_t)(r.bh / a.H) * a.sb + (int64_t)(r.bh % a.H) * a.sh;
        const int row = span_merged_row<PACKED>(a, r);
        store_once(&a.out[base + (int64_t)row * a.sn + t], (bf16_t)to_bf16_bits(lt > 0.f ? sum / lt : 0.f));
        if (t == 0) a.lse[span_lse_at<PACKED>(a, r.bh) + row] = lt > 0.f ? (mx + fast_log2(lt)) * kLn2 : 0.f;
    }
}

// Query side of the backward over the same blocks: S^T and dP^T = V_block x dO^T, p =
// exp2(s - lse), w = p dP.  A span inside the block has its whole row here, so delta = sum w
// and dS = w - delta p are final and dQ = scale * dS K_block (r_anc drops out: the dS of a row
// sum to zero).  An ancestor stores the partial sums A = W K, Bv = P K, delta, which the merge
// kernel turns into dQ = scale * (sum A - delta * sum Bv).
template <bool DROP, bool G16, bool PACKED = false>   // G16: dQ leaves rounded to bf16
__global__ void __launch_bounds__(kTileThreads, 3) bwd_q_span_tile_kernel(const SpanArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, j = lane & 15;
    bf16_t* k_s = reinterpret_cast<bf16_t*>(smem) + (size_t)wave * kSpanTok * kVStride;
    const int nblk = a.n / kSpanTok;
    const int item = blockIdx.x * kTileWaves + wave;
    if (item >= a.BH * nblk) return;
    const int bh = item / nblk, blk = item - bh * nblk, t0 = blk * kSpanTok;
    const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
    const float qscale = a.scale * kLog2e;
    const int ngroups = a.L > kSpanInLevels ? 3 : 2;
    const int nanc = a.L - kSpanInLevels;
    const int len = seq_length(a.seq_len, bh / a.H, a.n);

    if (t0 >= len) {   // wave-uniform: a block past the end of a shorter sequence
        span_block_gone(a, bh, t0, base, false, lane);
        return;
    }
    // packed batch: see fwd_span_tile_kernel
    const int dvec = PACKED ? load_delta(a.delta, a.BH / a.H, bh / a.H, lane, a.L + 1) : 0;
    // the Q and dO rows and the lse of all three groups are asked for together with the block's K and V:
    // one round trip to memory per block instead of four
    bf16x8_t qall[3][2], gall[3][2];
    float lall[3];
#pragma unroll
    for (int grp = 0; grp < 3; ++grp) {
        int level, loc;
        bool valid;
        span_slot(min(grp, ngroups - 1), j, a.L, level, loc, valid);
        int idx = (t0 >> level) + loc, shift_row = 0;
        if (PACKED) {
            idx = min(idx, ((len + (1 << level) - 1) >> level) - 1);
            shift_row = __shfl(dvec, level);
        }
        const int row = span_level_offset(a.n, level) + idx + shift_row;
        const bf16_t* qrow = a.Q + base + (int64_t)row * a.sn + 16 * g;
        const bf16_t* grow = a.dout + base + (int64_t)row * a.sn + 16 * g;
        qall[grp][0] = *reinterpret_cast<const bf16x8_t*>(qrow);
        qall[grp][1] = *reinterpret_cast<const bf16x8_t*>(qrow + 8);
        gall[grp][0] = *reinterpret_cast<const bf16x8_t*>(grow);
        gall[grp][1] = *reinterpret_cast<const bf16x8_t*>(grow + 8);
        lall[grp] = a.lse_r[span_lse_at<PACKED>(a, bh) + row];
    }
    bf16x8_t ka[2][2], va[2][2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int tk = PACKED ? min(t0 + 16 * c + j, len - 1) + level_delta(dvec, 0) : t0 + 16 * c + j;
        const int64_t at = base + (int64_t)tk * a.sn + 16 * g;
        const uint4 k0 = *reinterpret_cast<const uint4*>(a.K + at), k1 = *reinterpret_cast<const uint4*>(a.K + at + 8);
        ka[c][0] = __builtin_bit_cast(bf16x8_t, k0);
        ka[c][1] = __builtin_bit_cast(bf16x8_t, k1);
        va[c][0] = *reinterpret_cast<const bf16x8_t*>(a.V + at);
        va[c][1] = *reinterpret_cast<const bf16x8_t*>(a.V + at + 8);
        uint2* d = reinterpret_cast<uint2*>(k_s + (16 * c + j) * kVStride + 16 * g);
        d[0] = make_uint2(k0.x, k0.y);
        d[1] = make_uint2(k0.z, k0.w);
        d[2] = make_uint2(k1.x, k1.y);
        d[3] = make_uint2(k1.z, k1.w);
    }
    wave_lds_sync();
    bf16x8_t kB[4];
#pragma unroll
    for (int f = 0; f < 4; ++f) kB[f] = lds_transposed_b(k_s, kVStride, f, g, j);
    const int r8 = lane >> 3, piece = lane & 7;   // k_s is free from here on: it carries the finished rows on their way out

#pragma unroll
    for (int grp = 0; grp < 3; ++grp) {
        if (grp >= ngroups) break;   // wave-uniform
        int level, loc;
        bool valid;
        span_slot(grp, j, a.L, level, loc, valid);
        const int node = span_level_offset(a.n, level) + (t0 >> level) + loc;
        const bf16x8_t qb0 = qall[grp][0], qb1 = qall[grp][1], gb0 = gall[grp][0], gb1 = gall[grp][1];
        const float lse2 = lall[grp] * kLog2e;
        const float shift = span_shift(a, level, g, qb0, qb1, qscale);
        const uint32_t rowh = DROP ? drop_row_hash(drop_bh_hash(a.drop_seed, bh), node) : 0u;
        float p[2][4], wgt[2][4], dl = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            f32x4_t s4 = {0.f, 0.f, 0.f, 0.f}, d4 = {0.f, 0.f, 0.f, 0.f};
            s4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[c][0], qb0, s4, 0, 0, 0);
            s4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka[c][1], qb1, s4, 0, 0, 0);
            d4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[c][0], gb0, d4, 0, 0, 0);
            d4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va[c][1], gb1, d4, 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int tt = 16 * c + 4 * g + r;
                const bool member = valid && (grp == 2 || (tt >> level) == loc) && t0 + tt < len;
                p[c][r] = member ? fast_exp2(s4[r] * qscale + shift - lse2) : 0.f;
                const float keep = DROP ? drop_scale(rowh, drop_edge_x(false, 0, t0 + tt), a.drop_thr, a.drop_inv_keep) : 1.f;
                wgt[c][r] = p[c][r] * d4[r] * keep;
                dl += wgt[c][r];
            }
        }
        dl += __shfl_xor(dl, 16);
        dl += __shfl_xor(dl, 32);
        if (grp < 2) {
            uint32_t hi[4], lo[4];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                split_pack(wgt[c][0] - dl * p[c][0], wgt[c][1] - dl * p[c][1], hi[2 * c], lo[2 * c]);
                split_pack(wgt[c][2] - dl * p[c][2], wgt[c][3] - dl * p[c][3], hi[2 * c + 1], lo[2 * c + 1]);
            }
            const u32x4 xh = {hi[0], hi[1], hi[2], hi[3]}, xl = {lo[0], lo[1], lo[2], lo[3]};
            const bf16x8_t sH = __builtin_bit_cast(bf16x8_t, xh), sL = __builtin_bit_cast(bf16x8_t, xl);
            f32x4_t dq[4];
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                dq[f] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                // transposed (the operands changed places): this lane holds features 16f + 4g .. + 3 of query j
                dq[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kB[f], sH, dq[f], 0, 0, 0);
                dq[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kB[f], sL, dq[f], 0, 0, 0);
            }
            if (g == 0 && valid)
                a.stat[(int64_t)bh * a.N + node] = make_float2((((t0 >> level) + loc) << level) < len ? lse2 : kLseGone, dl);
            constexpr bool guard = PACKED;   // packed batch: a span past the end of the sequence has no row
            // the rows go through k_s and leave whole, 16 bytes per lane
            wave_lds_sync();   // the previous group's rows have been read
            if (G16) {
#pragma unroll
                for (int f = 0; f < 4; ++f)
                    *reinterpret_cast<uint2*>(k_s + j * kVStride + 16 * f + 4 * g) =
                        make_uint2(pack_bf16(a.scale * dq[f][0], a.scale * dq[f][1]), pack_bf16(a.scale * dq[f][2], a.scale * dq[f][3]));
                wave_lds_sync();
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int slot = 8 * h + r8;
                    const int row = span_slot_row<PACKED>(a, grp, slot, t0, dvec);
                    if (grp == 1 && slot == 15) continue;
                    if (guard && !span_slot_kept(a, grp, slot, t0, len)) continue;
                    const uint2* src = reinterpret_cast<const uint2*>(k_s + slot * kVStride + piece * 8);
                    const uint2 x0 = src[0], x1 = src[1];
                    store_once(reinterpret_cast<uint4*>(reinterpret_cast<bf16_t*>(a.dQ) + base + (int64_t)row * a.sn + piece * 8),
                               make_uint4(x0.x, x0.y, x1.x, x1.y));
                }
            } else {
                float* stage = reinterpret_cast<float*>(k_s);   // [16 queries][kDqStride]: exactly the 32 staged K rows
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    const f32x4_t x = {a.scale * dq[f][0], a.scale * dq[f][1], a.scale * dq[f][2], a.scale * dq[f][3]};
                    *reinterpret_cast<f32x4_t*>(stage + j * kDqStride + 16 * f + 4 * g) = x;
                }
                wave_lds_sync();
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    const int slot = 4 * h + g;
                    const int row = span_slot_row<PACKED>(a, grp, slot, t0, dvec);
                    if (grp == 1 && slot == 15) continue;
                    if (guard && !span_slot_kept(a, grp, slot, t0, len)) continue;
                    store_once(reinterpret_cast<float4*>(a.dQ + base + (int64_t)row * a.sn + 4 * j),
                               *reinterpret_cast<const float4*>(stage + slot * kDqStride + 4 * j));
                }
            }
        } else {
            uint32_t whi[4], wlo[4], phi[4], plo[4];
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                split_pack(wgt[c][0], wgt[c][1], whi[2 * c], wlo[2 * c]);
                split_pack(wgt[c][2], wgt[c][3], whi[2 * c + 1], wlo[2 * c + 1]);
                split_pack(p[c][0], p[c][1], phi[2 * c], plo[2 * c]);
                split_pack(p[c][2], p[c][3], phi[2 * c + 1], plo[2 * c + 1]);
            }
            const u32x4 wh = {whi[0], whi[1], whi[2], whi[3]}, wl = {wlo[0], wlo[1], wlo[2], wlo[3]};
            const u32x4 ph = {phi[0], phi[1], phi[2], phi[3]}, pl = {plo[0], plo[1], plo[2], plo[3]};
            const bf16x8_t wH = __builtin_bit_cast(bf16x8_t, wh), wL = __builtin_bit_cast(bf16x8_t, wl);
            const bf16x8_t pH = __builtin_bit_cast(bf16x8_t, ph), pL = __builtin_bit_cast(bf16x8_t, pl);
            f32x4_t ow[4], op[4];
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                ow[f] = op[f] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                ow[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kB[f], wH, ow[f], 0, 0, 0);   // transposed as well
                ow[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kB[f], wL, ow[f], 0, 0, 0);
                op[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kB[f], pH, op[f], 0, 0, 0);
                op[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kB[f], pL, op[f], 0, 0, 0);
            }
            if (g == 0 && valid) a.part[(((int64_t)bh * nanc + j) * nblk + blk) * kQPartStride + 2 * kD] = dl;
            if (j < nanc) {   // features 16f + 4g .. + 3 of ancestor j: 16 bytes at a time
                float* dst = a.part + (((int64_t)bh * nanc + j) * nblk + blk) * kQPartStride + 4 * g;
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    *reinterpret_cast<f32x4_t*>(dst + 16 * f) = ow[f];
                    *reinterpret_cast<f32x4_t*>(dst + kD + 16 * f) = op[f];
                }
            }
        }
    }
}

template <bool PACKED>
__device__ __forceinline__ void bwd_q_span_merge_small(const SpanArgs& a, int item, int first, int rows) {
    const int lane = threadIdx.x & 63;
    SpanRow r;
    if (!span_merge_row(a, item, first, rows, kQPartStride, r)) return;
    if (r.cnt == 0 && a.leave_unkept) {   // the sequence does not keep the node: only the switch for the key side
        if (lane == 0) a.stat[(int64_t)r.bh * a.N + r.v] = make_float2(kLseGone, 0.f);
        return;
    }
    float xa[kSpanSmallMax], xb[kSpanSmallMax], xd[kSpanSmallMax];
#pragma unroll
    for (int b = 0; b < kSpanSmallMax; ++b) {
        const float* pb = r.src + (int64_t)max(min(b, r.cnt - 1), 0) * kQPartStride;
        xa[b] = pb[lane];
        xb[b] = pb[kD + lane];
        xd[b] = pb[2 * kD];
    }
    float sa = 0.f, sb = 0.f, dl = 0.f;
#pragma unroll
    for (int b = 0; b < kSpanSmallMax; ++b)
        if (b < r.cnt) {
            sa += xa[b];
            sb += xb[b];
            dl += xd[b];
        }
    const int64_t base = (int64_t)(r.bh / a.H) * a.sb + (int64_t)(r.bh % a.H) * a.sh;
    store_grad(a.dQ, base + (int64_t)span_merged_row<PACKED>(a, r) * a.sn + lane, a.scale * (sa - dl * sb), a.grad_bf16);
    if (lane == 0) a.stat[(int64_t)r.bh * a.N + r.v] = make_float2(span_row_lse2<PACKED>(a, r), dl);
}

template <bool PACKED>
__global__ void __launch_bounds__(kSpanBigThreads) bwd_q_span_merge_kernel(const SpanArgs a, int first, int rows_small,
                                                                           int first_big, int rows_big, int small_blocks) {
    __shared__ float s_a[64][kD + 4], s_b[64][kD + 4];
    __shared__ float s_d[64];
    const int big_blocks = a.BH * rows_big;
    if ((int)blockIdx.x >= big_blocks) {
        bwd_q_span_merge_small<PACKED>(a, (blockIdx.x - big_blocks) * (kSpanBigThreads / 64) + (threadIdx.x >> 6), first, rows_small);
        return;
    }
    SpanRow r;
    const int big_item = (blockIdx.x % a.BH) * rows_big + (rows_big - 1 - blockIdx.x / a.BH);
    if (!span_merge_row(a, big_item, first_big, rows_big, kQPartStride, r)) return;
    if (r.cnt == 0 && a.leave_unkept) {
        if (threadIdx.x == 0) a.stat[(int64_t)r.bh * a.N + r.v] = make_float2(kLseGone, 0.f);
        return;
    }
    const int t = threadIdx.x, fq = t & 15, pl = t >> 4;
    float4 sa = make_float4(0.f, 0.f, 0.f, 0.f), sb = sa;
    float dl = 0.f;
#pragma unroll 4
    for (int b = pl; b < r.cnt; b += 64) {
        const float* pb = r.src + (int64_t)b * kQPartStride;
        const float4 x = *reinterpret_cast<const float4*>(pb + 4 * fq), y = *reinterpret_cast<const float4*>(pb + kD + 4 * fq);
        dl += pb[2 * kD];
        sa.x += x.x; sa.y += x.y; sa.z += x.z; sa.w += x.w;
        sb.x += y.x; sb.y += y.y; sb.z += y.z; sb.w += y.w;
    }
    *reinterpret_cast<float4*>(&s_a[pl][4 * fq]) = sa;
    *reinterpret_cast<float4*>(&s_b[pl][4 * fq]) = sb;
    if (fq == 0) s_d[pl] = dl;
    __syncthreads();
    if (t < 64) {
        float ta = 0.f, tb = 0.f, td = 0.f;
        for (int p = 0; p < 64; ++p) {
            ta += s_a[p][t];
            tb += s_b[p][t];
            td += s_d[p];
        }
        const int64_t base = (int64_t)(r.bh / a.H) * a.sb + (int64_t)(r.bh % a.H) * a.sh;
        store_grad(a.dQ, base + (int64_t)span_merged_row<PACKED>(a, r) * a.sn + t, a.scale * (ta - td * tb), a.grad_bf16);
        if (t == 0) a.stat[(int64_t)r.bh * a.N + r.v] = make_float2(span_row_lse2<PACKED>(a, r), td);
    }
}

}  // namespace
}  // namespace bpt
