// Graph self-attention with tree relative positions (paper Sec. 3.1 eq. (6),
// Sec. 3.4 eq. (8)) forward and backward for gfx950.
//
// Work decomposition.  A row of an adjacency (query node u with its key nodes, or
// key node v with its query nodes) is cut into segments of at most kSeg edges; one
// 64-lane wavefront processes one segment.  Inside the wavefront 8 lanes share one
// edge: each lane holds 8 of the 64 features, so a 128-byte bf16 row is one 16-byte
// load per lane and 8 edges are in flight per wavefront instruction.  Each 8-lane
// group keeps its own online-softmax state; the 8 groups are merged once per
// segment.  The edge loop is software pipelined: neighbour indices are fetched two
// iterations ahead and the gathered rows one iteration ahead, so the dependent
// index -> row latency overlaps the arithmetic of the current edges.
//
// Workgroups are persistent: each walks a strided list of tiles inside the share of
// its XCD, so workgroups that run together on one XCD touch neighbouring rows and
// the rows they share stay in that XCD's L2.
//
// The relative-position table is staged in LDS once per workgroup when it fits.
// For span rows every edge carries the same r_anc(level), which only shifts all
// scores of the row by scale*q.r_anc: it is applied once per row.
#include <algorithm>

#include "bpt_internal.h"

namespace bpt {
namespace {

typedef uint16_t bf16_t;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kNegBig = -1.0e30f;
constexpr int kThreads = 512;            // 8 wavefronts per workgroup
constexpr int kWaves = kThreads / 64;
constexpr int kQPartStride = 132;        // query-side partial: A[64], Bv[64], delta, padding

struct AttnArgs {
    // tensors
    const void *Q, *K, *V, *rel, *dout;
    void* out;
    float* lse_w;
    const float* lse_r;
    float *dQ, *dK, *dV, *d_rel;
    float2* stat;            // per (batch*head, node): (lse * log2(e), delta), written by the query side
    float2* wp;              // per (batch*head, edge of a token row): (p_e dP_e, p_e), written by the query side
    int64_t e_tok;           // edges of token rows (they come first in the CSR)
    float *part, *drel_part;
    int64_t sb, sh, sn;
    int32_t row_bytes;       // sn * sizeof(T): distance between the rows of two nodes
    uint32_t slab_bytes;     // extent of one (batch, head) slab of Q/K/V/dout
    uint32_t idx_bytes;      // extent of ia / ib
    int32_t BH, H, N, n_tokens;
    float scale;
    // adjacency: ptr[rows+1]; ia = other endpoint (col / t_src); ib = relative-position id
    const int32_t *ptr, *ia, *ib;
    // schedule
    const int32_t *seg_row, *seg_begin, *seg_part, *tile_ptr;
    int32_t num_tiles, num_part;
    int32_t rel_rows_lds;   // rows of the r table staged in LDS (0: read it from global memory)
    int32_t drel_rows;      // rows of d_rel that token rows can touch (levels with contextual edges)
    int32_t drel_block;     // token rows per block of rel_grad_kernel
    int32_t rel_rows;       // rows of the whole table
};

// ---- lane helpers ---------------------------------------------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_move(float x) {
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
// sum over the 8 lanes that share an edge; every one of them gets the result
__device__ __forceinline__ float sum8(float x) {
    x += dpp_move<0xB1>(x);   // quad_perm [1,0,3,2]
    x += dpp_move<0x4E>(x);   // quad_perm [2,3,0,1]
    x += dpp_move<0x141>(x);  // row_half_mirror: the other quad of the 8-lane group
    return x;
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// all 8 groups (lanes with the same feature chunk) get the sum / max
__device__ __forceinline__ float slots_sum(float x) {
    x += __shfl_xor(x, 8);
    x += __shfl_xor(x, 16);
    x += __shfl_xor(x, 32);
    return x;
}
__device__ __forceinline__ float slots_max(float x) {
    x = fmaxf(x, __shfl_xor(x, 8));
    x = fmaxf(x, __shfl_xor(x, 16));
    x = fmaxf(x, __shfl_xor(x, 32));
    return x;
}
// Sum x[0..7] over the 8 groups with 7 exchanges instead of 24: at every step a lane
// keeps one half of its values and hands the other half to its partner.  Returns
// the total of element slot_elem(lane) of the lane's feature chunk.
__device__ __forceinline__ int slot_elem(int lane) {
    return ((lane >> 5) & 1) * 4 + ((lane >> 4) & 1) * 2 + ((lane >> 3) & 1);
}
__device__ __forceinline__ float reduce_slots8(const float (&x)[8], int lane) {
    const bool h32 = lane & 32, h16 = lane & 16, h8 = lane & 8;
    float y[4], z[2];
#pragma unroll
    for (int i = 0; i < 4; ++i) y[i] = (h32 ? x[i + 4] : x[i]) + __shfl_xor(h32 ? x[i] : x[i + 4], 32);
#pragma unroll
    for (int i = 0; i < 2; ++i) z[i] = (h16 ? y[i + 2] : y[i]) + __shfl_xor(h16 ? y[i] : y[i + 2], 16);
    return (h8 ? z[1] : z[0]) + __shfl_xor(h8 ? z[0] : z[1], 8);
}

// ---- 8 consecutive features of one row, as loaded -----------------------------------
template <typename T>
struct Row;
template <>
struct Row<bf16_t> {
    uint4 w;
};
template <>
struct Row<float> {
    float4 a, b;
};
__device__ __forceinline__ Row<bf16_t> load_row(const bf16_t* p) {
    Row<bf16_t> r;
    r.w = *reinterpret_cast<const uint4*>(p);
    return r;
}
__device__ __forceinline__ Row<float> load_row(const float* p) {
    Row<float> r;
    r.a = *reinterpret_cast<const float4*>(p);
    r.b = *reinterpret_cast<const float4*>(p + 4);
    return r;
}
__device__ __forceinline__ void unpack(const Row<bf16_t>& r, float (&x)[8]) {
    x[0] = __uint_as_float(r.w.x << 16); x[1] = __uint_as_float(r.w.x & 0xFFFF0000u);
    x[2] = __uint_as_float(r.w.y << 16); x[3] = __uint_as_float(r.w.y & 0xFFFF0000u);
    x[4] = __uint_as_float(r.w.z << 16); x[5] = __uint_as_float(r.w.z & 0xFFFF0000u);
    x[6] = __uint_as_float(r.w.w << 16); x[7] = __uint_as_float(r.w.w & 0xFFFF0000u);
}
__device__ __forceinline__ void unpack(const Row<float>& r, float (&x)[8]) {
    x[0] = r.a.x; x[1] = r.a.y; x[2] = r.a.z; x[3] = r.a.w;
    x[4] = r.b.x; x[5] = r.b.y; x[6] = r.b.z; x[7] = r.b.w;
}
template <typename T>
__device__ __forceinline__ void load8(const T* p, float (&x)[8]) {
    unpack(load_row(p), x);
}
// c + dot product of two 8-feature chunks, fp32 accumulation.  bf16 rows stay packed:
// v_dot2c_f32_bf16 multiplies two pairs per instruction, so neither row is unpacked.
typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2_t;
__device__ __forceinline__ float dot2_bf16(uint32_t x, uint32_t y, float c) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, x), __builtin_bit_cast(bf16x2_t, y), c, false);
}
__device__ __forceinline__ float dot8(const Row<bf16_t>& x, const Row<bf16_t>& y, float c) {
    c = dot2_bf16(x.w.x, y.w.x, c);
    c = dot2_bf16(x.w.y, y.w.y, c);
    c = dot2_bf16(x.w.z, y.w.z, c);
    return dot2_bf16(x.w.w, y.w.w, c);
}
__device__ __forceinline__ float dot8(const Row<float>& x, const Row<float>& y, float c) {
    c += x.a.x * y.a.x; c += x.a.y * y.a.y; c += x.a.z * y.a.z; c += x.a.w * y.a.w;
    c += x.b.x * y.b.x; c += x.b.y * y.b.y; c += x.b.z * y.b.z; c += x.b.w * y.b.w;
    return c;
}
// Gathers go through buffer loads: a 32-bit byte offset per lane against a
// wave-uniform descriptor (cheap addressing, out-of-range offsets read 0), and,
// being intrinsics rather than plain loads, they stay where the software pipeline
// puts them instead of being sunk to their first use.
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* p, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, (int)bytes, 0x00020000);
}
__device__ __forceinline__ int buf_i32(rsrc_t r, int byte_off) {
    return (int)__builtin_amdgcn_raw_buffer_load_b32(r, byte_off, 0, 0);
}
__device__ __forceinline__ float2 buf_f2(rsrc_t r, int byte_off) {
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, 0, 0);
    return make_float2(__uint_as_float(v.x), __uint_as_float(v.y));
}
__device__ __forceinline__ void buf_row(rsrc_t r, int byte_off, Row<bf16_t>& out) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0);
    out.w = make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void buf_row(rsrc_t r, int byte_off, Row<float>& out) {
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off, 0, 0);
    const u32x4 w = __builtin_amdgcn_raw_buffer_load_b128(r, byte_off + 16, 0, 0);
    out.a = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
    out.b = make_float4(__uint_as_float(w.x), __uint_as_float(w.y), __uint_as_float(w.z), __uint_as_float(w.w));
}
// the lane's 8 features of the row of `node`
template <typename T>
__device__ __forceinline__ Row<T> gather_row(rsrc_t r, int node, int row_bytes, int lane_off) {
    Row<T> out;
    buf_row(r, (int)__umul24(node, row_bytes) + lane_off, out);
    return out;
}

__device__ __forceinline__ uint32_t to_bf16_bits(float f) {  // round to nearest even (v_cvt_pk_bf16_f32)
    return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)f);
}
__device__ __forceinline__ void store8(float* p, const float (&x)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(x[4], x[5], x[6], x[7]);
}
__device__ __forceinline__ void store8(bf16_t* p, const float (&x)[8]) {
    uint4 w;
    w.x = to_bf16_bits(x[0]) | (to_bf16_bits(x[1]) << 16);
    w.y = to_bf16_bits(x[2]) | (to_bf16_bits(x[3]) << 16);
    w.z = to_bf16_bits(x[4]) | (to_bf16_bits(x[5]) << 16);
    w.w = to_bf16_bits(x[6]) | (to_bf16_bits(x[7]) << 16);
    *reinterpret_cast<uint4*>(p) = w;
}
__device__ __forceinline__ void store1(float* p, float x) { *p = x; }
__device__ __forceinline__ void store1(bf16_t* p, float x) { *p = (bf16_t)to_bf16_bits(x); }

// Copy `count` table elements (a multiple of 8) into LDS, 16 bytes per thread per step.
template <typename T>
__device__ __forceinline__ void stage_table(T* dst, const T* src, int count) {
    constexpr int per = 16 / sizeof(T);
    for (int i = threadIdx.x * per; i < count; i += blockDim.x * per)
        *reinterpret_cast<uint4*>(dst + i) = *reinterpret_cast<const uint4*>(src + i);
}

// Tiles of this workgroup: the (batch*head, tile) space is split into 8 contiguous
// shares, one per XCD (workgroup w runs on XCD w mod 8); inside a share the
// workgroups of that XCD interleave, so they sweep it together.
struct TileWalk {
    int t, t_end, step;
    __device__ TileWalk(int total) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3, wgs = gridDim.x >> 3;
        const int per = (total + 7) >> 3;
        t = xcd * per + j;
        t_end = min(total, (xcd + 1) * per);
        step = wgs;
    }
};

// ---- forward --------------------------------------------------------------------
// One segment [e0, e1) of row u (e1 > e0).  SPAN: the row is a span node.
template <typename T, bool REL_LDS, bool SPAN>
__device__ __forceinline__ void fwd_segment(const AttnArgs& a, const T* rel_s, rsrc_t rK, rsrc_t rV, rsrc_t rIa,
                                            rsrc_t rIb, int bh, int64_t base, int u, int e0, int e1, int part,
                                            int lane) {
    const int slot = lane >> 3, sub = lane & 7;
    const int lane_off = sub * 8 * (int)sizeof(T);
    const T* relg = static_cast<const T*>(a.rel) + sub * 8;

    // indices two iterations ahead, rows one iteration ahead.  Lanes past the end of
    // the segment read the next rows' indices (or 0 past the array): valid nodes,
    // and their contribution is masked.
    int eo = (e0 + slot) * 4;
    const int c0 = buf_i32(rIa, eo);
    int c1 = buf_i32(rIa, eo + 32);
    int r0 = 0, r1 = 0;
    if (!SPAN) {
        r0 = buf_i32(rIb, eo);
        r1 = buf_i32(rIb, eo + 32);
    }
    Row<T> k0 = gather_row<T>(rK, c0, a.row_bytes, lane_off), v0 = gather_row<T>(rV, c0, a.row_bytes, lane_off);

    const Row<T> q = load_row(static_cast<const T*>(a.Q) + base + (int64_t)u * a.sn + sub * 8);
    const float qscale = a.scale * kLog2e;
    float shift = 0.f;
    if (SPAN)  // r_anc(level) is common to the whole row
        shift = sum8(dot8(q, load_row(relg + (int64_t)a.ib[e0] * kD), 0.f)) * qscale;
    float m = kNegBig, l = 0.f, acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;

    // One iteration: prefetch (indices of iteration +2, rows of iteration +1 into kn/vn),
    // then work on the rows kc/vc fetched one iteration ago.  Called alternately with
    // the two row buffers swapped, so nothing has to be copied between iterations.
    auto step = [&](int eb, const Row<T>& kc, const Row<T>& vc, Row<T>& kn, Row<T>& vn) {
        const int c2 = buf_i32(rIa, eo + 64);
        int r2 = 0;
        if (!SPAN) r2 = buf_i32(rIb, eo + 64);
        kn = gather_row<T>(rK, c1, a.row_bytes, lane_off);
        vn = gather_row<T>(rV, c1, a.row_bytes, lane_off);
        eo += 32;

        const bool valid = eb + slot < e1;
        float vv[8], d = 0.f;
        if (!SPAN) {
            const int rid = valid ? r0 : 0;  // a masked lane may hold an id of some other row
            d = dot8(q, REL_LDS ? load_row(rel_s + rid * kD + sub * 8) : load_row(relg + (int64_t)rid * kD), 0.f);
        }
        d = dot8(q, kc, d);
        float sc = sum8(d) * qscale + shift;
        sc = valid ? sc : kNegBig;
        // online softmax with one exponential: of exp2(m - mn) and exp2(sc - mn) one is 1
        const bool up = sc > m;
        const float e = fast_exp2(up ? m - sc : sc - m);
        const float corr = up ? e : 1.f;
        const float p = valid ? (up ? 1.f : e) : 0.f;
        m = up ? sc : m;
        unpack(vc, vv);
        l *= corr;
        l += p;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            acc[i] *= corr;
            acc[i] = fmaf(p, vv[i], acc[i]);
        }
        c1 = c2;
        r0 = r1;
        r1 = r2;
    };
    Row<T> k1, v1;
    for (int eb = e0; eb < e1; eb += 16) {
        step(eb, k0, v0, k1, v1);
        if (eb + 8 >= e1) break;
        step(eb + 8, k1, v1, k0, v0);
    }
    // merge the 8 groups: common max, rescale, then sum
    const float mall = slots_max(m);
    const float c = fast_exp2(m - mall);
    l = slots_sum(l * c);
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] *= c;
    const float mine = reduce_slots8(acc, lane);
    const int col = sub * 8 + slot_elem(lane);
    if (part < 0) {
        store1(static_cast<T*>(a.out) + base + (int64_t)u * a.sn + col, l > 0.f ? mine / l : 0.f);
        if (lane == 0) a.lse_w[(int64_t)bh * a.N + u] = (mall + fast_log2(l)) * kLn2;
    } else {
        float* dst = a.part + ((int64_t)bh * a.num_part + part) * kPartStride;
        dst[col] = mine;
        if (lane == 0) {
            dst[64] = mall;
            dst[65] = l;
        }
    }
}

// Eight consecutive span rows of one level (equal degree deg <= 64, keys = the deg
// consecutive tokens each span contains), one row per 8-lane group: no neighbour
// indices to fetch, no masking, and nothing to merge between the groups -- each
// group finishes its own row.  Short span rows are most of the rows of the graph,
// and one wavefront per row would spend its time in row set-up.
template <typename T>
__device__ __forceinline__ void fwd_span8(const AttnArgs& a, rsrc_t rK, rsrc_t rV, int bh, int64_t base, int u0, int e0,
                                          int deg, int lane) {
    const int slot = lane >> 3, sub = lane & 7;
    const int lane_off = sub * 8 * (int)sizeof(T);
    const int u = u0 + slot;
    const int tok0 = a.ia[e0 + slot * deg];  // first token of this group's span
    Row<T> k0 = gather_row<T>(rK, tok0, a.row_bytes, lane_off), v0 = gather_row<T>(rV, tok0, a.row_bytes, lane_off);
    const Row<T> q = load_row(static_cast<const T*>(a.Q) + base + (int64_t)u * a.sn + sub * 8);
    const float qscale = a.scale * kLog2e;
    const float shift =
        sum8(dot8(q, load_row(static_cast<const T*>(a.rel) + (int64_t)a.ib[e0] * kD + sub * 8), 0.f)) * qscale;
    float m = kNegBig, l = 0.f, acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    auto step = [&](int i, const Row<T>& kc, const Row<T>& vc, Row<T>& kn, Row<T>& vn) {
        const int nxt = tok0 + min(i + 1, deg - 1);
        kn = gather_row<T>(rK, nxt, a.row_bytes, lane_off);
        vn = gather_row<T>(rV, nxt, a.row_bytes, lane_off);
        const float sc = sum8(dot8(q, kc, 0.f)) * qscale + shift;
        const bool up = sc > m;
        const float e = fast_exp2(up ? m - sc : sc - m);
        const float corr = up ? e : 1.f, p = up ? 1.f : e;
        m = up ? sc : m;
        float vv[8];
        unpack(vc, vv);
        l *= corr;
        l += p;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            acc[x] *= corr;
            acc[x] = fmaf(p, vv[x], acc[x]);
        }
    };
    Row<T> k1, v1;
    for (int i = 0; i < deg; i += 2) {  // deg is a power of two >= 2
        step(i, k0, v0, k1, v1);
        step(i + 1, k1, v1, k0, v0);
    }
    const float inv = 1.f / l;
#pragma unroll
    for (int x = 0; x < 8; ++x) acc[x] *= inv;
    store8(static_cast<T*>(a.out) + base + (int64_t)u * a.sn + sub * 8, acc);
    if (sub == 0) a.lse_w[(int64_t)bh * a.N + u] = (m + fast_log2(l)) * kLn2;
}

template <typename T, bool REL_LDS>
__global__ void __launch_bounds__(kThreads) fwd_kernel(const AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    T* rel_s = reinterpret_cast<T*>(smem);
    if (REL_LDS) {
        stage_table(rel_s, static_cast<const T*>(a.rel), a.rel_rows_lds * kD);
        __syncthreads();
    }
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform: row bookkeeping stays scalar
    const int nwaves = blockDim.x >> 6;
    const rsrc_t rIa = make_rsrc(a.ia, a.idx_bytes), rIb = make_rsrc(a.ib, a.idx_bytes);
    for (TileWalk w(a.BH * a.num_tiles); w.t < w.t_end; w.t += w.step) {
        const int bh = w.t / a.num_tiles, tile = w.t - bh * a.num_tiles;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        const rsrc_t rK = make_rsrc(static_cast<const T*>(a.K) + base, a.slab_bytes);
        const rsrc_t rV = make_rsrc(static_cast<const T*>(a.V) + base, a.slab_bytes);
        const int s1 = a.tile_ptr[tile + 1];
        for (int s = a.tile_ptr[tile] + wave; s < s1; s += nwaves) {
            const int u = a.seg_row[s];
            const int e0 = a.seg_begin[s];
            const int e1 = min(e0 + kSeg, a.ptr[u + 1]);
            const int part = a.seg_part[s];
            if (e1 <= e0) continue;  // no row of this adjacency is empty
            if (part == kPartSpan8)
                fwd_span8<T>(a, rK, rV, bh, base, u, e0, a.ptr[u + 1] - e0, lane);
            else if (u >= a.n_tokens)
                fwd_segment<T, REL_LDS, true>(a, rel_s, rK, rV, rIa, rIb, bh, base, u, e0, e1, part, lane);
            else
                fwd_segment<T, REL_LDS, false>(a, rel_s, rK, rV, rIa, rIb, bh, base, u, e0, e1, part, lane);
        }
    }
}

// one wavefront per (batch*head, row with several segments); lane = feature
template <typename T>
__global__ void __launch_bounds__(256) fwd_merge_kernel(const AttnArgs a, const int32_t* __restrict__ multi_row,
                                                        const int32_t* __restrict__ multi_ptr, int num_multi) {
    const int lane = threadIdx.x & 63;
    const int item = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (item >= a.BH * num_multi) return;
    const int bh = item / num_multi, j = item - bh * num_multi;
    const int u = multi_row[j];
    float m = kNegBig, l = 0.f, acc = 0.f;
    for (int p = multi_ptr[j]; p < multi_ptr[j + 1]; ++p) {
        const float* src = a.part + ((int64_t)bh * a.num_part + p) * kPartStride;
        const float mo = src[64], lo = src[65], ao = src[lane];
        const float mn = fmaxf(m, mo);
        const float c1 = fast_exp2(m - mn), c2 = fast_exp2(mo - mn);
        l = l * c1 + lo * c2;
        acc = acc * c1 + ao * c2;
        m = mn;
    }
    const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
    store1(static_cast<T*>(a.out) + base + (int64_t)u * a.sn + lane, l > 0.f ? acc / l : 0.f);
    if (lane == 0) a.lse_w[(int64_t)bh * a.N + u] = (m + fast_log2(l)) * kLn2;
}

// ---- backward, query side: delta and dQ ------------------------------------------------
// With w_e = p_e dP_e:  delta_u = sum_e w_e  and
//   dQ_u = scale * sum_e p_e (dP_e - delta_u)(k_e + r_e) = scale * (A - delta_u * Bv),
//   A = sum_e w_e (k_e + r_e),  Bv = sum_e p_e (k_e + r_e),
// so one pass over the row gives delta exactly (in fp32, not through the rounded
// `out`) and dQ.  For a span row r_anc drops out of dQ because the dS of a row sum to 0.
template <typename T, bool REL_LDS, bool SPAN>
__device__ __forceinline__ void bwd_q_segment(const AttnArgs& a, const T* rel_s, rsrc_t rK, rsrc_t rV, rsrc_t rIa,
                                              rsrc_t rIb, int bh, int64_t base, int u, int e0, int e1, int part,
                                              int lane) {
    const int slot = lane >> 3, sub = lane & 7;
    const int lane_off = sub * 8 * (int)sizeof(T);
    const T* relg = static_cast<const T*>(a.rel) + sub * 8;

    int eo = (e0 + slot) * 4;
    const int c0 = buf_i32(rIa, eo);
    int c1 = buf_i32(rIa, eo + 32);
    int r0 = 0, r1 = 0;
    if (!SPAN) {
        r0 = buf_i32(rIb, eo);
        r1 = buf_i32(rIb, eo + 32);
    }
    Row<T> k0 = gather_row<T>(rK, c0, a.row_bytes, lane_off), v0 = gather_row<T>(rV, c0, a.row_bytes, lane_off);

    float qs[8];
    load8(static_cast<const T*>(a.Q) + base + (int64_t)u * a.sn + sub * 8, qs);
    const Row<T> g = load_row(static_cast<const T*>(a.dout) + base + (int64_t)u * a.sn + sub * 8);
    const float qscale = a.scale * kLog2e;
#pragma unroll
    for (int i = 0; i < 8; ++i) qs[i] *= qscale;
    const float lse2 = a.lse_r[(int64_t)bh * a.N + u] * kLog2e;
    float shift = 0.f;
    if (SPAN) {
        float r[8], d = 0.f;
        load8(relg + (int64_t)a.ib[e0] * kD, r);
#pragma unroll
        for (int i = 0; i < 8; ++i) d += qs[i] * r[i];
        shift = sum8(d);
    }
    float A[8], Bv[8], dl = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) A[i] = Bv[i] = 0.f;

    auto step = [&](int eb, const Row<T>& kc, const Row<T>& vc, Row<T>& kn, Row<T>& vn) {
        const int c2 = buf_i32(rIa, eo + 64);
        int r2 = 0;
        if (!SPAN) r2 = buf_i32(rIb, eo + 64);
        kn = gather_row<T>(rK, c1, a.row_bytes, lane_off);
        vn = gather_row<T>(rV, c1, a.row_bytes, lane_off);

        const bool valid = eb + slot < e1;
        float kk[8];
        unpack(kc, kk);
        if (!SPAN) {
            float r[8];
            const int rid = valid ? r0 : 0;  // a masked lane may hold an id of some other row
            if (REL_LDS)
                load8(rel_s + rid * kD + sub * 8, r);
            else
                load8(relg + (int64_t)rid * kD, r);
#pragma unroll
            for (int i = 0; i < 8; ++i) kk[i] += r[i];
        }
        float d = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) d += qs[i] * kk[i];
        const float sc = sum8(d) + shift;
        const float dP = sum8(dot8(g, vc, 0.f));
        const float p = valid ? fast_exp2(sc - lse2) : 0.f;
        const float wgt = p * dP;
        dl += wgt;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            A[i] = fmaf(wgt, kk[i], A[i]);
            Bv[i] = fmaf(p, kk[i], Bv[i]);
        }
        // what d_rel needs of this edge (dS_e = w_e - delta_u p_e once delta_u is known)
        if (!SPAN && valid && sub == 0) a.wp[(int64_t)bh * a.e_tok + (eo >> 2)] = make_float2(wgt, p);
        eo += 32;
        c1 = c2;
        r0 = r1;
        r1 = r2;
    };
    Row<T> k1, v1;
    for (int eb = e0; eb < e1; eb += 16) {
        step(eb, k0, v0, k1, v1);
        if (eb + 8 >= e1) break;
        step(eb + 8, k1, v1, k0, v0);
    }
    dl = slots_sum(dl);
    const int col = sub * 8 + slot_elem(lane);
    if (part < 0) {
#pragma unroll
        for (int i = 0; i < 8; ++i) A[i] -= dl * Bv[i];
        a.dQ[base + (int64_t)u * a.sn + col] = a.scale * reduce_slots8(A, lane);
        if (lane == 0) a.stat[(int64_t)bh * a.N + u] = make_float2(lse2, dl);
    } else {
        float* dst = a.part + ((int64_t)bh * a.num_part + part) * kQPartStride;
        dst[col] = reduce_slots8(A, lane);
        dst[kD + col] = reduce_slots8(Bv, lane);
        if (lane == 0) dst[2 * kD] = dl;
    }
}

// Query side of eight consecutive short span rows, one row per 8-lane group (see fwd_span8).
template <typename T>
__device__ __forceinline__ void bwd_q_span8(const AttnArgs& a, rsrc_t rK, rsrc_t rV, int bh, int64_t base, int u0,
                                            int e0, int deg, int lane) {
    const int slot = lane >> 3, sub = lane & 7;
    const int lane_off = sub * 8 * (int)sizeof(T);
    const int u = u0 + slot;
    const int tok0 = a.ia[e0 + slot * deg];
    Row<T> k0 = gather_row<T>(rK, tok0, a.row_bytes, lane_off), v0 = gather_row<T>(rV, tok0, a.row_bytes, lane_off);
    float qs[8];
    load8(static_cast<const T*>(a.Q) + base + (int64_t)u * a.sn + sub * 8, qs);
    const Row<T> g = load_row(static_cast<const T*>(a.dout) + base + (int64_t)u * a.sn + sub * 8);
    const float qscale = a.scale * kLog2e;
#pragma unroll
    for (int i = 0; i < 8; ++i) qs[i] *= qscale;
    const float lse2 = a.lse_r[(int64_t)bh * a.N + u] * kLog2e;
    float shift;
    {
        float r[8], d = 0.f;
        load8(static_cast<const T*>(a.rel) + (int64_t)a.ib[e0] * kD + sub * 8, r);
#pragma unroll
        for (int i = 0; i < 8; ++i) d += qs[i] * r[i];
        shift = sum8(d);
    }
    float A[8], Bv[8], dl = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) A[i] = Bv[i] = 0.f;
    auto step = [&](int i, const Row<T>& kc, const Row<T>& vc, Row<T>& kn, Row<T>& vn) {
        const int nxt = tok0 + min(i + 1, deg - 1);
        kn = gather_row<T>(rK, nxt, a.row_bytes, lane_off);
        vn = gather_row<T>(rV, nxt, a.row_bytes, lane_off);
        float kk[8], d = 0.f;
        unpack(kc, kk);
#pragma unroll
        for (int x = 0; x < 8; ++x) d += qs[x] * kk[x];
        const float p = fast_exp2(sum8(d) + shift - lse2);
        const float wgt = p * sum8(dot8(g, vc, 0.f));
        dl += wgt;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            A[x] = fmaf(wgt, kk[x], A[x]);
            Bv[x] = fmaf(p, kk[x], Bv[x]);
        }
    };
    Row<T> k1, v1;
    for (int i = 0; i < deg; i += 2) {
        step(i, k0, v0, k1, v1);
        step(i + 1, k1, v1, k0, v0);
    }
#pragma unroll
    for (int x = 0; x < 8; ++x) A[x] = a.scale * (A[x] - dl * Bv[x]);
    store8(a.dQ + base + (int64_t)u * a.sn + sub * 8, A);
    if (sub == 0) a.stat[(int64_t)bh * a.N + u] = make_float2(lse2, dl);
}

template <typename T, bool REL_LDS>
__global__ void __launch_bounds__(kThreads) bwd_q_kernel(const AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    T* rel_s = reinterpret_cast<T*>(smem);
    if (REL_LDS) {
        stage_table(rel_s, static_cast<const T*>(a.rel), a.rel_rows_lds * kD);
        __syncthreads();
    }
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const rsrc_t rIa = make_rsrc(a.ia, a.idx_bytes), rIb = make_rsrc(a.ib, a.idx_bytes);
    for (TileWalk w(a.BH * a.num_tiles); w.t < w.t_end; w.t += w.step) {
        const int bh = w.t / a.num_tiles, tile = w.t - bh * a.num_tiles;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        const rsrc_t rK = make_rsrc(static_cast<const T*>(a.K) + base, a.slab_bytes);
        const rsrc_t rV = make_rsrc(static_cast<const T*>(a.V) + base, a.slab_bytes);
        const int s1 = a.tile_ptr[tile + 1];
        for (int s = a.tile_ptr[tile] + wave; s < s1; s += nwaves) {
            const int u = a.seg_row[s];
            const int e0 = a.seg_begin[s];
            const int e1 = min(e0 + kSeg, a.ptr[u + 1]);
            const int part = a.seg_part[s];
            if (e1 <= e0) continue;
            if (part == kPartSpan8)
                bwd_q_span8<T>(a, rK, rV, bh, base, u, e0, a.ptr[u + 1] - e0, lane);
            else if (u >= a.n_tokens)
                bwd_q_segment<T, REL_LDS, true>(a, rel_s, rK, rV, rIa, rIb, bh, base, u, e0, e1, part, lane);
            else
                bwd_q_segment<T, REL_LDS, false>(a, rel_s, rK, rV, rIa, rIb, bh, base, u, e0, e1, part, lane);
        }
    }
}

// rows cut into several segments: combine (A, Bv, delta) partials in segment order
__global__ void __launch_bounds__(256) bwd_q_merge_kernel(const AttnArgs a, const int32_t* __restrict__ multi_row,
                                                          const int32_t* __restrict__ multi_ptr, int num_multi) {
    const int lane = threadIdx.x & 63;
    const int item = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (item >= a.BH * num_multi) return;
    const int bh = item / num_multi, j = item - bh * num_multi;
    const int u = multi_row[j];
    float sa = 0.f, sb = 0.f, dl = 0.f;
    for (int p = multi_ptr[j]; p < multi_ptr[j + 1]; ++p) {
        const float* src = a.part + ((int64_t)bh * a.num_part + p) * kQPartStride;
        sa += src[lane];
        sb += src[kD + lane];
        dl += src[2 * kD];
    }
    const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
    a.dQ[base + (int64_t)u * a.sn + lane] = a.scale * (sa - dl * sb);
    if (lane == 0) a.stat[(int64_t)bh * a.N + u] = make_float2(a.lse_r[(int64_t)bh * a.N + u] * kLog2e, dl);
}

// ---- backward, key side: dK, dV over the transposed adjacency -------------------------
// One wavefront per (segment of a) key node v; the rows q_u, dout_u and the pair
// (lse_u, delta_u) of its queries u are gathered.  No atomics: every key row is
// reduced by one wavefront (or by the merge kernel, in segment order).
template <typename T, bool REL_LDS>
__device__ __forceinline__ void bwd_kv_segment(const AttnArgs& a, const T* rel_s, rsrc_t rQ, rsrc_t rG, rsrc_t rS,
                                               rsrc_t rIa, rsrc_t rIb, int bh, int64_t base, int v, int e0, int e1,
                                               int part, int lane) {
    const int slot = lane >> 3, sub = lane & 7;
    const int lane_off = sub * 8 * (int)sizeof(T);
    const T* relg = static_cast<const T*>(a.rel) + sub * 8;
    const float qscale = a.scale * kLog2e;

    float dk[8], dv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) dk[i] = dv[i] = 0.f;

    if (e1 > e0) {
        int eo = (e0 + slot) * 4;
        const int u0 = buf_i32(rIa, eo);
        int u1 = buf_i32(rIa, eo + 32);
        int r0 = buf_i32(rIb, eo), r1 = buf_i32(rIb, eo + 32);
        Row<T> q0 = gather_row<T>(rQ, u0, a.row_bytes, lane_off), g0 = gather_row<T>(rG, u0, a.row_bytes, lane_off);
        float2 st0 = buf_f2(rS, u0 * 8);
        const Row<T> kk = load_row(static_cast<const T*>(a.K) + base + (int64_t)v * a.sn + sub * 8);
        const Row<T> vv = load_row(static_cast<const T*>(a.V) + base + (int64_t)v * a.sn + sub * 8);

        auto step = [&](int eb, const Row<T>& qc, const Row<T>& gc, const float2& stc, Row<T>& qn, Row<T>& gn,
                        float2& stn) {
            const int u2 = buf_i32(rIa, eo + 64);
            const int r2 = buf_i32(rIb, eo + 64);
            qn = gather_row<T>(rQ, u1, a.row_bytes, lane_off);
            gn = gather_row<T>(rG, u1, a.row_bytes, lane_off);
            stn = buf_f2(rS, u1 * 8);
            eo += 32;

            const bool valid = eb + slot < e1;
            float q[8], g[8];
            float d = dot8(qc, REL_LDS ? load_row(rel_s + r0 * kD + sub * 8) : load_row(relg + (int64_t)r0 * kD), 0.f);
            d = dot8(qc, kk, d);
            const float sc = sum8(d) * qscale;
            const float dP = sum8(dot8(gc, vv, 0.f));
            unpack(qc, q);
            unpack(gc, g);
            const float p = valid ? fast_exp2(sc - stc.x) : 0.f;
            const float dS = p * (dP - stc.y);
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                dk[i] = fmaf(dS, q[i], dk[i]);
                dv[i] = fmaf(p, g[i], dv[i]);
            }
            u1 = u2;
            r0 = r1;
            r1 = r2;
        };
        Row<T> q1, g1;
        float2 st1;
        for (int eb = e0; eb < e1; eb += 16) {
            step(eb, q0, g0, st0, q1, g1, st1);
            if (eb + 8 >= e1) break;
            step(eb + 8, q1, g1, st1, q0, g0, st0);
        }
    }
    const float tk = reduce_slots8(dk, lane), tv = reduce_slots8(dv, lane);
    const int col = sub * 8 + slot_elem(lane);
    if (part < 0) {
        a.dK[base + (int64_t)v * a.sn + col] = tk * a.scale;
        a.dV[base + (int64_t)v * a.sn + col] = tv;
    } else {
        float* dst = a.part + ((int64_t)bh * a.num_part + part) * (2 * kD);
        dst[col] = tk * a.scale;
        dst[kD + col] = tv;
    }
}

template <typename T, bool REL_LDS>
__global__ void __launch_bounds__(kThreads) bwd_kv_kernel(const AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    T* rel_s = reinterpret_cast<T*>(smem);
    if (REL_LDS) {
        stage_table(rel_s, static_cast<const T*>(a.rel), a.rel_rows_lds * kD);
        __syncthreads();
    }
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const rsrc_t rIa = make_rsrc(a.ia, a.idx_bytes), rIb = make_rsrc(a.ib, a.idx_bytes);
    for (TileWalk w(a.BH * a.num_tiles); w.t < w.t_end; w.t += w.step) {
        const int bh = w.t / a.num_tiles, tile = w.t - bh * a.num_tiles;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        const rsrc_t rQ = make_rsrc(static_cast<const T*>(a.Q) + base, a.slab_bytes);
        const rsrc_t rG = make_rsrc(static_cast<const T*>(a.dout) + base, a.slab_bytes);
        const rsrc_t rS = make_rsrc(a.stat + (int64_t)bh * a.N, (uint32_t)a.N * 8u);
        const int s1 = a.tile_ptr[tile + 1];
        for (int s = a.tile_ptr[tile] + wave; s < s1; s += nwaves) {
            const int v = a.seg_row[s];
            const int e0 = a.seg_begin[s];
            const int e1 = min(e0 + kSeg, a.ptr[v + 1]);
            bwd_kv_segment<T, REL_LDS>(a, rel_s, rQ, rG, rS, rIa, rIb, bh, base, v, e0, e1, a.seg_part[s], lane);
        }
    }
}

// ---- backward: gradient of the relative-position table ---------------------------------
// d_rel[id] = scale * sum over (batch, head, token row u, edge e of u with id_e = id) of
// dS_e q_u.  Within a token row every edge has a different id, so for a block of R
// consecutive token rows this is the dense contraction  d_rel += DS^T Q  with
// DS[r][id] = dS of row r's edge with that id (0 if it has none) and Q the block's
// query rows.  A workgroup builds DS (from the (w,p) pairs the query side stored and
// delta) and Q in LDS, then every thread accumulates IPW outputs in registers:
// wavefront g owns ids [g*IPW, (g+1)*IPW) of the workgroup's chunk of 8*IPW ids,
// lane = feature.  Blocks are assigned statically and summed in a fixed
// order, so d_rel is run-to-run identical.  blockIdx.y selects the chunk of ids.
template <typename T, int IPW>
__global__ void __launch_bounds__(kThreads) rel_grad_kernel(const AttnArgs a) {
    constexpr int kDrelIdsPerWave = IPW, kDrelChunk = IPW * kWaves;
    extern __shared__ __align__(16) unsigned char smem[];
    const int R = a.drel_block;
    float* ds_s = reinterpret_cast<float*>(smem);           // [R][kDrelChunk]
    float* q_s = ds_s + (size_t)R * kDrelChunk;             // [R][kD]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int id0 = blockIdx.y * kDrelChunk;                // first id of this workgroup's chunk
    const int blocks_per_bh = a.n_tokens / R;
    const int total = a.BH * blocks_per_bh;

    float acc[kDrelIdsPerWave];
#pragma unroll
    for (int i = 0; i < kDrelIdsPerWave; ++i) acc[i] = 0.f;

    for (int blk = blockIdx.x; blk < total; blk += gridDim.x) {
        const int bh = blk / blocks_per_bh, row0 = (blk - bh * blocks_per_bh) * R;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        for (int i = threadIdx.x; i < R * kDrelChunk; i += blockDim.x) ds_s[i] = 0.f;
        {   // Q rows of the block: 8 lanes per row
            const T* Qb = static_cast<const T*>(a.Q) + base;
            for (int i = threadIdx.x; i < R * 8; i += blockDim.x) {
                const int r = i >> 3, c = (i & 7) * 8;
                float x[8];
                load8(Qb + (int64_t)(row0 + r) * a.sn + c, x);
#pragma unroll
                for (int j = 0; j < 8; ++j) q_s[r * kD + c + j] = x[j];
            }
        }
        __syncthreads();
        // scatter dS of every edge of the block's rows: one wavefront per row, lanes over edges
        const float2* wp_b = a.wp + (int64_t)bh * a.e_tok;
        for (int r = wave; r < R; r += kWaves) {
            const int u = row0 + r;
            const float delta = a.stat[(int64_t)bh * a.N + u].y;
            const int e1 = a.ptr[u + 1];
            for (int e = a.ptr[u] + lane; e < e1; e += 64) {
                const int id = a.ib[e] - id0;
                if (id >= 0 && id < kDrelChunk) {
                    const float2 x = wp_b[e];
                    ds_s[r * kDrelChunk + id] = x.x - delta * x.y;
                }
            }
        }
        __syncthreads();
        const float* dsw = ds_s + wave * kDrelIdsPerWave;
        for (int r = 0; r < R; ++r) {
            const float qv = q_s[r * kD + lane];
#pragma unroll
            for (int i = 0; i < kDrelIdsPerWave; i += 4) {
                const float4 d4 = *reinterpret_cast<const float4*>(dsw + r * kDrelChunk + i);  // same address in all lanes
                acc[i] += d4.x * qv;
                acc[i + 1] += d4.y * qv;
                acc[i + 2] += d4.z * qv;
                acc[i + 3] += d4.w * qv;
            }
        }
        __syncthreads();
    }
    // this workgroup's copy: [gridDim.x][drel_rows][kD]
    float* dst = a.drel_part + (int64_t)blockIdx.x * a.drel_rows * kD;
#pragma unroll
    for (int i = 0; i < kDrelIdsPerWave; ++i) {
        const int id = id0 + wave * kDrelIdsPerWave + i;
        if (id < a.drel_rows) dst[id * kD + lane] = acc[i] * a.scale;
    }
}


// The same contraction on the matrix cores, for bf16 tensors.  dS is fp32; it is
// split into two bf16 numbers (hi + lo carries 16 mantissa bits) so that the products
// with the bf16 query features are exact and accumulate in fp32.  Per block of 32
// token rows the workgroup keeps DS^T (hi and lo, [id][row]) and Q^T ([feature][row])
// in LDS, rows padded to 80 bytes so that the 16-byte operand reads of 8 lanes fall
// into 8 different bank quads.  v_mfma_f32_16x16x32_bf16: A[m][k] sits in lane
// m + 16*(k/8) (8 consecutive k per lane), B[k][n] in lane n + 16*(k/8), and
// C[m][n] in lane n + 16*(m/4), register m%4.  Here m = relative-position id,
// n = feature, k = row of the block.  Wavefront w owns the 16-id chunks w and w+8
// of the workgroup's 256 ids (blockIdx.y selects the 256).
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
constexpr int kRgRows = 32;     // token rows per block = K of one MFMA
constexpr int kRgStride = 40;   // bf16 elements per LDS row (32 + padding)
constexpr int kRgIds = 256;     // ids per workgroup

__global__ void __launch_bounds__(kThreads) rel_grad_mfma_kernel(const AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int id0 = blockIdx.y * kRgIds;
    const int nids = min(kRgIds, (a.drel_rows - id0 + 31) & ~31);   // ids of this workgroup, padded to 32
    bf16_t* ds_hi = reinterpret_cast<bf16_t*>(smem);                // [nids][kRgStride]
    bf16_t* ds_lo = ds_hi + nids * kRgStride;
    bf16_t* q_t = ds_lo + nids * kRgStride;                         // [kD][kRgStride]
    __shared__ int row_s[kRgRows + 1];
    __shared__ float delta_s[kRgRows];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, j = lane & 15;
    const int blocks_per_bh = (a.n_tokens + kRgRows - 1) / kRgRows;
    const int total = a.BH * blocks_per_bh;
    const int nchunks = nids >> 4;

    f32x4_t acc[2][4];
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int f = 0; f < 4; ++f) acc[c][f] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    for (int blk = blockIdx.x; blk < total; blk += gridDim.x) {
        const int bh = blk / blocks_per_bh, row0 = (blk - bh * blocks_per_bh) * kRgRows;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        // clear DS^T (hi and lo are adjacent)
        for (int i = threadIdx.x * 8; i < 2 * nids * kRgStride; i += blockDim.x * 8)
            *reinterpret_cast<uint4*>(ds_hi + i) = make_uint4(0u, 0u, 0u, 0u);
        // Q^T: thread -> (row, 8 features); rows past the sequence are zero
        for (int i = threadIdx.x; i < kRgRows * 8; i += blockDim.x) {
            const int r = i >> 3, c = (i & 7) * 8;
            uint4 w = make_uint4(0u, 0u, 0u, 0u);
            if (row0 + r < a.n_tokens)
                w = *reinterpret_cast<const uint4*>(static_cast<const bf16_t*>(a.Q) + base +
                                                    (int64_t)(row0 + r) * a.sn + c);
            const uint32_t x[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                q_t[(c + 2 * t) * kRgStride + r] = (bf16_t)(x[t] & 0xFFFFu);
                q_t[(c + 2 * t + 1) * kRgStride + r] = (bf16_t)(x[t] >> 16);
            }
        }
        // row pointers and delta of the block's rows
        if (threadIdx.x <= kRgRows) row_s[threadIdx.x] = a.ptr[min(row0 + (int)threadIdx.x, a.n_tokens)];
        if (threadIdx.x < kRgRows && row0 + (int)threadIdx.x < a.n_tokens)
            delta_s[threadIdx.x] = a.stat[(int64_t)bh * a.N + row0 + threadIdx.x].y;
        __syncthreads();
        // scatter dS = w - delta*p of every edge of the block's rows; the edges of the block
        // are contiguous in the CSR, one thread per edge, its row found by bisection
        const float2* wp_b = a.wp + (int64_t)bh * a.e_tok;
        const int e_end = row_s[kRgRows];
        for (int e = row_s[0] + threadIdx.x; e < e_end; e += blockDim.x) {
            const int id = a.ib[e] - id0;
            const float2 x = wp_b[e];
            int r = 0;
#pragma unroll
            for (int w = kRgRows / 2; w > 0; w >>= 1)
                if (row_s[r + w] <= e) r += w;
            if (id >= 0 && id < nids) {
                const float ds = x.x - delta_s[r] * x.y;
                const uint32_t hi = to_bf16_bits(ds);
                const uint32_t lo = to_bf16_bits(ds - __uint_as_float(hi << 16));
                ds_hi[id * kRgStride + r] = (bf16_t)hi;
                ds_lo[id * kRgStride + r] = (bf16_t)lo;
            }
        }
        __syncthreads();
        bf16x8_t qb[4];
#pragma unroll
        for (int f = 0; f < 4; ++f)
            qb[f] = *reinterpret_cast<const bf16x8_t*>(q_t + (16 * f + j) * kRgStride + 8 * g);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int chunk = wave + kWaves * c;
            if (chunk < nchunks) {
                const int off = (16 * chunk + j) * kRgStride + 8 * g;
                const bf16x8_t ah = *reinterpret_cast<const bf16x8_t*>(ds_hi + off);
                const bf16x8_t al = *reinterpret_cast<const bf16x8_t*>(ds_lo + off);
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    acc[c][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, qb[f], acc[c][f], 0, 0, 0);
                    acc[c][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, qb[f], acc[c][f], 0, 0, 0);
                }
            }
        }
        __syncthreads();
    }
    // this workgroup's copy: [gridDim.x][drel_rows][kD]
    float* dst = a.drel_part + (int64_t)blockIdx.x * a.drel_rows * kD;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int chunk = wave + kWaves * c;
        if (chunk < nchunks) {
#pragma unroll
            for (int f = 0; f < 4; ++f)
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    const int id = id0 + 16 * chunk + 4 * g + m;
                    if (id < a.drel_rows) dst[id * kD + 16 * f + j] = acc[c][f][m] * a.scale;
                }
        }
    }
}


// ---- forward over dense tiles of token rows, on the matrix cores (bf16) ---------------
// A wavefront computes 16 consecutive token rows against the union U of their key
// nodes (tile metadata of the graph).  Consecutive tokens share almost all coarse
// neighbours, so the 16 x |U| score tile is more than half full and the products
// Q K^T and P V are real dense contractions:
//   S^T chunk [16 columns x 16 tokens] = K_chunk (A, rows straight from memory) x Q^T (B),
//   bias^T [ids x 16 tokens]            = Rel (A, from LDS)                    x Q^T (B),
//   out [16 tokens x 64]               += P (A) x V_chunk (B, transposed through LDS).
// With v_mfma_f32_16x16x32_bf16 the result C[m][n] lives in lane n + 16*(m/4),
// register m%4 -- for S^T that is token n = lane%16 and columns 4*(lane/16)..+3, which
// is exactly the A-operand layout P needs for the second product (A[m][k] in lane
// m + 16*(k/8)) once the columns of two chunks are interleaved as k = 8g+i:
// i<4 -> chunk 2c, column 4g+i; i>=4 -> chunk 2c+1, column 4g+i-4.  The feature
// dimension of the first product is permuted the same way in both operands (lane
// group g owns features 16g..16g+15), which leaves the dot products unchanged.
// Softmax runs online over groups of 8 chunks; masked and padding columns carry
// the id -1 in the tile map.
constexpr int kTileThreads = 256;
constexpr int kTileWaves = kTileThreads / 64;
constexpr int kRelStride = 72;   // bf16 per LDS row of the compact table (64 + padding: 144 B)
constexpr int kVStride = 68;     // bf16 per LDS row of a staged V row (136 B)
constexpr int kRowStride = 72;   // bf16 per LDS row where rows are written and read 16 bytes at a time (144 B)

struct TileArgs {
    const bf16_t *Q, *K, *V, *rel;
    bf16_t* out;
    float* lse;
    int64_t sb, sh, sn;
    int32_t BH, H, N;
    float scale;
    const int32_t *chunk_ptr, *cols, *cid_to_id;
    const int16_t* map;
    int32_t num_tiles, num_chunks, num_cids, cid_pad, bias_stride;
    int32_t row_bytes;
    uint32_t slab_bytes;
    // backward, query side
    const bf16_t* dout;
    const float* lse_r;
    float* dQ;
    float2 *stat, *wp;
};

__device__ __forceinline__ void wave_lds_sync() {  // order LDS traffic between the lanes of one wavefront
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}
// two floats -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32)
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    typedef __bf16 bf16x2v_t __attribute__((ext_vector_type(2)));
    const bf16x2v_t v = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, v);
}
// two floats -> packed bf16 pair of their leading parts and packed bf16 pair of the remainders
__device__ __forceinline__ void split_pack(float x, float y, uint32_t& hi, uint32_t& lo) {
    hi = pack_bf16(x, y);
    lo = pack_bf16(x - __uint_as_float(hi << 16), y - __uint_as_float(hi & 0xFFFF0000u));
}
// B operand of v_mfma_f32_16x16x32_bf16 out of rows staged in LDS: `rows` points at 32
// staged rows (two chunks of 16) of `stride` bf16 each.  Lane (g, j) receives feature
// 16f + j of rows 4g..4g+3 of the first chunk and of the second chunk -- the k order in
// which the score tiles' C layout serves as the A operand.  ds_read_b64_tr_b16 reads,
// per 16-lane group, a 4-row x 16-column block (lane 4r + c addresses columns 4c..4c+3
// of row r) and hands lane i column i of the 4 rows.
typedef short s16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8_t lds_transposed_b(const bf16_t* rows, int stride, int f, int g, int j) {
    typedef __attribute__((address_space(3))) s16x4_t* lds_ptr_t;
    const bf16_t* p = rows + (4 * g + (j >> 2)) * stride + 16 * f + 4 * (j & 3);
    const s16x4_t x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)p);
    const s16x4_t y = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 16 * stride));
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    const s16x8_t xy = {x[0], x[1], x[2], x[3], y[0], y[1], y[2], y[3]};
    return __builtin_bit_cast(bf16x8_t, xy);
}

// Position of a wavefront in its sequence of (token tile, pair of chunks); wave-uniform.
struct TileCursor {
    int t, pair, npairs, cp0, bh, tile;
    bool valid;
};

// REL_LDS: the compact relative-position table is staged in LDS; otherwise (large tables) its rows
// are read from memory when a tile forms its bias table.
template <bool REL_LDS>
__global__ void __launch_bounds__(kTileThreads, 2) fwd_tile_kernel(const TileArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* rel_s = reinterpret_cast<bf16_t*>(smem);                                   // [cid_pad][kRelStride]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, j = lane & 15;
    const int r8 = lane >> 3, piece = lane & 7;   // coalesced row fetches: row of the instruction, 16-byte piece
    const size_t rel_bytes = REL_LDS ? (size_t)a.cid_pad * kRelStride * sizeof(bf16_t) : 0;
    float* bias_s = reinterpret_cast<float*>(smem + rel_bytes) +
                    (size_t)wave * 16 * a.bias_stride;                                  // [16 tokens][bias_stride]
    bf16_t* k_s = reinterpret_cast<bf16_t*>(smem + rel_bytes + (size_t)kTileWaves * 16 * a.bias_stride * sizeof(float)) +
                  (size_t)wave * 64 * kRowStride;                                       // [32 columns][kRowStride]: K rows
    bf16_t* v_s = k_s + 32 * kRowStride;                                                // the same for V rows
    // compact relative-position table, zero rows as padding
    if (REL_LDS) {
        for (int i = threadIdx.x; i < a.cid_pad * 8; i += blockDim.x) {
            const int cid = i >> 3, c8 = (i & 7) * 8;
            uint4 w = make_uint4(0u, 0u, 0u, 0u);
            if (cid < a.num_cids) w = *reinterpret_cast<const uint4*>(a.rel + (int64_t)a.cid_to_id[cid] * kD + c8);
            *reinterpret_cast<uint4*>(rel_s + cid * kRelStride + c8) = w;
        }
    }
    __syncthreads();

    const float qscale = a.scale * kLog2e;
    const rsrc_t rC = make_rsrc(a.cols, (uint32_t)a.num_chunks * 64u);   // [chunks][16] int32
    const rsrc_t rM = make_rsrc(a.map, (uint32_t)a.num_chunks * 512u);   // [chunks][16][16] int16
    const int groups_per_bh = (a.num_tiles + kTileWaves - 1) / kTileWaves;
    const TileWalk w(a.BH * groups_per_bh);

    // One sequence of pairs of chunks through the wavefront's tiles, software pipelined as in
    // bwd_q_tile_kernel: `cc` is computed, the rows of `cr` and the ids of `ci` are in flight.
    auto enter_tile = [&](TileCursor& c) {
        c.valid = false;
        c.pair = 0;
        c.npairs = 1;
        for (; c.t < w.t_end; c.t += w.step) {
            c.bh = c.t / groups_per_bh;
            c.tile = (c.t - c.bh * groups_per_bh) * kTileWaves + wave;
            if (c.tile < a.num_tiles) {
                c.cp0 = a.chunk_ptr[c.tile];
                c.npairs = (a.chunk_ptr[c.tile + 1] - c.cp0) >> 1;
                c.valid = true;
                return;
            }
        }
    };
    auto advance = [&](TileCursor& c) {
        if (c.valid && ++c.pair == c.npairs) {
            c.t += w.step;
            enter_tile(c);
        }
    };
    int node_n[2][2];
    uint2 mp_n[2];
    auto load_idx = [&](const TileCursor& c) {
#pragma unroll
        for (int ci = 0; ci < 2; ++ci) {
            const int at = (c.cp0 + 2 * c.pair + ci) * 16;
            node_n[ci][0] = buf_i32(rC, (at + r8) * 4);
            node_n[ci][1] = buf_i32(rC, (at + 8 + r8) * 4);
            const u32x2 m2 = __builtin_amdgcn_raw_buffer_load_b64(rM, (at + j) * 32 + 8 * g, 0, 0);
            mp_n[ci] = make_uint2(m2.x, m2.y);
        }
    };
    Row<bf16_t> kr[2][2], vr[2][2];   // [chunk][half of its rows]: this lane's 16-byte piece
    bf16x8_t qn0, qn1;                // Q^T operand of the tile whose first pair is in flight
    auto request_rows = [&](const TileCursor& c) {
        const int64_t base = (int64_t)(c.bh / a.H) * a.sb + (int64_t)(c.bh % a.H) * a.sh;
        const rsrc_t rK = make_rsrc(a.K + base, a.slab_bytes), rV = make_rsrc(a.V + base, a.slab_bytes);
#pragma unroll
        for (int ci = 0; ci < 2; ++ci)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int off = (int)__umul24(node_n[ci][h], a.row_bytes) + piece * 16;
                buf_row(rK, off, kr[ci][h]);
                buf_row(rV, off, vr[ci][h]);
            }
        if (c.pair == 0) {   // token j, features 16g..16g+15
            const int64_t at = base + (int64_t)(c.tile * 16 + j) * a.sn + 16 * g;
            qn0 = *reinterpret_cast<const bf16x8_t*>(a.Q + at);
            qn1 = *reinterpret_cast<const bf16x8_t*>(a.Q + at + 8);
        }
    };

    TileCursor cc, cr, ci;
    cc.t = w.t;
    enter_tile(cc);
    if (!cc.valid) return;
    load_idx(cc);
    request_rows(cc);
    uint2 mp[2] = {mp_n[0], mp_n[1]};
    cr = cc;
    advance(cr);
    if (cr.valid) load_idx(cr);
    ci = cr;
    advance(ci);

    bf16x8_t qb0, qb1;
    float m_run = kNegBig, l_part = 0.f;
    f32x4_t o[4];

    while (cc.valid) {
        if (cc.pair == 0) {   // a new tile: its Q rows arrived with the rows of this pair
            qb0 = qn0;
            qb1 = qn1;
            m_run = kNegBig;
            l_part = 0.f;
#pragma unroll
            for (int f = 0; f < 4; ++f) o[f] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            // bias^T = Rel x Q^T, kept in LDS as [token][compact id]
            for (int c = 0; c < a.cid_pad; c += 16) {
                bf16x8_t r0, r1;
                if (REL_LDS) {
                    const bf16_t* rrow = rel_s + (c + j) * kRelStride + 16 * g;
                    r0 = *reinterpret_cast<const bf16x8_t*>(rrow);
                    r1 = *reinterpret_cast<const bf16x8_t*>(rrow + 8);
                } else {   // padding ids repeat the last real one; no column carries them
                    const bf16_t* rrow = a.rel + (int64_t)a.cid_to_id[min(c + j, a.num_cids - 1)] * kD + 16 * g;
                    r0 = *reinterpret_cast<const bf16x8_t*>(rrow);
                    r1 = *reinterpret_cast<const bf16x8_t*>(rrow + 8);
                }
                f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r0, qb0, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r1, qb1, acc, 0, 0, 0);
                *reinterpret_cast<f32x4_t*>(bias_s + j * a.bias_stride + c + 4 * g) = acc;
            }
        }
        wave_lds_sync();  // the previous pair's reads of k_s, v_s (and the previous tile's of bias_s) are done
#pragma unroll
        for (int ci2 = 0; ci2 < 2; ++ci2)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int row = 16 * ci2 + 8 * h + r8;
                *reinterpret_cast<uint4*>(k_s + row * kRowStride + piece * 8) = kr[ci2][h].w;
                *reinterpret_cast<uint4*>(v_s + row * kRowStride + piece * 8) = vr[ci2][h].w;
            }
        __builtin_amdgcn_sched_barrier(0);
        // the row registers are free: request the next pair's rows, then the ids of the pair after it
        const uint2 mpc[2] = {mp[0], mp[1]};
        if (cr.valid) {
            request_rows(cr);
            mp[0] = mp_n[0];
            mp[1] = mp_n[1];
        }
        if (ci.valid) load_idx(ci);
        __builtin_amdgcn_sched_barrier(0);
        wave_lds_sync();

        int cid[2][4];
        float bv[2][4];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            cid[c][0] = (int)(short)(mpc[c].x & 0xFFFFu);
            cid[c][1] = (int)(short)(mpc[c].x >> 16);
            cid[c][2] = (int)(short)(mpc[c].y & 0xFFFFu);
            cid[c][3] = (int)(short)(mpc[c].y >> 16);
#pragma unroll
            for (int r = 0; r < 4; ++r) bv[c][r] = bias_s[j * a.bias_stride + max(cid[c][r], 0)];
        }
        f32x4_t s4[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const bf16_t* krow = k_s + (16 * c + j) * kRowStride + 16 * g;
            s4[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            s4[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(krow), qb0, s4[c], 0, 0, 0);
            s4[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(krow + 8), qb1, s4[c], 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) asm volatile("" : "+v"(bv[c][r]));  // reads stay out of branches on the mask
        // online softmax over the pair's 32 columns
        float sc[2][4], gm = kNegBig;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                sc[c][r] = cid[c][r] >= 0 ? (s4[c][r] + bv[c][r]) * qscale : kNegBig;
                gm = fmaxf(gm, sc[c][r]);
            }
        gm = fmaxf(gm, __shfl_xor(gm, 16));
        gm = fmaxf(gm, __shfl_xor(gm, 32));
        const float mn = fmaxf(m_run, gm);
        const float corr = fast_exp2(m_run - mn);
        m_run = mn;
        float psum = 0.f;
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = sc[c][r] > 0.5f * kNegBig ? fast_exp2(sc[c][r] - mn) : 0.f;
                sc[c][r] = p;
                psum += p;
            }
        l_part = l_part * corr + psum;
        // the accumulators hold tokens 4g..4g+3: fetch their correction factors
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float cr4 = __shfl(corr, 4 * g + r);
#pragma unroll
            for (int f = 0; f < 4; ++f) o[f][r] *= cr4;
        }
        u32x4 pa;
        pa.x = pack_bf16(sc[0][0], sc[0][1]);
        pa.y = pack_bf16(sc[0][2], sc[0][3]);
        pa.z = pack_bf16(sc[1][0], sc[1][1]);
        pa.w = pack_bf16(sc[1][2], sc[1][3]);
        const bf16x8_t pA = __builtin_bit_cast(bf16x8_t, pa);
#pragma unroll
        for (int f = 0; f < 4; ++f)
            o[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pA, lds_transposed_b(v_s, kRowStride, f, g, j), o[f], 0, 0, 0);

        if (cc.pair == cc.npairs - 1) {   // the tile is complete
            const int64_t base = (int64_t)(cc.bh / a.H) * a.sb + (int64_t)(cc.bh % a.H) * a.sh;
            const int t0 = cc.tile * 16;
            // row sums: token j is spread over the 4 lane groups
            float l = l_part + __shfl_xor(l_part, 16);
            l += __shfl_xor(l, 32);
            if (g == 0) a.lse[(int64_t)cc.bh * a.N + t0 + j] = (m_run + fast_log2(l)) * kLn2;
            bf16_t* orow = a.out + base + (int64_t)t0 * a.sn + j;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float inv = 1.f / __shfl(l, 4 * g + r);
#pragma unroll
                for (int f = 0; f < 4; ++f)
                    orow[(int64_t)(4 * g + r) * a.sn + 16 * f] = (bf16_t)to_bf16_bits(o[f][r] * inv);
            }
        }
        cc = cr;
        cr = ci;
        advance(ci);
    }
}


// ---- backward, query side, over the same dense tiles (bf16) --------------------------
// Per tile: S^T and dP^T = V_chunk x dO^T on the matrix cores, p = exp2(s - lse),
// w = p dP, delta = sum w; then, with K staged in LDS as the B operand,
//   dQ_K = scale * (W K_U - delta * P K_U)       (the key part of dQ; lse is known, so
// no online softmax and no second pass).  (w, p) of every edge goes to `wp` in CSR
// order for the d_rel kernel, which also adds the relative-position part of dQ.
// REL_LDS: the compact relative-position table is staged in LDS; otherwise (large tables) its rows
// are read from memory when a tile forms its bias table.
template <bool REL_LDS>
__global__ void __launch_bounds__(kTileThreads, 2) bwd_q_tile_kernel(const TileArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    bf16_t* rel_s = reinterpret_cast<bf16_t*>(smem);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, j = lane & 15;
    const int r8 = lane >> 3, piece = lane & 7;   // coalesced row fetches: row of the instruction, 16-byte piece
    const size_t rel_bytes = REL_LDS ? (size_t)a.cid_pad * kRelStride * sizeof(bf16_t) : 0;
    float* bias_s = reinterpret_cast<float*>(smem + rel_bytes) +
                    (size_t)wave * 16 * a.bias_stride;
    bf16_t* k_s = reinterpret_cast<bf16_t*>(smem + rel_bytes + (size_t)kTileWaves * 16 * a.bias_stride * sizeof(float)) +
                  (size_t)wave * 64 * kRowStride;                      // [32 columns][kRowStride]: K rows
    bf16_t* v_s = k_s + 32 * kRowStride;                                // the same for V rows
    if (REL_LDS) {
        for (int i = threadIdx.x; i < a.cid_pad * 8; i += blockDim.x) {
            const int cid = i >> 3, c8 = (i & 7) * 8;
            uint4 w = make_uint4(0u, 0u, 0u, 0u);
            if (cid < a.num_cids) w = *reinterpret_cast<const uint4*>(a.rel + (int64_t)a.cid_to_id[cid] * kD + c8);
            *reinterpret_cast<uint4*>(rel_s + cid * kRelStride + c8) = w;
        }
    }
    __syncthreads();

    const float qscale = a.scale * kLog2e;
    const rsrc_t rC = make_rsrc(a.cols, (uint32_t)a.num_chunks * 64u);
    const rsrc_t rM = make_rsrc(a.map, (uint32_t)a.num_chunks * 512u);
    const int groups_per_bh = (a.num_tiles + kTileWaves - 1) / kTileWaves;
    const TileWalk w(a.BH * groups_per_bh);

    // The wavefront's work is one sequence of pairs of chunks running through its tiles.
    // Three positions move along it: `cc` is computed, the rows of `cr` (one pair ahead) are
    // in flight, the column ids and map words of `ci` (two pairs ahead) are in flight.
    auto enter_tile = [&](TileCursor& c) {
        c.valid = false;
        c.pair = 0;
        c.npairs = 1;
        for (; c.t < w.t_end; c.t += w.step) {
            c.bh = c.t / groups_per_bh;
            c.tile = (c.t - c.bh * groups_per_bh) * kTileWaves + wave;
            if (c.tile < a.num_tiles) {
                c.cp0 = a.chunk_ptr[c.tile];
                c.npairs = (a.chunk_ptr[c.tile + 1] - c.cp0) >> 1;
                c.valid = true;
                return;
            }
        }
    };
    auto advance = [&](TileCursor& c) {
        if (c.valid && ++c.pair == c.npairs) {
            c.t += w.step;
            enter_tile(c);
        }
    };
    int node_n[2][2];
    uint2 mp_n[2];
    auto load_idx = [&](const TileCursor& c) {
#pragma unroll
        for (int ci = 0; ci < 2; ++ci) {
            const int at = (c.cp0 + 2 * c.pair + ci) * 16;
            node_n[ci][0] = buf_i32(rC, (at + r8) * 4);
            node_n[ci][1] = buf_i32(rC, (at + 8 + r8) * 4);
            const u32x2 m2 = __builtin_amdgcn_raw_buffer_load_b64(rM, (at + j) * 32 + 8 * g, 0, 0);
            mp_n[ci] = make_uint2(m2.x, m2.y);
        }
    };
    Row<bf16_t> kr[2][2], vr[2][2];   // [chunk][half of its rows]: this lane's 16-byte piece
    bf16x8_t qn0, qn1, gn0, gn1;      // operands of the tile whose first pair is in flight
    float lse_n = 0.f;
    auto request_rows = [&](const TileCursor& c) {
        const int64_t base = (int64_t)(c.bh / a.H) * a.sb + (int64_t)(c.bh % a.H) * a.sh;
        const rsrc_t rK = make_rsrc(a.K + base, a.slab_bytes), rV = make_rsrc(a.V + base, a.slab_bytes);
#pragma unroll
        for (int ci = 0; ci < 2; ++ci)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int off = (int)__umul24(node_n[ci][h], a.row_bytes) + piece * 16;
                buf_row(rK, off, kr[ci][h]);
                buf_row(rV, off, vr[ci][h]);
            }
        if (c.pair == 0) {   // the tile's own rows: Q^T and dO^T operands (token j, features 16g..16g+15)
            const int64_t at = base + (int64_t)(c.tile * 16 + j) * a.sn + 16 * g;
            qn0 = *reinterpret_cast<const bf16x8_t*>(a.Q + at);
            qn1 = *reinterpret_cast<const bf16x8_t*>(a.Q + at + 8);
            gn0 = *reinterpret_cast<const bf16x8_t*>(a.dout + at);
            gn1 = *reinterpret_cast<const bf16x8_t*>(a.dout + at + 8);
            lse_n = a.lse_r[(int64_t)c.bh * a.N + c.tile * 16 + j];
        }
    };

    TileCursor cc, cr, ci;
    cc.t = w.t;
    enter_tile(cc);
    if (!cc.valid) return;
    load_idx(cc);
    request_rows(cc);
    uint2 mp[2] = {mp_n[0], mp_n[1]};
    cr = cc;
    advance(cr);
    if (cr.valid) load_idx(cr);
    ci = cr;
    advance(ci);

    bf16x8_t qb0, qb1, gb0, gb1;
    float lse2 = 0.f, dl_part = 0.f;
    float2* wp_t = a.wp;   // this (batch, head)'s pairs, in tile order: [chunk][token][16 columns]
    f32x4_t ow[4], op[4];

    while (cc.valid) {
        if (cc.pair == 0) {   // a new tile: its operands arrived with the rows of this pair
            qb0 = qn0; qb1 = qn1; gb0 = gn0; gb1 = gn1;
            lse2 = lse_n * kLog2e;
            wp_t = a.wp + (int64_t)cc.bh * a.num_chunks * 256;
            dl_part = 0.f;
#pragma unroll
            for (int f = 0; f < 4; ++f) ow[f] = op[f] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            // bias^T = Rel x Q^T, kept in LDS as [token][compact id]
            for (int c = 0; c < a.cid_pad; c += 16) {
                bf16x8_t r0, r1;
                if (REL_LDS) {
                    const bf16_t* rrow = rel_s + (c + j) * kRelStride + 16 * g;
                    r0 = *reinterpret_cast<const bf16x8_t*>(rrow);
                    r1 = *reinterpret_cast<const bf16x8_t*>(rrow + 8);
                } else {   // padding ids repeat the last real one; no column carries them
                    const bf16_t* rrow = a.rel + (int64_t)a.cid_to_id[min(c + j, a.num_cids - 1)] * kD + 16 * g;
                    r0 = *reinterpret_cast<const bf16x8_t*>(rrow);
                    r1 = *reinterpret_cast<const bf16x8_t*>(rrow + 8);
                }
                f32x4_t acc = {0.f, 0.f, 0.f, 0.f};
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r0, qb0, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(r1, qb1, acc, 0, 0, 0);
                *reinterpret_cast<f32x4_t*>(bias_s + j * a.bias_stride + c + 4 * g) = acc;
            }
        }
        wave_lds_sync();  // the previous pair's reads of k_s, v_s (and the previous tile's of bias_s) are done
#pragma unroll
        for (int ci2 = 0; ci2 < 2; ++ci2)
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int row = 16 * ci2 + 8 * h + r8;
                *reinterpret_cast<uint4*>(k_s + row * kRowStride + piece * 8) = kr[ci2][h].w;
                *reinterpret_cast<uint4*>(v_s + row * kRowStride + piece * 8) = vr[ci2][h].w;
            }
        __builtin_amdgcn_sched_barrier(0);
        // the row registers are free: request the next pair's rows, then the ids of the pair after it
        const uint2 mpc[2] = {mp[0], mp[1]};
        if (cr.valid) {
            request_rows(cr);
            mp[0] = mp_n[0]; mp[1] = mp_n[1];
        }
        if (ci.valid) load_idx(ci);
        __builtin_amdgcn_sched_barrier(0);
        wave_lds_sync();

        // scores and dP of the pair, the relative-position terms read unconditionally
        int cid[2][4];
        float bv[2][4];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            cid[c][0] = (int)(short)(mpc[c].x & 0xFFFFu);
            cid[c][1] = (int)(short)(mpc[c].x >> 16);
            cid[c][2] = (int)(short)(mpc[c].y & 0xFFFFu);
            cid[c][3] = (int)(short)(mpc[c].y >> 16);
#pragma unroll
            for (int r = 0; r < 4; ++r) bv[c][r] = bias_s[j * a.bias_stride + max(cid[c][r], 0)];
        }
        f32x4_t s4[2], d4[2];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const bf16_t* krow = k_s + (16 * c + j) * kRowStride + 16 * g;
            const bf16_t* vrow = v_s + (16 * c + j) * kRowStride + 16 * g;
            s4[c] = d4[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            s4[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(krow), qb0, s4[c], 0, 0, 0);
            s4[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(krow + 8), qb1, s4[c], 0, 0, 0);
            d4[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(vrow), gb0, d4[c], 0, 0, 0);
            d4[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(*reinterpret_cast<const bf16x8_t*>(vrow + 8), gb1, d4[c], 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
            for (int r = 0; r < 4; ++r) asm volatile("" : "+v"(bv[c][r]));  // reads stay out of branches on the mask
        float pw[2][4], pp[2][4];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float p = cid[c][r] >= 0 ? fast_exp2((s4[c][r] + bv[c][r]) * qscale - lse2) : 0.f;
                const float wgt = p * d4[c][r];
                dl_part += wgt;
                pw[c][r] = wgt;
                pp[c][r] = p;
            }
            // (w, p) of this lane's 4 columns: 32 contiguous bytes, a chunk is 2 KB contiguous
            float4* dst = reinterpret_cast<float4*>(wp_t + ((int64_t)(cc.cp0 + 2 * cc.pair + c) * 16 + j) * 16 + 4 * g);
            dst[0] = make_float4(pw[c][0], pp[c][0], pw[c][1], pp[c][1]);
            dst[1] = make_float4(pw[c][2], pp[c][2], pw[c][3], pp[c][3]);
        }
        // W and P as A operands, each split into bf16 hi + lo: A - delta*Bv cancels when a
        // row's softmax is peaked, so the two products need more than 8 mantissa bits
        uint32_t whi[4], wlo[4], phi[4], plo[4];
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            split_pack(pw[c][0], pw[c][1], whi[2 * c], wlo[2 * c]);
            split_pack(pw[c][2], pw[c][3], whi[2 * c + 1], wlo[2 * c + 1]);
            split_pack(pp[c][0], pp[c][1], phi[2 * c], plo[2 * c]);
            split_pack(pp[c][2], pp[c][3], phi[2 * c + 1], plo[2 * c + 1]);
        }
        const u32x4 wh = {whi[0], whi[1], whi[2], whi[3]}, wl = {wlo[0], wlo[1], wlo[2], wlo[3]};
        const u32x4 ph = {phi[0], phi[1], phi[2], phi[3]}, pl = {plo[0], plo[1], plo[2], plo[3]};
        const bf16x8_t wH = __builtin_bit_cast(bf16x8_t, wh), wL = __builtin_bit_cast(bf16x8_t, wl);
        const bf16x8_t pH = __builtin_bit_cast(bf16x8_t, ph), pL = __builtin_bit_cast(bf16x8_t, pl);
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            const bf16x8_t kB = lds_transposed_b(k_s, kRowStride, f, g, j);
            ow[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wH, kB, ow[f], 0, 0, 0);
            ow[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wL, kB, ow[f], 0, 0, 0);
            op[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pH, kB, op[f], 0, 0, 0);
            op[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pL, kB, op[f], 0, 0, 0);
        }
        if (cc.pair == cc.npairs - 1) {   // the tile is complete
            const int64_t base = (int64_t)(cc.bh / a.H) * a.sb + (int64_t)(cc.bh % a.H) * a.sh;
            const int t0 = cc.tile * 16;
            float delta = dl_part + __shfl_xor(dl_part, 16);
            delta += __shfl_xor(delta, 32);
            if (g == 0) a.stat[(int64_t)cc.bh * a.N + t0 + j] = make_float2(lse2, delta);
            float* qrow_out = a.dQ + base + (int64_t)t0 * a.sn + j;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float dr = __shfl(delta, 4 * g + r);
#pragma unroll
                for (int f = 0; f < 4; ++f)
                    qrow_out[(int64_t)(4 * g + r) * a.sn + 16 * f] = a.scale * (ow[f][r] - dr * op[f][r]);
            }
        }
        cc = cr;
        cr = ci;
        advance(ci);
    }
}


// d_rel and the relative-position part of dQ over the token tiles' compact ids (bf16
// tensors, at most 256 ids in use).  Per block of 32 token rows the workgroup builds
// DS^T[id][row] (hi and lo halves) in LDS from the (w, p) pairs of the query side: every
// edge of a token row carries a 16-bit code = compact id * 32 + row % 32 (tile metadata),
// so an edge needs no search for its row and no lookup of its id.  Q rows are staged
// row-major and enter the products through transposing LDS reads:
//   d_rel[id][f] += DS^T (A, 16-byte rows) x Q (B, transposed read),
//   dQ[row][f]   += scale * DS (A, transposed read of DS^T) x Rel (B, transposed read).
// Wavefront w owns id chunks w and w + 8; its accumulators live across the blocks the
// workgroup walks and are written once, as this workgroup's copy, in compact-id order.
struct RelGradArgs {
    const bf16_t *Q, *rel;
    float* dQ;
    const float2 *stat, *wp;
    float* drel_part;
    const int32_t *chunk_ptr, *cid_to_id;
    const int16_t* map;
    int64_t sb, sh, sn;
    int32_t BH, H, N, n, num_tiles, num_chunks, num_cids, nids;   // nids = ids padded to 32
    float scale;
};
// 8 consecutive k of the operand row/column `col0 + j`: two transposing reads of 4 rows each
__device__ __forceinline__ bf16x8_t lds_tr8(const bf16_t* base, int stride, int row0, int col0, int j) {
    typedef __attribute__((address_space(3))) s16x4_t* lds_ptr_t;
    const bf16_t* p = base + (row0 + (j >> 2)) * stride + col0 + 4 * (j & 3);
    const s16x4_t x = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)p);
    const s16x4_t y = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(p + 4 * stride));
    typedef short s16x8_t __attribute__((ext_vector_type(8)));
    const s16x8_t xy = {x[0], x[1], x[2], x[3], y[0], y[1], y[2], y[3]};
    return __builtin_bit_cast(bf16x8_t, xy);
}

constexpr int kRgPrefetch = 8;   // tile slots per thread fetched one block ahead (512 threads: 16 chunks)
constexpr int kRgTileMaxIds = 512;
// CPW: 16-id chunks per wavefront (2: up to 256 ids, 4: up to 512)
template <int CPW>
__global__ void __launch_bounds__(kThreads) rel_grad_tile_kernel(const RelGradArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int nids = a.nids;
    bf16_t* ds_hi = reinterpret_cast<bf16_t*>(smem);                 // [nids][kRgStride]: DS^T, rows of the block along a line
    bf16_t* ds_lo = ds_hi + nids * kRgStride;
    bf16_t* q_s = ds_lo + nids * kRgStride;                          // [32 rows][kRowStride]
    bf16_t* rel_s = q_s + kRgRows * kRowStride;                      // [nids][kRelStride], compact order
    __shared__ float delta_s[kRgRows];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, j = lane & 15;
    for (int i = threadIdx.x; i < nids * 8; i += blockDim.x) {
        const int cid = i >> 3, c8 = (i & 7) * 8;
        uint4 w = make_uint4(0u, 0u, 0u, 0u);
        if (cid < a.num_cids) w = *reinterpret_cast<const uint4*>(a.rel + (int64_t)a.cid_to_id[cid] * kD + c8);
        *reinterpret_cast<uint4*>(rel_s + cid * kRelStride + c8) = w;
    }
    const int blocks_per_bh = (a.n + kRgRows - 1) / kRgRows;
    const int total = a.BH * blocks_per_bh;
    const int nchunks = nids >> 4;
    const rsrc_t rMap = make_rsrc(a.map, (uint32_t)a.num_chunks * 512u);

    f32x4_t acc[CPW][4];
#pragma unroll
    for (int c = 0; c < CPW; ++c)
#pragma unroll
        for (int f = 0; f < 4; ++f) acc[c][f] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // What a block needs from memory is requested one block ahead, so that it arrives while
    // the current block's products run: the thread's piece of a Q row (or a delta), and its
    // first kRgPrefetch tile slots (compact id from the tile map, (w, p) pair).  The slots of
    // the block's two token tiles are contiguous: [chunk][token][16 columns].
    uint4 qpiece = make_uint4(0u, 0u, 0u, 0u);
    float dl_own = 0.f;
    int code[kRgPrefetch];
    float2 wpv[kRgPrefetch];
    int s_begin = 0, s_mid = 0, s_end = 0;   // first slot of the block, of its second tile, and the end
    auto prefetch = [&](int blk) {
        const int bh = blk / blocks_per_bh, b2 = 2 * (blk - bh * blocks_per_bh), row0 = 16 * b2;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        s_begin = a.chunk_ptr[b2] * 256;
        s_mid = a.chunk_ptr[min(b2 + 1, a.num_tiles)] * 256;
        s_end = a.chunk_ptr[min(b2 + 2, a.num_tiles)] * 256;
        qpiece = make_uint4(0u, 0u, 0u, 0u);
        if (threadIdx.x < kRgRows * 8) {
            const int r = threadIdx.x >> 3, c = (threadIdx.x & 7) * 8;
            if (row0 + r < a.n) qpiece = *reinterpret_cast<const uint4*>(a.Q + base + (int64_t)(row0 + r) * a.sn + c);
        } else if (threadIdx.x < kRgRows * 8 + kRgRows) {
            const int r = threadIdx.x - kRgRows * 8;
            dl_own = row0 + r < a.n ? a.stat[(int64_t)bh * a.N + row0 + r].y : 0.f;
        }
        const rsrc_t rWp = make_rsrc(a.wp + (int64_t)bh * a.num_chunks * 256, (uint32_t)a.num_chunks * 2048u);
#pragma unroll
        for (int k = 0; k < kRgPrefetch; ++k) {
            const int sl = s_begin + (int)threadIdx.x + k * kThreads;
            const uint32_t off = sl < s_end ? (uint32_t)sl : 0x1FFFFFFFu;   // past the block: an offset outside the buffers
            code[k] = (int)(short)__builtin_amdgcn_raw_buffer_load_b16(rMap, (int)(off * 2u), 0, 0);
            wpv[k] = buf_f2(rWp, (int)(off * 8u));
        }
    };
    if ((int)blockIdx.x < total) prefetch(blockIdx.x);

    for (int blk = blockIdx.x; blk < total; blk += gridDim.x) {
        const int bh = blk / blocks_per_bh, row0 = (blk - bh * blocks_per_bh) * kRgRows;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        // clear DS^T (hi and lo are adjacent), stage the block's Q rows and deltas
        for (int i = threadIdx.x * 8; i < 2 * nids * kRgStride; i += blockDim.x * 8)
            *reinterpret_cast<uint4*>(ds_hi + i) = make_uint4(0u, 0u, 0u, 0u);
        if (threadIdx.x < kRgRows * 8)
            *reinterpret_cast<uint4*>(q_s + (threadIdx.x >> 3) * kRowStride + (threadIdx.x & 7) * 8) = qpiece;
        else if (threadIdx.x < kRgRows * 8 + kRgRows)
            delta_s[threadIdx.x - kRgRows * 8] = dl_own;
        __syncthreads();
        // scatter dS = w - delta * p of the block's tile slots, one thread per slot; a masked slot
        // has the id -1; the row of a slot follows from its position
        const int cur_begin = s_begin, cur_mid = s_mid, cur_end = s_end;
        auto scatter = [&](int sl, int cid, float2 x) {
            if (cid < 0) return;
            const int r = ((sl >> 4) & 15) + (sl >= cur_mid ? 16 : 0);
            const float ds = x.x - delta_s[r] * x.y;
            uint32_t hi, lo;
            split_pack(ds, 0.f, hi, lo);
            ds_hi[cid * kRgStride + r] = (bf16_t)hi;
            ds_lo[cid * kRgStride + r] = (bf16_t)lo;
        };
#pragma unroll
        for (int k = 0; k < kRgPrefetch; ++k) {
            const int sl = cur_begin + (int)threadIdx.x + k * kThreads;
            if (sl < cur_end) scatter(sl, code[k], wpv[k]);
        }
        {   // blocks with more slots than were fetched ahead
            const float2* wp_b = a.wp + (int64_t)bh * a.num_chunks * 256;
            for (int sl = cur_begin + (int)threadIdx.x + kRgPrefetch * kThreads; sl < cur_end; sl += kThreads)
                scatter(sl, a.map[sl], wp_b[sl]);
        }
        // the dQ values this thread will add to, and everything the next block needs
        const int mc = wave >> 2, fc = wave & 3;
        float dq_old[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            const int row = row0 + 16 * mc + 4 * g + m;
            dq_old[m] = row < a.n ? a.dQ[base + (int64_t)row * a.sn + 16 * fc + j] : 0.f;
        }
        if (blk + (int)gridDim.x < total) prefetch(blk + gridDim.x);
        __syncthreads();
        {   // dQ of the block: wavefront -> 16 rows x 16 features
            f32x4_t dq = {0.f, 0.f, 0.f, 0.f};
            for (int ks = 0; ks < nids; ks += 32) {
                const bf16x8_t rb = lds_tr8(rel_s, kRelStride, ks + 8 * g, 16 * fc, j);
                dq = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lds_tr8(ds_hi, kRgStride, ks + 8 * g, 16 * mc, j), rb, dq, 0, 0, 0);
                dq = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lds_tr8(ds_lo, kRgStride, ks + 8 * g, 16 * mc, j), rb, dq, 0, 0, 0);
            }
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                const int row = row0 + 16 * mc + 4 * g + m;
                if (row < a.n) a.dQ[base + (int64_t)row * a.sn + 16 * fc + j] = dq_old[m] + a.scale * dq[m];
            }
        }
        bf16x8_t qb[4];
#pragma unroll
        for (int f = 0; f < 4; ++f) qb[f] = lds_tr8(q_s, kRowStride, 8 * g, 16 * f, j);
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            const int chunk = wave + kWaves * c;
            if (chunk < nchunks) {
                const int off = (16 * chunk + j) * kRgStride + 8 * g;
                const bf16x8_t ah = *reinterpret_cast<const bf16x8_t*>(ds_hi + off);
                const bf16x8_t al = *reinterpret_cast<const bf16x8_t*>(ds_lo + off);
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    acc[c][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, qb[f], acc[c][f], 0, 0, 0);
                    acc[c][f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, qb[f], acc[c][f], 0, 0, 0);
                }
            }
        }
        __syncthreads();
    }
    // this workgroup's copy: [gridDim.x][nids][kD], compact-id order
    float* dst = a.drel_part + (int64_t)blockIdx.x * nids * kD;
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int chunk = wave + kWaves * c;
        if (chunk < nchunks) {
#pragma unroll
            for (int f = 0; f < 4; ++f)
#pragma unroll
                for (int m = 0; m < 4; ++m) dst[(16 * chunk + 4 * g + m) * kD + 16 * f + j] = acc[c][f][m] * a.scale;
        }
    }
}

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

    // the block's K rows as A operands (token j of chunk c, features 16g..16g+15); V rows into LDS
    bf16x8_t ka[2][2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int64_t at = base + (int64_t)(t0 + 16 * c + j) * a.sn + 16 * g;
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

    for (int grp = 0; grp < ngroups; ++grp) {
        int level, loc;
        bool valid;
        span_slot(grp, j, a.L, level, loc, valid);
        const int node = span_level_offset(a.n, level) + (t0 >> level) + loc;
        const bf16_t* qrow = a.Q + base + (int64_t)node * a.sn + 16 * g;
        const bf16x8_t qb0 = *reinterpret_cast<const bf16x8_t*>(qrow);
        const bf16x8_t qb1 = *reinterpret_cast<const bf16x8_t*>(qrow + 8);
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
                const bool member = valid && (grp == 2 || (tt >> level) == loc);
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
            o[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pA, lds_transposed_b(v_s, kVStride, f, g, j), o[f], 0, 0, 0);
        }
        // C[m = query][n = feature]: this lane holds queries 4g..4g+3, feature 16f + j
        if (grp < 2) {
            if (g == 0 && valid) a.lse[(int64_t)bh * a.N + node] = (m + fast_log2(l)) * kLn2;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int slot = 4 * g + r;
                const float lq = __shfl(l, slot);
                if (grp == 1 && slot == 15) continue;
                bf16_t* orow = a.out + base + (int64_t)span_slot_node(grp, slot, a.L, a.n, t0) * a.sn + j;
                const float inv = 1.f / lq;
#pragma unroll
                for (int f = 0; f < 4; ++f) orow[16 * f] = (bf16_t)to_bf16_bits(o[f][r] * inv);
            }
        } else {
            // partial of the ancestor at level 6 + slot: [bh][level][block][66]
            if (g == 0 && valid) {
                float* dst = a.part + (((int64_t)bh * nanc + j) * nblk + blk) * kPartStride;
                dst[64] = m;
                dst[65] = l;
            }
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int slot = 4 * g + r;
                if (slot < nanc) {
                    float* dst = a.part + (((int64_t)bh * nanc + slot) * nblk + blk) * kPartStride + j;
#pragma unroll
                    for (int f = 0; f < 4; ++f) dst[16 * f] = o[f][r];
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
    int bh, v, cnt;
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
    r.cnt = 1 << (level - kSpanInLevels);
    r.src = a.part + (((int64_t)r.bh * nanc + (level - kSpanInLevels - 1)) * nblk + (int64_t)mi * r.cnt) * stride;
    return true;
}

__global__ void __launch_bounds__(256) fwd_span_merge_small_kernel(const SpanArgs a, int first, int rows) {
    const int lane = threadIdx.x & 63;
    SpanRow r;
    if (!span_merge_row(a, blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6), first, rows, kPartStride, r)) return;
    float o[kSpanSmallMax], m[kSpanSmallMax], l[kSpanSmallMax];
#pragma unroll
    for (int b = 0; b < kSpanSmallMax; ++b) {
        const float* pb = r.src + (int64_t)min(b, r.cnt - 1) * kPartStride;
        o[b] = pb[lane];
        m[b] = b < r.cnt ? pb[64] : kNegBig;
        l[b] = pb[65];
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
    a.out[base + (int64_t)r.v * a.sn + lane] = (bf16_t)to_bf16_bits(acc / ls);
    if (lane == 0) a.lse[(int64_t)r.bh * a.N + r.v] = (mx + fast_log2(ls)) * kLn2;
}

__global__ void __launch_bounds__(kSpanBigThreads) fwd_span_merge_big_kernel(const SpanArgs a, int first, int rows) {
    __shared__ float s_acc[64][kD + 4];
    __shared__ float s_l[64];
    __shared__ float s_m[kSpanBigThreads / 64];
    SpanRow r;
    if (!span_merge_row(a, blockIdx.x, first, rows, kPartStride, r)) return;   // uniform for the workgroup
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
        a.out[base + (int64_t)r.v * a.sn + t] = (bf16_t)to_bf16_bits(sum / lt);
        if (t == 0) a.lse[(int64_t)r.bh * a.N + r.v] = (mx + fast_log2(lt)) * kLn2;
    }
}

// Query side of the backward over the same blocks: S^T and dP^T = V_block x dO^T, p =
// exp2(s - lse), w = p dP.  A span inside the block has its whole row here, so delta = sum w
// and dS = w - delta p are final and dQ = scale * dS K_block (r_anc drops out: the dS of a row
// sum to zero).  An ancestor stores the partial sums A = W K, Bv = P K, delta, which the merge
// kernel turns into dQ = scale * (sum A - delta * sum Bv).
__global__ void __launch_bounds__(kTileThreads) bwd_q_span_tile_kernel(const SpanArgs a) {
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

    bf16x8_t ka[2][2], va[2][2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
        const int64_t at = base + (int64_t)(t0 + 16 * c + j) * a.sn + 16 * g;
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

    for (int grp = 0; grp < ngroups; ++grp) {
        int level, loc;
        bool valid;
        span_slot(grp, j, a.L, level, loc, valid);
        const int node = span_level_offset(a.n, level) + (t0 >> level) + loc;
        const bf16_t* qrow = a.Q + base + (int64_t)node * a.sn + 16 * g;
        const bf16_t* grow = a.dout + base + (int64_t)node * a.sn + 16 * g;
        const bf16x8_t qb0 = *reinterpret_cast<const bf16x8_t*>(qrow);
        const bf16x8_t qb1 = *reinterpret_cast<const bf16x8_t*>(qrow + 8);
        const bf16x8_t gb0 = *reinterpret_cast<const bf16x8_t*>(grow);
        const bf16x8_t gb1 = *reinterpret_cast<const bf16x8_t*>(grow + 8);
        const float lse2 = a.lse_r[(int64_t)bh * a.N + node] * kLog2e;
        const float shift = span_shift(a, level, g, qb0, qb1, qscale);
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
                const bool member = valid && (grp == 2 || (tt >> level) == loc);
                p[c][r] = member ? fast_exp2(s4[r] * qscale + shift - lse2) : 0.f;
                wgt[c][r] = p[c][r] * d4[r];
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
                dq[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sH, kB[f], dq[f], 0, 0, 0);
                dq[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sL, kB[f], dq[f], 0, 0, 0);
            }
            if (g == 0 && valid) a.stat[(int64_t)bh * a.N + node] = make_float2(lse2, dl);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int slot = 4 * g + r;
                if (grp == 1 && slot == 15) continue;
                float* orow = a.dQ + base + (int64_t)span_slot_node(grp, slot, a.L, a.n, t0) * a.sn + j;
#pragma unroll
                for (int f = 0; f < 4; ++f) orow[16 * f] = a.scale * dq[f][r];
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
                ow[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wH, kB[f], ow[f], 0, 0, 0);
                ow[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wL, kB[f], ow[f], 0, 0, 0);
                op[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pH, kB[f], op[f], 0, 0, 0);
                op[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pL, kB[f], op[f], 0, 0, 0);
            }
            if (g == 0 && valid) a.part[(((int64_t)bh * nanc + j) * nblk + blk) * kQPartStride + 2 * kD] = dl;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int slot = 4 * g + r;
                if (slot < nanc) {
                    float* dst = a.part + (((int64_t)bh * nanc + slot) * nblk + blk) * kQPartStride + j;
#pragma unroll
                    for (int f = 0; f < 4; ++f) {
                        dst[16 * f] = ow[f][r];
                        dst[kD + 16 * f] = op[f][r];
                    }
                }
            }
        }
    }
}

__global__ void __launch_bounds__(256) bwd_q_span_merge_small_kernel(const SpanArgs a, int first, int rows) {
    const int lane = threadIdx.x & 63;
    SpanRow r;
    if (!span_merge_row(a, blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6), first, rows, kQPartStride, r)) return;
    float xa[kSpanSmallMax], xb[kSpanSmallMax], xd[kSpanSmallMax];
#pragma unroll
    for (int b = 0; b < kSpanSmallMax; ++b) {
        const float* pb = r.src + (int64_t)min(b, r.cnt - 1) * kQPartStride;
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
    a.dQ[base + (int64_t)r.v * a.sn + lane] = a.scale * (sa - dl * sb);
    if (lane == 0) a.stat[(int64_t)r.bh * a.N + r.v] = make_float2(a.lse_r[(int64_t)r.bh * a.N + r.v] * kLog2e, dl);
}

__global__ void __launch_bounds__(kSpanBigThreads) bwd_q_span_merge_big_kernel(const SpanArgs a, int first, int rows) {
    __shared__ float s_a[64][kD + 4], s_b[64][kD + 4];
    __shared__ float s_d[64];
    SpanRow r;
    if (!span_merge_row(a, blockIdx.x, first, rows, kQPartStride, r)) return;
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
        a.dQ[base + (int64_t)r.v * a.sn + t] = a.scale * (ta - td * tb);
        if (t == 0) a.stat[(int64_t)r.bh * a.N + r.v] = make_float2(a.lse_r[(int64_t)r.bh * a.N + r.v] * kLog2e, td);
    }
}

// ---- backward, key side, over dense tiles of key nodes (bf16) --------------------------
// A wavefront owns up to 16 consecutive key nodes of one level and walks (a slice of)
// the nodes that attend to them, 32 at a time.  With the queries on the M side,
//   S[query][key]  = Q_chunk (A, rows from memory) x K_tile^T (B, rows from memory),
//   dP[query][key] = dO_chunk x V_tile^T,   bias[query][id] = Q_chunk x Rel_sel^T,
// the result C[m][n] has key n = lane%16 and queries 4*(lane/16)..+3 in the registers,
// which is the A-operand layout of the second products (contraction over queries):
//   dK[key][f] += dS^T x Q_chunk,   dV[key][f] += P^T x dO_chunk
// with Q and dO rows read transposed out of LDS.  lse and the exact delta of every
// query come from the query side (`stat`), so dS is formed in fp32 before it is
// rounded to bf16 for the product.  No atomics: a tile whose query list is cut into
// several tasks is summed by kv_tile_merge_kernel in task order.
constexpr int kMaxBiasChunks = 6;
struct KeyArgs {
    const bf16_t *Q, *K, *V, *rel, *dout;
    const float2* stat;
    float *dK, *dV, *part;
    int64_t sb, sh, sn;
    int32_t BH, H, N, num_levels;
    float scale;
    int32_t row_bytes;
    uint32_t slab_bytes;
    const int32_t *tile_node0, *tile_info, *cols, *task_tile, *task_c0, *task_nch, *task_part;
    const int16_t* map;
    int32_t num_tasks, num_part, num_chunks, nb_pad, W, zero;
};

template <int NBC>
__global__ void __launch_bounds__(kTileThreads, 2) bwd_kv_tile_kernel(const KeyArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, j = lane & 15;
    const int r8 = lane >> 3, piece = lane & 7;   // coalesced row fetches: row of the instruction, 16-byte piece
    const int bstride = a.nb_pad + 1;
    float* bias_s = reinterpret_cast<float*>(smem) + (size_t)wave * 32 * bstride;               // [32 queries][ids]
    bf16_t* q_s = reinterpret_cast<bf16_t*>(smem + (size_t)kTileWaves * 32 * bstride * sizeof(float)) +
                  (size_t)wave * 64 * kRowStride;                                                // [32 queries][kRowStride]
    bf16_t* g_s = q_s + 32 * kRowStride;
    float2* stat_s = reinterpret_cast<float2*>(smem + (size_t)kTileWaves * (32 * bstride * sizeof(float) +
                                                                            64 * kRowStride * sizeof(bf16_t))) +
                     (size_t)wave * 32;                                                          // [32 queries] (lse, delta)
    const float qscale = a.scale * kLog2e;
    const int groups = (a.num_tasks + kTileWaves - 1) / kTileWaves;
    const rsrc_t rC = make_rsrc(a.cols, (uint32_t)a.num_chunks * 64u);    // [chunks][16] int32
    const rsrc_t rM = make_rsrc(a.map, (uint32_t)a.num_chunks * 512u);    // [chunks][16][16] int16

    for (TileWalk w(a.BH * groups); w.t < w.t_end; w.t += w.step) {
        const int bh = w.t / groups;
        const int task = (w.t - bh * groups) * kTileWaves + wave;
        if (task >= a.num_tasks) continue;
        const int kt = a.task_tile[task], c0 = a.task_c0[task], nch = a.task_nch[task], part = a.task_part[task];
        const int node0 = a.tile_node0[kt], info = a.tile_info[kt];
        const int level = info & 255, nkeys = info >> 8;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        const rsrc_t rQ = make_rsrc(a.Q + base, a.slab_bytes), rG = make_rsrc(a.dout + base, a.slab_bytes);
        const rsrc_t rS = make_rsrc(a.stat + (int64_t)bh * a.N, (uint32_t)a.N * 8u);

        // Software pipeline over pairs of chunks.  `Idx` = what has to be known before a pair's
        // rows can be requested (its column ids and map words); the rows of pair i+1 are
        // requested in the middle of pair i, as soon as the registers of pair i's rows are free,
        // and the ids of pair i+2 right after, so the gathers overlap the second products.
        int node[2][2];   // [chunk][half]: query node whose row this lane helps to fetch
        uint2 mpn[2];
        auto load_idx = [&](int c2) {   // a pair past the end repeats the last one (valid addresses, results unused)
            const int cc = c0 + min(c2, nch - 2);
#pragma unroll
            for (int ci = 0; ci < 2; ++ci) {
                const int at = (cc + ci) * 16;
                node[ci][0] = buf_i32(rC, (at + r8) * 4);
                node[ci][1] = buf_i32(rC, (at + 8 + r8) * 4);
                const u32x2 m2 = __builtin_amdgcn_raw_buffer_load_b64(rM, (at + j) * 32 + 8 * g, 0, 0);
                mpn[ci] = make_uint2(m2.x, m2.y);
            }
        };
        // Row fetches are coalesced: 8 consecutive lanes take the 8 16-byte pieces of one row, an
        // instruction fetches 8 whole rows (two per 16-row chunk).  The rows go through LDS to get
        // into the operand layouts of the matrix instructions.
        Row<bf16_t> qa[2][2], ga[2][2];
        float2 stn[2][2];   // (lse, delta) of the row, kept by the lane that fetches its first piece
        auto load_rows = [&]() {
#pragma unroll
            for (int ci = 0; ci < 2; ++ci)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int off = (int)__umul24(node[ci][h], a.row_bytes) + piece * 16;
                    buf_row(rQ, off, qa[ci][h]);
                    buf_row(rG, off, ga[ci][h]);
                    stn[ci][h] = buf_f2(rS, node[ci][h] * 8);
                }
        };
        load_idx(0);

        // B operands: the tile's keys (lane j <-> key j) and the rows of the table this level can meet
        const int64_t krow = base + (int64_t)(node0 + min(j, nkeys - 1)) * a.sn + 16 * g;
        const bf16x8_t kb0 = *reinterpret_cast<const bf16x8_t*>(a.K + krow);
        const bf16x8_t kb1 = *reinterpret_cast<const bf16x8_t*>(a.K + krow + 8);
        const bf16x8_t vb0 = *reinterpret_cast<const bf16x8_t*>(a.V + krow);
        const bf16x8_t vb1 = *reinterpret_cast<const bf16x8_t*>(a.V + krow + 8);
        bf16x8_t rb[NBC][2];
#pragma unroll
        for (int bc = 0; bc < NBC; ++bc) {
            const int bid = 16 * bc + j;
            int row = 0;
            if (bid < a.W)
                row = level * a.W + bid;                        // (level, order)
            else if (bid - a.W + 1 < a.num_levels)
                row = (bid - a.W + 1) * a.W + a.zero;            // r_anc of the ancestor's level
            const bf16_t* rr = a.rel + (int64_t)row * kD + 16 * g;
            rb[bc][0] = *reinterpret_cast<const bf16x8_t*>(rr);
            rb[bc][1] = *reinterpret_cast<const bf16x8_t*>(rr + 8);
        }
        load_rows();     // pair 0 (waits for its ids)
        uint2 mp[2] = {mpn[0], mpn[1]};
        load_idx(2);     // ids of pair 1

        f32x4_t dk[4], dv[4];
#pragma unroll
        for (int f = 0; f < 4; ++f) dk[f] = dv[f] = f32x4_t{0.f, 0.f, 0.f, 0.f};

        for (int c2 = 0; c2 < nch; c2 += 2) {
            wave_lds_sync();  // the previous pair's LDS reads are done
#pragma unroll
            for (int ci = 0; ci < 2; ++ci)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int row = 16 * ci + 8 * h + r8;
                    *reinterpret_cast<uint4*>(q_s + row * kRowStride + piece * 8) = qa[ci][h].w;
                    *reinterpret_cast<uint4*>(g_s + row * kRowStride + piece * 8) = ga[ci][h].w;
                    if (piece == 0) stat_s[row] = stn[ci][h];
                }
            __builtin_amdgcn_sched_barrier(0);
            // the row registers are free: request the next pair's rows, then the ids of the pair after it
            const uint2 mpc[2] = {mp[0], mp[1]};
            load_rows();
            mp[0] = mpn[0];
            mp[1] = mpn[1];
            load_idx(c2 + 4);
            __builtin_amdgcn_sched_barrier(0);
            wave_lds_sync();
            f32x4_t s4[2], d4[2];
#pragma unroll
            for (int ci = 0; ci < 2; ++ci) {
                const bf16_t* qr = q_s + (16 * ci + j) * kRowStride + 16 * g;
                const bf16_t* gr = g_s + (16 * ci + j) * kRowStride + 16 * g;
                const bf16x8_t q0 = *reinterpret_cast<const bf16x8_t*>(qr), q1 = *reinterpret_cast<const bf16x8_t*>(qr + 8);
                const bf16x8_t g0 = *reinterpret_cast<const bf16x8_t*>(gr), g1 = *reinterpret_cast<const bf16x8_t*>(gr + 8);
                s4[ci] = d4[ci] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                s4[ci] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(q0, kb0, s4[ci], 0, 0, 0);
                s4[ci] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(q1, kb1, s4[ci], 0, 0, 0);
                d4[ci] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(g0, vb0, d4[ci], 0, 0, 0);
                d4[ci] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(g1, vb1, d4[ci], 0, 0, 0);
#pragma unroll
                for (int bc = 0; bc < NBC; ++bc) {
                    f32x4_t b4 = {0.f, 0.f, 0.f, 0.f};
                    b4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(q0, rb[bc][0], b4, 0, 0, 0);
                    b4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(q1, rb[bc][1], b4, 0, 0, 0);
#pragma unroll
                    for (int r = 0; r < 4; ++r) bias_s[(16 * ci + 4 * g + r) * bstride + 16 * bc + j] = b4[r];
                }
            }
            wave_lds_sync();
            float ds[2][4], pp[2][4], bv[2][4];
            float2 st[2][4];
            int bid[2][4];
#pragma unroll
            for (int ci = 0; ci < 2; ++ci) {
                const float4 x = *reinterpret_cast<const float4*>(stat_s + 16 * ci + 4 * g);
                const float4 y = *reinterpret_cast<const float4*>(stat_s + 16 * ci + 4 * g + 2);
                st[ci][0] = make_float2(x.x, x.y);
                st[ci][1] = make_float2(x.z, x.w);
                st[ci][2] = make_float2(y.x, y.y);
                st[ci][3] = make_float2(y.z, y.w);
            }
#pragma unroll
            for (int ci = 0; ci < 2; ++ci) {
                bid[ci][0] = (int)(short)(mpc[ci].x & 0xFFFFu);
                bid[ci][1] = (int)(short)(mpc[ci].x >> 16);
                bid[ci][2] = (int)(short)(mpc[ci].y & 0xFFFFu);
                bid[ci][3] = (int)(short)(mpc[ci].y >> 16);
#pragma unroll
                for (int r = 0; r < 4; ++r) bv[ci][r] = bias_s[(16 * ci + 4 * g + r) * bstride + max(bid[ci][r], 0)];
            }
#pragma unroll
            for (int ci = 0; ci < 2; ++ci)
#pragma unroll
                for (int r = 0; r < 4; ++r) asm volatile("" : "+v"(bv[ci][r]));  // reads stay out of branches on the mask
#pragma unroll
            for (int ci = 0; ci < 2; ++ci)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float p = bid[ci][r] >= 0 ? fast_exp2((s4[ci][r] + bv[ci][r]) * qscale - st[ci][r].x) : 0.f;
                    pp[ci][r] = p;
                    ds[ci][r] = p * (d4[ci][r] - st[ci][r].y);
                }
            // dS and P as A operands, each as bf16 hi + lo: the sums run over up to thousands of
            // queries and the tolerance is absolute, so 8 mantissa bits are not enough
            uint32_t shi[4], slo[4], phi[4], plo[4];
#pragma unroll
            for (int ci = 0; ci < 2; ++ci) {
                split_pack(ds[ci][0], ds[ci][1], shi[2 * ci], slo[2 * ci]);
                split_pack(ds[ci][2], ds[ci][3], shi[2 * ci + 1], slo[2 * ci + 1]);
                split_pack(pp[ci][0], pp[ci][1], phi[2 * ci], plo[2 * ci]);
                split_pack(pp[ci][2], pp[ci][3], phi[2 * ci + 1], plo[2 * ci + 1]);
            }
            const u32x4 xsh = {shi[0], shi[1], shi[2], shi[3]}, xsl = {slo[0], slo[1], slo[2], slo[3]};
            const u32x4 xph = {phi[0], phi[1], phi[2], phi[3]}, xpl = {plo[0], plo[1], plo[2], plo[3]};
            const bf16x8_t sH = __builtin_bit_cast(bf16x8_t, xsh), sL = __builtin_bit_cast(bf16x8_t, xsl);
            const bf16x8_t pH = __builtin_bit_cast(bf16x8_t, xph), pL = __builtin_bit_cast(bf16x8_t, xpl);
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const bf16x8_t qB = lds_transposed_b(q_s, kRowStride, f, g, j), gB = lds_transposed_b(g_s, kRowStride, f, g, j);
                dk[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sH, qB, dk[f], 0, 0, 0);
                dk[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sL, qB, dk[f], 0, 0, 0);
                dv[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pH, gB, dv[f], 0, 0, 0);
                dv[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pL, gB, dv[f], 0, 0, 0);
            }
        }
        // C[m = key][n = feature]: lane holds keys 4g..4g+3, feature 16f + j
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int key = 4 * g + r;
            if (key < nkeys) {
                if (part < 0) {
                    const int64_t at = base + (int64_t)(node0 + key) * a.sn + j;
#pragma unroll
                    for (int f = 0; f < 4; ++f) {
                        a.dK[at + 16 * f] = a.scale * dk[f][r];
                        a.dV[at + 16 * f] = dv[f][r];
                    }
                } else {
                    float* dst = a.part + (((int64_t)bh * a.num_part + part) * 16 + key) * (2 * kD) + j;
#pragma unroll
                    for (int f = 0; f < 4; ++f) {
                        dst[16 * f] = a.scale * dk[f][r];
                        dst[kD + 16 * f] = dv[f][r];
                    }
                }
            }
        }
        wave_lds_sync();
    }
}

// tiles whose query list was cut into several tasks: sum the partial (dK, dV) of the
// tile's keys in task order.  One workgroup per (batch*head, tile); thread -> (key, feature pair).
__global__ void __launch_bounds__(256) kv_tile_merge_kernel(const KeyArgs a, const int32_t* __restrict__ multi_tile,
                                                            const int32_t* __restrict__ multi_ptr, int num_multi) {
    const int bh = blockIdx.x / num_multi, mt = blockIdx.x - bh * num_multi;
    const int kt = multi_tile[mt];
    const int node0 = a.tile_node0[kt], nkeys = a.tile_info[kt] >> 8;
    const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
    for (int i = threadIdx.x; i < nkeys * kD; i += blockDim.x) {
        const int key = i >> 6, f = i & 63;
        float sk = 0.f, sv = 0.f;
        for (int p = multi_ptr[mt]; p < multi_ptr[mt + 1]; ++p) {
            const float* src = a.part + (((int64_t)bh * a.num_part + p) * 16 + key) * (2 * kD) + f;
            sk += src[0];
            sv += src[kD];
        }
        const int64_t at = base + (int64_t)(node0 + key) * a.sn + f;
        a.dK[at] = sk;
        a.dV[at] = sv;
    }
}

// nodes no one attends to (levels above the coarsest contextual level): zero gradients
__global__ void kv_zero_rows_kernel(const KeyArgs a, int first_row) {
    const int rows = a.N - first_row;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (int64_t)a.BH * rows * kD) return;
    const int f = (int)(i & 63);
    const int64_t rr = i >> 6;
    const int bh = (int)(rr / rows), row = first_row + (int)(rr - (int64_t)bh * rows);
    const int64_t at = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh + (int64_t)row * a.sn + f;
    a.dK[at] = 0.f;
    a.dV[at] = 0.f;
}

// key nodes cut into several segments: sum the (dK, dV) partials in segment order
__global__ void __launch_bounds__(256) bwd_kv_merge_kernel(const AttnArgs a, const int32_t* __restrict__ multi_row,
                                                           const int32_t* __restrict__ multi_ptr, int num_multi) {
    const int lane = threadIdx.x & 63;
    const int item = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (item >= a.BH * num_multi) return;
    const int bh = item / num_multi, j = item - bh * num_multi;
    float sk = 0.f, sv = 0.f;
    for (int p = multi_ptr[j]; p < multi_ptr[j + 1]; ++p) {
        const float* src = a.part + ((int64_t)bh * a.num_part + p) * (2 * kD);
        sk += src[lane];
        sv += src[kD + lane];
    }
    const int64_t at = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh + (int64_t)multi_row[j] * a.sn + lane;
    a.dK[at] = sk;
    a.dV[at] = sv;
}

// d_rel = sum of the workgroups' copies, in a fixed order; rows the copies do not
// cover are zero.  One workgroup per row of 64 features: 16 wavefronts each sum a
// sixteenth of the copies (lane = feature, coalesced 256-byte reads, four
// independent partial sums in flight), then combine in a fixed tree.
// With `id_to_cid` the copies are in the token tiles' compact-id order and hold
// `covered_rows` rows each: row `id` of d_rel is copy row id_to_cid[id] (or zero).
__global__ void __launch_bounds__(1024) drel_reduce_kernel(const float* __restrict__ parts, int num_parts,
                                                           int covered_rows, const int32_t* __restrict__ id_to_cid,
                                                           float* __restrict__ d_rel) {
    __shared__ float s[16][kD];
    const int row = blockIdx.x, lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int prow = id_to_cid ? id_to_cid[row] : row;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    if (prow >= 0 && prow < covered_rows) {
        const float* src = parts + (int64_t)prow * kD + lane;
        const int64_t stride = (int64_t)covered_rows * kD;
        int p = grp;
        for (; p + 48 < num_parts; p += 64) {
            a0 += src[p * stride];
            a1 += src[(p + 16) * stride];
            a2 += src[(p + 32) * stride];
            a3 += src[(p + 48) * stride];
        }
        for (; p < num_parts; p += 16) a0 += src[p * stride];
    }
    s[grp][lane] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    for (int w = 8; w > 0; w >>= 1) {
        if (grp < w) s[grp][lane] += s[grp + w][lane];
        __syncthreads();
    }
    if (grp == 0) d_rel[row * kD + lane] = s[0][lane];
}

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
    if ((int64_t)s->B * s->H > (int64_t)INT32_MAX / std::max(g->fwd.num_tiles, g->tr.num_tiles))
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
    a.n_tokens = g->n;
    a.scale = s->scale > 0.f ? s->scale : 0.125f;  // 1/sqrt(64)
    a.rel_rows = g->num_levels * g->rel_width;
    const int64_t es = s->dtype == BPT_BF16 ? 2 : 4;
    a.row_bytes = (int32_t)(s->stride_n * es);
    a.slab_bytes = (uint32_t)(((int64_t)(g->num_nodes - 1) * s->stride_n + kD) * es);
    a.idx_bytes = (uint32_t)(g->num_edges * 4);
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
TilePlan plan_tiles(const bpt_graph* g, const DeviceLimits& lim) {
    TilePlan t;
    if (g->tiles.num_tiles == 0) return t;
    t.cid_pad = (g->tiles.num_cids + 15) & ~15;
    t.bias_stride = t.cid_pad + ((4 - t.cid_pad % 32) + 32) % 32;  // = 4 mod 32: the 16 token rows hit different banks
    const size_t rel = (size_t)t.cid_pad * kRelStride * sizeof(bf16_t);
    const size_t rest = (size_t)kTileWaves * 16 * t.bias_stride * sizeof(float) +
                        (size_t)kTileWaves * 64 * kRowStride * sizeof(bf16_t);
    t.rel_lds = rel + rest <= lim.lds;
    t.lds = t.rel_lds ? rel + rest : rest;
    t.ok = t.lds <= lim.lds;
    return t;
}

void fill_tile_args(TileArgs& t, const bpt_graph* g, const AttnArgs& a, const TilePlan& tp);

template <typename K>
int launch_tiles(const char* name, K kernel, const TileArgs& t, const DeviceLimits& lim, size_t lds, hipStream_t st) {
    if (lds > 65536)
        BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    const int grid = std::max(8, lim.cus * resident_blocks(kernel, kTileThreads, lds, lim) / 8 * 8);
    BPT_LAUNCH(name, kernel, dim3(grid), dim3(kTileThreads), lds, st, t);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

// bf16 backward, query side of the token rows on dense tiles
int run_bwd_q_tiles(const bpt_graph* g, const AttnArgs& a, const DeviceLimits& lim, hipStream_t st) {
    const TilePlan tp = plan_tiles(g, lim);
    TileArgs t = {};
    fill_tile_args(t, g, a, tp);
    return tp.rel_lds ? launch_tiles("bwd_q_tile_kernel", bwd_q_tile_kernel<true>, t, lim, tp.lds, st)
                      : launch_tiles("bwd_q_tile_kernel", bwd_q_tile_kernel<false>, t, lim, tp.lds, st);
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
}
// forward == true: out and lse of all span rows; else delta, lse and dQ of all span rows
int run_span_tiles(const bpt_graph* g, const AttnArgs& a, bool forward, hipStream_t st) {
    SpanArgs t;
    fill_span_args(t, g, a);
    const int64_t items = (int64_t)a.BH * (g->n / kSpanTok);
    const unsigned grid = (unsigned)((items + kTileWaves - 1) / kTileWaves);
    const size_t lds = (size_t)kTileWaves * kSpanTok * kVStride * sizeof(bf16_t);
    if (forward)
        BPT_LAUNCH("fwd_span_tile_kernel", fwd_span_tile_kernel, dim3(grid), dim3(kTileThreads), lds, st, t);
    else
        BPT_LAUNCH("bwd_q_span_tile_kernel", bwd_q_span_tile_kernel, dim3(grid), dim3(kTileThreads), lds, st, t);
    BPT_HIP(hipGetLastError());
    if (t.L > kSpanInLevels) {
        // rows of levels 6..9 (at most 16 partials each), then the longer rows
        const int first = 2 * g->n - ((2 * g->n) >> (kSpanInLevels + 1));
        const int big_level = kSpanInLevels + 1 + kSpanSmallLevels;
        const int first_big = t.L >= big_level ? 2 * g->n - ((2 * g->n) >> big_level) : g->num_nodes;
        const int rows_small = first_big - first, rows_big = g->num_nodes - first_big;
        const unsigned sgrid = (unsigned)(((int64_t)a.BH * rows_small + 3) / 4);
        if (forward)
            BPT_LAUNCH("fwd_span_merge_small_kernel", fwd_span_merge_small_kernel, dim3(sgrid), dim3(256), 0, st, t, first,
                       rows_small);
        else
            BPT_LAUNCH("bwd_q_span_merge_small_kernel", bwd_q_span_merge_small_kernel, dim3(sgrid), dim3(256), 0, st, t,
                       first, rows_small);
        BPT_HIP(hipGetLastError());
        if (rows_big > 0) {
            const unsigned bgrid = (unsigned)((int64_t)a.BH * rows_big);
            if (forward)
                BPT_LAUNCH("fwd_span_merge_big_kernel", fwd_span_merge_big_kernel, dim3(bgrid), dim3(kSpanBigThreads), 0, st,
                           t, first_big, rows_big);
            else
                BPT_LAUNCH("bwd_q_span_merge_big_kernel", bwd_q_span_merge_big_kernel, dim3(bgrid), dim3(kSpanBigThreads), 0,
                           st, t, first_big, rows_big);
            BPT_HIP(hipGetLastError());
        }
    }
    return BPT_OK;
}

// bf16 forward: token rows as dense tiles on the matrix cores, span rows with the gather kernel
int run_fwd_tiles(const bpt_graph* g, AttnArgs& a, const DeviceLimits& lim, const TilePlan& tp, hipStream_t st) {
    TileArgs t = {};
    fill_tile_args(t, g, a, tp);
    return tp.rel_lds ? launch_tiles("fwd_tile_kernel", fwd_tile_kernel<true>, t, lim, tp.lds, st)
                      : launch_tiles("fwd_tile_kernel", fwd_tile_kernel<false>, t, lim, tp.lds, st);
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
struct BwdPlan {
    int drel_rows = 0;        // d_rel rows token rows can touch
    bool drel_mfma = false;   // bf16 tensors: rel_grad_mfma_kernel; fp32: rel_grad_kernel
    bool drel_tile = false;   // bf16 tensors with token tiles and at most 256 ids in use: rel_grad_tile_kernel
    int drel_part_rows = 0;   // rows of one workgroup's copy of d_rel
    bool q_tiles = false;     // query side of token rows on dense tiles (bwd_q_tile_kernel)
    bool kv_tiles = false;    // key side on dense tiles of key nodes (bwd_kv_tile_kernel)
    size_t kv_lds = 0;
    int drel_ipw = 32;        // ids per wavefront: 8, 16 or 32
    int drel_block = 32;      // token rows per block
    int drel_grid_x = 8, drel_grid_y = 1;
    size_t drel_lds = 0;
    size_t off_stat = 0, off_wp = 0, off_qpart = 0, off_kvpart = 0, off_drel = 0, total = 0;
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
        }
        if (g->ktiles.num_tasks > 0 && g->ktiles.nb_pad <= 16 * kMaxBiasChunks) {
            p->kv_lds = (size_t)kTileWaves * (32 * (g->ktiles.nb_pad + 1) * sizeof(float) + 64 * kRowStride * sizeof(bf16_t) +
                                              32 * sizeof(float2));
            p->kv_tiles = p->kv_lds <= lim.lds;
        }
        p->drel_grid_y = p->drel_tile ? 1 : (p->drel_rows + kRgIds - 1) / kRgIds;
        blocks = (int64_t)s->B * s->H * ((g->n + kRgRows - 1) / kRgRows);
    } else {
        p->drel_ipw = p->drel_rows <= 64 ? 8 : p->drel_rows <= 128 ? 16 : 32;
        const int chunk = p->drel_ipw * kWaves;
        p->drel_block = std::min(g->n, chunk > 128 ? 32 : 64);
        p->drel_lds = (size_t)p->drel_block * (chunk + kD) * sizeof(float);
        p->drel_grid_y = (p->drel_rows + chunk - 1) / chunk;
        blocks = (int64_t)s->B * s->H * (g->n / p->drel_block);
    }
    const int per_cu = (int)std::max<size_t>(1, std::min<size_t>(4, lim.lds_cu / p->drel_lds));
    p->drel_grid_x = (int)std::max<int64_t>(1, std::min<int64_t>(blocks, (int64_t)lim.cus * per_cu / p->drel_grid_y));
    const size_t bh = (size_t)s->B * s->H;
    size_t off = 0;
    p->off_stat = off;
    off += align_up(bh * g->num_nodes * sizeof(float2));
    p->off_wp = off;
    // (w, p) pairs: per edge of a token row in CSR order, or per slot of the token tiles
    off += align_up(bh * (p->q_tiles ? (size_t)g->tiles.num_chunks * 256 : (size_t)g->num_token_edges) * sizeof(float2));
    p->off_qpart = off;
    off += align_up(bh * std::max<size_t>(std::max(g->fwd.num_part, g->fwd_span.num_part), span_partials(g)) *
                    kQPartStride * sizeof(float));
    p->off_kvpart = off;
    off += align_up(bh * std::max<size_t>(g->tr.num_part, p->kv_tiles ? (size_t)g->ktiles.num_part * 16 : 0) * 2 * kD *
                    sizeof(float));
    p->off_drel = off;
    if (!p->drel_tile) p->drel_part_rows = p->drel_rows;
    off += align_up((size_t)p->drel_grid_x * p->drel_part_rows * kD * sizeof(float));
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
        if ((rc = run_bwd_q_tiles(g, a, lim, st))) return rc;
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
        if (p.drel_part_rows <= 256) {
            if (p.drel_lds > 65536)
                BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(rel_grad_tile_kernel<2>),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.drel_lds));
            BPT_LAUNCH("rel_grad_tile_kernel", rel_grad_tile_kernel<2>, dim3(p.drel_grid_x), dim3(kThreads), p.drel_lds, st, t);
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
               p.drel_part_rows, p.drel_tile ? g->tiles.id_to_cid : nullptr, a.d_rel);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

template <int NBC>
int launch_kv_tiles(const KeyArgs& t, const BwdPlan& p, const DeviceLimits& lim, hipStream_t st) {
    if (p.kv_lds > 65536)
        BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_kv_tile_kernel<NBC>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.kv_lds));
    const int grid = std::max(8, lim.cus * resident_blocks(bwd_kv_tile_kernel<NBC>, kTileThreads, p.kv_lds, lim) / 8 * 8);
    BPT_LAUNCH("bwd_kv_tile_kernel", bwd_kv_tile_kernel<NBC>, dim3(grid), dim3(kTileThreads), p.kv_lds, st, t);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

// bf16 key side on dense tiles of key nodes
int run_bwd_kv_tiles(const bpt_graph* g, const BwdPlan& p, const AttnArgs& a, const DeviceLimits& lim, hipStream_t st) {
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
    t.map = kt.map;
    t.num_tasks = kt.num_tasks;
    t.num_part = kt.num_part;
    t.nb_pad = kt.nb_pad;
    t.W = g->rel_width;
    t.zero = g->k + 1;
    t.num_chunks = kt.num_chunks;
    int rc = BPT_ERR_UNSUPPORTED;
    switch (kt.nb_pad / 16) {
        case 1: rc = launch_kv_tiles<1>(t, p, lim, st); break;
        case 2: rc = launch_kv_tiles<2>(t, p, lim, st); break;
        case 3: rc = launch_kv_tiles<3>(t, p, lim, st); break;
        case 4: rc = launch_kv_tiles<4>(t, p, lim, st); break;
        case 5: rc = launch_kv_tiles<5>(t, p, lim, st); break;
        case 6: rc = launch_kv_tiles<6>(t, p, lim, st); break;
        default: break;
    }
    if (rc) return rc;
    if (kt.num_multi > 0) {
        BPT_LAUNCH("kv_tile_merge_kernel", kv_tile_merge_kernel, dim3(a.BH * kt.num_multi), dim3(256), 0, st, t, kt.multi_tile,
                           kt.multi_ptr, kt.num_multi);
        BPT_HIP(hipGetLastError());
    }
    const int64_t zero_elems = (int64_t)a.BH * (a.N - kt.first_uncovered) * kD;
    if (zero_elems > 0) {
        BPT_LAUNCH("kv_zero_rows_kernel", kv_zero_rows_kernel, dim3((unsigned)((zero_elems + 255) / 256)), dim3(256), 0, st, t,
                           kt.first_uncovered);
        BPT_HIP(hipGetLastError());
    }
    return BPT_OK;
}

template <typename T>
int run_bwd_kv(const bpt_graph* g, const BwdPlan& p, AttnArgs& a, hipStream_t st) {
    DeviceLimits lim;
    int rc = device_limits(g, &lim);
    if (rc) return rc;
    if (p.kv_tiles) return run_bwd_kv_tiles(g, p, a, lim, st);
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

enum { kStageQ = 1, kStageKV = 2 };

int backward(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K, const void* V, const void* rel,
             const float* lse, const void* dout, float* dQ, float* dK, float* dV, float* d_rel, void* workspace,
             size_t workspace_bytes, void* stream, int stages) {
    int rc = check_shape(g, s);
    if (rc) return rc;
    if (!Q || !K || !V || !rel || !lse || !dout) return BPT_ERR_INVALID_ARG;
    if ((stages & kStageQ) && (!dQ || !d_rel)) return BPT_ERR_INVALID_ARG;
    if ((stages & kStageKV) && (!dK || !dV)) return BPT_ERR_INVALID_ARG;
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(rel) || misaligned(dout) || misaligned(dQ) ||
        misaligned(dK) || misaligned(dV) || misaligned(d_rel) || misaligned(workspace))
        return BPT_ERR_INVALID_ARG;
    BwdPlan p;
    if ((rc = plan_bwd(g, s, &p))) return rc;
    if (!workspace || workspace_bytes < p.total) return BPT_ERR_INVALID_ARG;
    unsigned char* ws = static_cast<unsigned char*>(workspace);
    AttnArgs a;
    fill_common(a, g, s);
    a.Q = Q;
    a.K = K;
    a.V = V;
    a.rel = rel;
    a.lse_r = lse;
    a.dout = dout;
    a.dQ = dQ;
    a.dK = dK;
    a.dV = dV;
    a.d_rel = d_rel;
    a.stat = reinterpret_cast<float2*>(ws + p.off_stat);
    a.wp = reinterpret_cast<float2*>(ws + p.off_wp);
    a.e_tok = g->num_token_edges;
    a.drel_part = reinterpret_cast<float*>(ws + p.off_drel);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = s->dtype == BPT_BF16;
    if (stages & kStageQ) {
        a.part = reinterpret_cast<float*>(ws + p.off_qpart);
        if ((rc = bf ? run_bwd_q<bf16_t>(g, p, a, st) : run_bwd_q<float>(g, p, a, st))) return rc;
    }
    if (stages & kStageKV) {
        a.part = reinterpret_cast<float*>(ws + p.off_kvpart);
        if ((rc = bf ? run_bwd_kv<bf16_t>(g, p, a, st) : run_bwd_kv<float>(g, p, a, st))) return rc;
    }
    return BPT_OK;
}

}  // namespace
}  // namespace bpt

extern "C" {

size_t bpt_attn_fwd_workspace(const bpt_graph_t* g, const bpt_shape_t* s) {
    if (bpt::check_shape(g, s) != BPT_OK) return 0;
    return bpt::align_up((size_t)s->B * s->H *
                         std::max<size_t>(std::max(g->fwd.num_part, g->fwd_span.num_part), bpt::span_partials(g)) *
                         bpt::kPartStride * sizeof(float));
}

size_t bpt_attn_bwd_workspace(const bpt_graph_t* g, const bpt_shape_t* s) {
    if (bpt::check_shape(g, s) != BPT_OK) return 0;
    bpt::BwdPlan p;
    if (bpt::plan_bwd(g, s, &p) != BPT_OK) return 0;
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
    if (need > 0 && (!workspace || workspace_bytes < need)) return BPT_ERR_INVALID_ARG;
    bpt::AttnArgs a;
    bpt::fill_common(a, g, s);
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

int bpt_attn_bwd(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K, const void* V,
                 const void* rel, const float* lse, const void* dout, float* dQ, float* dK, float* dV, float* d_rel,
                 void* workspace, size_t workspace_bytes, void* stream) {
    return bpt::backward(g, s, Q, K, V, rel, lse, dout, dQ, dK, dV, d_rel, workspace, workspace_bytes, stream,
                         bpt::kStageQ | bpt::kStageKV);
}

int bpt_attn_bwd_query_side(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K, const void* V,
                            const void* rel, const float* lse, const void* dout, float* dQ, float* d_rel,
                            void* workspace, size_t workspace_bytes, void* stream) {
    return bpt::backward(g, s, Q, K, V, rel, lse, dout, dQ, nullptr, nullptr, d_rel, workspace, workspace_bytes,
                         stream, bpt::kStageQ);
}

int bpt_attn_bwd_key_side(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K, const void* V,
                          const void* rel, const float* lse, const void* dout, float* dK, float* dV, void* workspace,
                          size_t workspace_bytes, void* stream) {
    return bpt::backward(g, s, Q, K, V, rel, lse, dout, nullptr, dK, dV, nullptr, workspace, workspace_bytes, stream,
                         bpt::kStageKV);
}

}  // extern "C"
