// Device-side helpers shared by the attention kernels: kernel arguments, lane and row helpers,
// buffer loads, bf16 packing, the XCD-aware walk over work items.
#pragma once

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
    const int32_t* seq_len; // [B] tokens of every sequence, or null: all have n_tokens
    int32_t leave_unkept;   // with seq_len: rows of nodes a sequence does not keep are left unwritten, not zero-filled
    int32_t lg;             // log2(n_tokens)
    // dropout on the attention weights: an edge is kept iff its hash >= drop_thr (0: no dropout)
    uint32_t drop_thr, drop_seed;
    float drop_inv_keep;    // 1 / (1 - p)
    int32_t* queue;         // backward workspace: task counters of the key-tile kernel
    int32_t grad_bf16;      // dQ, dK, dV leave rounded to bf16 (the three pointers then address bf16 elements)
    // packed batch on the tile kernels: delta[level][sequence] or null; lse of (bh, node u) at
    // (bh / H) * lse_sb + (bh % H) * lse_sh + row of u
    const int32_t* delta;
    int64_t lse_sb, lse_sh;
};

// ---- dropout on the attention weights ---------------------------------------------------
// Inverted dropout after the softmax (the p_a of the paper's hyper-parameter tables): the weight
// of a kept edge is multiplied by 1/(1-p), that of a dropped one by 0, in the weighted sum of
// values; lse stays that of the full softmax.  The mask is a counter-based hash of (seed,
// batch*heads index, query node, x) with x = relative-position id of the edge for a token row
// and 2^31 + key node for a span row -- both name the edge within its row, and every kernel
// that meets the edge (forward, query side, key side) can form them:
//   keep = mix(mix(mix(seed ^ 0x9E3779B9 * bh) + u) + x) >= floor(p * 2^32).
__device__ __forceinline__ uint32_t mix32(uint32_t z) {
    z ^= z >> 16;
    z *= 0x7FEB352Du;
    z ^= z >> 15;
    z *= 0x846CA68Bu;
    z ^= z >> 16;
    return z;
}
__device__ __forceinline__ uint32_t drop_bh_hash(uint32_t seed, int bh) { return mix32(seed ^ (0x9E3779B9u * (uint32_t)bh)); }
__device__ __forceinline__ uint32_t drop_row_hash(uint32_t bh_hash, int u) { return mix32(bh_hash + (uint32_t)u); }
__device__ __forceinline__ uint32_t drop_edge_x(bool token_row, int rel_id, int key_node) {
    return token_row ? (uint32_t)rel_id : 0x80000000u + (uint32_t)key_node;
}
// multiplier of the edge's weight: 1/(1-p) or 0 (thr == 0: always inv_keep == 1)
__device__ __forceinline__ float drop_scale(uint32_t row_hash, uint32_t x, uint32_t thr, float inv_keep) {
    return mix32(row_hash + x) >= thr ? inv_keep : 0.f;
}

// ---- wave-uniform loads of read-only tables -------------------------------------------
// Graph metadata and sequence lengths are written by no attention kernel, and the tile kernels
// read them at addresses that are the same in all lanes.  Read as scalar loads from the constant
// address space they stay out of the vector-memory queue: vector loads return in order, so a
// wait for such a value issued as a vector load would also wait for every row fetch in flight
// (which is what a software-pipelined loop must not do at each tile boundary).
typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr;
__device__ __forceinline__ int uniform_i32(const int32_t* p, int idx) {
    return reinterpret_cast<const_i32_ptr>(reinterpret_cast<uintptr_t>(p))[__builtin_amdgcn_readfirstlane(idx)];
}

// ---- sequences shorter than n ------------------------------------------------------
// A batch entry with len < n tokens keeps the nodes whose first token exists; an edge counts
// iff both of its nodes are kept.  Rows of nodes that are not kept produce zeros.
__device__ __forceinline__ int seq_length(const int32_t* seq_len, int b, int n) {
    return seq_len ? min(max(seq_len[b], 0), n) : n;
}
// the same for a wave-uniform batch index
__device__ __forceinline__ int seq_length_u(const int32_t* seq_len, int b, int n) {
    return seq_len ? min(max(uniform_i32(seq_len, b), 0), n) : n;
}
// first token of a node of the tree over n = 2^lg tokens (ids are level-major)
__device__ __forceinline__ int node_first_token(int id, int lg) {
    const int x = (2 << lg) - id;                  // (n >> l) < x <= (2n >> l) on level l
    const int level = lg - (31 - __clz(x - 1));
    return (((2 << lg) >> level) - x) << level;
}
// Rows of a packed batch (one graph for a batch of sequences, rows only for kept nodes): node (level l, index m) of
// sequence b is row first_row[l][b] + m, that is its id in the tree over n plus delta[l][b] with
// delta[l][b] = first_row[l][b] - (first id of level l).  The tile kernels keep walking the tree of one sequence
// (ids, tile metadata, lengths) and translate an id only where a row of a caller's tensor is addressed: lane l of a
// wavefront holds delta[l][b] of the sequence it works on (`dvec`), and the level of a node follows from its id.
__device__ __forceinline__ int node_level(int id, int lg) {
    const int x = (2 << lg) - id;                  // (n >> l) < x <= (2n >> l) on level l
    return lg - (31 - __clz(x - 1));
}
__device__ __forceinline__ int load_delta(const int32_t* delta, int nbatch, int b, int lane, int levels) {
    return lane < levels ? delta[lane * nbatch + b] : 0;
}
// the row of node `id` (any lane-varying id); dvec as loaded by load_delta
// (ds_bpermute takes the byte address of the source lane's value; a level is below 64, so no wrap-around is needed)
__device__ __forceinline__ int packed_row(int id, int lg, int dvec) {
    return id + __builtin_amdgcn_ds_bpermute(node_level(id, lg) << 2, dvec);
}
// delta of a level that is the same in all lanes
__device__ __forceinline__ int level_delta(int dvec, int level) {
    return __builtin_amdgcn_readlane(dvec, __builtin_amdgcn_readfirstlane(level));
}

// whether a sequence of `len` tokens keeps `node`.  Without seq_len every row of the graph is a kept node (also
// in the graph of a packed batch, whose rows are not the nodes of one tree).
__device__ __forceinline__ bool node_kept(const AttnArgs& a, int node, int len) {
    return !a.seq_len || node_first_token(node, a.lg) < len;
}
// The walk over (batch*head, tile) gives every XCD a contiguous share.  With sequences of
// different lengths the shares are cut head-major (all batch entries of a head together), so that
// every XCD gets the same mix of lengths instead of a few whole batch entries.
__device__ __forceinline__ int walk_bh(const int32_t* seq_len, int idx, int BH, int H) {
    if (!seq_len) return idx;
    const int B = BH / H;
    return (idx % B) * H + idx / B;
}
// A persistent workgroup steps through the work items with a stride that usually divides the
// number of items per (batch, head), so it would meet the same positions of every sequence -- and a
// workgroup on the late positions would find most of them past the end.  With sequences of different
// lengths the positions are therefore rotated by a different amount for every (batch, head).
__device__ __forceinline__ int walk_pos(const int32_t* seq_len, int slab, int pos, int count) {
    if (!seq_len) return pos;
    // fractional part of slab * golden ratio, scaled to the item count: rotations of consecutive
    // (batch, head)s are spread evenly, so a workgroup's positions cover the sequences evenly
    const unsigned rot = (unsigned)(((unsigned long long)((unsigned)slab * 0x9E3779B1u) * (unsigned)count) >> 32);
    return (int)(((unsigned)pos + rot) % (unsigned)count);
}
constexpr float kLseGone = 1.0e30f;   // stands for lse * log2(e) of a row that is not kept: exp2(s - kLseGone) = 0

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
// the same for 8 bytes that are read once: the non-temporal bit of the cache policy (aux bit 1)
__device__ __forceinline__ float2 buf_f2_once(rsrc_t r, int byte_off) {
    const u32x2 v = __builtin_amdgcn_raw_buffer_load_b64(r, byte_off, 0, 2);
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

// Stores of results that no kernel of this library reads again (out, dQ, dK, dV): marked non-temporal, so
// that the lines do not push the rows the gathers share out of L2 (lm: forward + backward 0.588 -> 0.564 ms).
template <typename T>
__device__ __forceinline__ void store_once(T* p, T v) {
    __builtin_nontemporal_store(v, p);
}
// 16 bytes of a row that a kernel reads once (the backward's own Q, dO and K, V tiles, as opposed to the rows
// it gathers): non-temporal as well (-1 % on the two backward kernels; the forward's Q tile is better off plain)
template <typename V>
__device__ __forceinline__ V load_once16(const void* p) {
    typedef uint32_t vec4 __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(V, __builtin_nontemporal_load(reinterpret_cast<const vec4*>(p)));
}
__device__ __forceinline__ void store_once(float4* p, float4 v) {
    typedef float vec4 __attribute__((ext_vector_type(4)));
    __builtin_nontemporal_store(vec4{v.x, v.y, v.z, v.w}, reinterpret_cast<vec4*>(p));
}
__device__ __forceinline__ void store_once(uint4* p, uint4 v) {
    typedef uint32_t vec4 __attribute__((ext_vector_type(4)));
    __builtin_nontemporal_store(vec4{v.x, v.y, v.z, v.w}, reinterpret_cast<vec4*>(p));
}
// Gradient rows (dQ, dK, dV) leave as fp32 or, on request, rounded to bf16 (round to nearest even): `tensor` is
// the caller's pointer, `elem` an element offset (strides count elements of either type), and with as_bf16 the
// pointer addresses bf16 elements.  as_bf16 is the same in all lanes.
__device__ __forceinline__ void store_grad(float* tensor, int64_t elem, float v, bool as_bf16) {
    if (as_bf16)
        store_once(reinterpret_cast<bf16_t*>(tensor) + elem, (bf16_t)to_bf16_bits(v));
    else
        store_once(tensor + elem, v);
}
// four consecutive elements (elem a multiple of 4)
__device__ __forceinline__ void store_grad4(float* tensor, int64_t elem, float4 v, bool as_bf16) {
    if (as_bf16) {
        typedef uint32_t vec2 __attribute__((ext_vector_type(2)));
        const vec2 w = {to_bf16_bits(v.x) | (to_bf16_bits(v.y) << 16), to_bf16_bits(v.z) | (to_bf16_bits(v.w) << 16)};
        __builtin_nontemporal_store(w, reinterpret_cast<vec2*>(reinterpret_cast<bf16_t*>(tensor) + elem));
    } else {
        store_once(reinterpret_cast<float4*>(tensor + elem), v);
    }
}
__device__ __forceinline__ float4 load_grad4(const float* tensor, int64_t elem, bool as_bf16) {
    if (as_bf16) {
        const uint2 w = *reinterpret_cast<const uint2*>(reinterpret_cast<const bf16_t*>(tensor) + elem);
        return make_float4(__uint_as_float(w.x << 16), __uint_as_float(w.x & 0xFFFF0000u), __uint_as_float(w.y << 16),
                           __uint_as_float(w.y & 0xFFFF0000u));
    }
    return *reinterpret_cast<const float4*>(tensor + elem);
}
__device__ __forceinline__ float load_grad(const float* tensor, int64_t elem, bool as_bf16) {
    return as_bf16 ? __uint_as_float((uint32_t)reinterpret_cast<const bf16_t*>(tensor)[elem] << 16) : tensor[elem];
}

}  // namespace
}  // namespace bpt
