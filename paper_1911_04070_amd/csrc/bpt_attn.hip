// Graph self-attention with tree relative positions (paper Sec. 3.1 eq. (6),
// Sec. 3.4 eq. (8)) forward and backward for gfx950.
//
// Work decomposition.  A row of an adjacency (query node u with its key nodes, or
// key node v with its query nodes) is cut into segments of at most kSeg edges; one
// 64-lane wavefront processes one segment.  Inside the wavefront 8 lanes share one
// edge: each lane holds 8 of the 64 features, so a 128-byte bf16 row is one 16-byte
// load per lane and 8 edges are in flight per wavefront instruction.  Each 8-lane
// group keeps its own online-softmax state; the 8 groups are merged once per
// segment.  Workgroups are persistent: each walks a strided list of tiles inside
// the share of its XCD, so workgroups that run together on one XCD touch
// neighbouring rows and the K/V rows they share stay in that XCD's L2.
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
constexpr int kThreads = 512;            // 8 wavefronts per workgroup (forward, query-side backward)
constexpr int kWaves = kThreads / 64;
constexpr int kThreadsKV = 1024;         // 16 wavefronts share one LDS copy of d_rel (key-side backward)
constexpr int kQPartStride = 132;        // query-side partial: A[64], Bv[64], delta, padding

struct AttnArgs {
    // tensors
    const void *Q, *K, *V, *rel, *dout;
    void* out;
    float* lse_w;
    const float* lse_r;
    float *dQ, *dK, *dV, *d_rel;
    float *delta, *part, *drel_part;
    int64_t sb, sh, sn;
    int32_t BH, H, N, n_tokens;
    float scale;
    // adjacency: ptr[rows+1]; ia = other endpoint (col / t_src); ib = relative-position id
    const int32_t *ptr, *ia, *ib;
    // schedule
    const int32_t *seg_row, *seg_begin, *seg_part, *tile_ptr;
    int32_t num_tiles, num_part;
    int32_t rel_rows_lds;   // rows of the r table staged in LDS (0: read it from global memory)
    int32_t drel_rows_lds;  // rows of d_rel accumulated in LDS (0: global atomics)
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

__device__ __forceinline__ void load8(const float* p, float (&x)[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t* p, float (&x)[8]) {
    const uint4 w = *reinterpret_cast<const uint4*>(p);
    x[0] = __uint_as_float(w.x << 16); x[1] = __uint_as_float(w.x & 0xFFFF0000u);
    x[2] = __uint_as_float(w.y << 16); x[3] = __uint_as_float(w.y & 0xFFFF0000u);
    x[4] = __uint_as_float(w.z << 16); x[5] = __uint_as_float(w.z & 0xFFFF0000u);
    x[6] = __uint_as_float(w.w << 16); x[7] = __uint_as_float(w.w & 0xFFFF0000u);
}
__device__ __forceinline__ void store8(float* p, const float (&x)[8]) {
    *reinterpret_cast<float4*>(p) = make_float4(x[0], x[1], x[2], x[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(x[4], x[5], x[6], x[7]);
}
__device__ __forceinline__ uint32_t to_bf16_bits(float f) {  // round to nearest even
    uint32_t u = __float_as_uint(f);
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
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
    const int slot = lane >> 3, sub = lane & 7;
    const float qscale = a.scale * kLog2e;
    const T* relg = static_cast<const T*>(a.rel);

    for (TileWalk w(a.BH * a.num_tiles); w.t < w.t_end; w.t += w.step) {
        const int bh = w.t / a.num_tiles, tile = w.t - bh * a.num_tiles;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        const T* Qb = static_cast<const T*>(a.Q) + base;
        const T* Kb = static_cast<const T*>(a.K) + base;
        const T* Vb = static_cast<const T*>(a.V) + base;
        const int s1 = a.tile_ptr[tile + 1];
        for (int s = a.tile_ptr[tile] + wave; s < s1; s += kWaves) {
            const int u = a.seg_row[s];
            const int e0 = a.seg_begin[s];
            const int e1 = min(e0 + kSeg, a.ptr[u + 1]);
            const int part = a.seg_part[s];
            const bool span = u >= a.n_tokens;

            float q[8];
            load8(Qb + (int64_t)u * a.sn + sub * 8, q);
#pragma unroll
            for (int i = 0; i < 8; ++i) q[i] *= qscale;
            float shift = 0.f;
            if (span && e1 > e0) {  // r_anc(level) is common to the whole row
                float r[8];
                load8(relg + (int64_t)a.ib[e0] * kD + sub * 8, r);
                float d = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) d += q[i] * r[i];
                shift = sum8(d);
            }

            float m = kNegBig, l = 0.f, acc[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = 0.f;

            for (int eb = e0; eb < e1; eb += 8) {
                const bool valid = eb + slot < e1;
                const int e = valid ? eb + slot : e1 - 1;
                const int c = a.ia[e];
                float kk[8], vv[8];
                load8(Kb + (int64_t)c * a.sn + sub * 8, kk);
                load8(Vb + (int64_t)c * a.sn + sub * 8, vv);
                float d = 0.f;
                if (!span) {
                    const int rid = a.ib[e];
                    float r[8];
                    if (REL_LDS)
                        load8(rel_s + rid * kD + sub * 8, r);
                    else
                        load8(relg + (int64_t)rid * kD + sub * 8, r);
#pragma unroll
                    for (int i = 0; i < 8; ++i) d += q[i] * (kk[i] + r[i]);
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) d += q[i] * kk[i];
                }
                float sc = sum8(d) + shift;
                sc = valid ? sc : kNegBig;
                const float mn = fmaxf(m, sc);
                const float corr = fast_exp2(m - mn);
                const float p = valid ? fast_exp2(sc - mn) : 0.f;
                l = l * corr + p;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = acc[i] * corr + p * vv[i];
                m = mn;
            }
            // merge the 8 groups
#pragma unroll
            for (int mask = 8; mask < 64; mask <<= 1) {
                const float mo = __shfl_xor(m, mask), lo = __shfl_xor(l, mask);
                const float mn = fmaxf(m, mo);
                const float c1 = fast_exp2(m - mn), c2 = fast_exp2(mo - mn);
                l = l * c1 + lo * c2;
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[i] = acc[i] * c1 + __shfl_xor(acc[i], mask) * c2;
                m = mn;
            }
            if (part < 0) {
                const float inv = l > 0.f ? 1.f / l : 0.f;
                if (slot == 0) {
                    float o[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) o[i] = acc[i] * inv;
                    store8(static_cast<T*>(a.out) + base + (int64_t)u * a.sn + sub * 8, o);
                }
                if (lane == 0) a.lse_w[(int64_t)bh * a.N + u] = (m + fast_log2(l)) * kLn2;
            } else {
                float* dst = a.part + ((int64_t)bh * a.num_part + part) * kPartStride;
                if (slot == 0) store8(dst + sub * 8, acc);
                if (lane == 0) {
                    dst[64] = m;
                    dst[65] = l;
                }
            }
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
    const int slot = lane >> 3, sub = lane & 7;
    const float qscale = a.scale * kLog2e;
    const T* relg = static_cast<const T*>(a.rel);

    for (TileWalk w(a.BH * a.num_tiles); w.t < w.t_end; w.t += w.step) {
        const int bh = w.t / a.num_tiles, tile = w.t - bh * a.num_tiles;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        const T* Qb = static_cast<const T*>(a.Q) + base;
        const T* Kb = static_cast<const T*>(a.K) + base;
        const T* Vb = static_cast<const T*>(a.V) + base;
        const T* Gb = static_cast<const T*>(a.dout) + base;
        const int s1 = a.tile_ptr[tile + 1];
        for (int s = a.tile_ptr[tile] + wave; s < s1; s += kWaves) {
            const int u = a.seg_row[s];
            const int e0 = a.seg_begin[s];
            const int e1 = min(e0 + kSeg, a.ptr[u + 1]);
            const int part = a.seg_part[s];
            const bool span = u >= a.n_tokens;

            float qs[8], g[8];
            load8(Qb + (int64_t)u * a.sn + sub * 8, qs);
            load8(Gb + (int64_t)u * a.sn + sub * 8, g);
#pragma unroll
            for (int i = 0; i < 8; ++i) qs[i] *= qscale;
            const float lse2 = a.lse_r[(int64_t)bh * a.N + u] * kLog2e;
            float shift = 0.f;
            if (span && e1 > e0) {
                float r[8], d = 0.f;
                load8(relg + (int64_t)a.ib[e0] * kD + sub * 8, r);
#pragma unroll
                for (int i = 0; i < 8; ++i) d += qs[i] * r[i];
                shift = sum8(d);
            }
            float A[8], Bv[8], dl = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) A[i] = Bv[i] = 0.f;

            for (int eb = e0; eb < e1; eb += 8) {
                const bool valid = eb + slot < e1;
                const int e = valid ? eb + slot : e1 - 1;
                const int c = a.ia[e];
                float kk[8], vv[8];
                load8(Kb + (int64_t)c * a.sn + sub * 8, kk);
                load8(Vb + (int64_t)c * a.sn + sub * 8, vv);
                if (!span) {
                    const int rid = a.ib[e];
                    float r[8];
                    if (REL_LDS)
                        load8(rel_s + rid * kD + sub * 8, r);
                    else
                        load8(relg + (int64_t)rid * kD + sub * 8, r);
#pragma unroll
                    for (int i = 0; i < 8; ++i) kk[i] += r[i];
                }
                float d = 0.f, dp = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    d += qs[i] * kk[i];
                    dp += g[i] * vv[i];
                }
                const float sc = sum8(d) + shift;
                const float dP = sum8(dp);
                const float p = valid ? fast_exp2(sc - lse2) : 0.f;
                const float wgt = p * dP;
                dl += wgt;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    A[i] += wgt * kk[i];
                    Bv[i] += p * kk[i];
                }
            }
#pragma unroll
            for (int mask = 8; mask < 64; mask <<= 1) {
                dl += __shfl_xor(dl, mask);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    A[i] += __shfl_xor(A[i], mask);
                    Bv[i] += __shfl_xor(Bv[i], mask);
                }
            }
            if (part < 0) {
                if (slot == 0) {
#pragma unroll
                    for (int i = 0; i < 8; ++i) A[i] = a.scale * (A[i] - dl * Bv[i]);
                    store8(a.dQ + base + (int64_t)u * a.sn + sub * 8, A);
                }
                if (lane == 0) a.delta[(int64_t)bh * a.N + u] = dl;
            } else {
                float* dst = a.part + ((int64_t)bh * a.num_part + part) * kQPartStride;
                if (slot == 0) {
                    store8(dst + sub * 8, A);
                    store8(dst + kD + sub * 8, Bv);
                }
                if (lane == 0) dst[2 * kD] = dl;
            }
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
    if (lane == 0) a.delta[(int64_t)bh * a.N + u] = dl;
}

// ---- backward, key side: dK, dV and d_rel over the transposed adjacency ---------------
// One wavefront per (segment of a) key node v; its queries u are gathered.  d_rel is
// accumulated here because q_u and the exact dS_e are both at hand: each 8-lane group
// sums the contributions of consecutive edges that share a relative-position id in
// registers (for a coarse span the id changes only every 2^level queries) and adds
// the run to the workgroup's LDS copy of d_rel with ds_add_f32; the copies are
// summed by drel_reduce_kernel.  Edges whose query is a span carry r_anc, whose
// gradient is zero, and are skipped.
template <typename T, bool REL_LDS, bool DREL_LDS>
__device__ __forceinline__ void flush_run(const AttnArgs& a, float* drel_s, int id, int sub, float (&dr)[8]) {
    float* dst = (DREL_LDS ? drel_s : a.d_rel) + (int64_t)id * kD + sub * 8;
#pragma unroll
    for (int i = 0; i < 8; ++i) atomicAdd(dst + i, dr[i] * a.scale);
}

template <typename T, bool REL_LDS, bool DREL_LDS>
__global__ void __launch_bounds__(kThreadsKV) bwd_kv_kernel(const AttnArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    T* rel_s = reinterpret_cast<T*>(smem);
    float* drel_s = reinterpret_cast<float*>(smem + (REL_LDS ? (size_t)a.rel_rows_lds * kD * sizeof(T) : 0));
    if (REL_LDS) stage_table(rel_s, static_cast<const T*>(a.rel), a.rel_rows_lds * kD);
    if (DREL_LDS)
        for (int i = threadIdx.x; i < a.drel_rows_lds * kD; i += blockDim.x) drel_s[i] = 0.f;
    if (REL_LDS || DREL_LDS) __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = blockDim.x >> 6;
    const int slot = lane >> 3, sub = lane & 7;
    const float qscale = a.scale * kLog2e;
    const T* relg = static_cast<const T*>(a.rel);

    for (TileWalk w(a.BH * a.num_tiles); w.t < w.t_end; w.t += w.step) {
        const int bh = w.t / a.num_tiles, tile = w.t - bh * a.num_tiles;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        const T* Qb = static_cast<const T*>(a.Q) + base;
        const T* Kb = static_cast<const T*>(a.K) + base;
        const T* Vb = static_cast<const T*>(a.V) + base;
        const T* Gb = static_cast<const T*>(a.dout) + base;
        const float* lse_b = a.lse_r + (int64_t)bh * a.N;
        const float* delta_b = a.delta + (int64_t)bh * a.N;
        const int s1 = a.tile_ptr[tile + 1];
        for (int s = a.tile_ptr[tile] + wave; s < s1; s += nwaves) {
            const int v = a.seg_row[s];
            const int e0 = a.seg_begin[s];
            const int e1 = min(e0 + kSeg, a.ptr[v + 1]);
            const int part = a.seg_part[s];

            float kk[8], vv[8], dk[8], dv[8], dr[8];
            load8(Kb + (int64_t)v * a.sn + sub * 8, kk);
            load8(Vb + (int64_t)v * a.sn + sub * 8, vv);
#pragma unroll
            for (int i = 0; i < 8; ++i) dk[i] = dv[i] = dr[i] = 0.f;
            int cur = -1;

            for (int eb = e0; eb < e1; eb += 8) {
                const bool valid = eb + slot < e1;
                const int e = valid ? eb + slot : e1 - 1;
                const int u = a.ia[e];
                const int rid = a.ib[e];
                float q[8], g[8], r[8];
                load8(Qb + (int64_t)u * a.sn + sub * 8, q);
                load8(Gb + (int64_t)u * a.sn + sub * 8, g);
                const float lse2 = lse_b[u] * kLog2e;
                const float delta = delta_b[u];
                if (REL_LDS)
                    load8(rel_s + rid * kD + sub * 8, r);
                else
                    load8(relg + (int64_t)rid * kD + sub * 8, r);
                float d = 0.f, dp = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    d += q[i] * (kk[i] + r[i]);
                    dp += g[i] * vv[i];
                }
                const float sc = sum8(d) * qscale;
                const float dP = sum8(dp);
                const float p = valid ? fast_exp2(sc - lse2) : 0.f;
                const float dS = p * (dP - delta);
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    dk[i] += dS * q[i];
                    dv[i] += p * g[i];
                }
                if (valid && u < a.n_tokens) {
                    if (rid != cur) {
                        if (cur >= 0) flush_run<T, REL_LDS, DREL_LDS>(a, drel_s, cur, sub, dr);
                        cur = rid;
#pragma unroll
                        for (int i = 0; i < 8; ++i) dr[i] = 0.f;
                    }
#pragma unroll
                    for (int i = 0; i < 8; ++i) dr[i] += dS * q[i];
                }
            }
            if (cur >= 0) flush_run<T, REL_LDS, DREL_LDS>(a, drel_s, cur, sub, dr);
#pragma unroll
            for (int mask = 8; mask < 64; mask <<= 1) {
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    dk[i] += __shfl_xor(dk[i], mask);
                    dv[i] += __shfl_xor(dv[i], mask);
                }
            }
            if (slot == 0) {
#pragma unroll
                for (int i = 0; i < 8; ++i) dk[i] *= a.scale;
                if (part < 0) {
                    store8(a.dK + base + (int64_t)v * a.sn + sub * 8, dk);
                    store8(a.dV + base + (int64_t)v * a.sn + sub * 8, dv);
                } else {
                    float* dst = a.part + ((int64_t)bh * a.num_part + part) * (2 * kD);
                    store8(dst + sub * 8, dk);
                    store8(dst + kD + sub * 8, dv);
                }
            }
        }
    }
    if (DREL_LDS) {
        __syncthreads();
        float* dst = a.drel_part + (int64_t)blockIdx.x * a.drel_rows_lds * kD;
        for (int i = threadIdx.x; i < a.drel_rows_lds * kD; i += blockDim.x) dst[i] = drel_s[i];
    }
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

// d_rel = sum of the workgroups' LDS copies (rows the copies do not cover are zero)
__global__ void drel_reduce_kernel(const float* __restrict__ parts, int num_parts, int lds_elems,
                                   float* __restrict__ d_rel, int total_elems) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= total_elems) return;
    float acc = 0.f;
    if (i < lds_elems)
        for (int p = 0; p < num_parts; ++p) acc += parts[(int64_t)p * lds_elems + i];
    d_rel[i] = acc;
}

__global__ void fill_zero_kernel(float* __restrict__ p, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0.f;
}

// ---- host side --------------------------------------------------------------------
constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct DeviceLimits {
    int cus = 0;
    size_t lds = 0;
};

int device_limits(const bpt_graph* g, DeviceLimits* out) {
    int lds = 0;
    BPT_HIP(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, g->device));
    out->cus = g->num_cus > 0 ? g->num_cus : 256;
    out->lds = lds > 0 ? (size_t)lds : 65536;
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
    return BPT_OK;
}

inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline size_t elem_size(const bpt_shape_t* s) { return s->dtype == BPT_BF16 ? 2 : 4; }

// Resident workgroups per CU for a persistent launch, from the runtime's occupancy
// calculator; the grid is that times the CU count, rounded down to a multiple of 8
// (one share of the tile space per XCD).
template <typename K>
int persistent_grid(K kernel, int threads, size_t lds, const DeviceLimits& lim, int* grid) {
    if (lds > 65536)
        BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)lds));
    int per_cu = 0;
    BPT_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, lds));
    per_cu = std::max(1, per_cu);
    *grid = std::max(8, lim.cus * per_cu / 8 * 8);
    return BPT_OK;
}

template <typename K>
int launch(K kernel, int grid, int threads, size_t lds, hipStream_t st, const AttnArgs& a) {
    hipLaunchKernelGGL(kernel, dim3(grid), dim3(threads), lds, st, a);
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
}

void use_schedule(AttnArgs& a, const Schedule& sc) {
    a.seg_row = sc.seg_row;
    a.seg_begin = sc.seg_begin;
    a.seg_part = sc.seg_part;
    a.tile_ptr = sc.tile_ptr;
    a.num_tiles = sc.num_tiles;
    a.num_part = sc.num_part;
}

template <typename T>
int run_fwd(const bpt_graph* g, AttnArgs& a, hipStream_t st) {
    DeviceLimits lim;
    int rc = device_limits(g, &lim);
    if (rc) return rc;
    const int ctx_rows = g->ctx_levels * g->rel_width;
    const size_t rel_b = (size_t)ctx_rows * kD * sizeof(T);
    const bool rel_lds = rel_b <= lim.lds;
    a.rel_rows_lds = rel_lds ? ctx_rows : 0;
    const size_t lds = rel_lds ? rel_b : 0;
    int grid = 8;
    if (rel_lds) {
        if ((rc = persistent_grid(fwd_kernel<T, true>, kThreads, lds, lim, &grid))) return rc;
        rc = launch(fwd_kernel<T, true>, grid, kThreads, lds, st, a);
    } else {
        if ((rc = persistent_grid(fwd_kernel<T, false>, kThreads, 0, lim, &grid))) return rc;
        rc = launch(fwd_kernel<T, false>, grid, kThreads, 0, st, a);
    }
    if (rc) return rc;
    if (g->fwd.num_multi > 0) {
        const int items = a.BH * g->fwd.num_multi;
        hipLaunchKernelGGL(fwd_merge_kernel<T>, dim3((items + 3) / 4), dim3(256), 0, st, a, g->fwd.multi_row,
                           g->fwd.multi_ptr, g->fwd.num_multi);
        BPT_HIP(hipGetLastError());
    }
    return BPT_OK;
}

// Workspace layout and LDS use of the backward.
struct BwdPlan {
    int rel_rows_kv = 0, drel_rows_kv = 0;  // LDS rows of the key-side kernel (0: global memory)
    size_t lds_kv = 0;
    int grid_kv = 8;
    size_t off_delta = 0, off_qpart = 0, off_kvpart = 0, off_drel = 0, total = 0;
};

int plan_bwd(const bpt_graph* g, const bpt_shape_t* s, BwdPlan* p) {
    DeviceLimits lim;
    int rc = device_limits(g, &lim);
    if (rc) return rc;
    const size_t es = elem_size(s);
    const int ctx_rows = g->ctx_levels * g->rel_width;
    const int all_rows = g->num_levels * g->rel_width;
    const size_t rel_b = (size_t)all_rows * kD * es, drel_b = (size_t)ctx_rows * kD * sizeof(float);
    if (rel_b + drel_b <= lim.lds) {
        p->rel_rows_kv = all_rows;
        p->drel_rows_kv = ctx_rows;
        p->lds_kv = rel_b + drel_b;
    } else if (drel_b <= lim.lds) {
        p->drel_rows_kv = ctx_rows;
        p->lds_kv = drel_b;
    } else if (rel_b <= lim.lds) {
        p->rel_rows_kv = all_rows;
        p->lds_kv = rel_b;
    }
    p->grid_kv = std::max(8, lim.cus / 8 * 8);  // one 16-wavefront workgroup per CU
    const size_t bh = (size_t)s->B * s->H;
    size_t off = 0;
    p->off_delta = off;
    off += align_up(bh * g->num_nodes * sizeof(float));
    p->off_qpart = off;
    off += align_up(bh * g->fwd.num_part * kQPartStride * sizeof(float));
    p->off_kvpart = off;
    off += align_up(bh * g->tr.num_part * 2 * kD * sizeof(float));
    p->off_drel = off;
    off += align_up((size_t)p->grid_kv * p->drel_rows_kv * kD * sizeof(float));
    p->total = off;
    return BPT_OK;
}

template <typename T>
int run_bwd_q(const bpt_graph* g, AttnArgs& a, hipStream_t st) {
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
    int grid = 8;
    if (rel_lds) {
        if ((rc = persistent_grid(bwd_q_kernel<T, true>, kThreads, rel_b, lim, &grid))) return rc;
        rc = launch(bwd_q_kernel<T, true>, grid, kThreads, rel_b, st, a);
    } else {
        if ((rc = persistent_grid(bwd_q_kernel<T, false>, kThreads, 0, lim, &grid))) return rc;
        rc = launch(bwd_q_kernel<T, false>, grid, kThreads, 0, st, a);
    }
    if (rc) return rc;
    if (g->fwd.num_multi > 0) {
        const int items = a.BH * g->fwd.num_multi;
        hipLaunchKernelGGL(bwd_q_merge_kernel, dim3((items + 3) / 4), dim3(256), 0, st, a, g->fwd.multi_row,
                           g->fwd.multi_ptr, g->fwd.num_multi);
        BPT_HIP(hipGetLastError());
    }
    return BPT_OK;
}

template <typename T, bool REL_LDS, bool DREL_LDS>
int launch_kv(const BwdPlan& p, hipStream_t st, const AttnArgs& a) {
    if (p.lds_kv > 65536)
        BPT_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(bwd_kv_kernel<T, REL_LDS, DREL_LDS>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds_kv));
    return launch(bwd_kv_kernel<T, REL_LDS, DREL_LDS>, p.grid_kv, kThreadsKV, p.lds_kv, st, a);
}

template <typename T>
int run_bwd_kv(const bpt_graph* g, const BwdPlan& p, AttnArgs& a, hipStream_t st) {
    a.ptr = g->t_ptr;
    a.ia = g->t_src;
    a.ib = g->t_rel;
    use_schedule(a, g->tr);
    a.rel_rows_lds = p.rel_rows_kv;
    a.drel_rows_lds = p.drel_rows_kv;
    const int rel_elems = a.rel_rows * kD;
    int rc;
    if (p.drel_rows_kv == 0) {  // global atomics accumulate into d_rel itself
        hipLaunchKernelGGL(fill_zero_kernel, dim3((rel_elems + 255) / 256), dim3(256), 0, st, a.d_rel, rel_elems);
        BPT_HIP(hipGetLastError());
    }
    if (p.rel_rows_kv && p.drel_rows_kv)
        rc = launch_kv<T, true, true>(p, st, a);
    else if (p.drel_rows_kv)
        rc = launch_kv<T, false, true>(p, st, a);
    else if (p.rel_rows_kv)
        rc = launch_kv<T, true, false>(p, st, a);
    else
        rc = launch_kv<T, false, false>(p, st, a);
    if (rc) return rc;
    if (p.drel_rows_kv) {
        hipLaunchKernelGGL(drel_reduce_kernel, dim3((rel_elems + 255) / 256), dim3(256), 0, st, a.drel_part, p.grid_kv,
                           p.drel_rows_kv * kD, a.d_rel, rel_elems);
        BPT_HIP(hipGetLastError());
    }
    if (g->tr.num_multi > 0) {
        const int items = a.BH * g->tr.num_multi;
        hipLaunchKernelGGL(bwd_kv_merge_kernel, dim3((items + 3) / 4), dim3(256), 0, st, a, g->tr.multi_row,
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
    if ((stages & kStageQ) && !dQ) return BPT_ERR_INVALID_ARG;
    if ((stages & kStageKV) && (!dK || !dV || !d_rel)) return BPT_ERR_INVALID_ARG;
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
    a.delta = reinterpret_cast<float*>(ws + p.off_delta);
    a.drel_part = reinterpret_cast<float*>(ws + p.off_drel);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = s->dtype == BPT_BF16;
    if (stages & kStageQ) {
        a.part = reinterpret_cast<float*>(ws + p.off_qpart);
        if ((rc = bf ? run_bwd_q<bf16_t>(g, a, st) : run_bwd_q<float>(g, a, st))) return rc;
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
    return bpt::align_up((size_t)s->B * s->H * g->fwd.num_part * bpt::kPartStride * sizeof(float));
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
                            const void* rel, const float* lse, const void* dout, float* dQ, void* workspace,
                            size_t workspace_bytes, void* stream) {
    return bpt::backward(g, s, Q, K, V, rel, lse, dout, dQ, nullptr, nullptr, nullptr, workspace, workspace_bytes,
                         stream, bpt::kStageQ);
}

int bpt_attn_bwd_key_side(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K, const void* V,
                          const void* rel, const float* lse, const void* dout, float* dK, float* dV, float* d_rel,
                          void* workspace, size_t workspace_bytes, void* stream) {
    return bpt::backward(g, s, Q, K, V, rel, lse, dout, nullptr, dK, dV, d_rel, workspace, workspace_bytes, stream,
                         bpt::kStageKV);
}

}  // extern "C"
