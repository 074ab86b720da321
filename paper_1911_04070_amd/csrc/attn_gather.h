// Gather kernels (vector ALU): forward, query side and key side of the backward over CSR /
// transposed adjacency, and the dense d_rel contractions that read the CSR.  fp32 tensors and fallback.
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
#pragma once

#include "attn_device.h"

namespace bpt {
namespace {

// ---- forward --------------------------------------------------------------------
// One segment [e0, e1) of row u (e1 > e0).  SPAN: the row is a span node.
template <typename T, bool REL_LDS, bool SPAN>
__device__ __forceinline__ void fwd_segment(const AttnArgs& a, const T* rel_s, rsrc_t rK, rsrc_t rV, rsrc_t rIa,
                                            rsrc_t rIb, int bh, int64_t base, int u, int e0, int e1, int part,
                                            int lane, int len) {
    const int slot = lane >> 3, sub = lane & 7;
    const int lane_off = sub * 8 * (int)sizeof(T);
    const T* relg = static_cast<const T*>(a.rel) + sub * 8;
    const bool row_kept = node_kept(a, u, len);
    const uint32_t rowh = drop_row_hash(drop_bh_hash(a.drop_seed, bh), u);

    // indices two iterations ahead, rows one iteration ahead.  Lanes past the end of
    // the segment read the next rows' indices (or 0 past the array): valid nodes,
    // and their contribution is masked.
    int eo = (e0 + slot) * 4;
    const int c0 = buf_i32(rIa, eo);
    int cnow = c0;   // key node of the rows in work
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

        const bool valid = eb + slot < e1 && row_kept && node_kept(a, cnow, len);
        const float keep = a.drop_thr ? drop_scale(rowh, drop_edge_x(!SPAN, r0, cnow), a.drop_thr, a.drop_inv_keep) : 1.f;
        cnow = c1;
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
        const float pk = p * keep;   // dropout acts on the weighted sum only
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            acc[i] *= corr;
            acc[i] = fmaf(pk, vv[i], acc[i]);
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
        if (lane == 0) a.lse_w[(int64_t)bh * a.N + u] = l > 0.f ? (mall + fast_log2(l)) * kLn2 : 0.f;
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
                                          int deg, int lane, int len) {
    const int slot = lane >> 3, sub = lane & 7;
    const int lane_off = sub * 8 * (int)sizeof(T);
    const int u = u0 + slot;
    const int tok0 = a.ia[e0 + slot * deg];  // first token of this group's span
    Row<T> k0 = gather_row<T>(rK, tok0, a.row_bytes, lane_off), v0 = gather_row<T>(rV, tok0, a.row_bytes, lane_off);
    const Row<T> q = load_row(static_cast<const T*>(a.Q) + base + (int64_t)u * a.sn + sub * 8);
    const float qscale = a.scale * kLog2e;
    const float shift =
        sum8(dot8(q, load_row(static_cast<const T*>(a.rel) + (int64_t)a.ib[e0] * kD + sub * 8), 0.f)) * qscale;
    const uint32_t rowh = drop_row_hash(drop_bh_hash(a.drop_seed, bh), u);
    float m = kNegBig, l = 0.f, acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[i] = 0.f;
    auto step = [&](int i, const Row<T>& kc, const Row<T>& vc, Row<T>& kn, Row<T>& vn) {
        const int nxt = tok0 + min(i + 1, deg - 1);
        kn = gather_row<T>(rK, nxt, a.row_bytes, lane_off);
        vn = gather_row<T>(rV, nxt, a.row_bytes, lane_off);
        const bool valid = tok0 + i < len;
        const float sc = valid ? sum8(dot8(q, kc, 0.f)) * qscale + shift : kNegBig;
        const bool up = sc > m;
        const float e = fast_exp2(up ? m - sc : sc - m);
        const float corr = up ? e : 1.f, p = valid ? (up ? 1.f : e) : 0.f;
        m = up ? sc : m;
        float vv[8];
        unpack(vc, vv);
        l *= corr;
        l += p;
        const float pk = a.drop_thr ? p * drop_scale(rowh, drop_edge_x(false, 0, tok0 + i), a.drop_thr, a.drop_inv_keep) : p;
#pragma unroll
        for (int x = 0; x < 8; ++x) {
            acc[x] *= corr;
            acc[x] = fmaf(pk, vv[x], acc[x]);
        }
    };
    Row<T> k1, v1;
    for (int i = 0; i < deg; i += 2) {  // deg is a power of two >= 2
        step(i, k0, v0, k1, v1);
        step(i + 1, k1, v1, k0, v0);
    }
    const float inv = l > 0.f ? 1.f / l : 0.f;   // l == 0: a span past the end of a shorter sequence
#pragma unroll
    for (int x = 0; x < 8; ++x) acc[x] *= inv;
    store8(static_cast<T*>(a.out) + base + (int64_t)u * a.sn + sub * 8, acc);
    if (sub == 0) a.lse_w[(int64_t)bh * a.N + u] = l > 0.f ? (m + fast_log2(l)) * kLn2 : 0.f;
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
        const int len = seq_length(a.seq_len, bh / a.H, a.n_tokens);
        const int s1 = a.tile_ptr[tile + 1];
        for (int s = a.tile_ptr[tile] + wave; s < s1; s += nwaves) {
            const int u = a.seg_row[s];
            const int e0 = a.seg_begin[s];
            const int e1 = min(e0 + kSeg, a.ptr[u + 1]);
            const int part = a.seg_part[s];
            if (e1 <= e0) continue;  // no row of this adjacency is empty
            if (part == kPartSpan8)
                fwd_span8<T>(a, rK, rV, bh, base, u, e0, a.ptr[u + 1] - e0, lane, len);
            else if (u >= a.n_tokens)
                fwd_segment<T, REL_LDS, true>(a, rel_s, rK, rV, rIa, rIb, bh, base, u, e0, e1, part, lane, len);
            else
                fwd_segment<T, REL_LDS, false>(a, rel_s, rK, rV, rIa, rIb, bh, base, u, e0, e1, part, lane, len);
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
    if (lane == 0) a.lse_w[(int64_t)bh * a.N + u] = l > 0.f ? (m + fast_log2(l)) * kLn2 : 0.f;
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
                                              int lane, int len) {
    const int slot = lane >> 3, sub = lane & 7;
    const int lane_off = sub * 8 * (int)sizeof(T);
    const T* relg = static_cast<const T*>(a.rel) + sub * 8;
    const bool row_kept = node_kept(a, u, len);
    const uint32_t rowh = drop_row_hash(drop_bh_hash(a.drop_seed, bh), u);

    int eo = (e0 + slot) * 4;
    const int c0 = buf_i32(rIa, eo);
    int cnow = c0;   // key node of the rows in work
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

        const bool inside = eb + slot < e1;
        const bool valid = inside && row_kept && node_kept(a, cnow, len);
        const float keep = a.drop_thr ? drop_scale(rowh, drop_edge_x(!SPAN, r0, cnow), a.drop_thr, a.drop_inv_keep) : 1.f;
        cnow = c1;
        float kk[8];
        unpack(kc, kk);
        if (!SPAN) {
            float r[8];
            const int rid = inside ? r0 : 0;  // a lane past the end may hold an id of some other row
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
        const float dP = sum8(dot8(g, vc, 0.f)) * keep;   // out = sum keep p v: dP carries the mask
        const float p = valid ? fast_exp2(sc - lse2) : 0.f;
        const float wgt = p * dP;
        dl += wgt;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            A[i] = fmaf(wgt, kk[i], A[i]);
            Bv[i] = fmaf(p, kk[i], Bv[i]);
        }
        // what d_rel needs of this edge (dS_e = w_e - delta_u p_e once delta_u is known)
        if (!SPAN && inside && sub == 0) a.wp[(int64_t)bh * a.e_tok + (eo >> 2)] = make_float2(wgt, p);
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
        store_grad(a.dQ, base + (int64_t)u * a.sn + col, a.scale * reduce_slots8(A, lane), a.grad_bf16);
        if (lane == 0) a.stat[(int64_t)bh * a.N + u] = make_float2(row_kept ? lse2 : kLseGone, dl);
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
                                            int e0, int deg, int lane, int len) {
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
    const uint32_t rowh = drop_row_hash(drop_bh_hash(a.drop_seed, bh), u);
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
        const float p = tok0 + i < len ? fast_exp2(sum8(d) + shift - lse2) : 0.f;
        const float keep = a.drop_thr ? drop_scale(rowh, drop_edge_x(false, 0, tok0 + i), a.drop_thr, a.drop_inv_keep) : 1.f;
        const float wgt = p * sum8(dot8(g, vc, 0.f)) * keep;
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
    store_grad4(a.dQ, base + (int64_t)u * a.sn + sub * 8, make_float4(A[0], A[1], A[2], A[3]), a.grad_bf16);
    store_grad4(a.dQ, base + (int64_t)u * a.sn + sub * 8 + 4, make_float4(A[4], A[5], A[6], A[7]), a.grad_bf16);
    if (sub == 0) a.stat[(int64_t)bh * a.N + u] = make_float2(tok0 < len ? lse2 : kLseGone, dl);
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
        const int len = seq_length(a.seq_len, bh / a.H, a.n_tokens);
        const int s1 = a.tile_ptr[tile + 1];
        for (int s = a.tile_ptr[tile] + wave; s < s1; s += nwaves) {
            const int u = a.seg_row[s];
            const int e0 = a.seg_begin[s];
            const int e1 = min(e0 + kSeg, a.ptr[u + 1]);
            const int part = a.seg_part[s];
            if (e1 <= e0) continue;
            if (part == kPartSpan8)
                bwd_q_span8<T>(a, rK, rV, bh, base, u, e0, a.ptr[u + 1] - e0, lane, len);
            else if (u >= a.n_tokens)
                bwd_q_segment<T, REL_LDS, true>(a, rel_s, rK, rV, rIa, rIb, bh, base, u, e0, e1, part, lane, len);
            else
                bwd_q_segment<T, REL_LDS, false>(a, rel_s, rK, rV, rIa, rIb, bh, base, u, e0, e1, part, lane, len);
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
    store_grad(a.dQ, base + (int64_t)u * a.sn + lane, a.scale * (sa - dl * sb), a.grad_bf16);
    const bool kept = node_kept(a, u, seq_length(a.seq_len, bh / a.H, a.n_tokens));
    if (lane == 0) a.stat[(int64_t)bh * a.N + u] = make_float2(kept ? a.lse_r[(int64_t)bh * a.N + u] * kLog2e : kLseGone, dl);
}

// ---- backward, key side: dK, dV over the transposed adjacency -------------------------
// One wavefront per (segment of a) key node v; the rows q_u, dout_u and the pair
// (lse_u, delta_u) of its queries u are gathered.  No atomics: every key row is
// reduced by one wavefront (or by the merge kernel, in segment order).
template <typename T, bool REL_LDS>
__device__ __forceinline__ void bwd_kv_segment(const AttnArgs& a, const T* rel_s, rsrc_t rQ, rsrc_t rG, rsrc_t rS,
                                               rsrc_t rIa, rsrc_t rIb, int bh, int64_t base, int v, int e0, int e1,
                                               int part, int lane, int len) {
    const int slot = lane >> 3, sub = lane & 7;
    const int lane_off = sub * 8 * (int)sizeof(T);
    const T* relg = static_cast<const T*>(a.rel) + sub * 8;
    const float qscale = a.scale * kLog2e;

    float dk[8], dv[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) dk[i] = dv[i] = 0.f;

    // queries that are not kept carry kLseGone in `stat`; a key that is not kept has no edge at all
    if (e1 > e0 && node_kept(a, v, len)) {
        int eo = (e0 + slot) * 4;
        const int u0 = buf_i32(rIa, eo);
        int unow = u0;   // query node of the rows in work
        const uint32_t bhh = drop_bh_hash(a.drop_seed, bh);
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
            const float keep = a.drop_thr ? drop_scale(drop_row_hash(bhh, unow), drop_edge_x(unow < a.n_tokens, r0, v), a.drop_thr,
                                                       a.drop_inv_keep)
                                          : 1.f;
            unow = u1;
            const float dP = sum8(dot8(gc, vv, 0.f)) * keep;
            unpack(qc, q);
            unpack(gc, g);
            const float p = valid ? fast_exp2(sc - stc.x) : 0.f;
            const float dS = p * (dP - stc.y);
            const float pk = p * keep;
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                dk[i] = fmaf(dS, q[i], dk[i]);
                dv[i] = fmaf(pk, g[i], dv[i]);
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
        store_grad(a.dK, base + (int64_t)v * a.sn + col, tk * a.scale, a.grad_bf16);
        store_grad(a.dV, base + (int64_t)v * a.sn + col, tv, a.grad_bf16);
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
            bwd_kv_segment<T, REL_LDS>(a, rel_s, rQ, rG, rS, rIa, rIb, bh, base, v, e0, e1, a.seg_part[s], lane,
                                       seq_length(a.seq_len, bh / a.H, a.n_tokens));
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
    const int blocks_per_bh = (a.n_tokens + R - 1) / R;   // the last block of a batch graph may be short
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
                if (row0 + r < a.n_tokens) {
                    load8(Qb + (int64_t)(row0 + r) * a.sn + c, x);
                } else {
#pragma unroll
                    for (int j = 0; j < 8; ++j) x[j] = 0.f;
                }
#pragma unroll
                for (int j = 0; j < 8; ++j) q_s[r * kD + c + j] = x[j];
            }
        }
        __syncthreads();
        // scatter dS of every edge of the block's rows: one wavefront per row, lanes over edges
        const float2* wp_b = a.wp + (int64_t)bh * a.e_tok;
        for (int r = wave; r < R && row0 + r < a.n_tokens; r += kWaves) {
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

}  // namespace
}  // namespace bpt
