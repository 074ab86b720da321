// Matrix-core key side of the backward over dense tiles of key nodes (bf16), its merges, and
// the fixed-order reduction of the d_rel copies.
#pragma once

#include "attn_token_tiles.h"

namespace bpt {
namespace {

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
constexpr int kMaxBiasChunks = 10;   // 16-id chunks of the table a key tile can meet (W + levels - 1 ids <= 160)
constexpr int kKvOutStride = 2 * kD + 4;   // floats per key row of the output staging in LDS (528 bytes)
constexpr int kRegBiasChunks = 6;    // of which this many are register operands; the others are parked in LDS
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
    const int32_t *task_ntiles, *chunk_ptr;   // chained tasks: tiles the task walks, first chunk of every tile
    const int16_t* map;
    int32_t num_tasks, num_part, num_chunks, nb_pad, W, zero;
    const int32_t* seq_len;   // [B] tokens of every sequence, or null
    int32_t leave_unkept;     // rows of nodes a shorter sequence does not keep: left unwritten instead of zero-filled
    int32_t grad_bf16;        // dK, dV leave rounded to bf16
    const int32_t* delta;     // packed batch: delta[level][sequence] (see attn_device.h), or null
    int32_t n;
    uint32_t drop_thr, drop_seed;   // dropout on the attention weights (DROP variants)
    float drop_inv_keep;
    // 8 task counters (one per XCD, 64 bytes apart), zero when the kernel starts: cleared by the last kernel
    // of the query side when both sides run in one call, else by zero_ints_kernel
    int32_t* queue;
};

// `count` ints = 0 (a fill kernel, so that the call can be captured in a graph)
__global__ void zero_ints_kernel(int32_t* p, int count) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0;
}

// PACKED: the rows of the caller's tensors are those of a packed batch (KeyArgs.delta; see attn_device.h)
template <int NBC, bool DROP, bool PACKED = false>
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
    // table operands beyond the kRegBiasChunks kept in registers: every lane parks and re-reads its own 32 bytes
    constexpr int kParked = NBC > kRegBiasChunks ? NBC - kRegBiasChunks : 0;
    // DROP: hash of (seed, batch*head, query node) of the 32 queries, what the mask of their edges is drawn from
    uint32_t* rowh_s = reinterpret_cast<uint32_t*>(smem + (size_t)kTileWaves * (32 * bstride * sizeof(float) +
                                                                                64 * kRowStride * sizeof(bf16_t) +
                                                                                32 * sizeof(float2))) +
                       (size_t)wave * 32;
    uint4* rb_s = reinterpret_cast<uint4*>(smem + (size_t)kTileWaves * (32 * bstride * sizeof(float) +
                                                                        64 * kRowStride * sizeof(bf16_t) + 32 * sizeof(float2) +
                                                                        32 * sizeof(uint32_t))) +
                  ((size_t)wave * (kParked > 0 ? kParked : 1) * 64 + lane) * 2;
    const float qscale = a.scale * kLog2e;
    // The (batch*head, task) space is split into 8 contiguous shares, one per XCD (workgroup w runs on
    // XCD w mod 8).  The wavefronts of an XCD take the tasks of its share in order from a shared counter:
    // tasks differ 16-fold in length, and with a fixed assignment the wavefronts drift apart until the XCD
    // works on many (batch, head)s at once and their rows push each other out of its L2.  Taken in order,
    // the wavefronts stay within a few hundred consecutive tasks.  Which wavefront computes a task changes
    // no result.
    const int xcd = blockIdx.x & 7;
    const int total = a.BH * a.num_tasks, per = (total + 7) >> 3;
    const int share_begin = xcd * per, share_end = min(total, share_begin + per);
    const rsrc_t rC = make_rsrc(a.cols, (uint32_t)a.num_chunks * 64u);    // [chunks][16] int32
    const rsrc_t rM = make_rsrc(a.map, (uint32_t)a.num_chunks * 512u);    // [chunks][16][16] int16

    for (;;) {
        int item = 0;
        if (lane == 0) item = atomicAdd(a.queue + xcd * 16, 1);
        item = __builtin_amdgcn_readfirstlane(item) + share_begin;
        // every wavefront gets here: the counter only grows from zero
        if (item >= share_end) break;
        const int slab = item / a.num_tasks;
        const int bh = walk_bh(a.seq_len, slab, a.BH, a.H);
        const int task = item - slab * a.num_tasks;
        const int kt = uniform_i32(a.task_tile, task), c0 = uniform_i32(a.task_c0, task), part = uniform_i32(a.task_part, task);
        const int node0 = uniform_i32(a.tile_node0, kt), info = uniform_i32(a.tile_info, kt);
        const int level = info & 255, nkeys = info >> 8;
        // a shorter sequence keeps the first ceil(len / 2^level) nodes of the level; queries that are
        // not kept carry kLseGone in `stat`
        const int len = seq_length_u(a.seq_len, bh / a.H, a.n);
        const int kept_keys = ((len + (1 << level) - 1) >> level) - (node0 - (2 * a.n - ((2 * a.n) >> level)));
        const bool key_kept = j < kept_keys;
        const int nch = uniform_i32(a.task_nch, task);
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        // wave-uniform: no key of the tile exists in this sequence; kv_tile_merge_kernel writes the zero rows
        if (kept_keys <= 0) continue;
        const rsrc_t rQ = make_rsrc(a.Q + base, a.slab_bytes), rG = make_rsrc(a.dout + base, a.slab_bytes);
        const rsrc_t rS = make_rsrc(a.stat + (int64_t)bh * a.N, (uint32_t)a.N * 8u);
        // packed batch: rows of the caller's tensors are node ids moved by the sequence's delta of the node's level
        // (`stat` is workspace and stays indexed by node id); keys the sequence does not keep have no row
        const int dvec = PACKED ? load_delta(a.delta, a.BH / a.H, bh / a.H, lane, a.num_levels) : 0;
        const int dlev = PACKED ? level_delta(dvec, level) : 0;
        const int nstore = PACKED ? min(nkeys, kept_keys) : nkeys;

        // Software pipeline over pairs of chunks.  `Idx` = what has to be known before a pair's
        // rows can be requested (its column ids and map words); the rows of pair i+1 are
        // requested in the middle of pair i, as soon as the registers of pair i's rows are free,
        // and the ids of pair i+2 right after, so the gathers overlap the second products.
        // the 32 query nodes of a pair arrive with one instruction, node l in lane l (and l + 32); the lane that
        // fetches a piece of row 16 ci + 8 h + r8 reads its id from there, and lane l fetches (lse, delta) of node l
        int colv;
        uint2 mpn[2];
        auto load_idx = [&](int c2) {   // a pair past the end repeats the last one (valid addresses, results unused)
            const int cc = c0 + min(c2, nch - 2);
            colv = buf_i32(rC, (cc * 16 + (lane & 31)) * 4);
#pragma unroll
            for (int ci = 0; ci < 2; ++ci) {
                const u32x2 m2 = __builtin_amdgcn_raw_buffer_load_b64(rM, ((cc + ci) * 16 + j) * 32 + 8 * g, 0, 0);
                mpn[ci] = make_uint2(m2.x, m2.y);
            }
        };
        // Row fetches are coalesced: 8 consecutive lanes take the 8 16-byte pieces of one row, an
        // instruction fetches 8 whole rows (two per 16-row chunk).  The rows go through LDS to get
        // into the operand layouts of the matrix instructions.
        Row<bf16_t> qa[2][2], ga[2][2];
        float2 stn;         // (lse, delta) of query node `lane % 32` of the pair
        uint32_t rhn = 0;   // DROP: its hash
        const uint32_t bhh = DROP ? drop_bh_hash(a.drop_seed, bh) : 0u;
        auto load_rows = [&]() {
#pragma unroll
            for (int ci = 0; ci < 2; ++ci)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int node = __shfl(colv, 16 * ci + 8 * h + r8);
                    const int row = PACKED ? packed_row(node, a.num_levels - 1, dvec) : node;
                    const int off = (int)__umul24(row, a.row_bytes) + piece * 16;
                    buf_row(rQ, off, qa[ci][h]);
                    buf_row(rG, off, ga[ci][h]);
                }
            stn = buf_f2(rS, colv * 8);
            if (DROP) rhn = drop_row_hash(bhh, colv);
        };
        load_idx(0);

        // B operands: the tile's keys (lane j <-> key j) and the rows of the table this level can meet
        const int64_t krow = base + (int64_t)(node0 + dlev + min(j, nstore - 1)) * a.sn + 16 * g;
        const bf16x8_t kb0 = load_once16<bf16x8_t>(a.K + krow);
        const bf16x8_t kb1 = load_once16<bf16x8_t>(a.K + krow + 8);
        const bf16x8_t vb0 = load_once16<bf16x8_t>(a.V + krow);
        const bf16x8_t vb1 = load_once16<bf16x8_t>(a.V + krow + 8);
        constexpr int kInRegs = NBC < kRegBiasChunks ? NBC : kRegBiasChunks;
        bf16x8_t rb[kInRegs][2];
#pragma unroll
        for (int bc = 0; bc < NBC; ++bc) {
            const int bid = 16 * bc + j;
            int row = 0;
            if (bid < a.W)
                row = level * a.W + bid;                        // (level, order)
            else if (bid - a.W + 1 < a.num_levels)
                row = (bid - a.W + 1) * a.W + a.zero;            // r_anc of the ancestor's level
            const bf16_t* rr = a.rel + (int64_t)row * kD + 16 * g;
            if (bc < kInRegs) {
                rb[bc][0] = *reinterpret_cast<const bf16x8_t*>(rr);
                rb[bc][1] = *reinterpret_cast<const bf16x8_t*>(rr + 8);
            } else {
                rb_s[(bc - kInRegs) * 128] = *reinterpret_cast<const uint4*>(rr);
                rb_s[(bc - kInRegs) * 128 + 1] = *reinterpret_cast<const uint4*>(rr + 8);
            }
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
                }
            if (lane < 32) stat_s[lane] = stn;
            if (DROP && lane < 32) rowh_s[lane] = rhn;
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
                    bf16x8_t r0, r1;
                    if (bc < kInRegs) {
                        r0 = rb[bc][0];
                        r1 = rb[bc][1];
                    } else {
                        r0 = __builtin_bit_cast(bf16x8_t, rb_s[(bc - kInRegs) * 128]);
                        r1 = __builtin_bit_cast(bf16x8_t, rb_s[(bc - kInRegs) * 128 + 1]);
                    }
                    b4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(q0, r0, b4, 0, 0, 0);
                    b4 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(q1, r1, b4, 0, 0, 0);
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
                    const float p = bid[ci][r] >= 0 && key_kept ? fast_exp2((s4[ci][r] + bv[ci][r]) * qscale - st[ci][r].x) : 0.f;
                    if (DROP) {
                        // a token row's edge is named by its relative-position id, a span row's by the key node;
                        // out = sum keep p v: dV takes keep p, and dP carries the mask into dS
                        const uint32_t x = bid[ci][r] < a.W ? (uint32_t)(level * a.W + bid[ci][r]) : 0x80000000u + (uint32_t)(node0 + j);
                        const float keep = drop_scale(rowh_s[16 * ci + 4 * g + r], x, a.drop_thr, a.drop_inv_keep);
                        pp[ci][r] = p * keep;
                        ds[ci][r] = p * (d4[ci][r] * keep - st[ci][r].y);
                    } else {
                        pp[ci][r] = p;
                        ds[ci][r] = p * (d4[ci][r] - st[ci][r].y);
                    }
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
                // transposed, C[m = feature][n = key] (the operands of dS^T Q changed places, the registers are the
                // same): a lane holds features 16f + 4g .. + 3 of key j
                dk[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qB, sH, dk[f], 0, 0, 0);
                dk[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qB, sL, dk[f], 0, 0, 0);
                dv[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gB, pH, dv[f], 0, 0, 0);
                dv[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gB, pL, dv[f], 0, 0, 0);
            }
        }
        // Stored from the registers, a wavefront instruction would write 64-byte pieces of 16 rows (measured: the key
        // side 21 % slower than with whole lines); the sums go through LDS (the row buffers are free now), 16 bytes
        // per lane in and out, and leave as rows of 256 contiguous bytes.
        wave_lds_sync();   // the last pair's reads of q_s, g_s are done
        float* o_s = reinterpret_cast<float*>(q_s);   // [16 keys][kKvOutStride]: 64 dK | 64 dV
#pragma unroll
        for (int f = 0; f < 4; ++f) {
            const f32x4_t xk = {a.scale * dk[f][0], a.scale * dk[f][1], a.scale * dk[f][2], a.scale * dk[f][3]};
            *reinterpret_cast<f32x4_t*>(o_s + j * kKvOutStride + 16 * f + 4 * g) = xk;
            *reinterpret_cast<f32x4_t*>(o_s + j * kKvOutStride + kD + 16 * f + 4 * g) = dv[f];
        }
        wave_lds_sync();
        if (part < 0 && a.grad_bf16) {   // rounded to bf16: 8 bytes per lane
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int idx = lane + 64 * i, key = idx >> 5, q4 = (idx & 31) * 4;
                if (key < nstore)
                    store_grad4(q4 < kD ? a.dK : a.dV, base + (int64_t)(node0 + dlev + key) * a.sn + (q4 & (kD - 1)),
                                *reinterpret_cast<const float4*>(o_s + key * kKvOutStride + q4), true);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int idx = lane + 64 * i, key = idx >> 5, q4 = (idx & 31) * 4;
                if (key < (part < 0 ? nstore : nkeys)) {
                    const float4 v = *reinterpret_cast<const float4*>(o_s + key * kKvOutStride + q4);
                    float* dst;
                    if (part < 0)
                        dst = (q4 < kD ? a.dK + q4 : a.dV + (q4 - kD)) + base + (int64_t)(node0 + dlev + key) * a.sn;
                    else
                        dst = a.part + (((int64_t)bh * a.num_part + part) * 16 + key) * (2 * kD) + q4;
                    if (part < 0)
                        store_once(reinterpret_cast<float4*>(dst), v);
                    else   // the merge kernel reads the partial sums
                        *reinterpret_cast<float4*>(dst) = v;
                }
            }
        }
        wave_lds_sync();
    }
}

// The same products for the graphs whose key tiles meet at most 32 relative-position ids, with two changes
// that matter for the fine levels, where a tile has only one to four pairs of chunks and the start of a task
// (task counter, tile description, column ids, first rows: four dependent round trips to memory) costs more
// than its products.  (1) A task walks `task_ntiles` consecutive tiles of one level: their chunks are
// consecutive in `cols` and `map`, so the software pipeline runs through the tile boundaries -- the rows of
// the next tile's first pair are requested while the last pair of this one is computed, its K and V rows one
// tile ahead.  At a boundary the sums go to a staging area in LDS and are stored from there in the next
// iteration, before that iteration's loads are requested: the loop waits for loads only, and a store
// requested behind them would be waited for as well (the two return through the same counter).  (2) The
// bias of (query, id) is not staged through LDS: the product Q_chunk x Rel_sel^T leaves bias[query 4g + r][id j]
// in lane (g, j), register r, and the lane that needs it reads it from there (ds_bpermute), which makes room
// for the staging area.
// G16: dK and dV leave rounded to bf16 (a compile-time switch: the stores sit inside the pipelined loop)
template <int NBC, bool DROP, bool G16, bool PACKED = false>
__global__ void __launch_bounds__(kTileThreads, 2) bwd_kv_chain_kernel(const KeyArgs a) {
    static_assert(NBC == 1 || NBC == 2, "the bias is looked up across the 16 lanes of a group, for up to two chunks of ids");
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, j = lane & 15;
    const int r8 = lane >> 3, piece = lane & 7;
    constexpr size_t kRowsBytes = 64 * kRowStride * sizeof(bf16_t), kStageBytes = 16 * kKvOutStride * sizeof(float);
    bf16_t* q_s = reinterpret_cast<bf16_t*>(smem) + (size_t)wave * 64 * kRowStride;                       // [32 queries][kRowStride]
    bf16_t* g_s = q_s + 32 * kRowStride;
    float* o_s = reinterpret_cast<float*>(smem + (size_t)kTileWaves * kRowsBytes) + (size_t)wave * 16 * kKvOutStride;   // [16 keys][64 dK | 64 dV]
    float2* stat_s = reinterpret_cast<float2*>(smem + (size_t)kTileWaves * (kRowsBytes + kStageBytes)) + (size_t)wave * 32;
    uint32_t* rowh_s = reinterpret_cast<uint32_t*>(smem + (size_t)kTileWaves * (kRowsBytes + kStageBytes + 32 * sizeof(float2))) +
                       (size_t)wave * 32;
    const float qscale = a.scale * kLog2e;
    const int xcd = blockIdx.x & 7;
    const int total = a.BH * a.num_tasks, per = (total + 7) >> 3;
    const int share_begin = xcd * per, share_end = min(total, share_begin + per);
    const rsrc_t rC = make_rsrc(a.cols, (uint32_t)a.num_chunks * 64u);
    const rsrc_t rM = make_rsrc(a.map, (uint32_t)a.num_chunks * 512u);

    for (;;) {
        int item = 0;
        if (lane == 0) item = atomicAdd(a.queue + xcd * 16, 1);
        item = __builtin_amdgcn_readfirstlane(item) + share_begin;
        if (item >= share_end) break;   // every wavefront gets here: the counter only grows from zero
        const int slab = item / a.num_tasks, task = item - slab * a.num_tasks;
        const int bh = walk_bh(a.seq_len, slab, a.BH, a.H);
        const int kt0 = uniform_i32(a.task_tile, task), c0 = uniform_i32(a.task_c0, task), part = uniform_i32(a.task_part, task);
        const int nch = uniform_i32(a.task_nch, task), ntiles = uniform_i32(a.task_ntiles, task);
        const int level = uniform_i32(a.tile_info, kt0) & 255;   // the same for all tiles of the task
        const int len = seq_length_u(a.seq_len, bh / a.H, a.n);
        const int level_node0 = 2 * a.n - ((2 * a.n) >> level), level_kept = (len + (1 << level) - 1) >> level;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        // the tile at work: its keys, how many the sequence keeps, and the chunk (relative to c0) at which it ends
        int kt = kt0;
        int node0 = uniform_i32(a.tile_node0, kt), nkeys = uniform_i32(a.tile_info, kt) >> 8;
        int kept_keys = level_kept - (node0 - level_node0);
        if (kept_keys <= 0) continue;   // no key of the first tile exists in this sequence, nor of the ones behind it
        int tile_end = ntiles > 1 ? uniform_i32(a.chunk_ptr, kt + 1) - c0 : nch;
        const rsrc_t rQ = make_rsrc(a.Q + base, a.slab_bytes), rG = make_rsrc(a.dout + base, a.slab_bytes);
        const rsrc_t rK = make_rsrc(a.K + base, a.slab_bytes), rV = make_rsrc(a.V + base, a.slab_bytes);
        const rsrc_t rS = make_rsrc(a.stat + (int64_t)bh * a.N, (uint32_t)a.N * 8u);
        // packed batch: see bwd_kv_tile_kernel
        const int dvec = PACKED ? load_delta(a.delta, a.BH / a.H, bh / a.H, lane, a.num_levels) : 0;
        const int dlev = PACKED ? level_delta(dvec, level) : 0;

        // the 32 query nodes of a pair arrive with one instruction, node l in lane l (and l + 32); the lane that
        // fetches a piece of row 16 ci + 8 h + r8 reads its id from there, and lane l fetches (lse, delta) of node l
        int colv;
        uint2 mpn[2];
        auto load_idx = [&](int c2) {   // a pair past the end repeats the last one (valid addresses, results unused)
            const int cc = c0 + min(c2, nch - 2);
            colv = buf_i32(rC, (cc * 16 + (lane & 31)) * 4);
#pragma unroll
            for (int ci = 0; ci < 2; ++ci) {
                const u32x2 m2 = __builtin_amdgcn_raw_buffer_load_b64(rM, ((cc + ci) * 16 + j) * 32 + 8 * g, 0, 0);
                mpn[ci] = make_uint2(m2.x, m2.y);
            }
        };
        Row<bf16_t> qa[2][2], ga[2][2];
        float2 stn;
        uint32_t rhn = 0;
        const uint32_t bhh = DROP ? drop_bh_hash(a.drop_seed, bh) : 0u;
        auto load_rows = [&]() {
#pragma unroll
            for (int ci = 0; ci < 2; ++ci)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int node = __shfl(colv, 16 * ci + 8 * h + r8);
                    const int row = PACKED ? packed_row(node, a.num_levels - 1, dvec) : node;
                    const int off = (int)__umul24(row, a.row_bytes) + piece * 16;
                    buf_row(rQ, off, qa[ci][h]);
                    buf_row(rG, off, ga[ci][h]);
                }
            stn = buf_f2(rS, colv * 8);
            if (DROP) rhn = drop_row_hash(bhh, colv);
        };
        // B operands: the keys of a tile (lane j <-> key j) ...
        Row<bf16_t> kk[2], vv[2], kn[2], vn[2];
        auto load_keys = [&](int first, int count, Row<bf16_t> (&ko)[2], Row<bf16_t> (&vo)[2]) {
            const int off = (int)__umul24(first + dlev + min(j, count - 1), a.row_bytes) + 32 * g;
            buf_row(rK, off, ko[0]);
            buf_row(rK, off + 16, ko[1]);
            buf_row(rV, off, vo[0]);
            buf_row(rV, off + 16, vo[1]);
        };
        load_idx(0);
        load_keys(node0, nkeys, kk, vv);
        // ... and the rows of the table this level can meet
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
        // sums of a finished tile wait in o_s for the next iteration: where they go
        bool staged = false;
        int st_node0 = 0, st_nkeys = 0;   // st_node0: first row of the finished tile's keys in dK, dV; st_nkeys: rows to store
        auto store_staged = [&]() {
            if (G16 && part < 0) {   // rounded to bf16: 8 bytes per lane, rows of 256 contiguous bytes
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int idx = lane + 64 * i, key = idx >> 5, q4 = (idx & 31) * 4;
                    if (key < st_nkeys)
                        store_grad4(q4 < kD ? a.dK : a.dV, base + (int64_t)(st_node0 + key) * a.sn + (q4 & (kD - 1)),
                                    *reinterpret_cast<const float4*>(o_s + key * kKvOutStride + q4), true);
                }
                return;
            }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int idx = lane + 64 * i, key = idx >> 5, q4 = (idx & 31) * 4;
                if (key < st_nkeys) {
                    const float4 v = *reinterpret_cast<const float4*>(o_s + key * kKvOutStride + q4);
                    if (part < 0) {
                        float* dst = (q4 < kD ? a.dK + q4 : a.dV + (q4 - kD)) + base + (int64_t)(st_node0 + key) * a.sn;
                        store_once(reinterpret_cast<float4*>(dst), v);
                    } else {   // the merge kernel reads the partial sums
                        float* dst = a.part + (((int64_t)bh * a.num_part + part) * 16 + key) * (2 * kD) + q4;
                        *reinterpret_cast<float4*>(dst) = v;
                    }
                }
            }
        };

        bool fetch_next_keys = ntiles > 1;   // the next tile's K and V rows are requested with the first pair of this one
        for (int c2 = 0; c2 < nch; c2 += 2) {
            wave_lds_sync();  // the previous pair's LDS reads are done
#pragma unroll
            for (int ci = 0; ci < 2; ++ci)
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    const int row = 16 * ci + 8 * h + r8;
                    *reinterpret_cast<uint4*>(q_s + row * kRowStride + piece * 8) = qa[ci][h].w;
                    *reinterpret_cast<uint4*>(g_s + row * kRowStride + piece * 8) = ga[ci][h].w;
                }
            if (lane < 32) stat_s[lane] = stn;
            if (DROP && lane < 32) rowh_s[lane] = rhn;
            __builtin_amdgcn_sched_barrier(0);
            if (staged) {   // wave-uniform: the tile finished by the previous pair
                store_staged();
                staged = false;
            }
            // the row registers are free: request the next pair's rows, then the ids of the pair after it
            const uint2 mpc[2] = {mp[0], mp[1]};
            load_rows();
            mp[0] = mpn[0];
            mp[1] = mpn[1];
            load_idx(c2 + 4);
            if (fetch_next_keys) {   // wave-uniform
                const int nx = kt + 1;
                load_keys(uniform_i32(a.tile_node0, nx), uniform_i32(a.tile_info, nx) >> 8, kn, vn);
                fetch_next_keys = false;
            }
            __builtin_amdgcn_sched_barrier(0);
            wave_lds_sync();
            const bool key_kept = j < kept_keys;
            const bf16x8_t kb0 = __builtin_bit_cast(bf16x8_t, kk[0].w), kb1 = __builtin_bit_cast(bf16x8_t, kk[1].w);
            const bf16x8_t vb0 = __builtin_bit_cast(bf16x8_t, vv[0].w), vb1 = __builtin_bit_cast(bf16x8_t, vv[1].w);
            f32x4_t s4[2], d4[2], b4[2][NBC];
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
                    b4[ci][bc] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                    b4[ci][bc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(q0, rb[bc][0], b4[ci][bc], 0, 0, 0);
                    b4[ci][bc] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(q1, rb[bc][1], b4[ci][bc], 0, 0, 0);
                }
            }
            float ds[2][4], pp[2][4];
#pragma unroll
            for (int ci = 0; ci < 2; ++ci) {
                const float4 x = *reinterpret_cast<const float4*>(stat_s + 16 * ci + 4 * g);
                const float4 y = *reinterpret_cast<const float4*>(stat_s + 16 * ci + 4 * g + 2);
                const float2 st[4] = {make_float2(x.x, x.y), make_float2(x.z, x.w), make_float2(y.x, y.y), make_float2(y.z, y.w)};
                const int bid[4] = {(int)(short)(mpc[ci].x & 0xFFFFu), (int)(short)(mpc[ci].x >> 16),
                                    (int)(short)(mpc[ci].y & 0xFFFFu), (int)(short)(mpc[ci].y >> 16)};
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    // bias[query 4g + r][id] sits in lane (g, id % 16), register r of the id's chunk
                    const int src = (lane & 48) | (max(bid[r], 0) & 15);
                    float bv = __shfl(b4[ci][0][r], src);
                    if (NBC == 2) {
                        const float bv1 = __shfl(b4[ci][1][r], src);
                        bv = bid[r] >= 16 ? bv1 : bv;
                    }
                    const float p = bid[r] >= 0 && key_kept ? fast_exp2((s4[ci][r] + bv) * qscale - st[r].x) : 0.f;
                    if (DROP) {
                        const uint32_t x2 = bid[r] < a.W ? (uint32_t)(level * a.W + bid[r]) : 0x80000000u + (uint32_t)(node0 + j);
                        const float keep = drop_scale(rowh_s[16 * ci + 4 * g + r], x2, a.drop_thr, a.drop_inv_keep);
                        pp[ci][r] = p * keep;
                        ds[ci][r] = p * (d4[ci][r] * keep - st[r].y);
                    } else {
                        pp[ci][r] = p;
                        ds[ci][r] = p * (d4[ci][r] - st[r].y);
                    }
                }
            }
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
                // transposed, C[m = feature][n = key] (the operands of dS^T Q changed places, the registers are the
                // same): a lane holds features 16f + 4g .. + 3 of key j
                dk[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qB, sH, dk[f], 0, 0, 0);
                dk[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qB, sL, dk[f], 0, 0, 0);
                dv[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gB, pH, dv[f], 0, 0, 0);
                dv[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(gB, pL, dv[f], 0, 0, 0);
            }
            if (c2 + 2 == tile_end) {   // wave-uniform: the tile is complete
                // o_s was read (if at all) at the top of this iteration, before a barrier of the wavefront
#pragma unroll
                for (int f = 0; f < 4; ++f) {
                    const f32x4_t xk = {a.scale * dk[f][0], a.scale * dk[f][1], a.scale * dk[f][2], a.scale * dk[f][3]};
                    *reinterpret_cast<f32x4_t*>(o_s + j * kKvOutStride + 16 * f + 4 * g) = xk;
                    *reinterpret_cast<f32x4_t*>(o_s + j * kKvOutStride + kD + 16 * f + 4 * g) = dv[f];
                    dk[f] = dv[f] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                }
                staged = true;
                st_node0 = node0 + dlev;
                // (packed batch: keys the sequence does not keep have no row; partial sums keep all of the tile's keys)
                st_nkeys = PACKED && part < 0 ? min(nkeys, kept_keys) : nkeys;
                if (c2 + 2 < nch) {   // on to the next tile of the task
                    ++kt;
                    node0 = uniform_i32(a.tile_node0, kt);
                    nkeys = uniform_i32(a.tile_info, kt) >> 8;
                    kept_keys = level_kept - (node0 - level_node0);
                    tile_end = uniform_i32(a.chunk_ptr, kt + 1) - c0;
                    kk[0] = kn[0];
                    kk[1] = kn[1];
                    vv[0] = vn[0];
                    vv[1] = vn[1];
                    fetch_next_keys = kt + 1 < kt0 + ntiles;
                    if (kept_keys <= 0) break;   // this tile and the ones behind it lie past the end of the sequence
                }
            }
        }
        wave_lds_sync();
        if (staged) store_staged();
        wave_lds_sync();
    }
}

// Tiles whose query list was cut into several tasks: sum the partial (dK, dV) of the
// tile's keys in task order.  One workgroup per (batch*head, tile); thread -> (key, feature).
// The workgroups after those write the zero gradients of the nodes no one attends to
// (levels above the coarsest contextual level, from `first_zero` on).
template <bool PACKED>
__global__ void __launch_bounds__(256) kv_tile_merge_kernel(const KeyArgs a, const int32_t* __restrict__ multi_tile,
                                                            const int32_t* __restrict__ multi_ptr, int num_multi,
                                                            int first_zero) {
    const int merge_blocks = a.BH * num_multi;
    if ((int)blockIdx.x >= merge_blocks) {
        // zero rows: without seq_len the nodes from first_zero on; with seq_len also those a shorter sequence
        // does not keep (which the tile kernel steps over).  A wavefront looks at 64 consecutive nodes, one
        // per lane, and then writes the rows found two at a time: 16 lanes x 16 bytes for each of dK and dV
        // of a row.
        const int row0 = a.seq_len && !a.leave_unkept ? 0 : (first_zero & ~63), waves_per_bh = (a.N - row0 + 63) >> 6;
        const int64_t gw = ((int64_t)(blockIdx.x - merge_blocks) * blockDim.x + threadIdx.x) >> 6;
        if (gw >= (int64_t)a.BH * waves_per_bh) return;
        const int lane = threadIdx.x & 63;
        const int bh = (int)(gw / waves_per_bh), first = row0 + 64 * (int)(gw - (int64_t)bh * waves_per_bh);
        const int row = first + lane;
        bool gone = row < a.N && row >= first_zero;
        if (a.seq_len && row < a.N) {
            const bool unkept = node_first_token(row, 31 - __clz(a.n)) >= seq_length(a.seq_len, bh / a.H, a.n);
            gone = a.leave_unkept ? gone && !unkept : gone || unkept;
        }
        uint64_t todo = __ballot(gone);
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        while (todo) {   // wave-uniform
            const int ra = __builtin_ctzll(todo);
            todo &= todo - 1;
            const int rb = todo ? __builtin_ctzll(todo) : -1;
            if (todo) todo &= todo - 1;
            const int r = lane < 32 ? ra : rb;
            if (r >= 0) {
                int at = first + r;
                if (PACKED) at += a.delta[node_level(at, a.num_levels - 1) * (a.BH / a.H) + bh / a.H];   // its packed row
                store_grad4((lane & 16) ? a.dV : a.dK, base + (int64_t)at * a.sn + 4 * (lane & 15),
                            make_float4(0.f, 0.f, 0.f, 0.f), a.grad_bf16);
            }
        }
        return;
    }
    const int bh = blockIdx.x / num_multi, mt = blockIdx.x - bh * num_multi;
    const int kt = multi_tile[mt];
    const int node0 = a.tile_node0[kt], nkeys = a.tile_info[kt] >> 8, level = a.tile_info[kt] & 255;
    const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
    // a tile none of whose keys exists in this (shorter) sequence has no partial sums: zeros
    const int len = seq_length(a.seq_len, bh / a.H, a.n);
    const int kept_keys = ((len + (1 << level) - 1) >> level) - (node0 - (2 * a.n - ((2 * a.n) >> level)));
    const bool gone = kept_keys <= 0;
    if (gone && a.leave_unkept) return;   // uniform for the workgroup
    // packed batch: the tile's keys begin at the sequence's delta of the level; keys it does not keep have no row
    const int dlev = PACKED ? a.delta[level * (a.BH / a.H) + bh / a.H] : 0;
    const int nstore = PACKED ? min(nkeys, kept_keys) : nkeys;
    // thread -> (key, 4 consecutive values of its 64 dK | 64 dV); four partial sums in flight, combined in a fixed order
    const int p0 = gone ? multi_ptr[mt + 1] : multi_ptr[mt], p1 = multi_ptr[mt + 1];
    for (int i = threadIdx.x; i < nstore * 32; i += blockDim.x) {
        const int key = i >> 5, q4 = (i & 31) * 4;
        const float* src = a.part + (((int64_t)bh * a.num_part) * 16 + key) * (2 * kD) + q4;
        const int64_t pstride = (int64_t)16 * 2 * kD;
        float4 s0 = make_float4(0.f, 0.f, 0.f, 0.f), s1 = s0, s2 = s0, s3 = s0;
        int p = p0;
        for (; p + 3 < p1; p += 4) {
            const float4 x0 = *reinterpret_cast<const float4*>(src + p * pstride);
            const float4 x1 = *reinterpret_cast<const float4*>(src + (p + 1) * pstride);
            const float4 x2 = *reinterpret_cast<const float4*>(src + (p + 2) * pstride);
            const float4 x3 = *reinterpret_cast<const float4*>(src + (p + 3) * pstride);
            s0.x += x0.x; s0.y += x0.y; s0.z += x0.z; s0.w += x0.w;
            s1.x += x1.x; s1.y += x1.y; s1.z += x1.z; s1.w += x1.w;
            s2.x += x2.x; s2.y += x2.y; s2.z += x2.z; s2.w += x2.w;
            s3.x += x3.x; s3.y += x3.y; s3.z += x3.z; s3.w += x3.w;
        }
        for (; p < p1; ++p) {
            const float4 x0 = *reinterpret_cast<const float4*>(src + p * pstride);
            s0.x += x0.x; s0.y += x0.y; s0.z += x0.z; s0.w += x0.w;
        }
        const float4 t = make_float4((s0.x + s1.x) + (s2.x + s3.x), (s0.y + s1.y) + (s2.y + s3.y),
                                     (s0.z + s1.z) + (s2.z + s3.z), (s0.w + s1.w) + (s2.w + s3.w));
        store_grad4(q4 < kD ? a.dK : a.dV, base + (int64_t)(node0 + dlev + key) * a.sn + (q4 & (kD - 1)), t, a.grad_bf16);
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
    store_grad(a.dK, at, sk, a.grad_bf16);
    store_grad(a.dV, at, sv, a.grad_bf16);
}

// d_rel = sum of the workgroups' copies, in a fixed order; rows the copies do not
// cover are zero.  One workgroup per row of 64 features: 16 wavefronts each sum a
// sixteenth of the copies (lane = feature, coalesced 256-byte reads, four
// independent partial sums in flight), then combine in a fixed tree.
// With `id_to_cid` the copies are in the token tiles' compact-id order and hold
// `covered_rows` rows each: row `id` of d_rel is copy row id_to_cid[id] (or zero).
// The first workgroup also clears the `zero_count` ints at `zero`: the task counters of the key side,
// which runs after the query side that ends with this kernel.
__global__ void __launch_bounds__(1024) drel_reduce_kernel(const float* __restrict__ parts, int num_parts,
                                                           int covered_rows, const int32_t* __restrict__ id_to_cid,
                                                           float* __restrict__ d_rel, int32_t* __restrict__ zero,
                                                           int zero_count) {
    __shared__ float s[16][kD];
    if (blockIdx.x == 0 && (int)threadIdx.x < zero_count) zero[threadIdx.x] = 0;
    const int row = blockIdx.x, lane = threadIdx.x & 63, grp = threadIdx.x >> 6;
    const int prow = id_to_cid ? id_to_cid[row] : row;
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f, a4 = 0.f, a5 = 0.f, a6 = 0.f, a7 = 0.f;
    if (prow >= 0 && prow < covered_rows) {
        const float* src = parts + (int64_t)prow * kD + lane;
        const int64_t stride = (int64_t)covered_rows * kD;
        int p = grp;
        for (; p + 112 < num_parts; p += 128) {   // eight loads in flight per round trip
            const float x0 = src[p * stride], x1 = src[(p + 16) * stride], x2 = src[(p + 32) * stride];
            const float x3 = src[(p + 48) * stride], x4 = src[(p + 64) * stride], x5 = src[(p + 80) * stride];
            const float x6 = src[(p + 96) * stride], x7 = src[(p + 112) * stride];
            a0 += x0; a1 += x1; a2 += x2; a3 += x3; a4 += x4; a5 += x5; a6 += x6; a7 += x7;
        }
        for (; p < num_parts; p += 16) a0 += src[p * stride];
    }
    s[grp][lane] = ((a0 + a1) + (a2 + a3)) + ((a4 + a5) + (a6 + a7));
    __syncthreads();
    for (int w = 8; w > 0; w >>= 1) {
        if (grp < w) s[grp][lane] += s[grp + w][lane];
        __syncthreads();
    }
    if (grp == 0) d_rel[row * kD + lane] = s[0][lane];
}

}  // namespace
}  // namespace bpt
