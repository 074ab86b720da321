// Matrix-core kernels over dense tiles of 16 token rows (bf16): forward, query side of the
// backward, and d_rel / the relative-position part of dQ from the tiles' (w, p) pairs.
#pragma once

#include "attn_device.h"
#include "attn_gather.h"

namespace bpt {
namespace {

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
constexpr int kDqStride = 68;    // floats per row of a tile's fp32 dQ rows on their way out through LDS (16 rows fit the K row buffer)

constexpr int kDenseChunks = 8;   // 16-id chunks the dense variant of bwd_q_tile_kernel keeps d_rel sums for
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
    float* drel_part;   // DENSE variant: the workgroups' copies of d_rel, [workgroup][cid_pad][64]
    // sequences shorter than n
    const int32_t *seq_len, *id_to_cid;
    int32_t leave_unkept;   // rows of nodes a shorter sequence does not keep: left unwritten instead of zero-filled
    int32_t grad_bf16;      // dQ leaves rounded to bf16
    int32_t n, k, W, ctx_levels, causal;
    // packed batch: delta[level][sequence] (see attn_device.h) or null; lse of (batch*head index bh, node u) is at
    // (bh / H) * lse_sb + (bh % H) * lse_sh + row of u
    const int32_t* delta;
    int32_t levels, lg;
    int64_t lse_sb, lse_sh;
    // dropout on the attention weights (DROP variants of the kernels)
    uint32_t drop_thr, drop_seed;
    float drop_inv_keep;
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

// 4 consecutive k (rows row0 .. row0 + 3) of the operand column `col0 + j`: one transposing read, the
// operand of v_mfma_f32_16x16x16_bf16 for k = 4g .. 4g + 3
__device__ __forceinline__ s16x4_t lds_tr4(const bf16_t* base, int stride, int row0, int col0, int j) {
    typedef __attribute__((address_space(3))) s16x4_t* lds_ptr_t;
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr_t)(base + (row0 + (j >> 2)) * stride + col0 + 4 * (j & 3)));
}

// Sequences shorter than n: the bias entries of edges such a sequence does not have are set to
// kMaskBias, which drives their softmax weight to 0 without touching the loop over the chunks --
// every entry of a token past the end, and for the other tokens the right-side nodes past the
// end.  The i-th node to join on the right at level l is node p_l + i - 1 of that level, with
// p_0 = t + 1 and p_{l+1} = ceil((p_l + k) / 2) (Algorithm 1: k nodes, one more when the run would
// not end on a parent boundary), and level l keeps ceil(len / 2^l) nodes.  Lane (g, j) works on
// token j of the tile; the four lane groups share the ids.
constexpr float kMaskBias = -1.0e30f;
__device__ __forceinline__ void mask_bias(const TileArgs& a, float* bias_s, int t0, int len, int g, int j) {
    const int t = t0 + j;
    float* row = bias_s + j * a.bias_stride;
    if (t >= len) {
        for (int c = 4 * g; c < a.cid_pad; c += 16) *reinterpret_cast<f32x4_t*>(row + c) = f32x4_t{kMaskBias, kMaskBias, kMaskBias, kMaskBias};
    } else if (!a.causal) {
        int p = t + 1;
        for (int l = 0; l < a.ctx_levels; ++l) {
            const int cnt = (len + (1 << l) - 1) >> l;            // nodes the level keeps
            for (int o = max(cnt - p + 1, 1) + g; o <= a.k + 1; o += 4) {
                const int cid = a.id_to_cid[l * a.W + a.k + 1 + o];
                if (cid >= 0) row[cid] = kMaskBias;
            }
            p = (p + a.k + 1) >> 1;
        }
    }
}

// Batches of sequences of different lengths: entry b keeps its first ceil(len_b / 16) token tiles, so the
// tiles that exist can be numbered in closed form from a prefix sum over the batch, head-major --
// i -> (head i / S, entry b with pref[b] <= i % S < pref[b + 1], tile i % S - pref[b]), S = pref[B] -- and
// so can the ones that do not (entry b has num_tiles - count_b of them, after the kept ones).  A
// kernel that walks these numbers instead of all (batch, head, tile) triples gives every wavefront
// the same number of tiles to compute, whatever the lengths.  Up to kMaxLenBatch entries.
constexpr int kMaxLenBatch = 256;
// whole workgroup; pref[0 .. B] in LDS; ends with a barrier
__device__ __forceinline__ void live_tiles_prefix(int* pref, const int32_t* seq_len, int B, int n, int num_tiles) {
    if (threadIdx.x < 64) {
        int carry = 0;
        for (int b0 = 0; b0 < B; b0 += 64) {
            const int b = b0 + (int)threadIdx.x;
            const int cnt = b < B ? min(num_tiles, (min(max(seq_len[b], 0), n) + 15) >> 4) : 0;
            int incl = cnt;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const int up = __shfl_up(incl, d);
                if ((int)threadIdx.x >= d) incl += up;
            }
            if (b < B) pref[b] = carry + incl - cnt;
            carry += __shfl(incl, 63);
        }
        if (threadIdx.x == 0) pref[B] = carry;
    }
    __syncthreads();
}
// the idx-th tile that exists (dead == false) or that does not (dead == true); wave-uniform arguments
__device__ __forceinline__ void nth_tile(const int* pref, int B, int H, int num_tiles, bool dead, int idx, int& bh, int& tile) {
    const int per_head = dead ? B * num_tiles - pref[B] : pref[B];
    const int h = idx / per_head, r = idx - h * per_head;
    int lo = 0, hi = B - 1;   // the last entry whose tiles begin at or before r
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        const int start = dead ? mid * num_tiles - pref[mid] : pref[mid];
        if (start <= r) lo = mid; else hi = mid - 1;
    }
    const int start = dead ? lo * num_tiles - pref[lo] : pref[lo];
    bh = lo * H + h;
    tile = dead ? (pref[lo + 1] - pref[lo]) + (r - start) : r - start;
}

// Position of a wavefront in its sequence of (token tile, pair of chunks); wave-uniform.
struct TileCursor {
    int t, pair, npairs, cp0, bh, tile;
    int dvec;   // packed batch: this lane's delta of the sequence the tile belongs to (0 otherwise)
    bool valid;
};
// Says that everything but dvec is the same in all lanes.  With a lane's own dvec among the fields the compiler keeps
// the whole cursor in vector registers, and what follows from it -- the divisions by the number of heads and by the
// tiles per sequence, the tensors' base offsets: some hundred instructions per pair of chunks -- is done per lane.
__device__ __forceinline__ void cursor_uniform(TileCursor& c) {
    c.t = __builtin_amdgcn_readfirstlane(c.t);
    c.pair = __builtin_amdgcn_readfirstlane(c.pair);
    c.npairs = __builtin_amdgcn_readfirstlane(c.npairs);
    c.cp0 = __builtin_amdgcn_readfirstlane(c.cp0);
    c.bh = __builtin_amdgcn_readfirstlane(c.bh);
    c.tile = __builtin_amdgcn_readfirstlane(c.tile);
    c.valid = __builtin_amdgcn_readfirstlane((int)c.valid) != 0;
}

// REL_LDS: the compact relative-position table is staged in LDS; otherwise (large tables) its rows
// are read from memory when a tile forms its bias table.
// PACKED: the rows of the caller's tensors are those of a packed batch (TileArgs.delta; see attn_device.h)
template <bool REL_LDS, bool DROP, bool PACKED = false>
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
    // DROP: relative-position id of every compact id, what the dropout mask of an edge is drawn from
    int32_t* relid_s = reinterpret_cast<int32_t*>(smem + rel_bytes + (size_t)kTileWaves * 16 * a.bias_stride * sizeof(float) +
                                                  (size_t)kTileWaves * 64 * kRowStride * sizeof(bf16_t));   // [cid_pad]
    if (DROP)
        for (int i = threadIdx.x; i < a.cid_pad; i += blockDim.x) relid_s[i] = i < a.num_cids ? a.cid_to_id[i] : 0;
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
    // sequences of different lengths: walk the tiles that exist, and first write the zero rows of the others
    __shared__ int pref_s[kMaxLenBatch + 1];
    const int nbatch = a.BH / a.H;
    const bool compact = a.seq_len && nbatch <= kMaxLenBatch;
    int live_total = 0;
    auto zero_rows = [&](int bh, int tile) {   // out and lse of a tile past the end of its sequence
        if (a.leave_unkept) return;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        bf16_t* orow = a.out + base + (int64_t)(tile * 16 + r8) * a.sn + piece * 8;
        *reinterpret_cast<uint4*>(orow) = make_uint4(0u, 0u, 0u, 0u);
        *reinterpret_cast<uint4*>(orow + 8 * a.sn) = make_uint4(0u, 0u, 0u, 0u);
        if (lane < 16) a.lse[(int64_t)bh * a.N + tile * 16 + lane] = 0.f;   // (never with PACKED: its rows are left unwritten)
    };
    if (compact) {
        live_tiles_prefix(pref_s, a.seq_len, nbatch, a.n, a.num_tiles);
        live_total = a.H * pref_s[nbatch];
        const int dead_total = a.leave_unkept ? 0 : a.BH * a.num_tiles - live_total;
        for (TileWalk wd((dead_total + kTileWaves - 1) / kTileWaves); wd.t < wd.t_end; wd.t += wd.step) {
            const int idx = wd.t * kTileWaves + wave;
            if (idx < dead_total) {
                int bh, tile;
                nth_tile(pref_s, nbatch, a.H, a.num_tiles, true, idx, bh, tile);
                zero_rows(bh, tile);
            }
        }
    }
    const TileWalk w(compact ? (live_total + kTileWaves - 1) / kTileWaves : a.BH * groups_per_bh);

    // One sequence of pairs of chunks through the wavefront's tiles, software pipelined as in
    // bwd_q_tile_kernel: `cc` is computed, the rows of `cr` and the ids of `ci` are in flight.
    // A tile whose 16 tokens all lie past the end of a shorter sequence is not computed: whoever
    // walks over it (every tile is entered by exactly one cursor, the others are copies) writes
    // its zero rows.
    auto enter_tile = [&](TileCursor& c) {
        c.valid = false;
        c.pair = 0;
        c.npairs = 1;
        c.dvec = 0;
        if (PACKED) c.t = __builtin_amdgcn_readfirstlane(c.t);   // (see cursor_uniform)
        if (compact) {   // the next tile that exists; the walk covers nothing else
            const int idx = c.t * kTileWaves + wave;
            if (c.t < w.t_end && idx < live_total) {
                nth_tile(pref_s, nbatch, a.H, a.num_tiles, false, idx, c.bh, c.tile);
                if (PACKED) {
                    c.bh = __builtin_amdgcn_readfirstlane(c.bh);
                    c.tile = __builtin_amdgcn_readfirstlane(c.tile);
                }
                c.cp0 = a.chunk_ptr[c.tile];
                c.npairs = (a.chunk_ptr[c.tile + 1] - c.cp0) >> 1;
                c.dvec = PACKED ? load_delta(a.delta, nbatch, c.bh / a.H, lane, a.levels) : 0;
                c.valid = true;
            }
            return;
        }
        for (; c.t < w.t_end; c.t += w.step) {
            const int slab = c.t / groups_per_bh;
            c.bh = walk_bh(a.seq_len, slab, a.BH, a.H);
            c.tile = walk_pos(a.seq_len, slab, c.t - slab * groups_per_bh, groups_per_bh) * kTileWaves + wave;
            if (c.tile >= a.num_tiles) continue;
            if (a.seq_len && c.tile * 16 >= seq_length_u(a.seq_len, c.bh / a.H, a.n)) {
                zero_rows(c.bh, c.tile);
                continue;
            }
            c.cp0 = a.chunk_ptr[c.tile];
            c.npairs = (a.chunk_ptr[c.tile + 1] - c.cp0) >> 1;
            c.dvec = PACKED ? load_delta(a.delta, nbatch, c.bh / a.H, lane, a.levels) : 0;
            c.valid = true;
            return;
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
                const int node = PACKED ? packed_row(node_n[ci][h], a.lg, c.dvec) : node_n[ci][h];
                const int off = (int)__umul24(node, a.row_bytes) + piece * 16;
                buf_row(rK, off, kr[ci][h]);
                buf_row(rV, off, vr[ci][h]);
            }
        if (c.pair == 0) {   // token j, features 16g..16g+15
            // (packed batch: a token past the end of the sequence reads the sequence's last row instead of another node's)
            const int tq = PACKED ? min(c.tile * 16 + j, seq_length_u(a.seq_len, c.bh / a.H, a.n) - 1) + level_delta(c.dvec, 0)
                                   : c.tile * 16 + j;
            const int64_t at = base + (int64_t)tq * a.sn + 16 * g;
            qn0 = *reinterpret_cast<const bf16x8_t*>(a.Q + at);
            qn1 = *reinterpret_cast<const bf16x8_t*>(a.Q + at + 8);
        }
    };

    TileCursor cc, cr, ci;
    cc.t = w.t;
    enter_tile(cc);
    if (!cc.valid) return;
    if (PACKED) cursor_uniform(cc);
    load_idx(cc);
    request_rows(cc);
    uint2 mp[2] = {mp_n[0], mp_n[1]};
    cr = cc;
    advance(cr);
    if (PACKED) cursor_uniform(cr);
    if (cr.valid) load_idx(cr);
    ci = cr;
    advance(ci);

    bf16x8_t qb0, qb1;
    float m_run = kNegBig, l_part = 0.f;
    f32x4_t o[4];
    uint32_t rowh = 0;   // DROP: hash of (seed, batch*head, token j of the tile)

    while (cc.valid) {
        if (PACKED) {
            cursor_uniform(cc);
            cursor_uniform(cr);
            cursor_uniform(ci);
        }
        if (cc.pair == 0) {   // a new tile: its Q rows arrived with the rows of this pair
            if (DROP) rowh = drop_row_hash(drop_bh_hash(a.drop_seed, cc.bh), cc.tile * 16 + j);
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
            if (a.seq_len) {   // uniform
                wave_lds_sync();
                mask_bias(a, bias_s, cc.tile * 16, seq_length_u(a.seq_len, cc.bh / a.H, a.n), g, j);
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
        if (DROP) {   // dropout acts on the weighted sum of values only: the row sum keeps every edge
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    sc[c][r] *= drop_scale(rowh, (uint32_t)relid_s[max(cid[c][r], 0)], a.drop_thr, a.drop_inv_keep);
        }
        // the accumulators hold out^T, C[m = feature][n = token]: all four values of a lane belong to its token j
#pragma unroll
        for (int f = 0; f < 4; ++f)
#pragma unroll
            for (int r = 0; r < 4; ++r) o[f][r] *= corr;
        u32x4 pa;
        pa.x = pack_bf16(sc[0][0], sc[0][1]);
        pa.y = pack_bf16(sc[0][2], sc[0][3]);
        pa.z = pack_bf16(sc[1][0], sc[1][1]);
        pa.w = pack_bf16(sc[1][2], sc[1][3]);
        const bf16x8_t pA = __builtin_bit_cast(bf16x8_t, pa);
#pragma unroll
        for (int f = 0; f < 4; ++f)
            o[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lds_transposed_b(v_s, kRowStride, f, g, j), pA, o[f], 0, 0, 0);

        if (cc.pair == cc.npairs - 1) {   // the tile is complete
            const int64_t base = (int64_t)(cc.bh / a.H) * a.sb + (int64_t)(cc.bh % a.H) * a.sh;
            const int t0 = cc.tile * 16;
            const int len = seq_length_u(a.seq_len, cc.bh / a.H, a.n);   // tokens past the end give zeros
            // row sums: token j is spread over the 4 lane groups
            float l = l_part + __shfl_xor(l_part, 16);
            l += __shfl_xor(l, 32);
            // packed batch: the token rows of the sequence begin at row level_delta(.., 0), and a row past the end of
            // the sequence is some other node's row: nothing is stored there
            const int row0 = PACKED ? t0 + level_delta(cc.dvec, 0) : t0;
            constexpr bool guard = PACKED;
            const int64_t lse_at = PACKED ? (int64_t)(cc.bh / a.H) * a.lse_sb + (int64_t)(cc.bh % a.H) * a.lse_sh : (int64_t)cc.bh * a.N;
            if (g == 0 && !(guard && t0 + j >= len)) a.lse[lse_at + row0 + j] = t0 + j < len ? (m_run + fast_log2(l)) * kLn2 : 0.f;
            // out^T = V^T P^T (the operands of P V changed places: the same registers): lane (g, j) holds features
            // 16f + 4g .. + 3 of token j.  The rows go through k_s (this pair's products have read it; the next
            // pair's rows are written behind the barrier at the top of the loop) and leave as whole rows, 16 bytes
            // per lane: a store instruction writes eight rows of 128 contiguous bytes.
            const float inv = t0 + j < len ? 1.f / l : 0.f;
            wave_lds_sync();
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const u32x2 w = {pack_bf16(o[f][0] * inv, o[f][1] * inv), pack_bf16(o[f][2] * inv, o[f][3] * inv)};
                *reinterpret_cast<u32x2*>(k_s + j * kRowStride + 16 * f + 4 * g) = w;
            }
            wave_lds_sync();
            bf16_t* orow = a.out + base + (int64_t)row0 * a.sn + piece * 8;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const int row = 8 * h + r8;
                if (guard && t0 + row >= len) continue;
                store_once(reinterpret_cast<uint4*>(orow + (int64_t)row * a.sn),
                           *reinterpret_cast<const uint4*>(k_s + row * kRowStride + piece * 8));
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
// no online softmax and no second pass).  Without DENSE, (w, p) of every tile slot goes to `wp` in
// tile order for rel_grad_tile_kernel, which also adds the relative-position part of dQ.
// REL_LDS: the compact relative-position table is staged in LDS; otherwise (large tables) its rows
// are read from memory when a tile forms its bias table.
// DENSE (needs REL_LDS and cid_pad a multiple of 32): a tile's w = p dP and p are not stored per slot
// for rel_grad_tile_kernel but scattered into two LDS tables [token][compact id] (the ids of a token
// row are distinct).  When the tile is complete and delta is known, dS = w - delta p is there as a
// dense 16 x cid_pad matrix (kept as bf16 hi + lo in the row buffers): the relative-position part of
// dQ, scale * dS x Rel, is taken at once (A operands from those tables, B operands by transposing
// reads of the staged table), and so is the tile's share of d_rel, dS^T x Q, with both operands from
// transposing reads, into accumulators the wavefront keeps over all its tiles (at most kDenseChunks
// chunks of 16 ids).  Nothing per slot or per tile leaves for a d_rel kernel; every workgroup writes
// one copy of d_rel at the end, and drel_reduce_kernel adds the copies in a fixed order.
template <bool REL_LDS, bool DROP, bool DENSE = false, bool PACKED = false>
__global__ void __launch_bounds__(kTileThreads, DENSE ? 1 : 2) bwd_q_tile_kernel(const TileArgs a) {
    static_assert(!DENSE || REL_LDS, "the dense variant multiplies by the staged table");
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
    int32_t* relid_s = reinterpret_cast<int32_t*>(smem + rel_bytes + (size_t)kTileWaves * 16 * a.bias_stride * sizeof(float) +
                                                  (size_t)kTileWaves * 64 * kRowStride * sizeof(bf16_t));   // [cid_pad], DROP
    // DENSE: (w, p) of the tile, [16 tokens][cid_pad + 2] pairs, after relid_s (the region is sized as two tables of
    // bias_stride floats per token; a row of cid_pad + 2 pairs puts 8 consecutive tokens on different banks)
    float* w_s = reinterpret_cast<float*>(relid_s + a.cid_pad) + (size_t)wave * 32 * a.bias_stride;
    float2* wp_s = reinterpret_cast<float2*>(w_s);
    const int wp_stride = a.cid_pad + 2;
    if (DROP)
        for (int i = threadIdx.x; i < a.cid_pad; i += blockDim.x) relid_s[i] = i < a.num_cids ? a.cid_to_id[i] : 0;
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
    // sequences of different lengths: walk the tiles that exist, and first write the zero rows of the others
    __shared__ int pref_s[kMaxLenBatch + 1];
    const int nbatch = a.BH / a.H;
    const bool compact = a.seq_len && nbatch <= kMaxLenBatch;
    int live_total = 0;
    auto zero_rows = [&](int bh, int tile) {   // dQ of a tile past the end of its sequence; `stat` switches its rows off on the key side
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        const int64_t qrow = base + (int64_t)(tile * 16 + r8) * a.sn + piece * 8;
        if (!a.leave_unkept) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                store_grad4(a.dQ, qrow + (int64_t)8 * h * a.sn, make_float4(0.f, 0.f, 0.f, 0.f), a.grad_bf16);
                store_grad4(a.dQ, qrow + (int64_t)8 * h * a.sn + 4, make_float4(0.f, 0.f, 0.f, 0.f), a.grad_bf16);
            }
        }
        if (lane < 16) a.stat[(int64_t)bh * a.N + tile * 16 + lane] = make_float2(kLseGone, 0.f);
    };
    if (compact) {
        live_tiles_prefix(pref_s, a.seq_len, nbatch, a.n, a.num_tiles);
        live_total = a.H * pref_s[nbatch];
        const int dead_total = a.BH * a.num_tiles - live_total;
        for (TileWalk wd((dead_total + kTileWaves - 1) / kTileWaves); wd.t < wd.t_end; wd.t += wd.step) {
            const int idx = wd.t * kTileWaves + wave;
            if (idx < dead_total) {
                int bh, tile;
                nth_tile(pref_s, nbatch, a.H, a.num_tiles, true, idx, bh, tile);
                zero_rows(bh, tile);
            }
        }
    }
    const TileWalk w(compact ? (live_total + kTileWaves - 1) / kTileWaves : a.BH * groups_per_bh);

    // The wavefront's work is one sequence of pairs of chunks running through its tiles.
    // Three positions move along it: `cc` is computed, the rows of `cr` (one pair ahead) are
    // in flight, the column ids and map words of `ci` (two pairs ahead) are in flight.
    // Tiles past the end of a shorter sequence are not computed (see fwd_tile_kernel): zero dQ rows,
    // and `stat` entries that switch the rows off on the key side; their (w, p) slots stay unwritten
    // and rel_grad_tile_kernel does not read them.
    auto enter_tile = [&](TileCursor& c) {
        c.valid = false;
        c.pair = 0;
        c.npairs = 1;
        c.dvec = 0;
        if (PACKED) c.t = __builtin_amdgcn_readfirstlane(c.t);   // (see cursor_uniform)
        if (compact) {   // the next tile that exists; the walk covers nothing else
            const int idx = c.t * kTileWaves + wave;
            if (c.t < w.t_end && idx < live_total) {
                nth_tile(pref_s, nbatch, a.H, a.num_tiles, false, idx, c.bh, c.tile);
                if (PACKED) {
                    c.bh = __builtin_amdgcn_readfirstlane(c.bh);
                    c.tile = __builtin_amdgcn_readfirstlane(c.tile);
                }
                c.cp0 = uniform_i32(a.chunk_ptr, c.tile);
                c.npairs = (uniform_i32(a.chunk_ptr, c.tile + 1) - c.cp0) >> 1;
                c.dvec = PACKED ? load_delta(a.delta, nbatch, c.bh / a.H, lane, a.levels) : 0;
                c.valid = true;
            }
            return;
        }
        for (; c.t < w.t_end; c.t += w.step) {
            const int slab = c.t / groups_per_bh;
            c.bh = walk_bh(a.seq_len, slab, a.BH, a.H);
            c.tile = walk_pos(a.seq_len, slab, c.t - slab * groups_per_bh, groups_per_bh) * kTileWaves + wave;
            if (c.tile >= a.num_tiles) continue;
            if (a.seq_len && c.tile * 16 >= seq_length_u(a.seq_len, c.bh / a.H, a.n)) {
                zero_rows(c.bh, c.tile);
                continue;
            }
            c.cp0 = uniform_i32(a.chunk_ptr, c.tile);
            c.npairs = (uniform_i32(a.chunk_ptr, c.tile + 1) - c.cp0) >> 1;
            c.dvec = PACKED ? load_delta(a.delta, nbatch, c.bh / a.H, lane, a.levels) : 0;
            c.valid = true;
            return;
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
                const int node = PACKED ? packed_row(node_n[ci][h], a.lg, c.dvec) : node_n[ci][h];
                const int off = (int)__umul24(node, a.row_bytes) + piece * 16;
                buf_row(rK, off, kr[ci][h]);
                buf_row(rV, off, vr[ci][h]);
            }
        if (c.pair == 0) {   // the tile's own rows: Q^T and dO^T operands (token j, features 16g..16g+15)
            // (packed batch: a token past the end of the sequence reads the sequence's last row instead of another node's)
            const int tq = PACKED ? min(c.tile * 16 + j, seq_length_u(a.seq_len, c.bh / a.H, a.n) - 1) + level_delta(c.dvec, 0)
                                   : c.tile * 16 + j;
            const int64_t at = base + (int64_t)tq * a.sn + 16 * g;
            qn0 = load_once16<bf16x8_t>(a.Q + at);
            qn1 = load_once16<bf16x8_t>(a.Q + at + 8);
            gn0 = load_once16<bf16x8_t>(a.dout + at);
            gn1 = load_once16<bf16x8_t>(a.dout + at + 8);
            lse_n = a.lse_r[(PACKED ? (int64_t)(c.bh / a.H) * a.lse_sb + (int64_t)(c.bh % a.H) * a.lse_sh : (int64_t)c.bh * a.N) + tq];
        }
    };

    // DENSE: this wavefront's d_rel sums over its tiles, [id chunk][feature chunk] in the C layout (id 4g + r
    // of the chunk, feature 16f + j); written once, as this wavefront's copy, in compact-id order
    f32x4_t racc[DENSE ? kDenseChunks : 1][4];
#pragma unroll
    for (int c = 0; c < (DENSE ? kDenseChunks : 1); ++c)
#pragma unroll
        for (int f = 0; f < 4; ++f) racc[c][f] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    // the four wavefronts' sums are added in wavefront order through LDS (all of it is free by then: every
    // wavefront of the workgroup comes here exactly once, at its end) and leave as the workgroup's copy
    auto write_drel = [&]() {
        if (!DENSE) return;
        __syncthreads();   // no wavefront of the workgroup still uses its tables
        float* sum_s = reinterpret_cast<float*>(smem);   // [4 wavefronts][cid_pad][64]
#pragma unroll
        for (int c = 0; c < (DENSE ? kDenseChunks : 1); ++c)
            if (16 * c < a.cid_pad) {
#pragma unroll
                for (int f = 0; f < 4; ++f)
#pragma unroll
                    for (int m = 0; m < 4; ++m)
                        sum_s[((size_t)wave * a.cid_pad + 16 * c + 4 * g + m) * kD + 16 * f + j] = racc[c][f][m];
            }
        __syncthreads();
        float* out = a.drel_part + (int64_t)blockIdx.x * a.cid_pad * kD;
        const int count = a.cid_pad * kD;
        for (int i = threadIdx.x * 4; i < count; i += kTileThreads * 4) {
            f32x4_t t = *reinterpret_cast<const f32x4_t*>(sum_s + i);
#pragma unroll
            for (int w2 = 1; w2 < kTileWaves; ++w2) {
                const f32x4_t x = *reinterpret_cast<const f32x4_t*>(sum_s + (size_t)w2 * count + i);
                t[0] += x[0]; t[1] += x[1]; t[2] += x[2]; t[3] += x[3];
            }
            *reinterpret_cast<f32x4_t*>(out + i) = f32x4_t{t[0] * a.scale, t[1] * a.scale, t[2] * a.scale, t[3] * a.scale};
        }
    };

    TileCursor cc, cr, ci;
    cc.t = w.t;
    enter_tile(cc);
    if (!cc.valid) {
        write_drel();
        return;
    }
    if (PACKED) cursor_uniform(cc);
    load_idx(cc);
    request_rows(cc);
    uint2 mp[2] = {mp_n[0], mp_n[1]};
    cr = cc;
    advance(cr);
    if (PACKED) cursor_uniform(cr);
    if (cr.valid) load_idx(cr);
    ci = cr;
    advance(ci);

    bf16x8_t qb0, qb1, gb0, gb1;
    float lse2 = 0.f, dl_part = 0.f;
    float2* wp_t = a.wp;   // this (batch, head)'s pairs, in tile order: [chunk][token][16 columns]
    f32x4_t ow[4], op[4];
    uint32_t rowh = 0;   // DROP: hash of (seed, batch*head, token j of the tile)
    bool tables_clear = false;   // DENSE: the (w, p) table holds zeros

    while (cc.valid) {
        if (PACKED) {
            cursor_uniform(cc);
            cursor_uniform(cr);
            cursor_uniform(ci);
        }
        if (cc.pair == 0) {   // a new tile: its operands arrived with the rows of this pair
            if (DROP) rowh = drop_row_hash(drop_bh_hash(a.drop_seed, cc.bh), cc.tile * 16 + j);
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
            if (a.seq_len) {   // uniform
                wave_lds_sync();
                mask_bias(a, bias_s, cc.tile * 16, seq_length_u(a.seq_len, cc.bh / a.H, a.n), g, j);
            }
            if (DENSE && !tables_clear) {   // the whole region once; later tiles find it cleared by the reads below
                for (int i = lane * 4; i < 32 * a.bias_stride; i += 256)
                    *reinterpret_cast<f32x4_t*>(w_s + i) = f32x4_t{0.f, 0.f, 0.f, 0.f};
                tables_clear = true;
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
                // with dropout out = sum keep p v, so dP carries the mask
                const float keep = DROP ? drop_scale(rowh, (uint32_t)relid_s[max(cid[c][r], 0)], a.drop_thr, a.drop_inv_keep) : 1.f;
                const float wgt = p * d4[c][r] * keep;
                dl_part += wgt;
                pw[c][r] = wgt;
                pp[c][r] = p;
            }
            if (DENSE) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    // a slot without an edge (w = p = 0) goes to the first padding column, which nothing reads
                    wp_s[j * wp_stride + (cid[c][r] >= 0 ? cid[c][r] : a.cid_pad)] = make_float2(pw[c][r], pp[c][r]);
            } else {
                // (w, p) of this lane's 4 columns: 32 contiguous bytes, a chunk is 2 KB contiguous
                float4* dst = reinterpret_cast<float4*>(wp_t + ((int64_t)(cc.cp0 + 2 * cc.pair + c) * 16 + j) * 16 + 4 * g);
                store_once(dst, make_float4(pw[c][0], pp[c][0], pw[c][1], pp[c][1]));
                store_once(dst + 1, make_float4(pw[c][2], pp[c][2], pw[c][3], pp[c][3]));
            }
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
            // transposed, C[m = feature][n = token] (the operands of W K changed places, the registers are the same):
            // all values of a lane belong to its token j, and a lane holds 4 consecutive features of the row
            ow[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kB, wH, ow[f], 0, 0, 0);
            ow[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kB, wL, ow[f], 0, 0, 0);
            op[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kB, pH, op[f], 0, 0, 0);
            op[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kB, pL, op[f], 0, 0, 0);
        }
        if (cc.pair == cc.npairs - 1) {   // the tile is complete
            const int64_t base = (int64_t)(cc.bh / a.H) * a.sb + (int64_t)(cc.bh % a.H) * a.sh;
            const int t0 = cc.tile * 16;
            float delta = dl_part + __shfl_xor(dl_part, 16);
            delta += __shfl_xor(delta, 32);
            const int len = seq_length_u(a.seq_len, cc.bh / a.H, a.n);
            if (g == 0) a.stat[(int64_t)cc.bh * a.N + t0 + j] = make_float2(t0 + j < len ? lse2 : kLseGone, delta);
            f32x4_t dqr[4];
#pragma unroll
            for (int f = 0; f < 4; ++f) dqr[f] = f32x4_t{0.f, 0.f, 0.f, 0.f};
            if (DENSE) {
                wave_lds_sync();   // the scattered w and p of all lanes are in place
                // dS as bf16 hi and lo, [16 tokens][cid_pad + 8], in the row buffers (free until the next pair is staged)
                const int dstride = a.cid_pad + 8;
                bf16_t* ds_h = k_s;
                bf16_t* ds_l = k_s + 16 * dstride;
                // relative-position part of dQ: dS [token j][ids] x Rel [ids][features]
                for (int ks = 0; ks < a.cid_pad; ks += 32) {
                    // 8 pairs of row j, (w, p) (w, p) in every 16 bytes; this lane is their only reader and leaves them
                    // cleared for the next tile
                    f32x4_t* pairs = reinterpret_cast<f32x4_t*>(wp_s + j * wp_stride + ks + 8 * g);
                    const f32x4_t x0 = pairs[0], x1 = pairs[1], x2 = pairs[2], x3 = pairs[3];
#pragma unroll
                    for (int i = 0; i < 4; ++i) pairs[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
                    uint32_t hi[4], lo[4];
                    split_pack(x0[0] - delta * x0[1], x0[2] - delta * x0[3], hi[0], lo[0]);
                    split_pack(x1[0] - delta * x1[1], x1[2] - delta * x1[3], hi[1], lo[1]);
                    split_pack(x2[0] - delta * x2[1], x2[2] - delta * x2[3], hi[2], lo[2]);
                    split_pack(x3[0] - delta * x3[1], x3[2] - delta * x3[3], hi[3], lo[3]);
                    const u32x4 xh = {hi[0], hi[1], hi[2], hi[3]}, xl = {lo[0], lo[1], lo[2], lo[3]};
                    const bf16x8_t aH = __builtin_bit_cast(bf16x8_t, xh), aL = __builtin_bit_cast(bf16x8_t, xl);
                    *reinterpret_cast<u32x4*>(ds_h + j * dstride + ks + 8 * g) = xh;
                    *reinterpret_cast<u32x4*>(ds_l + j * dstride + ks + 8 * g) = xl;
#pragma unroll
                    for (int f = 0; f < 4; ++f) {
                        const bf16x8_t rB = lds_tr8(rel_s, kRelStride, ks + 8 * g, 16 * f, j);
                        dqr[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rB, aH, dqr[f], 0, 0, 0);   // transposed as well
                        dqr[f] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rB, aL, dqr[f], 0, 0, 0);
                    }
                }
                // d_rel += dS^T [ids][16 tokens] x Q [16 tokens][features], 16 ids at a time: the A operand is one
                // transposing read of dS (tokens 4g .. 4g + 3 of id 16c + j), the B operand one of the tile's Q
                // rows, put row-major where the bias table was (dead once the tile is complete)
                bf16_t* q_t = reinterpret_cast<bf16_t*>(bias_s);   // [16 tokens][kRowStride]
                *reinterpret_cast<bf16x8_t*>(q_t + j * kRowStride + 16 * g) = qb0;
                *reinterpret_cast<bf16x8_t*>(q_t + j * kRowStride + 16 * g + 8) = qb1;
                wave_lds_sync();
                s16x4_t qB[4];
#pragma unroll
                for (int f = 0; f < 4; ++f) qB[f] = lds_tr4(q_t, kRowStride, 4 * g, 16 * f, j);
#pragma unroll
                for (int c = 0; c < kDenseChunks; ++c)
                    if (16 * c < a.cid_pad) {
                        const s16x4_t aH = lds_tr4(ds_h, dstride, 4 * g, 16 * c, j), aL = lds_tr4(ds_l, dstride, 4 * g, 16 * c, j);
#pragma unroll
                        for (int f = 0; f < 4; ++f) {
                            racc[c][f] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(aH, qB[f], racc[c][f], 0, 0, 0);
                            racc[c][f] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(aL, qB[f], racc[c][f], 0, 0, 0);
                        }
                    }
                wave_lds_sync();   // before the next tile clears the tables and forms its bias table
            }
            // dQ rows of the tile, lane (g, j): features 16f + 4g .. + 3 of token j.  They go through the row buffers
            // (free until the next pair is staged behind the barrier at the top of the loop) and leave as whole rows,
            // 16 bytes per lane: a store instruction writes four rows of 256 (fp32) or eight of 128 (bf16) contiguous
            // bytes.  Packed batch: the sequence's token rows begin at row level_delta(.., 0); a row past its end is
            // not stored.
            const int64_t qrow_out = base + (int64_t)(PACKED ? t0 + level_delta(cc.dvec, 0) : t0) * a.sn;
            const int live = PACKED ? len - t0 : 16;   // rows of the tile that may be stored
            if (j < live) {
                if (a.grad_bf16) {
                    bf16_t* dst = reinterpret_cast<bf16_t*>(a.dQ) + qrow_out + (int64_t)j * a.sn + 4 * g;
#pragma unroll
                    for (int f = 0; f < 4; ++f) {
                        float x[4];
#pragma unroll
                        for (int r = 0; r < 4; ++r) x[r] = a.scale * (ow[f][r] - delta * op[f][r] + dqr[f][r]);
                        typedef uint32_t vec2 __attribute__((ext_vector_type(2)));
                        const vec2 w = {pack_bf16(x[0], x[1]), pack_bf16(x[2], x[3])};
                        __builtin_nontemporal_store(w, reinterpret_cast<vec2*>(dst + 16 * f));
                    }
                } else {
                    float* dst = a.dQ + qrow_out + (int64_t)j * a.sn + 4 * g;
#pragma unroll
                    for (int f = 0; f < 4; ++f) {
                        float4 x;
                        x.x = a.scale * (ow[f][0] - delta * op[f][0] + dqr[f][0]);
                        x.y = a.scale * (ow[f][1] - delta * op[f][1] + dqr[f][1]);
                        x.z = a.scale * (ow[f][2] - delta * op[f][2] + dqr[f][2]);
                        x.w = a.scale * (ow[f][3] - delta * op[f][3] + dqr[f][3]);
                        store_once(reinterpret_cast<float4*>(dst + 16 * f), x);
                    }
                }
            }
        }
        cc = cr;
        cr = ci;
        advance(ci);
    }
    write_drel();
}


// d_rel and the relative-position part of dQ over the token tiles' compact ids (bf16
// tensors, at most 256 ids in use).  Per block of 32 token rows the workgroup builds
// DS^T[id][row] (hi and lo halves) in LDS from the (w, p) pairs of the query side: every
// edge of a token row carries a 16-bit code = compact id * 32 + row % 32 (tile metadata),
// so an edge needs no search for its row and no lookup of its id.  Q rows are staged
// row-major and enter the products through transposing LDS reads:
//   d_rel[id][f] += DS^T (A, 16-byte rows) x Q (B, transposed read),
//   dQ[row][f]   += scale * DS x Rel, formed transposed (Rel^T DS^T, both operands transposed reads) so that a
//                   lane adds to 16 contiguous bytes of a row.
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
    const int32_t* seq_len;   // [B] tokens of every sequence, or null
    int32_t grad_bf16;        // dQ holds bf16 elements
    const int32_t* delta;     // packed batch: delta[level][sequence] (only the token level is used here), or null
};
// tile slots per thread fetched one block ahead: 8 (512 threads: 16 chunks) with up to 256 ids, 24 with more --
// those graphs have 25..30 slots per thread and block, and one workgroup per compute unit to hide their latency
template <int CPW>
struct RgPrefetch {
    static constexpr int value = CPW == 2 ? 8 : 32;
};
constexpr int kRgTileMaxIds = 512;
// CPW: 16-id chunks per wavefront (2: up to 256 ids, 4: up to 512)
template <int CPW, bool PACKED = false>
__global__ void __launch_bounds__(kThreads, CPW == 2 ? 4 : 2) rel_grad_tile_kernel(const RelGradArgs a) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int kRgPrefetch = RgPrefetch<CPW>::value;
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
        const int bh = blk / blocks_per_bh, b2 = 2 * walk_pos(a.seq_len, bh, blk - bh * blocks_per_bh, blocks_per_bh), row0 = 16 * b2;
        const int64_t base = (int64_t)(bh / a.H) * a.sb + (int64_t)(bh % a.H) * a.sh;
        // token tiles past the end of a shorter sequence were not computed: their slots do not count
        const int len = seq_length_u(a.seq_len, bh / a.H, a.n);
        s_begin = uniform_i32(a.chunk_ptr, b2) * 256;
        s_mid = uniform_i32(a.chunk_ptr, min(b2 + 1, a.num_tiles)) * 256;
        s_end = row0 + 16 < len ? uniform_i32(a.chunk_ptr, min(b2 + 2, a.num_tiles)) * 256 : s_mid;
        qpiece = make_uint4(0u, 0u, 0u, 0u);
        if (threadIdx.x < kRgRows * 8) {
            const int r = threadIdx.x >> 3, c = (threadIdx.x & 7) * 8;
            // packed batch: the sequence's token rows begin at its delta of level 0; rows past its end are other nodes'
            const int live = PACKED ? len : a.n, tok0 = PACKED ? a.delta[bh / a.H] : 0;
            if (row0 + r < live) qpiece = *reinterpret_cast<const uint4*>(a.Q + base + (int64_t)(row0 + r + tok0) * a.sn + c);
        } else if (threadIdx.x < kRgRows * 8 + kRgRows) {
            const int r = threadIdx.x - kRgRows * 8;
            dl_own = row0 + r < a.n ? a.stat[(int64_t)bh * a.N + row0 + r].y : 0.f;
        }
        const rsrc_t rWp = make_rsrc(a.wp + (int64_t)bh * a.num_chunks * 256, (uint32_t)a.num_chunks * 2048u);
#pragma unroll
        for (int k = 0; k < kRgPrefetch; ++k) {
            if (k >= 8 && s_begin + k * kThreads >= s_end) break;   // uniform: no slot of the block is that far
            const int sl = s_begin + (int)threadIdx.x + k * kThreads;
            const uint32_t off = sl < s_end ? (uint32_t)sl : 0x1FFFFFFFu;   // past the block: an offset outside the buffers
            code[k] = (int)(short)__builtin_amdgcn_raw_buffer_load_b16(rMap, (int)(off * 2u), 0, 0);
            wpv[k] = buf_f2_once(rWp, (int)(off * 8u));
        }
    };
    // blocks past the end of a shorter sequence add nothing and are stepped over (uniform for the workgroup)
    auto next_block = [&](int blk) {
        if (a.seq_len)
            for (; blk < total; blk += gridDim.x) {
                const int bh = blk / blocks_per_bh;
                if (walk_pos(a.seq_len, bh, blk - bh * blocks_per_bh, blocks_per_bh) * kRgRows < seq_length_u(a.seq_len, bh / a.H, a.n)) break;
            }
        return blk;
    };
    int blk = next_block(blockIdx.x);
    if (blk < total) prefetch(blk);

    while (blk < total) {
        const int bh = blk / blocks_per_bh, row0 = walk_pos(a.seq_len, bh, blk - bh * blocks_per_bh, blocks_per_bh) * kRgRows;
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
        // (the product below is formed transposed, C[m = feature][n = row]: a lane holds features 16fc + 4g .. + 3 of row j)
        const int live = PACKED ? seq_length_u(a.seq_len, bh / a.H, a.n) : a.n, tok0 = PACKED ? a.delta[bh / a.H] : 0;
        const int dq_row = row0 + 16 * mc + j;
        const int64_t dq_at = base + (int64_t)(dq_row + tok0) * a.sn + 16 * fc + 4 * g;
        const float4 dq_old = dq_row < live ? load_grad4(a.dQ, dq_at, a.grad_bf16) : make_float4(0.f, 0.f, 0.f, 0.f);
        const int blk_next = next_block(blk + gridDim.x);
        if (blk_next < total) prefetch(blk_next);
        __syncthreads();
        {   // dQ of the block: wavefront -> 16 rows x 16 features
            f32x4_t dq = {0.f, 0.f, 0.f, 0.f};
            for (int ks = 0; ks < nids; ks += 32) {
                const bf16x8_t rb = lds_tr8(rel_s, kRelStride, ks + 8 * g, 16 * fc, j);
                dq = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rb, lds_tr8(ds_hi, kRgStride, ks + 8 * g, 16 * mc, j), dq, 0, 0, 0);
                dq = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rb, lds_tr8(ds_lo, kRgStride, ks + 8 * g, 16 * mc, j), dq, 0, 0, 0);
            }
            if (dq_row < live)
                store_grad4(a.dQ, dq_at,
                            make_float4(dq_old.x + a.scale * dq[0], dq_old.y + a.scale * dq[1], dq_old.z + a.scale * dq[2],
                                        dq_old.w + a.scale * dq[3]), a.grad_bf16);
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
        blk = blk_next;
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

}  // namespace
}  // namespace bpt
