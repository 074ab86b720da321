// Metadata of the matrix-core attention kernels, built on the GPU from the CSR of the
// binary-partition graph (paper Sec. 3.2): dense tiles over 16 consecutive token rows and
// dense tiles over 16 consecutive key nodes of one tree level (layouts in bpt_internal.h).
// Everything here is integer work whose result does not depend on thread order (the only
// atomics are integer min / max in LDS).
#include <algorithm>
#include <vector>

#include "bpt_internal.h"

namespace bpt {
namespace {

constexpr int kTB = 256;
constexpr int kScanItems = 16;
constexpr int kScanBlock = kTB * kScanItems;   // elements per block of the scan
constexpr int kMaxLevels = 24;                 // n <= 2^22
constexpr int kMaxSortedTasks = 1 << 16;       // key-tile tasks are put in stretch order up to this many (the ordering is quadratic)
constexpr int kMaxBuckets = 2 * kMaxLevels;
constexpr int kChainChunks = 16;               // key tiles of at most this many chunks are chained

__host__ __device__ inline int level_off(int n, int level) { return 2 * n - ((2 * n) >> level); }

struct DeviceBuf {  // frees on scope exit unless released
    void* p = nullptr;
    ~DeviceBuf() {
        if (p) (void)hipFree(p);
    }
    hipError_t alloc(size_t bytes) { return hipMalloc(&p, bytes ? bytes : 4); }
    template <typename T>
    T* as() const {
        return static_cast<T*>(p);
    }
    template <typename T>
    T* release() {
        T* r = static_cast<T*>(p);
        p = nullptr;
        return r;
    }
};

// ---- exclusive scan of int32, total written on the device ----------------------------
__global__ void tscan_blocks(const int32_t* __restrict__ in, int32_t* __restrict__ out, int32_t* __restrict__ block_sums,
                             int m) {
    __shared__ int32_t s[kTB];
    const int base = blockIdx.x * kScanBlock + threadIdx.x * kScanItems;
    int32_t v[kScanItems], sum = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        v[j] = base + j < m ? in[base + j] : 0;
        sum += v[j];
    }
    s[threadIdx.x] = sum;
    __syncthreads();
    for (int off = 1; off < kTB; off <<= 1) {
        const int32_t t = (int)threadIdx.x >= off ? s[threadIdx.x - off] : 0;
        __syncthreads();
        s[threadIdx.x] += t;
        __syncthreads();
    }
    int32_t run = s[threadIdx.x] - sum;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (base + j < m) out[base + j] = run;
        run += v[j];
    }
    if (threadIdx.x == kTB - 1) block_sums[blockIdx.x] = s[threadIdx.x];
}

// one block; nblocks <= kScanBlock; block_sums[nblocks] receives the grand total
__global__ void tscan_sums(int32_t* __restrict__ block_sums, int nblocks) {
    __shared__ int32_t s[kTB];
    const int base = threadIdx.x * kScanItems;
    int32_t v[kScanItems], sum = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        v[j] = base + j < nblocks ? block_sums[base + j] : 0;
        sum += v[j];
    }
    s[threadIdx.x] = sum;
    __syncthreads();
    for (int off = 1; off < kTB; off <<= 1) {
        const int32_t t = (int)threadIdx.x >= off ? s[threadIdx.x - off] : 0;
        __syncthreads();
        s[threadIdx.x] += t;
        __syncthreads();
    }
    int32_t run = s[threadIdx.x] - sum;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        if (base + j < nblocks) block_sums[base + j] = run;
        run += v[j];
    }
    if (threadIdx.x == kTB - 1) block_sums[nblocks] = s[threadIdx.x];
}

__global__ void tscan_add(int32_t* __restrict__ out, const int32_t* __restrict__ block_sums, int m, int nblocks,
                          int32_t* __restrict__ total_out) {
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < m) out[idx] += block_sums[idx / kScanBlock];
    if (idx == m) {
        out[m] = block_sums[nblocks];
        if (total_out) *total_out = block_sums[nblocks];
    }
}

// out[0..m] = exclusive prefix sums of in[0..m-1] (out[m] = total, also stored to *total_out)
int dev_scan(const int32_t* in, int32_t* out, int m, int32_t* block_sums, int32_t* total_out, hipStream_t st) {
    const int nblocks = (m + kScanBlock - 1) / kScanBlock;
    if (nblocks > kScanBlock) return BPT_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(tscan_blocks, dim3(std::max(nblocks, 1)), dim3(kTB), 0, st, in, out, block_sums, m);
    hipLaunchKernelGGL(tscan_sums, dim3(1), dim3(kTB), 0, st, block_sums, nblocks);
    hipLaunchKernelGGL(tscan_add, dim3((m + 1 + kTB - 1) / kTB), dim3(kTB), 0, st, out, block_sums, m, nblocks, total_out);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

// ---- token tiles ---------------------------------------------------------------------------
__global__ void mark_ids(const int32_t* __restrict__ rel, int32_t e_tok, int32_t* __restrict__ used) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e < e_tok) used[rel[e]] = 1;   // every writer stores the same value
}

__global__ void finish_ids(const int32_t* __restrict__ used, const int32_t* __restrict__ pos, int num_ids,
                           int32_t* __restrict__ id_to_cid, int32_t* __restrict__ cid_to_id) {
    const int id = blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= num_ids) return;
    if (used[id]) {
        id_to_cid[id] = pos[id];
        cid_to_id[pos[id]] = id;
    } else {
        id_to_cid[id] = -1;
    }
}

__device__ inline int token_bucket(int rel_id, int W, int zero) {   // 0: level 0; 2l-1 / 2l: left / right of level l
    const int lev = rel_id / W, ord = rel_id % W - zero;
    return lev == 0 ? 0 : 2 * lev - 1 + (ord > 0 ? 1 : 0);
}

// one workgroup (64 threads) per tile of 16 token rows: node range of every (level, side)
// bucket, the slot at which the bucket starts, and the number of 16-column chunks (even)
__global__ void token_tile_ranges(int tiles, int nb, int W, int zero, const int32_t* __restrict__ row_ptr,
                                  const int32_t* __restrict__ col, const int32_t* __restrict__ rel,
                                  int32_t* __restrict__ tile_lo, int32_t* __restrict__ tile_hi,
                                  int32_t* __restrict__ tile_first, int32_t* __restrict__ tile_nch) {
    __shared__ int lo[kMaxBuckets], hi[kMaxBuckets];
    const int t = blockIdx.x;
    for (int q = threadIdx.x; q < nb; q += blockDim.x) {
        lo[q] = INT32_MAX;
        hi[q] = -1;
    }
    __syncthreads();
    const int e1 = row_ptr[16 * t + 16];
    for (int e = row_ptr[16 * t] + threadIdx.x; e < e1; e += blockDim.x) {
        const int q = token_bucket(rel[e], W, zero), c = col[e];
        atomicMin(&lo[q], c);
        atomicMax(&hi[q], c);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int total = 0;
        for (int q = 0; q < nb; ++q) {
            tile_lo[(int64_t)t * nb + q] = lo[q];
            tile_hi[(int64_t)t * nb + q] = hi[q];
            tile_first[(int64_t)t * nb + q] = total;
            if (hi[q] >= 0) total += hi[q] - lo[q] + 1;
        }
        int nch = (total + 15) / 16;
        nch += nch & 1;   // even: the kernels consume chunks in pairs
        tile_nch[t] = nch;
    }
}

// one workgroup per tile: the node of every column; padding columns point at a real node and stay masked
__global__ void token_tile_cols(int nb, const int32_t* __restrict__ chunk_ptr, const int32_t* __restrict__ tile_lo,
                                const int32_t* __restrict__ tile_hi, const int32_t* __restrict__ tile_first,
                                int32_t* __restrict__ cols) {
    const int t = blockIdx.x;
    const int64_t c0 = (int64_t)chunk_ptr[t] * 16;
    const int ncols = (chunk_ptr[t + 1] - chunk_ptr[t]) * 16;
    for (int i = threadIdx.x; i < ncols; i += blockDim.x) cols[c0 + i] = 16 * t;
    __syncthreads();
    for (int q = 0; q < nb; ++q) {
        const int lo = tile_lo[(int64_t)t * nb + q], hi = tile_hi[(int64_t)t * nb + q];
        const int first = tile_first[(int64_t)t * nb + q];
        for (int v = lo + (int)threadIdx.x; hi >= 0 && v <= hi; v += blockDim.x) cols[c0 + first + (v - lo)] = v;
    }
}

// one thread per token row: the compact relative-position id of each of its edges at its (row, column) slot
__global__ void token_tile_map(int n, int nb, int W, int zero, const int32_t* __restrict__ row_ptr,
                               const int32_t* __restrict__ col, const int32_t* __restrict__ rel,
                               const int32_t* __restrict__ chunk_ptr, const int32_t* __restrict__ tile_lo,
                               const int32_t* __restrict__ tile_first, const int32_t* __restrict__ id_to_cid,
                               int16_t* __restrict__ map) {
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= n) return;
    const int t = u >> 4, r = u & 15;
    const int64_t m0 = (int64_t)chunk_ptr[t] * 256;
    const int e1 = row_ptr[u + 1];
    for (int e = row_ptr[u]; e < e1; ++e) {
        const int id = rel[e], q = token_bucket(id, W, zero);
        const int slot = tile_first[(int64_t)t * nb + q] + col[e] - tile_lo[(int64_t)t * nb + q];
        map[m0 + ((int64_t)(slot >> 4) * 16 + r) * 16 + (slot & 15)] = (int16_t)id_to_cid[id];
    }
}

// ---- key tiles -----------------------------------------------------------------------------
struct LevelBases {
    int32_t tile_base[kMaxLevels + 1];   // first tile of every level that has contextual edges
    int32_t chain[kMaxLevels];           // tiles of the level that one task walks (1: every tile has its own tasks)
};

// One thread per key tile: level, keys, the range of tokens that attend to it in each bucket
// (bucket 1: tokens that see the keys in their left context at a span level; bucket 0: the
// others, for token keys all of them and the keys themselves), where each bucket and the
// ancestors start, chunks, tasks.  The tokens attending to one node from one side are a
// contiguous range [first, first + count) (transposed-adjacency builder), so no atomics.
__global__ void key_tile_layout(int n, int num_levels, int ctx_levels, int nkt, int task_chunks, LevelBases lb,
                                const int32_t* __restrict__ cnt_l, const int32_t* __restrict__ min_l,
                                const int32_t* __restrict__ cnt_r, const int32_t* __restrict__ min_r,
                                int32_t* __restrict__ klo, int32_t* __restrict__ khi,
                                int32_t* __restrict__ tile_node0, int32_t* __restrict__ tile_info,
                                int32_t* __restrict__ kfirst, int32_t* __restrict__ anc_first,
                                int32_t* __restrict__ knch, int32_t* __restrict__ ntask, int32_t* __restrict__ npart,
                                int32_t* __restrict__ is_multi) {
    const int kt = blockIdx.x * blockDim.x + threadIdx.x;
    if (kt >= nkt) return;
    int l = 0;
    while (l + 1 < ctx_levels && lb.tile_base[l + 1] <= kt) ++l;
    const int m0 = (kt - lb.tile_base[l]) * 16, nkeys = min(16, (n >> l) - m0);
    const int node0 = level_off(n, l) + m0;
    tile_node0[kt] = node0;
    tile_info[kt] = l | (nkeys << 8);
    int lo[2] = {INT32_MAX, INT32_MAX}, hi[2] = {-1, -1};
    for (int key = 0; key < nkeys; ++key) {
        const int v = node0 + key;
        if (cnt_l[v] > 0) {   // tokens left of v: v is in their right context
            lo[0] = min(lo[0], min_l[v]);
            hi[0] = max(hi[0], min_l[v] + cnt_l[v] - 1);
        }
        if (cnt_r[v] > 0) {   // tokens right of v: v is in their left context
            const int b = l > 0 ? 1 : 0;
            lo[b] = min(lo[b], min_r[v]);
            hi[b] = max(hi[b], min_r[v] + cnt_r[v] - 1);
        }
        if (l == 0) {         // self edge
            lo[0] = min(lo[0], v);
            hi[0] = max(hi[0], v);
        }
    }
    int total = 0;
    for (int b = 0; b < 2; ++b) {
        klo[2 * kt + b] = lo[b];
        khi[2 * kt + b] = hi[b];
        kfirst[2 * kt + b] = total;
        if (hi[b] >= 0) total += hi[b] - lo[b] + 1;
    }
    anc_first[kt] = total;
    if (l == 0)   // ancestors of the tile's tokens, level by level
        for (int la = 1; la < num_levels; ++la) total += ((m0 + nkeys - 1) >> la) - (m0 >> la) + 1;
    int nch = (total + 15) / 16;
    nch += nch & 1;
    knch[kt] = nch;
    int nt = max(1, (nch + task_chunks - 1) / task_chunks);
    // a chained level: the first tile of every group of lb.chain[l] carries the group's one task
    if (lb.chain[l] > 1) nt = (kt - lb.tile_base[l]) % lb.chain[l] == 0 ? 1 : 0;
    ntask[kt] = nt;
    npart[kt] = nt > 1 ? nt : 0;
    is_multi[kt] = nt > 1 ? 1 : 0;
}

// one workgroup per key tile: the query node of every column (tokens of bucket 0, of bucket 1,
// then for token keys their ancestors level by level); padding columns: a real node, masked
__global__ void key_tile_cols(int n, int num_levels, const int32_t* __restrict__ kchunk_ptr,
                              const int32_t* __restrict__ tile_node0, const int32_t* __restrict__ tile_info,
                              const int32_t* __restrict__ klo, const int32_t* __restrict__ khi,
                              const int32_t* __restrict__ anc_first, int32_t* __restrict__ cols) {
    const int kt = blockIdx.x;
    const int64_t c0 = (int64_t)kchunk_ptr[kt] * 16;
    const int ncols = (kchunk_ptr[kt + 1] - kchunk_ptr[kt]) * 16;
    const int node0 = tile_node0[kt], level = tile_info[kt] & 255, nkeys = tile_info[kt] >> 8;
    const int cnt0 = khi[2 * kt] >= 0 ? khi[2 * kt] - klo[2 * kt] + 1 : 0;
    const int cnt1 = khi[2 * kt + 1] >= 0 ? khi[2 * kt + 1] - klo[2 * kt + 1] + 1 : 0;
    const int af = anc_first[kt], m0 = node0 - level_off(n, level);
    for (int i = threadIdx.x; i < ncols; i += blockDim.x) {
        int v = node0;
        if (i < cnt0) {
            v = klo[2 * kt] + i;
        } else if (i < cnt0 + cnt1) {
            v = klo[2 * kt + 1] + (i - cnt0);
        } else if (level == 0) {
            int p = i - af;
            for (int la = 1; la < num_levels; ++la) {
                const int a0 = m0 >> la, cnt = ((m0 + nkeys - 1) >> la) - a0 + 1;
                if (p < cnt) {
                    v = level_off(n, la) + a0 + p;
                    break;
                }
                p -= cnt;
            }
        }
        cols[c0 + i] = v;
    }
}

// one thread per token row: tile-local relative-position id (order + k + 1) of each of its edges
__global__ void key_tile_map_tokens(int n, int W, LevelBases lb, const int32_t* __restrict__ row_ptr,
                                    const int32_t* __restrict__ col, const int32_t* __restrict__ rel,
                                    const int32_t* __restrict__ kchunk_ptr, const int32_t* __restrict__ tile_node0,
                                    const int32_t* __restrict__ klo, const int32_t* __restrict__ kfirst,
                                    int16_t* __restrict__ map) {
    const int u = blockIdx.x * blockDim.x + threadIdx.x;
    if (u >= n) return;
    const int zero = (W - 1) / 2;
    const int e1 = row_ptr[u + 1];
    for (int e = row_ptr[u]; e < e1; ++e) {
        const int l = rel[e] / W, w = rel[e] % W;
        const int kt = lb.tile_base[l] + ((col[e] - level_off(n, l)) >> 4);
        const int b = 2 * kt + ((l > 0 && w - zero < 0) ? 1 : 0);
        const int slot = kfirst[b] + u - klo[b];
        const int key = col[e] - tile_node0[kt];
        map[((int64_t)kchunk_ptr[kt] + (slot >> 4)) * 256 + key * 16 + (slot & 15)] = (int16_t)w;
    }
}

// one thread per (tile of token keys, key): the affiliated edges, ancestor at level la <- token,
// with the tile-local id W + la - 1
__global__ void key_tile_map_ancestors(int num_levels, int W, int token_tiles, const int32_t* __restrict__ kchunk_ptr,
                                       const int32_t* __restrict__ tile_node0, const int32_t* __restrict__ tile_info,
                                       const int32_t* __restrict__ anc_first, int16_t* __restrict__ map) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    const int kt = i >> 4, key = i & 15;
    if (kt >= token_tiles) return;
    const int m0 = tile_node0[kt], nkeys = tile_info[kt] >> 8;   // level 0: node id = token index
    if (key >= nkeys) return;
    int slot0 = anc_first[kt];
    for (int la = 1; la < num_levels; ++la) {
        const int slot = slot0 + ((m0 + key) >> la) - (m0 >> la);
        map[((int64_t)kchunk_ptr[kt] + (slot >> 4)) * 256 + key * 16 + (slot & 15)] = (int16_t)(W + la - 1);
        slot0 += ((m0 + nkeys - 1) >> la) - (m0 >> la) + 1;
    }
}

// one thread per key tile: its tasks; tiles with several tasks also enter the merge list
__global__ void key_tile_tasks(int nkt, int ctx_levels, LevelBases lb, int task_chunks, int num_multi, int num_part,
                               const int32_t* __restrict__ kchunk_ptr, const int32_t* __restrict__ ntask,
                               const int32_t* __restrict__ task_ptr, const int32_t* __restrict__ part_base,
                               const int32_t* __restrict__ multi_idx, int32_t* __restrict__ task_tile,
                               int32_t* __restrict__ task_c0, int32_t* __restrict__ task_nch,
                               int32_t* __restrict__ task_part, int32_t* __restrict__ task_ntiles,
                               int32_t* __restrict__ multi_tile, int32_t* __restrict__ multi_ptr) {
    const int kt = blockIdx.x * blockDim.x + threadIdx.x;
    if (kt == 0) multi_ptr[num_multi] = num_part;
    if (kt >= nkt) return;
    const int c0 = kchunk_ptr[kt], nch = kchunk_ptr[kt + 1] - c0, nt = ntask[kt], tp = task_ptr[kt];
    int l = 0;
    while (l + 1 < ctx_levels && lb.tile_base[l + 1] <= kt) ++l;
    if (lb.chain[l] > 1) {   // one task for this tile and the following ones of its group (their chunks are consecutive)
        if (nt == 1) {
            const int last = min(kt + lb.chain[l], lb.tile_base[l + 1]);
            task_tile[tp] = kt;
            task_c0[tp] = c0;
            task_nch[tp] = kchunk_ptr[last] - c0;
            task_part[tp] = -1;
            task_ntiles[tp] = last - kt;
        }
        return;
    }
    for (int t = 0; t < nt; ++t) {
        task_tile[tp + t] = kt;
        task_c0[tp + t] = c0 + t * task_chunks;
        task_nch[tp + t] = max(0, min(task_chunks, nch - t * task_chunks));
        task_part[tp + t] = nt > 1 ? part_base[kt] + t : -1;
        task_ntiles[tp + t] = 1;
    }
    if (nt > 1) {
        multi_tile[multi_idx[kt]] = kt;
        multi_ptr[multi_idx[kt]] = part_base[kt];
    }
}

// Orders the tasks by the stretch of kSegTokens tokens in which their query lists begin, and inside
// a stretch keeps the order of the tiles (level-major).  The wavefronts of an XCD take the tasks in
// this order, so all levels of one stretch run together and read its Q and dO rows while they are
// in the L2 of the XCD, instead of every level sweeping the whole sequence again (the rows of one
// (batch, head) are about as large as that L2): 30 % fewer bytes fetched by the key-side kernel
// at n = 8192.  Inside a stretch the longest tasks come first: the wavefronts take tasks as they
// become free, and a long task started last would run on alone at the end of the kernel.  One
// thread per task counts the tasks that come before it.  Which wavefront computes a task changes
// no result: partial sums keep their slots.
constexpr int kSegTokens = 512;
__global__ void key_tile_task_order(int num_tasks, int n, const int32_t* __restrict__ cols,
                                    const int32_t* __restrict__ in_tile, const int32_t* __restrict__ in_c0,
                                    const int32_t* __restrict__ in_nch, const int32_t* __restrict__ in_part,
                                    const int32_t* __restrict__ in_ntiles, int32_t* __restrict__ task_tile,
                                    int32_t* __restrict__ task_c0, int32_t* __restrict__ task_nch,
                                    int32_t* __restrict__ task_part, int32_t* __restrict__ task_ntiles) {
    __shared__ int32_t keys_s[kTB];
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    // sort key: stretch ascending, then chunks descending (at most 2^12 chunks per task); a list that
    // begins with a span node (only ancestors) belongs to the last stretch
    auto key_of = [&](int task) {
        return (min(cols[(int64_t)in_c0[task] * 16], n - 1) / kSegTokens) * 4096 + (4095 - min(in_nch[task], 4095));
    };
    const int mine = t < num_tasks ? key_of(t) : 0;
    int rank = 0;
    for (int base = 0; base < num_tasks; base += kTB) {
        const int o = base + (int)threadIdx.x;
        keys_s[threadIdx.x] = o < num_tasks ? key_of(o) : 0x7FFFFFFF;
        __syncthreads();
        const int lim = min(kTB, num_tasks - base);
        for (int i = 0; i < lim; ++i) {
            const int other = keys_s[i];
            rank += (other < mine || (other == mine && base + i < t)) ? 1 : 0;
        }
        __syncthreads();
    }
    if (t < num_tasks) {
        task_tile[rank] = in_tile[t];
        task_c0[rank] = in_c0[t];
        task_nch[rank] = in_nch[t];
        task_part[rank] = in_part[t];
        task_ntiles[rank] = in_ntiles[t];
    }
}

template <typename T>
int device_alloc(T** p, size_t count) {
    BPT_HIP(hipMalloc((void**)p, std::max<size_t>(count, 1) * sizeof(T)));
    return BPT_OK;
}

}  // namespace

// Builds g->tiles and g->ktiles from the CSR already on the device and, per node, the count and
// the first of the tokens attending to it from its left / right (what the transposed-adjacency
// builder computes).  Leaves them empty (the
// gather kernels then do all the work) when a table would not fit its 16-bit ids or the size
// limits.  Synchronises `st` once, to learn the sizes to allocate.
int build_tile_metadata(bpt_graph* g, const int32_t* cnt_l, const int32_t* min_l, const int32_t* cnt_r,
                        const int32_t* min_r, hipStream_t st) {
    const int n = g->n, W = g->rel_width, zero = g->k + 1, num_levels = g->num_levels, ctx_levels = g->ctx_levels;
    const int64_t e_tok = g->num_token_edges;
    const int64_t num_ids64 = (int64_t)num_levels * W;
    if (n < 16 || e_tok >= ((int64_t)1 << 27) || num_ids64 > (1 << 20) || num_levels > kMaxLevels) return BPT_OK;
    const int num_ids = (int)num_ids64, tiles = n / 16, nb = 2 * num_levels;

    LevelBases lb = {};
    for (int l = 0; l < ctx_levels; ++l) lb.tile_base[l + 1] = lb.tile_base[l] + ((n >> l) + 15) / 16;
    const int task_chunks = key_task_chunks(n);
    for (int l = 0; l < ctx_levels; ++l) {
        // an upper bound of a tile's columns: the tokens that read its 16 keys from either side (a key of level l
        // is read by at most (k + 2) 2^l tokens on a side, the ranges of consecutive keys are 2^l apart), and for
        // token keys their ancestors; tiles of at most kChainChunks chunks are chained up to a task's length
        const int64_t cols = (int64_t)(g->causal ? 1 : 2) * (17 + g->k) * ((int64_t)1 << l) + (l == 0 ? 28 + num_levels : 0);
        const int64_t nch = ((cols + 15) / 16 + 1) & ~(int64_t)1;
        // (the chained kernel looks the bias up across lanes, which covers 32 ids)
        lb.chain[l] = nch <= kChainChunks && ((W + num_levels - 1 + 15) & ~15) <= 32 ? (int)std::max<int64_t>(1, task_chunks / nch) : 1;
    }
    const int nkt = lb.tile_base[ctx_levels];
    const bool want_keys = W + num_levels <= 32767;

    // ---- phase 1: everything whose size is known in advance ----
    DeviceBuf used, pos, sums, totals, tile_lo, tile_hi, tile_first, tile_nch;
    DeviceBuf klo, khi, kfirst, anc_first, knch, ntask, npart, is_multi, task_ptr, part_base, multi_idx;
    BPT_HIP(used.alloc(sizeof(int32_t) * (size_t)num_ids));
    BPT_HIP(pos.alloc(sizeof(int32_t) * ((size_t)num_ids + 1)));
    BPT_HIP(sums.alloc(sizeof(int32_t) * (kScanBlock + 1)));
    BPT_HIP(totals.alloc(sizeof(int32_t) * 8));
    BPT_HIP(tile_lo.alloc(sizeof(int32_t) * (size_t)tiles * nb));
    BPT_HIP(tile_hi.alloc(sizeof(int32_t) * (size_t)tiles * nb));
    BPT_HIP(tile_first.alloc(sizeof(int32_t) * (size_t)tiles * nb));
    BPT_HIP(tile_nch.alloc(sizeof(int32_t) * (size_t)tiles));
    int32_t* d_tot = totals.as<int32_t>();   // 0: ids in use, 1: token chunks, 2: key chunks, 3: tasks, 4: partials, 5: multi tiles
    BPT_HIP(hipMemsetAsync(d_tot, 0, sizeof(int32_t) * 8, st));
    BPT_HIP(hipMemsetAsync(used.p, 0, sizeof(int32_t) * (size_t)num_ids, st));

    TokenTiles& tt = g->tiles;
    int rc;
    if ((rc = device_alloc(&tt.id_to_cid, num_ids)) || (rc = device_alloc(&tt.cid_to_id, num_ids)) ||
        (rc = device_alloc(&tt.chunk_ptr, (size_t)tiles + 1)))
        return rc;
    hipLaunchKernelGGL(mark_ids, dim3((unsigned)((e_tok + kTB - 1) / kTB)), dim3(kTB), 0, st, g->rel, (int32_t)e_tok,
                       used.as<int32_t>());
    if ((rc = dev_scan(used.as<int32_t>(), pos.as<int32_t>(), num_ids, sums.as<int32_t>(), d_tot + 0, st))) return rc;
    hipLaunchKernelGGL(finish_ids, dim3((num_ids + kTB - 1) / kTB), dim3(kTB), 0, st, used.as<int32_t>(), pos.as<int32_t>(),
                       num_ids, tt.id_to_cid, tt.cid_to_id);
    hipLaunchKernelGGL(token_tile_ranges, dim3(tiles), dim3(64), 0, st, tiles, nb, W, zero, g->row_ptr, g->col,
                       g->rel, tile_lo.as<int32_t>(), tile_hi.as<int32_t>(), tile_first.as<int32_t>(),
                       tile_nch.as<int32_t>());
    if ((rc = dev_scan(tile_nch.as<int32_t>(), tt.chunk_ptr, tiles, sums.as<int32_t>(), d_tot + 1, st))) return rc;

    KeyTiles& kt = g->ktiles;
    if (want_keys) {
        BPT_HIP(klo.alloc(sizeof(int32_t) * 2 * (size_t)nkt));
        BPT_HIP(khi.alloc(sizeof(int32_t) * 2 * (size_t)nkt));
        BPT_HIP(kfirst.alloc(sizeof(int32_t) * 2 * (size_t)nkt));
        BPT_HIP(anc_first.alloc(sizeof(int32_t) * (size_t)nkt));
        BPT_HIP(knch.alloc(sizeof(int32_t) * (size_t)nkt));
        BPT_HIP(ntask.alloc(sizeof(int32_t) * (size_t)nkt));
        BPT_HIP(npart.alloc(sizeof(int32_t) * (size_t)nkt));
        BPT_HIP(is_multi.alloc(sizeof(int32_t) * (size_t)nkt));
        BPT_HIP(task_ptr.alloc(sizeof(int32_t) * ((size_t)nkt + 1)));
        BPT_HIP(part_base.alloc(sizeof(int32_t) * ((size_t)nkt + 1)));
        BPT_HIP(multi_idx.alloc(sizeof(int32_t) * ((size_t)nkt + 1)));
        if ((rc = device_alloc(&kt.tile_node0, nkt)) || (rc = device_alloc(&kt.tile_info, nkt)) ||
            (rc = device_alloc(&kt.chunk_ptr, (size_t)nkt + 1)))
            return rc;
        hipLaunchKernelGGL(key_tile_layout, dim3((nkt + kTB - 1) / kTB), dim3(kTB), 0, st, n, num_levels, ctx_levels, nkt,
                           task_chunks, lb, cnt_l, min_l, cnt_r, min_r, klo.as<int32_t>(), khi.as<int32_t>(), kt.tile_node0,
                           kt.tile_info,
                           kfirst.as<int32_t>(), anc_first.as<int32_t>(), knch.as<int32_t>(), ntask.as<int32_t>(),
                           npart.as<int32_t>(), is_multi.as<int32_t>());
        if ((rc = dev_scan(knch.as<int32_t>(), kt.chunk_ptr, nkt, sums.as<int32_t>(), d_tot + 2, st)) ||
            (rc = dev_scan(ntask.as<int32_t>(), task_ptr.as<int32_t>(), nkt, sums.as<int32_t>(), d_tot + 3, st)) ||
            (rc = dev_scan(npart.as<int32_t>(), part_base.as<int32_t>(), nkt, sums.as<int32_t>(), d_tot + 4, st)) ||
            (rc = dev_scan(is_multi.as<int32_t>(), multi_idx.as<int32_t>(), nkt, sums.as<int32_t>(), d_tot + 5, st)))
            return rc;
    }
    BPT_HIP(hipGetLastError());
    int32_t h_tot[8] = {0};
    BPT_HIP(hipMemcpyAsync(h_tot, d_tot, sizeof h_tot, hipMemcpyDeviceToHost, st));
    BPT_HIP(hipStreamSynchronize(st));

    // ---- phase 2: the tables whose sizes phase 1 produced ----
    const int num_cids = h_tot[0];
    const int64_t chunks = h_tot[1];
    const bool token_ok = num_cids <= 32767 && chunks * 512 <= ((int64_t)256 << 20);
    if (!token_ok) return BPT_OK;   // num_tiles stays 0: no tile path (the destroy call frees what was allocated)
    if ((rc = device_alloc(&tt.cols, (size_t)chunks * 16)) || (rc = device_alloc(&tt.map, (size_t)chunks * 256))) return rc;
    BPT_HIP(hipMemsetAsync(tt.map, 0xFF, sizeof(int16_t) * (size_t)chunks * 256, st));
    hipLaunchKernelGGL(token_tile_cols, dim3(tiles), dim3(64), 0, st, nb, tt.chunk_ptr, tile_lo.as<int32_t>(),
                       tile_hi.as<int32_t>(), tile_first.as<int32_t>(), tt.cols);
    hipLaunchKernelGGL(token_tile_map, dim3((n + kTB - 1) / kTB), dim3(kTB), 0, st, n, nb, W, zero, g->row_ptr, g->col,
                       g->rel, tt.chunk_ptr, tile_lo.as<int32_t>(), tile_first.as<int32_t>(), tt.id_to_cid, tt.map);
    BPT_HIP(hipGetLastError());
    tt.num_cids = num_cids;
    tt.num_chunks = (int32_t)chunks;
    tt.num_tiles = tiles;

    const int64_t kchunks = h_tot[2];
    if (want_keys && kchunks * 512 <= ((int64_t)512 << 20)) {
        const int num_tasks = h_tot[3], num_part = h_tot[4], num_multi = h_tot[5];
        if ((rc = device_alloc(&kt.cols, (size_t)kchunks * 16)) || (rc = device_alloc(&kt.map, (size_t)kchunks * 256)) ||
            (rc = device_alloc(&kt.task_tile, num_tasks)) || (rc = device_alloc(&kt.task_c0, num_tasks)) ||
            (rc = device_alloc(&kt.task_nch, num_tasks)) || (rc = device_alloc(&kt.task_part, num_tasks)) ||
            (rc = device_alloc(&kt.task_ntiles, num_tasks)) ||
            (rc = device_alloc(&kt.multi_tile, num_multi)) || (rc = device_alloc(&kt.multi_ptr, (size_t)num_multi + 1)))
            return rc;
        BPT_HIP(hipMemsetAsync(kt.map, 0xFF, sizeof(int16_t) * (size_t)kchunks * 256, st));
        hipLaunchKernelGGL(key_tile_cols, dim3(nkt), dim3(64), 0, st, n, num_levels, kt.chunk_ptr, kt.tile_node0, kt.tile_info,
                           klo.as<int32_t>(), khi.as<int32_t>(), anc_first.as<int32_t>(), kt.cols);
        hipLaunchKernelGGL(key_tile_map_tokens, dim3((n + kTB - 1) / kTB), dim3(kTB), 0, st, n, W, lb, g->row_ptr, g->col,
                           g->rel, kt.chunk_ptr, kt.tile_node0, klo.as<int32_t>(), kfirst.as<int32_t>(), kt.map);
        const int token_tiles = lb.tile_base[1];
        hipLaunchKernelGGL(key_tile_map_ancestors, dim3((token_tiles * 16 + kTB - 1) / kTB), dim3(kTB), 0, st, num_levels, W,
                           token_tiles, kt.chunk_ptr, kt.tile_node0, kt.tile_info, anc_first.as<int32_t>(), kt.map);
        const bool reorder = n > kSegTokens && num_tasks <= kMaxSortedTasks;
        DeviceBuf ut_tile, ut_c0, ut_nch, ut_part, ut_ntiles;   // the tasks in tile order, when they are put in another one
        if (reorder) {
            const size_t tbytes = sizeof(int32_t) * (size_t)std::max(num_tasks, 1);
            BPT_HIP(ut_tile.alloc(tbytes));
            BPT_HIP(ut_c0.alloc(tbytes));
            BPT_HIP(ut_nch.alloc(tbytes));
            BPT_HIP(ut_part.alloc(tbytes));
            BPT_HIP(ut_ntiles.alloc(tbytes));
        }
        hipLaunchKernelGGL(key_tile_tasks, dim3((nkt + kTB - 1) / kTB), dim3(kTB), 0, st, nkt, ctx_levels, lb, task_chunks,
                           num_multi, num_part, kt.chunk_ptr, ntask.as<int32_t>(), task_ptr.as<int32_t>(),
                           part_base.as<int32_t>(), multi_idx.as<int32_t>(), reorder ? ut_tile.as<int32_t>() : kt.task_tile,
                           reorder ? ut_c0.as<int32_t>() : kt.task_c0, reorder ? ut_nch.as<int32_t>() : kt.task_nch,
                           reorder ? ut_part.as<int32_t>() : kt.task_part, reorder ? ut_ntiles.as<int32_t>() : kt.task_ntiles,
                           kt.multi_tile, kt.multi_ptr);
        if (reorder && num_tasks > 0)
            hipLaunchKernelGGL(key_tile_task_order, dim3((num_tasks + kTB - 1) / kTB), dim3(kTB), 0, st, num_tasks, n, kt.cols,
                               ut_tile.as<int32_t>(), ut_c0.as<int32_t>(), ut_nch.as<int32_t>(), ut_part.as<int32_t>(),
                               ut_ntiles.as<int32_t>(), kt.task_tile, kt.task_c0, kt.task_nch, kt.task_part, kt.task_ntiles);
        BPT_HIP(hipGetLastError());
        if (reorder) BPT_HIP(hipStreamSynchronize(st));   // the lists in tile order are freed at the end of this block
        kt.num_chunks = (int32_t)kchunks;
        kt.nb_pad = (W + num_levels - 1 + 15) & ~15;
        kt.first_uncovered = level_off(n, ctx_levels);
        kt.num_multi = num_multi;
        kt.num_part = num_part;
        kt.num_tasks = num_tasks;
    }
    // the temporaries are freed when this function returns: wait for the kernels that read them
    BPT_HIP(hipStreamSynchronize(st));
    return BPT_OK;
}

}  // namespace bpt
