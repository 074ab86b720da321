// Binary-partition graph construction on the GPU (paper Sec. 3.2, Algorithm 1)
// plus the host-side launch schedules of the attention kernels.
//
// Kernels (all integer work, results independent of thread order):
//   token_degree   one thread per token runs the contextual-node recurrence and counts
//   scan_*         exclusive prefix sum -> row_ptr
//   fill_tokens    one thread per token emits (col, rel) of its row in canonical order
//   fill_spans     one thread per affiliated edge (closed form)
//   t_ranges       first and last query token on each side of every key node (no atomics)
//   t_fill         closed-form slot of every edge in the transposed adjacency
// The dense tiles of the matrix-core kernels are built by bpt_tiles.hip.
#include <algorithm>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <utility>
#include <vector>

#include "bpt_internal.h"

namespace bpt {
namespace {

constexpr int kScanThreads = 256;
constexpr int kScanItems = 16;
constexpr int kScanBlock = kScanThreads * kScanItems;  // elements per block

__host__ __device__ inline int64_t level_offset(int64_t n, int level) { return 2 * n - ((2 * n) >> level); }

// One side's walk over the tree levels for token i (Sec. 3.2.2, contextual
// edges): at level j the run covers the nodes [lo, hi]; `near` is the end next to
// the token.  k nodes per level; the run is clipped to the level and grows by
// one node when it would not end on a parent boundary, so that the next level
// starts exactly where this one ends.
struct LeftWalk {
    int q;  // nearest node of the current level; < 0 when the side is exhausted
    __device__ explicit LeftWalk(int i) : q(i - 1) {}
    __device__ bool alive() const { return q >= 0; }
    __device__ void run(int k, int& lo, int& hi) const {
        int e = q - k + 1;  // k <= 2^20 and q < 2^22: no overflow
        if (e < 0) e = 0;
        if (e & 1) e -= 1;  // ends on a right child: its sibling joins
        lo = e;
        hi = q;
    }
    __device__ void up(int lo) { q = (lo - 1 < 0) ? -1 : ((lo - 1) >> 1); }
};

struct RightWalk {
    int p, size;  // nearest node and node count of the current level
    __device__ RightWalk(int i, int n) : p(i + 1), size(n) {}
    __device__ bool alive() const { return p < size; }
    __device__ void run(int k, int& lo, int& hi) const {
        int e = (k - 1 > size - 1 - p) ? size - 1 : p + k - 1;  // min(p+k-1, size-1) without overflow
        if ((e & 1) == 0) e += 1;  // ends on a left child: its sibling joins (size is even)
        lo = p;
        hi = e;
    }
    __device__ void up(int hi) {
        int nxt = hi + 1;
        if (nxt >= size) {
            p = size;  // exhausted
        } else {
            p = nxt >> 1;
            size >>= 1;
        }
    }
};

__global__ void token_degree(int n, int k, int causal, int32_t* __restrict__ deg,
                             unsigned long long* __restrict__ total, int32_t* __restrict__ max_levels) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    int d = 0, used = 0;
    if (i < n) {
        d = 1;  // self (Algorithm 1 starts from N = {u})
        LeftWalk L(i);
        int lv = 0;
        while (L.alive()) {
            int lo, hi;
            L.run(k, lo, hi);
            d += hi - lo + 1;
            L.up(lo);
            ++lv;
        }
        used = lv;
        if (!causal) {
            RightWalk R(i, n);
            lv = 0;
            while (R.alive()) {
                int lo, hi;
                R.run(k, lo, hi);
                d += hi - lo + 1;
                R.up(hi);
                ++lv;
            }
            used = max(used, lv);
        }
        deg[i] = d;
    }
    // block totals -> one 64-bit atomic per block (integer: order does not matter)
    __shared__ unsigned long long s_sum[kScanThreads];
    __shared__ int s_lv[kScanThreads];
    s_sum[threadIdx.x] = (unsigned long long)d;
    s_lv[threadIdx.x] = used;
    __syncthreads();
    for (int w = blockDim.x / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            s_sum[threadIdx.x] += s_sum[threadIdx.x + w];
            s_lv[threadIdx.x] = max(s_lv[threadIdx.x], s_lv[threadIdx.x + w]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        atomicAdd(total, s_sum[0]);
        atomicMax(max_levels, s_lv[0]);
    }
}

// ---- exclusive scan of int32 (three phases) ------------------------------
__global__ void scan_blocks(const int32_t* __restrict__ in, int32_t* __restrict__ out, int32_t* __restrict__ block_sums,
                            int m) {
    __shared__ int32_t s[kScanThreads];
    int base = blockIdx.x * kScanBlock + threadIdx.x * kScanItems;
    int32_t v[kScanItems];
    int32_t sum = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        int idx = base + j;
        v[j] = idx < m ? in[idx] : 0;
        sum += v[j];
    }
    s[threadIdx.x] = sum;
    __syncthreads();
    for (int off = 1; off < kScanThreads; off <<= 1) {  // inclusive scan of the thread sums
        int32_t t = (int)threadIdx.x >= off ? s[threadIdx.x - off] : 0;
        __syncthreads();
        s[threadIdx.x] += t;
        __syncthreads();
    }
    int32_t run = s[threadIdx.x] - sum;  // exclusive prefix of this thread inside the block
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        int idx = base + j;
        if (idx < m) out[idx] = run;
        run += v[j];
    }
    if (threadIdx.x == kScanThreads - 1) block_sums[blockIdx.x] = s[threadIdx.x];
}

__global__ void scan_sums(int32_t* __restrict__ block_sums, int nblocks) {  // one block, nblocks <= kScanBlock
    __shared__ int32_t s[kScanThreads];
    int base = threadIdx.x * kScanItems;
    int32_t v[kScanItems];
    int32_t sum = 0;
#pragma unroll
    for (int j = 0; j < kScanItems; ++j) {
        v[j] = base + j < nblocks ? block_sums[base + j] : 0;
        sum += v[j];
    }
    s[threadIdx.x] = sum;
    __syncthreads();
    for (int off = 1; off < kScanThreads; off <<= 1) {
        int32_t t = (int)threadIdx.x >= off ? s[threadIdx.x - off] : 0;
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
}

__global__ void scan_add(int32_t* __restrict__ out, const int32_t* __restrict__ block_sums, int m, int32_t total) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx < m) out[idx] += block_sums[idx / kScanBlock];
    if (idx == m) out[m] = total;
}

// ---- CSR fill ---------------------------------------------------------------
__global__ void fill_tokens(int n, int k, int causal, const int32_t* __restrict__ row_ptr, int32_t* __restrict__ col,
                            int32_t* __restrict__ rel) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int W = 2 * (k + 1) + 1, zero = k + 1;
    int e = row_ptr[i];
    LeftWalk L(i);
    RightWalk R(i, causal ? 0 : n);  // size 0: never alive
    for (int j = 0; j == 0 || L.alive() || R.alive(); ++j) {
        const int off = (int)level_offset(n, j);
        if (L.alive()) {  // far -> near: orders -(count) .. -1
            int lo, hi;
            L.run(k, lo, hi);
            for (int x = lo; x <= hi; ++x) {
                col[e] = off + x;
                rel[e] = j * W + zero - (hi - x + 1);
                ++e;
            }
            L.up(lo);
        }
        if (j == 0) {  // self, r_self
            col[e] = i;
            rel[e] = zero;
            ++e;
        }
        if (R.alive()) {  // near -> far: orders +1 .. +count
            int lo, hi;
            R.run(k, lo, hi);
            for (int x = lo; x <= hi; ++x) {
                col[e] = off + x;
                rel[e] = j * W + zero + (x - lo + 1);
                ++e;
            }
            R.up(hi);
        }
    }
}

// Affiliated edges (Sec. 3.2.2): span (l,m) <- tokens m*2^l .. (m+1)*2^l-1.  The
// n edges of one level are simply the tokens 0..n-1 in order.
__global__ void fill_spans(int n, int k, int num_levels, int32_t e_tok, int32_t* __restrict__ row_ptr,
                           int32_t* __restrict__ col, int32_t* __restrict__ rel) {
    const int64_t a = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)n * (num_levels - 1);
    const int W = 2 * (k + 1) + 1, zero = k + 1;
    if (a < total) {
        int lev = 1 + (int)(a / n);
        int t = (int)(a % n);
        col[e_tok + a] = t;
        rel[e_tok + a] = lev * W + zero;  // r_anc(lev)
    }
    if (a < n - 1) {  // span row starts: a-th span node in level-major order
        int64_t node = n + a;
        int64_t x = 2 * (int64_t)n - node;                 // (n >> l) < x <= (2n >> l)
        int ceil_log2 = 64 - __clzll((unsigned long long)(x - 1));
        int lev = num_levels - ceil_log2;                  // log2(2n) = num_levels
        int64_t m = node - level_offset(n, lev);
        row_ptr[node] = (int32_t)(e_tok + (int64_t)(lev - 1) * n + (m << lev));
    }
    if (a == 0) row_ptr[2 * n - 1] = (int32_t)(e_tok + total);
}

// ---- transposed adjacency -----------------------------------------------------
// For a key node v the tokens attending to it from its left (they see v in their
// right context) form one contiguous range, and so do those on its right: the run
// boundaries of the walks above are monotone in the token index.  So the slot of
// an edge in v's list follows from counts and range starts alone.
__global__ void t_init(int num_nodes, int32_t* __restrict__ cnt_l, int32_t* __restrict__ cnt_r,
                       int32_t* __restrict__ min_l, int32_t* __restrict__ min_r) {
    int v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v < num_nodes) {
        cnt_l[v] = -1;  // until t_degree: the last token of the range (t_ranges), -1 = no token
        cnt_r[v] = -1;
        min_l[v] = INT32_MAX;
        min_r[v] = INT32_MAX;
    }
}

// First and last token of the range that attends to every node from each side, without
// atomics: token i is the first of node x's range iff token i-1 does not attend to x at that
// level, and the last iff token i+1 does not.  One thread per token walks the levels of
// tokens i-1, i and i+1 together.  `last_*` receive the last token (t_degree turns them into counts).
__global__ void t_ranges(int n, int k, int causal, int32_t* __restrict__ last_l, int32_t* __restrict__ last_r,
                         int32_t* __restrict__ min_l, int32_t* __restrict__ min_r) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const bool has_prev = i > 0, has_next = i + 1 < n;
    {   // nodes in the left context of i: i lies to their right
        LeftWalk A(i), P(i - 1), N(i + 1);
        for (int j = 0; A.alive(); ++j) {
            const int off = (int)level_offset(n, j);
            int lo, hi, plo = 0, phi = -1, nlo = 0, nhi = -1;
            A.run(k, lo, hi);
            const bool pa = has_prev && P.alive(), na = has_next && N.alive();
            if (pa) P.run(k, plo, phi);
            if (na) N.run(k, nlo, nhi);
            for (int x = lo; x <= hi; ++x) {
                if (!(pa && plo <= x && x <= phi)) min_r[off + x] = i;
                if (!(na && nlo <= x && x <= nhi)) last_r[off + x] = i;
            }
            A.up(lo);
            if (pa) P.up(plo);
            if (na) N.up(nlo);
        }
    }
    if (!causal) {   // nodes in the right context of i: i lies to their left
        RightWalk A(i, n), P(i - 1, n), N(i + 1, n);
        for (int j = 0; A.alive(); ++j) {
            const int off = (int)level_offset(n, j);
            int lo, hi, plo = 0, phi = -1, nlo = 0, nhi = -1;
            A.run(k, lo, hi);
            const bool pa = has_prev && P.alive(), na = has_next && N.alive();
            if (pa) P.run(k, plo, phi);
            if (na) N.run(k, nlo, nhi);
            for (int x = lo; x <= hi; ++x) {
                if (!(pa && plo <= x && x <= phi)) min_l[off + x] = i;
                if (!(na && nlo <= x && x <= nhi)) last_l[off + x] = i;
            }
            A.up(hi);
            if (pa) P.up(phi);
            if (na) N.up(nhi);
        }
    }
}

// counts from the (first, last) pairs, and the in-degree of every node
__global__ void t_degree(int n, int num_nodes, int num_levels, int32_t* __restrict__ cnt_l, int32_t* __restrict__ cnt_r,
                         const int32_t* __restrict__ min_l, const int32_t* __restrict__ min_r,
                         int32_t* __restrict__ t_deg) {
    int v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= num_nodes) return;
    const int cl = cnt_l[v] >= 0 ? cnt_l[v] - min_l[v] + 1 : 0, cr = cnt_r[v] >= 0 ? cnt_r[v] - min_r[v] + 1 : 0;
    cnt_l[v] = cl;
    cnt_r[v] = cr;
    t_deg[v] = cl + cr + (v < n ? num_levels : 0);  // self + one per ancestor
}

__global__ void t_fill_tokens(int n, int k, const int32_t* __restrict__ row_ptr, const int32_t* __restrict__ col,
                              const int32_t* __restrict__ rel, const int32_t* __restrict__ t_ptr,
                              const int32_t* __restrict__ cnt_l, const int32_t* __restrict__ min_l,
                              const int32_t* __restrict__ min_r, int32_t* __restrict__ t_src,
                              int32_t* __restrict__ t_eid, int32_t* __restrict__ t_rel) {
    int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int W = 2 * (k + 1) + 1, zero = k + 1;
    for (int e = row_ptr[i]; e < row_ptr[i + 1]; ++e) {
        int r = rel[e];
        int order = r % W - zero;
        int v = col[e];
        int pos = t_ptr[v];
        if (order > 0)
            pos += i - min_l[v];
        else if (order == 0)
            pos += cnt_l[v];
        else
            pos += cnt_l[v] + (v < n ? 1 : 0) + (i - min_r[v]);
        t_src[pos] = i;
        t_eid[pos] = e;
        t_rel[pos] = r;
    }
}

__global__ void t_fill_spans(int n, int num_levels, int32_t e_tok, const int32_t* __restrict__ rel,
                             const int32_t* __restrict__ t_ptr, const int32_t* __restrict__ cnt_l,
                             const int32_t* __restrict__ cnt_r, int32_t* __restrict__ t_src,
                             int32_t* __restrict__ t_eid, int32_t* __restrict__ t_rel) {
    const int64_t a = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= (int64_t)n * (num_levels - 1)) return;
    int lev = 1 + (int)(a / n);
    int t = (int)(a % n);
    int32_t e = (int32_t)(e_tok + a);
    int pos = t_ptr[t] + cnt_l[t] + 1 + cnt_r[t] + (lev - 1);  // after all token queries, by level
    t_src[pos] = (int32_t)(level_offset(n, lev) + (t >> lev));
    t_eid[pos] = e;
    t_rel[pos] = rel[e];
}

// ---- a batch of sequences of different lengths as one graph ----------------------------------
// The disjoint union of the graphs of B sequences (sequence b: len_b <= n tokens on the tree over n, keeping
// the nodes whose first token exists; an edge needs both of its nodes).  Rows are numbered level-major over
// the batch: the tokens of sequence 0, of sequence 1, ..., then the level-1 nodes of sequence 0, of sequence 1,
// and so on, so that token rows still come first and the tokens under a span are consecutive rows.
// first_row[l * B + b] is the row of node (l, 0) of sequence b; tok_off = first_row of level 0, with the total
// appended.  Level l of a sequence of len tokens keeps ceil(len / 2^l) nodes.
struct SeqToken {
    int b, t, len;
};
// sequence and position of packed token i: the last b with tok_off[b] <= i (empty sequences share their offset
// with the next one and are skipped by that rule)
__device__ inline SeqToken locate_token(const int32_t* __restrict__ tok_off, int B, int i) {
    int lo = 0, hi = B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (tok_off[mid] <= i)
            lo = mid;
        else
            hi = mid;
    }
    return SeqToken{lo, i - tok_off[lo], tok_off[lo + 1] - tok_off[lo]};
}

// RightWalk on the kept nodes of a sequence of `len` tokens: the run is clipped to the nodes the level keeps,
// and the alignment node joins only if it is kept.  len = 0: never alive.
struct RightWalkLen {
    int p, level, len;
    __device__ RightWalkLen(int t, int len_) : p(t + 1), level(0), len(len_) {}
    __device__ int count() const { return (len + (1 << level) - 1) >> level; }
    __device__ bool alive() const { return p < count(); }
    __device__ void run(int k, int& lo, int& hi) const {
        const int c = count();
        int e = (k - 1 > c - 1 - p) ? c - 1 : p + k - 1;
        if ((e & 1) == 0 && e + 1 < c) e += 1;
        lo = p;
        hi = e;
    }
    __device__ void up(int hi) {
        if (hi + 1 >= count()) {
            p = INT32_MAX;  // exhausted
        } else {
            p = (hi + 1) >> 1;
            ++level;
        }
    }
};

__global__ void batch_token_degree(int T, int k, int causal, int B, const int32_t* __restrict__ tok_off,
                                   int32_t* __restrict__ deg, unsigned long long* __restrict__ total,
                                   int32_t* __restrict__ max_levels) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    int d = 0, used = 0;
    if (i < T) {
        const SeqToken s = locate_token(tok_off, B, i);
        d = 1;
        LeftWalk L(s.t);
        int lv = 0;
        while (L.alive()) {
            int lo, hi;
            L.run(k, lo, hi);
            d += hi - lo + 1;
            L.up(lo);
            ++lv;
        }
        used = lv;
        RightWalkLen R(s.t, causal ? 0 : s.len);
        lv = 0;
        while (R.alive()) {
            int lo, hi;
            R.run(k, lo, hi);
            d += hi - lo + 1;
            R.up(hi);
            ++lv;
        }
        used = max(used, lv);
        deg[i] = d;
    }
    __shared__ unsigned long long s_sum[kScanThreads];
    __shared__ int s_lv[kScanThreads];
    s_sum[threadIdx.x] = (unsigned long long)d;
    s_lv[threadIdx.x] = used;
    __syncthreads();
    for (int w = blockDim.x / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) {
            s_sum[threadIdx.x] += s_sum[threadIdx.x + w];
            s_lv[threadIdx.x] = max(s_lv[threadIdx.x], s_lv[threadIdx.x + w]);
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        atomicAdd(total, s_sum[0]);
        atomicMax(max_levels, s_lv[0]);
    }
}

__global__ void batch_fill_tokens(int T, int k, int causal, int B, const int32_t* __restrict__ tok_off,
                                  const int32_t* __restrict__ first_row, const int32_t* __restrict__ row_ptr,
                                  int32_t* __restrict__ col, int32_t* __restrict__ rel) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T) return;
    const SeqToken s = locate_token(tok_off, B, i);
    const int W = 2 * (k + 1) + 1, zero = k + 1;
    int e = row_ptr[i];
    LeftWalk L(s.t);
    RightWalkLen R(s.t, causal ? 0 : s.len);
    for (int j = 0; j == 0 || L.alive() || R.alive(); ++j) {
        const int off = first_row[j * B + s.b];
        if (L.alive()) {
            int lo, hi;
            L.run(k, lo, hi);
            for (int x = lo; x <= hi; ++x) {
                col[e] = off + x;
                rel[e] = j * W + zero - (hi - x + 1);
                ++e;
            }
            L.up(lo);
        }
        if (j == 0) {
            col[e] = i;
            rel[e] = zero;
            ++e;
        }
        if (R.alive()) {
            int lo, hi;
            R.run(k, lo, hi);
            for (int x = lo; x <= hi; ++x) {
                col[e] = off + x;
                rel[e] = j * W + zero + (x - lo + 1);
                ++e;
            }
            R.up(hi);
        }
    }
}

// Affiliated edges: on every level above the tokens the kept spans of all sequences hold every token once,
// in row order -- the T edges of a level are the tokens 0..T-1.  Span (l, m) of sequence b starts at token
// m * 2^l of that sequence.
__global__ void batch_fill_spans(int T, int k, int B, int num_levels, int num_nodes, int32_t e_tok,
                                 const int32_t* __restrict__ tok_off, const int32_t* __restrict__ first_row,
                                 int32_t* __restrict__ row_ptr, int32_t* __restrict__ col, int32_t* __restrict__ rel) {
    const int64_t a = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t total = (int64_t)T * (num_levels - 1);
    const int W = 2 * (k + 1) + 1, zero = k + 1;
    if (a < total) {
        const int lev = 1 + (int)(a / T);
        col[e_tok + a] = (int)(a % T);
        rel[e_tok + a] = lev * W + zero;
    }
    if (a < num_nodes - T) {
        const int node = T + (int)a;
        int lev = 1;
        while (lev + 1 < num_levels && first_row[(lev + 1) * B] <= node) ++lev;
        const int32_t* fr = first_row + lev * B;
        int lo = 0, hi = B;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (fr[mid] <= node)
                lo = mid;
            else
                hi = mid;
        }
        const int64_t m = node - fr[lo];
        row_ptr[node] = (int32_t)(e_tok + (int64_t)(lev - 1) * T + tok_off[lo] + (m << lev));
    }
    if (a == 0) row_ptr[num_nodes] = (int32_t)(e_tok + total);
}

// t_ranges for the packed batch: the neighbours of a token are those of its own sequence
__global__ void batch_t_ranges(int T, int k, int causal, int B, const int32_t* __restrict__ tok_off,
                               const int32_t* __restrict__ first_row, int32_t* __restrict__ last_l,
                               int32_t* __restrict__ last_r, int32_t* __restrict__ min_l, int32_t* __restrict__ min_r) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= T) return;
    const SeqToken s = locate_token(tok_off, B, i);
    const bool has_prev = s.t > 0, has_next = s.t + 1 < s.len;
    {
        LeftWalk A(s.t), P(s.t - 1), N(s.t + 1);
        for (int j = 0; A.alive(); ++j) {
            const int off = first_row[j * B + s.b];
            int lo, hi, plo = 0, phi = -1, nlo = 0, nhi = -1;
            A.run(k, lo, hi);
            const bool pa = has_prev && P.alive(), na = has_next && N.alive();
            if (pa) P.run(k, plo, phi);
            if (na) N.run(k, nlo, nhi);
            for (int x = lo; x <= hi; ++x) {
                if (!(pa && plo <= x && x <= phi)) min_r[off + x] = i;
                if (!(na && nlo <= x && x <= nhi)) last_r[off + x] = i;
            }
            A.up(lo);
            if (pa) P.up(plo);
            if (na) N.up(nlo);
        }
    }
    if (!causal) {
        RightWalkLen A(s.t, s.len), P(s.t - 1, s.len), N(s.t + 1, s.len);
        for (int j = 0; A.alive(); ++j) {
            const int off = first_row[j * B + s.b];
            int lo, hi, plo = 0, phi = -1, nlo = 0, nhi = -1;
            A.run(k, lo, hi);
            // every walk climbs one level per step until it dies, so the three are on level j together
            const bool pa = has_prev && P.alive(), na = has_next && N.alive();
            if (pa) P.run(k, plo, phi);
            if (na) N.run(k, nlo, nhi);
            for (int x = lo; x <= hi; ++x) {
                if (!(pa && plo <= x && x <= phi)) min_l[off + x] = i;
                if (!(na && nlo <= x && x <= nhi)) last_l[off + x] = i;
            }
            A.up(hi);
            if (pa) P.up(phi);
            if (na) N.up(nhi);
        }
    }
}

__global__ void batch_t_fill_spans(int T, int B, int num_levels, int32_t e_tok, const int32_t* __restrict__ tok_off,
                                   const int32_t* __restrict__ first_row, const int32_t* __restrict__ rel,
                                   const int32_t* __restrict__ t_ptr, const int32_t* __restrict__ cnt_l,
                                   const int32_t* __restrict__ cnt_r, int32_t* __restrict__ t_src,
                                   int32_t* __restrict__ t_eid, int32_t* __restrict__ t_rel) {
    const int64_t a = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (a >= (int64_t)T * (num_levels - 1)) return;
    const int lev = 1 + (int)(a / T);
    const int i = (int)(a % T);
    const SeqToken s = locate_token(tok_off, B, i);
    const int32_t e = (int32_t)(e_tok + a);
    const int pos = t_ptr[i] + cnt_l[i] + 1 + cnt_r[i] + (lev - 1);
    t_src[pos] = first_row[lev * B + s.b] + (s.t >> lev);
    t_eid[pos] = e;
    t_rel[pos] = rel[e];
}

// ---- host helpers -------------------------------------------------------------
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
    void* release() {
        void* r = p;
        p = nullptr;
        return r;
    }
};

int exclusive_scan(const int32_t* in, int32_t* out, int m, int32_t total, int32_t* block_sums, hipStream_t st) {
    int nblocks = (m + kScanBlock - 1) / kScanBlock;
    if (nblocks > kScanBlock) return BPT_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(scan_blocks, dim3(nblocks), dim3(kScanThreads), 0, st, in, out, block_sums, m);
    hipLaunchKernelGGL(scan_sums, dim3(1), dim3(kScanThreads), 0, st, block_sums, nblocks);
    hipLaunchKernelGGL(scan_add, dim3((m + 1 + 255) / 256), dim3(256), 0, st, out, block_sums, m, total);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

void free_schedule(Schedule& s) {
    (void)hipFree(s.seg_row);
    (void)hipFree(s.seg_begin);
    (void)hipFree(s.seg_part);
    (void)hipFree(s.tile_ptr);
    (void)hipFree(s.multi_row);
    (void)hipFree(s.multi_ptr);
    s = Schedule();
}

template <typename T>
int upload(const std::vector<T>& h, T** d) {
    BPT_HIP(hipMalloc((void**)d, std::max<size_t>(h.size(), 1) * sizeof(T)));
    if (!h.empty()) BPT_HIP(hipMemcpy(*d, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice));
    return BPT_OK;
}

// Cut rows into segments of at most kSeg edges and group consecutive segments
// into tiles of about kTileWork work units.  Rows without edges still get one
// (empty) segment so that their outputs are written.
// Rows from `span_from` on are span rows: 8 consecutive ones of equal degree <= kSpan8MaxDeg, a power of two (a
// span of a batch graph that a sequence's end cuts short has any degree), become one segment marked kPartSpan8
// (pass the row count to disable).
int make_schedule(const std::vector<int32_t>& ptr, int32_t first_row, int32_t span_from, Schedule& out) {
    const int32_t rows = (int32_t)ptr.size() - 1;
    std::vector<int32_t> seg_row, seg_begin, seg_part, tile_ptr, multi_row, multi_ptr;
    seg_row.reserve(rows + rows / 8);
    seg_begin.reserve(rows + rows / 8);
    seg_part.reserve(rows + rows / 8);
    tile_ptr.push_back(0);
    multi_ptr.push_back(0);
    int64_t work = 0;
    int32_t parts = 0;
    for (int32_t u = first_row; u < rows; ++u) {
        const int32_t b = ptr[u], deg = ptr[u + 1] - b;
        if (u >= span_from && u + 8 <= rows && deg >= 2 && deg <= kSpan8MaxDeg && (deg & (deg - 1)) == 0 &&
            ptr[u + 8] - b == 8 * deg) {
            bool same = true;
            for (int32_t x = 1; x < 8; ++x) same = same && ptr[u + x + 1] - ptr[u + x] == deg;
            if (same) {
                seg_row.push_back(u);
                seg_begin.push_back(b);
                seg_part.push_back(kPartSpan8);
                work += 8 * deg + kRowCost;
                if (work >= kTileWork) {
                    tile_ptr.push_back((int32_t)seg_row.size());
                    work = 0;
                }
                u += 7;
                continue;
            }
        }
        const int32_t nseg = deg <= kSeg ? 1 : (deg + kSeg - 1) / kSeg;
        for (int32_t s = 0; s < nseg; ++s) {
            const int32_t len = std::min<int32_t>(kSeg, deg - s * kSeg);
            seg_row.push_back(u);
            seg_begin.push_back(b + s * kSeg);
            seg_part.push_back(nseg > 1 ? parts++ : -1);
            work += std::max<int32_t>(len, 0) + kRowCost;
            if (work >= kTileWork) {
                tile_ptr.push_back((int32_t)seg_row.size());
                work = 0;
            }
        }
        if (nseg > 1) {
            multi_row.push_back(u);
            multi_ptr.push_back(parts);
        }
    }
    if (tile_ptr.back() != (int32_t)seg_row.size()) tile_ptr.push_back((int32_t)seg_row.size());
    out.num_segs = (int32_t)seg_row.size();
    out.num_tiles = (int32_t)tile_ptr.size() - 1;
    out.num_multi = (int32_t)multi_row.size();
    out.num_part = parts;
    int rc;
    if ((rc = upload(seg_row, &out.seg_row)) || (rc = upload(seg_begin, &out.seg_begin)) ||
        (rc = upload(seg_part, &out.seg_part)) || (rc = upload(tile_ptr, &out.tile_ptr)) ||
        (rc = upload(multi_row, &out.multi_row)) || (rc = upload(multi_ptr, &out.multi_ptr)))
        return rc;
    return BPT_OK;
}

void free_tiles(TokenTiles& t) {
    (void)hipFree(t.chunk_ptr);
    (void)hipFree(t.cols);
    (void)hipFree(t.map);
    (void)hipFree(t.cid_to_id);
    (void)hipFree(t.id_to_cid);
    t = TokenTiles();
}

void free_key_tiles(KeyTiles& t) {
    (void)hipFree(t.chunk_ptr);
    (void)hipFree(t.tile_node0);
    (void)hipFree(t.tile_info);
    (void)hipFree(t.cols);
    (void)hipFree(t.map);
    (void)hipFree(t.task_tile);
    (void)hipFree(t.task_c0);
    (void)hipFree(t.task_nch);
    (void)hipFree(t.task_part);
    (void)hipFree(t.task_ntiles);
    (void)hipFree(t.multi_tile);
    (void)hipFree(t.multi_ptr);
    t = KeyTiles();
}

int build(int32_t n, int32_t k, int32_t causal, hipStream_t st, bpt_graph* g) {
    const int num_levels = 32 - __builtin_clz((unsigned)n);  // log2(n) + 1
    const int num_nodes = 2 * n - 1;
    g->n = n;
    g->n_tokens = n;
    g->k = k;
    g->causal = causal ? 1 : 0;
    g->num_nodes = num_nodes;
    g->num_levels = num_levels;
    g->rel_width = 2 * (k + 1) + 1;
    BPT_HIP(hipGetDevice(&g->device));
    hipDeviceProp_t prop;
    BPT_HIP(hipGetDeviceProperties(&prop, g->device));
    g->num_cus = prop.multiProcessorCount;

    const int tb = kScanThreads;
    const int token_blocks = (n + tb - 1) / tb;
    const int node_blocks = (num_nodes + tb - 1) / tb;

    DeviceBuf deg, counters, block_sums;
    BPT_HIP(deg.alloc(sizeof(int32_t) * (size_t)num_nodes));
    BPT_HIP(counters.alloc(16));
    BPT_HIP(block_sums.alloc(sizeof(int32_t) * kScanBlock));
    BPT_HIP(hipMemsetAsync(counters.p, 0, 16, st));
    unsigned long long* d_total = counters.as<unsigned long long>();
    int32_t* d_maxlev = counters.as<int32_t>() + 2;

    // 1. token degrees, their total, and the deepest contextual level
    hipLaunchKernelGGL(token_degree, dim3(token_blocks), dim3(tb), 0, st, n, k, g->causal, deg.as<int32_t>(), d_total,
                       d_maxlev);
    BPT_HIP(hipGetLastError());
    struct {
        unsigned long long total;
        int32_t maxlev, pad;
    } h = {0, 0, 0};
    BPT_HIP(hipMemcpyAsync(&h, counters.p, 16, hipMemcpyDeviceToHost, st));
    BPT_HIP(hipStreamSynchronize(st));
    const int64_t e_tok = (int64_t)h.total;
    const int64_t e_all = e_tok + (int64_t)n * (num_levels - 1);
    if (e_all > INT32_MAX) return BPT_ERR_OVERFLOW;
    g->num_edges = e_all;
    g->num_token_edges = e_tok;
    g->ctx_levels = std::max(1, (int)h.maxlev);

    // 2. row_ptr: scan of the token degrees; span rows are closed form (fill_spans)
    BPT_HIP(hipMalloc((void**)&g->row_ptr, sizeof(int32_t) * ((size_t)num_nodes + 1)));
    BPT_HIP(hipMalloc((void**)&g->col, sizeof(int32_t) * (size_t)e_all));
    BPT_HIP(hipMalloc((void**)&g->rel, sizeof(int32_t) * (size_t)e_all));
    int rc = exclusive_scan(deg.as<int32_t>(), g->row_ptr, n, (int32_t)e_tok, block_sums.as<int32_t>(), st);
    if (rc) return rc;

    // 3. fill
    hipLaunchKernelGGL(fill_tokens, dim3(token_blocks), dim3(tb), 0, st, n, k, g->causal, g->row_ptr, g->col, g->rel);
    const int64_t aff = (int64_t)n * (num_levels - 1);
    const int aff_blocks = (int)((std::max<int64_t>(aff, n) + tb - 1) / tb);
    hipLaunchKernelGGL(fill_spans, dim3(aff_blocks), dim3(tb), 0, st, n, k, num_levels, (int32_t)e_tok, g->row_ptr,
                       g->col, g->rel);
    BPT_HIP(hipGetLastError());

    // 4. transposed adjacency
    DeviceBuf cnt_l, cnt_r, min_l, min_r;
    const size_t nb = sizeof(int32_t) * (size_t)num_nodes;
    BPT_HIP(cnt_l.alloc(nb));
    BPT_HIP(cnt_r.alloc(nb));
    BPT_HIP(min_l.alloc(nb));
    BPT_HIP(min_r.alloc(nb));
    BPT_HIP(hipMalloc((void**)&g->t_ptr, sizeof(int32_t) * ((size_t)num_nodes + 1)));
    BPT_HIP(hipMalloc((void**)&g->t_src, sizeof(int32_t) * (size_t)e_all));
    BPT_HIP(hipMalloc((void**)&g->t_eid, sizeof(int32_t) * (size_t)e_all));
    BPT_HIP(hipMalloc((void**)&g->t_rel, sizeof(int32_t) * (size_t)e_all));
    hipLaunchKernelGGL(t_init, dim3(node_blocks), dim3(tb), 0, st, num_nodes, cnt_l.as<int32_t>(), cnt_r.as<int32_t>(),
                       min_l.as<int32_t>(), min_r.as<int32_t>());
    hipLaunchKernelGGL(t_ranges, dim3(token_blocks), dim3(tb), 0, st, n, k, g->causal, cnt_l.as<int32_t>(), cnt_r.as<int32_t>(),
                       min_l.as<int32_t>(), min_r.as<int32_t>());
    hipLaunchKernelGGL(t_degree, dim3(node_blocks), dim3(tb), 0, st, n, num_nodes, num_levels, cnt_l.as<int32_t>(),
                       cnt_r.as<int32_t>(), min_l.as<int32_t>(), min_r.as<int32_t>(), deg.as<int32_t>());
    BPT_HIP(hipGetLastError());
    rc = exclusive_scan(deg.as<int32_t>(), g->t_ptr, num_nodes, (int32_t)e_all, block_sums.as<int32_t>(), st);
    if (rc) return rc;
    hipLaunchKernelGGL(t_fill_tokens, dim3(token_blocks), dim3(tb), 0, st, n, k, g->row_ptr, g->col, g->rel, g->t_ptr,
                       cnt_l.as<int32_t>(), min_l.as<int32_t>(), min_r.as<int32_t>(), g->t_src, g->t_eid, g->t_rel);
    if (aff > 0)
        hipLaunchKernelGGL(t_fill_spans, dim3((int)((aff + tb - 1) / tb)), dim3(tb), 0, st, n, num_levels,
                           (int32_t)e_tok, g->rel, g->t_ptr, cnt_l.as<int32_t>(), cnt_r.as<int32_t>(), g->t_src,
                           g->t_eid, g->t_rel);
    BPT_HIP(hipGetLastError());

    // 5. launch schedules (host, from the two row-pointer arrays)
    std::vector<int32_t> h_ptr((size_t)num_nodes + 1), h_tptr((size_t)num_nodes + 1);
    BPT_HIP(hipMemcpyAsync(h_ptr.data(), g->row_ptr, sizeof(int32_t) * h_ptr.size(), hipMemcpyDeviceToHost, st));
    BPT_HIP(hipMemcpyAsync(h_tptr.data(), g->t_ptr, sizeof(int32_t) * h_tptr.size(), hipMemcpyDeviceToHost, st));
    BPT_HIP(hipStreamSynchronize(st));
    if ((rc = make_schedule(h_ptr, 0, n, g->fwd))) return rc;
    if ((rc = make_schedule(h_tptr, 0, num_nodes, g->tr))) return rc;
    // 6. dense tiles for the matrix-core kernels (GPU, from the CSR on the device)
    if ((rc = build_tile_metadata(g, cnt_l.as<int32_t>(), min_l.as<int32_t>(), cnt_r.as<int32_t>(), min_r.as<int32_t>(), st)))
        return rc;
    if (g->tiles.num_tiles > 0 && (rc = make_schedule(h_ptr, n, n, g->fwd_span))) return rc;
    return BPT_OK;
}

// The graph of a batch of sequences (see the kernels above): same steps as build(), no dense tiles -- the
// attention calls run the gather kernels on it.
// What the matrix-core kernels and the stack's readout need of a batch graph beyond its row layout: the tree of
// one sequence with its tile metadata (built here, or shared), the lengths and the row deltas on the device, the
// roots.  g->first_row / row_count / batch / n / num_levels are set.
int batch_tables(int32_t n, int32_t k, int32_t causal, const int32_t* lengths, int32_t B, hipStream_t st, bpt_graph* g,
                 const bpt_graph* shared_tree) {
    const int num_levels = g->num_levels;
    int rc;
    if (shared_tree) {
        g->tree = const_cast<bpt_graph*>(shared_tree);
        g->owns_tree = false;
    } else {
        g->tree = new (std::nothrow) bpt_graph();
        if (!g->tree) return BPT_ERR_ALLOC;
        g->owns_tree = true;
        if ((rc = build(n, k, causal, st, g->tree))) return rc;
    }
    g->ctx_levels = g->tree->ctx_levels;
    std::vector<int32_t> h_delta((size_t)num_levels * B);
    for (int l = 0; l < num_levels; ++l)
        for (int b = 0; b < B; ++b) h_delta[(size_t)l * B + b] = g->first_row[(size_t)l * B + b] - (int32_t)level_offset(n, l);
    std::vector<int32_t> h_len(lengths, lengths + B);
    if ((rc = upload(h_delta, &g->d_delta)) || (rc = upload(h_len, &g->d_lengths))) return rc;
    // the roots (the last level keeps one node of every sequence that has a token)
    std::vector<int32_t> h_root_row((size_t)B), h_root_seq;
    const size_t top = (size_t)(num_levels - 1) * B;
    g->first_root = g->first_row[top];
    for (int b = 0; b < B; ++b) {
        h_root_row[b] = g->row_count[top + b] > 0 ? g->first_row[top + b] : -1;
        if (g->row_count[top + b] > 0) h_root_seq.push_back(b);
    }
    if ((rc = upload(h_root_row, &g->d_root_row)) || (rc = upload(h_root_seq, &g->d_root_seq))) return rc;
    return BPT_OK;
}

// shared_tree: an existing graph of (n, k, causal) to use for the matrix-core kernels instead of building one (not
// owned); with_edges == false: the row layout only -- no CSR, no transposed adjacency, no gather schedules.
int build_batch(int32_t n, int32_t k, int32_t causal, const int32_t* lengths, int32_t B, hipStream_t st, bpt_graph* g,
                const bpt_graph* shared_tree = nullptr, bool with_edges = true) {
    const int num_levels = 32 - __builtin_clz((unsigned)n);
    g->n = n;
    g->k = k;
    g->causal = causal ? 1 : 0;
    g->num_levels = num_levels;
    g->rel_width = 2 * (k + 1) + 1;
    g->batch = B;
    if (shared_tree) {
        g->device = shared_tree->device;
        g->num_cus = shared_tree->num_cus;
    } else {
        BPT_HIP(hipGetDevice(&g->device));
        hipDeviceProp_t prop;
        BPT_HIP(hipGetDeviceProperties(&prop, g->device));
        g->num_cus = prop.multiProcessorCount;
    }

    // row numbering (host): level-major over the batch
    g->first_row.assign((size_t)num_levels * B, 0);
    g->row_count.assign((size_t)num_levels * B, 0);
    int64_t row = 0;
    for (int l = 0; l < num_levels; ++l)
        for (int b = 0; b < B; ++b) {
            const int64_t cnt = ((int64_t)lengths[b] + ((int64_t)1 << l) - 1) >> l;
            g->first_row[(size_t)l * B + b] = (int32_t)row;
            g->row_count[(size_t)l * B + b] = (int32_t)cnt;
            row += cnt;
            if (row > (1 << 23)) return BPT_ERR_UNSUPPORTED;
        }
    const int num_nodes = (int)row;
    std::vector<int32_t> h_tok_off((size_t)B + 1);
    for (int b = 0; b < B; ++b) h_tok_off[b] = g->first_row[b];
    const int T = B > 0 ? g->first_row[B - 1] + g->row_count[B - 1] : 0;
    h_tok_off[B] = T;
    if (T < 1) return BPT_ERR_INVALID_ARG;
    g->num_nodes = num_nodes;
    g->n_tokens = T;
    int rc = batch_tables(n, k, causal, lengths, B, st, g, shared_tree);
    if (rc || !with_edges) return rc;

    DeviceBuf tok_off, first_row, deg, counters, block_sums;
    BPT_HIP(tok_off.alloc(sizeof(int32_t) * h_tok_off.size()));
    BPT_HIP(first_row.alloc(sizeof(int32_t) * g->first_row.size()));
    BPT_HIP(hipMemcpyAsync(tok_off.p, h_tok_off.data(), sizeof(int32_t) * h_tok_off.size(), hipMemcpyHostToDevice, st));
    BPT_HIP(hipMemcpyAsync(first_row.p, g->first_row.data(), sizeof(int32_t) * g->first_row.size(), hipMemcpyHostToDevice, st));
    BPT_HIP(deg.alloc(sizeof(int32_t) * (size_t)num_nodes));
    BPT_HIP(counters.alloc(16));
    BPT_HIP(block_sums.alloc(sizeof(int32_t) * kScanBlock));
    BPT_HIP(hipMemsetAsync(counters.p, 0, 16, st));
    const int tb = kScanThreads;
    const int token_blocks = (T + tb - 1) / tb;
    const int node_blocks = (num_nodes + tb - 1) / tb;

    // 1. token degrees
    hipLaunchKernelGGL(batch_token_degree, dim3(token_blocks), dim3(tb), 0, st, T, k, g->causal, B, tok_off.as<int32_t>(),
                       deg.as<int32_t>(), counters.as<unsigned long long>(), counters.as<int32_t>() + 2);
    BPT_HIP(hipGetLastError());
    struct {
        unsigned long long total;
        int32_t maxlev, pad;
    } h = {0, 0, 0};
    BPT_HIP(hipMemcpyAsync(&h, counters.p, 16, hipMemcpyDeviceToHost, st));
    BPT_HIP(hipStreamSynchronize(st));   // also: the host arrays above have been read
    const int64_t e_tok = (int64_t)h.total;
    const int64_t aff = (int64_t)T * (num_levels - 1);
    const int64_t e_all = e_tok + aff;
    if (e_all > INT32_MAX) return BPT_ERR_OVERFLOW;
    g->num_edges = e_all;
    g->num_token_edges = e_tok;
    g->ctx_levels = std::max(1, (int)h.maxlev);

    // 2. row_ptr, 3. fill
    BPT_HIP(hipMalloc((void**)&g->row_ptr, sizeof(int32_t) * ((size_t)num_nodes + 1)));
    BPT_HIP(hipMalloc((void**)&g->col, sizeof(int32_t) * (size_t)e_all));
    BPT_HIP(hipMalloc((void**)&g->rel, sizeof(int32_t) * (size_t)e_all));
    rc = exclusive_scan(deg.as<int32_t>(), g->row_ptr, T, (int32_t)e_tok, block_sums.as<int32_t>(), st);
    if (rc) return rc;
    hipLaunchKernelGGL(batch_fill_tokens, dim3(token_blocks), dim3(tb), 0, st, T, k, g->causal, B, tok_off.as<int32_t>(),
                       first_row.as<int32_t>(), g->row_ptr, g->col, g->rel);
    const int64_t span_items = std::max<int64_t>(std::max<int64_t>(aff, num_nodes - T), 1);
    hipLaunchKernelGGL(batch_fill_spans, dim3((unsigned)((span_items + tb - 1) / tb)), dim3(tb), 0, st, T, k, B, num_levels,
                       num_nodes, (int32_t)e_tok, tok_off.as<int32_t>(), first_row.as<int32_t>(), g->row_ptr, g->col, g->rel);
    BPT_HIP(hipGetLastError());

    // 4. transposed adjacency
    DeviceBuf cnt_l, cnt_r, min_l, min_r;
    const size_t nb = sizeof(int32_t) * (size_t)num_nodes;
    BPT_HIP(cnt_l.alloc(nb));
    BPT_HIP(cnt_r.alloc(nb));
    BPT_HIP(min_l.alloc(nb));
    BPT_HIP(min_r.alloc(nb));
    BPT_HIP(hipMalloc((void**)&g->t_ptr, sizeof(int32_t) * ((size_t)num_nodes + 1)));
    BPT_HIP(hipMalloc((void**)&g->t_src, sizeof(int32_t) * (size_t)e_all));
    BPT_HIP(hipMalloc((void**)&g->t_eid, sizeof(int32_t) * (size_t)e_all));
    BPT_HIP(hipMalloc((void**)&g->t_rel, sizeof(int32_t) * (size_t)e_all));
    hipLaunchKernelGGL(t_init, dim3(node_blocks), dim3(tb), 0, st, num_nodes, cnt_l.as<int32_t>(), cnt_r.as<int32_t>(),
                       min_l.as<int32_t>(), min_r.as<int32_t>());
    hipLaunchKernelGGL(batch_t_ranges, dim3(token_blocks), dim3(tb), 0, st, T, k, g->causal, B, tok_off.as<int32_t>(),
                       first_row.as<int32_t>(), cnt_l.as<int32_t>(), cnt_r.as<int32_t>(), min_l.as<int32_t>(),
                       min_r.as<int32_t>());
    hipLaunchKernelGGL(t_degree, dim3(node_blocks), dim3(tb), 0, st, T, num_nodes, num_levels, cnt_l.as<int32_t>(),
                       cnt_r.as<int32_t>(), min_l.as<int32_t>(), min_r.as<int32_t>(), deg.as<int32_t>());
    BPT_HIP(hipGetLastError());
    rc = exclusive_scan(deg.as<int32_t>(), g->t_ptr, num_nodes, (int32_t)e_all, block_sums.as<int32_t>(), st);
    if (rc) return rc;
    hipLaunchKernelGGL(t_fill_tokens, dim3(token_blocks), dim3(tb), 0, st, T, k, g->row_ptr, g->col, g->rel, g->t_ptr,
                       cnt_l.as<int32_t>(), min_l.as<int32_t>(), min_r.as<int32_t>(), g->t_src, g->t_eid, g->t_rel);
    if (aff > 0)
        hipLaunchKernelGGL(batch_t_fill_spans, dim3((unsigned)((aff + tb - 1) / tb)), dim3(tb), 0, st, T, B, num_levels,
                           (int32_t)e_tok, tok_off.as<int32_t>(), first_row.as<int32_t>(), g->rel, g->t_ptr,
                           cnt_l.as<int32_t>(), cnt_r.as<int32_t>(), g->t_src, g->t_eid, g->t_rel);
    BPT_HIP(hipGetLastError());

    // 5. launch schedules
    std::vector<int32_t> h_ptr((size_t)num_nodes + 1), h_tptr((size_t)num_nodes + 1);
    BPT_HIP(hipMemcpyAsync(h_ptr.data(), g->row_ptr, sizeof(int32_t) * h_ptr.size(), hipMemcpyDeviceToHost, st));
    BPT_HIP(hipMemcpyAsync(h_tptr.data(), g->t_ptr, sizeof(int32_t) * h_tptr.size(), hipMemcpyDeviceToHost, st));
    BPT_HIP(hipStreamSynchronize(st));
    if ((rc = make_schedule(h_ptr, 0, T, g->fwd))) return rc;
    return make_schedule(h_tptr, 0, num_nodes, g->tr);
}

}  // namespace
}  // namespace bpt

namespace bpt {
namespace prof {
namespace {
struct Rec {
    const char* name;
    hipEvent_t a, b;
};
bool g_on = false;
std::vector<Rec> g_recs;
void clear() {
    for (Rec& r : g_recs) {
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_recs.clear();
}
}  // namespace
bool enabled() { return g_on; }
namespace {
bool g_open = false;   // begin() has pushed a record that end() still has to close
}
void begin(const char* name, hipStream_t st) {
    g_open = false;
    // no events inside a stream capture: they would become nodes of the captured graph
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) != hipSuccess) {
        (void)hipGetLastError();
        return;
    }
    if (cap != hipStreamCaptureStatusNone) return;
    Rec r{name, nullptr, nullptr};
    if (hipEventCreate(&r.a) != hipSuccess) {
        (void)hipGetLastError();
        return;
    }
    if (hipEventCreate(&r.b) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipEventDestroy(r.a);
        return;
    }
    if (hipEventRecord(r.a, st) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
        return;
    }
    g_recs.push_back(r);
    g_open = true;
}
void end(hipStream_t st) {
    if (!g_open) return;   // begin() made no record for this launch: nothing of an earlier launch is touched
    g_open = false;
    if (hipEventRecord(g_recs.back().b, st) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipEventDestroy(g_recs.back().a);
        (void)hipEventDestroy(g_recs.back().b);
        g_recs.pop_back();
    }
}
}  // namespace prof
}  // namespace bpt

namespace bpt {
namespace {
// Rows of 128 bytes read once each through a list of row numbers, 8 consecutive lanes per row and 16 bytes per
// lane -- the request shape of the attention kernels' row gathers -- and written back in list order.
__global__ void __launch_bounds__(256) calibrate_gather_kernel(const uint4* __restrict__ src, const int32_t* __restrict__ perm,
                                                               uint4* __restrict__ dst, int64_t rows) {
    const int64_t slot = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t r = slot >> 3;
    if (r >= rows) return;
    const int piece = (int)(slot & 7);
    dst[r * 8 + piece] = src[(int64_t)perm[r] * 8 + piece];
}
}  // namespace
}  // namespace bpt

extern "C" {

int bpt_calibrate_gather(const void* src, const int32_t* perm, void* dst, int64_t rows, void* stream) {
    if (!src || !perm || !dst || rows < 1 || rows > ((int64_t)1 << 31) - 1) return BPT_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst)) & 15u) return BPT_ERR_INVALID_ARG;
    const int64_t blocks = (rows * 8 + 255) / 256;
    if (blocks > INT32_MAX) return BPT_ERR_INVALID_ARG;
    hipStream_t st = static_cast<hipStream_t>(stream);
    BPT_LAUNCH("calibrate_gather_kernel", bpt::calibrate_gather_kernel, dim3((unsigned)blocks), dim3(256), 0, st,
               static_cast<const uint4*>(src), perm, static_cast<uint4*>(dst), rows);
    BPT_HIP(hipGetLastError());
    return BPT_OK;
}

int bpt_profile_enable(int on) {
    bpt::prof::clear();
    bpt::prof::g_on = on != 0;
    return BPT_OK;
}

int64_t bpt_profile_report(char* buf, size_t capacity) {
    using namespace bpt::prof;
    std::vector<std::pair<const char*, std::pair<int, double>>> agg;
    for (Rec& r : g_recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) {
            (void)hipGetLastError();
            return -1;
        }
        bool found = false;
        for (auto& e : agg)
            if (e.first == r.name) {
                e.second.first += 1;
                e.second.second += ms;
                found = true;
            }
        if (!found) agg.push_back({r.name, {1, (double)ms}});
    }
    std::string text;
    for (auto& e : agg) {
        char line[160];
        snprintf(line, sizeof line, "%s %d %.6f\n", e.first, e.second.first, e.second.second);
        text += line;
    }
    if (buf && capacity > 0) {
        const size_t ncopy = std::min(capacity - 1, text.size());
        memcpy(buf, text.data(), ncopy);
        buf[ncopy] = 0;
    }
    return (int64_t)text.size() + 1;
}

void bpt_graph_destroy(bpt_graph_t* g) {
    if (!g) return;
    (void)hipFree(g->row_ptr);
    (void)hipFree(g->col);
    (void)hipFree(g->rel);
    (void)hipFree(g->t_ptr);
    (void)hipFree(g->t_src);
    (void)hipFree(g->t_eid);
    (void)hipFree(g->t_rel);
    bpt::free_schedule(g->fwd);
    bpt::free_schedule(g->tr);
    bpt::free_schedule(g->fwd_span);
    bpt::free_tiles(g->tiles);
    bpt::free_key_tiles(g->ktiles);
    (void)hipFree(g->d_lengths);
    (void)hipFree(g->d_delta);
    (void)hipFree(g->d_root_row);
    (void)hipFree(g->d_root_seq);
    if (g->owns_tree) bpt_graph_destroy(g->tree);
    delete g;
}

int bpt_build_graph(int32_t n, int32_t k, int32_t causal, void* stream, bpt_graph_t** out) {
    if (!out) return BPT_ERR_INVALID_ARG;
    *out = nullptr;
    if (n < 2 || k < 1) return BPT_ERR_INVALID_ARG;
    if ((n & (n - 1)) != 0 || n > (1 << 22) || k > (1 << 20)) return BPT_ERR_UNSUPPORTED;
    bpt_graph* g = new (std::nothrow) bpt_graph();
    if (!g) return BPT_ERR_ALLOC;
    int rc;
    try {
        rc = bpt::build(n, k, causal, static_cast<hipStream_t>(stream), g);
        // set-up is also where the address of this device's static scratch is looked up (bpt_attn_fwd_static)
        void* scratch_ptr = nullptr;
        if (rc == BPT_OK) rc = bpt::static_scratch(g->device, &scratch_ptr);
    } catch (const std::bad_alloc&) {
        rc = BPT_ERR_ALLOC;
    }
    if (rc != BPT_OK) {
        bpt_graph_destroy(g);
        return rc;
    }
    *out = g;
    return BPT_OK;
}

int bpt_build_batch_graph(int32_t n, int32_t k, int32_t causal, const int32_t* lengths, int32_t batch, void* stream,
                          bpt_graph_t** out) {
    if (!out) return BPT_ERR_INVALID_ARG;
    *out = nullptr;
    if (n < 2 || k < 1 || !lengths || batch < 1) return BPT_ERR_INVALID_ARG;
    if ((n & (n - 1)) != 0 || n > (1 << 22) || k > (1 << 20) || batch > (1 << 16)) return BPT_ERR_UNSUPPORTED;
    for (int32_t b = 0; b < batch; ++b)
        if (lengths[b] < 0 || lengths[b] > n) return BPT_ERR_INVALID_ARG;
    bpt_graph* g = new (std::nothrow) bpt_graph();
    if (!g) return BPT_ERR_ALLOC;
    int rc;
    try {
        rc = bpt::build_batch(n, k, causal, lengths, batch, static_cast<hipStream_t>(stream), g);
        void* scratch_ptr = nullptr;
        if (rc == BPT_OK) rc = bpt::static_scratch(g->device, &scratch_ptr);
    } catch (const std::bad_alloc&) {
        rc = BPT_ERR_ALLOC;
    }
    if (rc != BPT_OK) {
        bpt_graph_destroy(g);
        return rc;
    }
    *out = g;
    return BPT_OK;
}

int bpt_build_batch_graph_on(const bpt_graph_t* tree, const int32_t* lengths, int32_t batch, int32_t with_edges, void* stream,
                             bpt_graph_t** out) {
    if (!out) return BPT_ERR_INVALID_ARG;
    *out = nullptr;
    if (!tree || tree->batch > 0 || !lengths || batch < 1) return BPT_ERR_INVALID_ARG;
    if (batch > (1 << 16)) return BPT_ERR_UNSUPPORTED;
    for (int32_t b = 0; b < batch; ++b)
        if (lengths[b] < 0 || lengths[b] > tree->n) return BPT_ERR_INVALID_ARG;
    int device = -1;
    if (hipGetDevice(&device) != hipSuccess || device != tree->device) return BPT_ERR_INVALID_ARG;
    bpt_graph* g = new (std::nothrow) bpt_graph();
    if (!g) return BPT_ERR_ALLOC;
    int rc;
    try {
        rc = bpt::build_batch(tree->n, tree->k, tree->causal, lengths, batch, static_cast<hipStream_t>(stream), g, tree,
                              with_edges != 0);
    } catch (const std::bad_alloc&) {
        rc = BPT_ERR_ALLOC;
    }
    if (rc != BPT_OK) {
        bpt_graph_destroy(g);
        return rc;
    }
    *out = g;
    return BPT_OK;
}

int bpt_graph_layout(const bpt_graph_t* g, int32_t* batch, int32_t* n_tokens, int32_t* first_row, int32_t* row_count) {
    if (!g) return BPT_ERR_INVALID_ARG;
    if (batch) *batch = g->batch > 0 ? g->batch : 1;
    if (n_tokens) *n_tokens = g->n_tokens;
    if (g->batch > 0) {
        if (first_row) std::copy(g->first_row.begin(), g->first_row.end(), first_row);
        if (row_count) std::copy(g->row_count.begin(), g->row_count.end(), row_count);
    } else {
        for (int l = 0; l < g->num_levels; ++l) {
            if (first_row) first_row[l] = (int32_t)bpt::level_offset(g->n, l);
            if (row_count) row_count[l] = g->n >> l;
        }
    }
    return BPT_OK;
}

int bpt_graph_info(const bpt_graph_t* g, int32_t* n, int32_t* k, int32_t* causal, int32_t* num_nodes,
                   int64_t* num_edges, int32_t* num_levels, int32_t* rel_width, int32_t* ctx_levels) {
    if (!g) return BPT_ERR_INVALID_ARG;
    if (n) *n = g->n;
    if (k) *k = g->k;
    if (causal) *causal = g->causal;
    if (num_nodes) *num_nodes = g->num_nodes;
    if (num_edges) *num_edges = g->num_edges;
    if (num_levels) *num_levels = g->num_levels;
    if (rel_width) *rel_width = g->rel_width;
    if (ctx_levels) *ctx_levels = g->ctx_levels;
    return BPT_OK;
}

int bpt_graph_csr(const bpt_graph_t* g, const int32_t** row_ptr, const int32_t** col, const int32_t** rel) {
    if (!g) return BPT_ERR_INVALID_ARG;
    if (!g->row_ptr) return BPT_ERR_UNSUPPORTED;   // a batch graph built without its edge lists
    if (row_ptr) *row_ptr = g->row_ptr;
    if (col) *col = g->col;
    if (rel) *rel = g->rel;
    return BPT_OK;
}

int bpt_graph_transposed(const bpt_graph_t* g, const int32_t** t_ptr, const int32_t** t_src, const int32_t** t_eid) {
    if (!g) return BPT_ERR_INVALID_ARG;
    if (!g->row_ptr) return BPT_ERR_UNSUPPORTED;   // a batch graph built without its edge lists
    if (t_ptr) *t_ptr = g->t_ptr;
    if (t_src) *t_src = g->t_src;
    if (t_eid) *t_eid = g->t_eid;
    return BPT_OK;
}

static int copy_out(int32_t* dst, const int32_t* src, size_t count) {
    if (dst && count) BPT_HIP(hipMemcpy(dst, src, count * sizeof(int32_t), hipMemcpyDeviceToHost));
    return BPT_OK;
}

int bpt_graph_to_host(const bpt_graph_t* g, int32_t* row_ptr, int32_t* col, int32_t* rel) {
    if (!g) return BPT_ERR_INVALID_ARG;
    if (!g->row_ptr) return BPT_ERR_UNSUPPORTED;   // a batch graph built without its edge lists
    int rc;
    if ((rc = copy_out(row_ptr, g->row_ptr, (size_t)g->num_nodes + 1))) return rc;
    if ((rc = copy_out(col, g->col, (size_t)g->num_edges))) return rc;
    return copy_out(rel, g->rel, (size_t)g->num_edges);
}

int bpt_graph_transposed_to_host(const bpt_graph_t* g, int32_t* t_ptr, int32_t* t_src, int32_t* t_eid) {
    if (!g) return BPT_ERR_INVALID_ARG;
    if (!g->row_ptr) return BPT_ERR_UNSUPPORTED;   // a batch graph built without its edge lists
    int rc;
    if ((rc = copy_out(t_ptr, g->t_ptr, (size_t)g->num_nodes + 1))) return rc;
    if ((rc = copy_out(t_src, g->t_src, (size_t)g->num_edges))) return rc;
    return copy_out(t_eid, g->t_eid, (size_t)g->num_edges);
}

int bpt_count_edges(int32_t n, int32_t k, int32_t causal, int32_t len, int64_t* edges) {
    if (!edges || n < 2 || k < 1 || len < 0 || len > n) return BPT_ERR_INVALID_ARG;
    if ((n & (n - 1)) != 0 || n > (1 << 22) || k > (1 << 20)) return BPT_ERR_UNSUPPORTED;
    int levels = 1;
    while ((1 << (levels - 1)) < n) ++levels;
    // span rows: on every level above the tokens the kept nodes hold each token once
    int64_t total = (int64_t)len * (levels - 1);
    for (int64_t i = 0; i < len; ++i) {
        int64_t d = 1;   // self
        for (int64_t q = i - 1; q >= 0;) {   // left side: everything left of a token is kept
            int64_t e = std::max<int64_t>(q - k + 1, 0);
            if (e & 1) e -= 1;
            d += q - e + 1;
            q = e >= 1 ? (e - 1) >> 1 : -1;
        }
        if (!causal) {
            int64_t p = i + 1;
            for (int l = 0;; ++l) {   // right side: level l keeps ceil(len / 2^l) nodes
                const int64_t cnt = (len + ((int64_t)1 << l) - 1) >> l;
                if (p >= cnt) break;
                int64_t e = std::min<int64_t>(p + k - 1, cnt - 1);
                if (!(e & 1) && e + 1 < cnt) e += 1;
                d += e - p + 1;
                if (e + 1 >= cnt) break;
                p = (e + 1) >> 1;
            }
        }
        total += d;
    }
    *edges = total;
    return BPT_OK;
}

const char* bpt_strerror(int status) {
    switch (status) {
        case BPT_OK: return "ok";
        case BPT_ERR_INVALID_ARG: return "invalid argument";
        case BPT_ERR_UNSUPPORTED: return "unsupported size, width or dtype";
        case BPT_ERR_ALLOC: return "allocation failed";
        case BPT_ERR_LAUNCH: return "HIP call or kernel launch failed";
        case BPT_ERR_OVERFLOW: return "graph has more than INT32_MAX edges";
        case BPT_ERR_SCRATCH: return "the call needs more scratch than the library's static buffer holds";
        default: return "unknown status";
    }
}

}  // extern "C"
