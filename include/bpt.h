/*
 * bpt.h -- C ABI of the MI355X (gfx950) BP-Transformer graph self-attention library.
 *
 * The library computes the hot path of BP-Transformer (arXiv 1911.04070):
 *   1. the binary-partition graph of a sequence (Sec. 3.2): tokens are the
 *      leaves of a perfect binary tree, spans its internal nodes; every span
 *      node attends to the tokens it contains (affiliated edges) and every
 *      token attends to itself and, per side and per tree level from fine to
 *      coarse, to k (+1 alignment) nodes (contextual edges, Algorithm 1);
 *   2. graph self-attention with tree relative positions over that graph
 *      (Sec. 3.1 eq. (6), Sec. 3.4 eq. (8)), forward and backward.
 *
 * Conventions
 *   - Every function returns a bpt_status_t code and never throws or aborts.
 *   - "device" pointers are HIP device memory of the current device, owned by
 *     the caller unless stated otherwise; "host" pointers are ordinary memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Attention calls are asynchronous on it.  bpt_build_graph and the
 *     *_to_host calls synchronise it.
 *   - Nodes are numbered level-major: id(l,m) = 2n - (2n >> l) + m, so tokens
 *     are 0..n-1, level-1 spans n..n+n/2-1, ..., the root is 2n-2.  N = 2n-1.
 *   - An edge u <- v ("u attends to v") is stored in row u of a CSR
 *     (row_ptr[N+1], col[E] = v, rel[E] = relative-position id).  The id packs
 *     (level j of v, signed order o) as  j*W + (o + k+1),  W = 2(k+1)+1:
 *     o = 0 at level 0 is r_self, o = 0 at level j>=1 is r_anc(j) (span rows),
 *     o = +i / -i is the i-th node to join on the right / left at level j,
 *     nearest first, i = 1..k+1 (Sec. 3.4).  Rows are sorted by id ascending
 *     (which also sorts them by col).
 *   - The relative-position table `rel` is [num_levels][W][D] in the tensor
 *     dtype, shared by all batches and heads (Sec. 3.4).
 *   - Q, K, V, out, dout and the fp32 gradients dQ, dK, dV are [B][H][N][D]
 *     with D contiguous and element strides stride_b, stride_h, stride_n
 *     (the same for all of them); lse is contiguous [B][H][N] fp32.
 *   - Outputs are fully overwritten, never accumulated into.
 *
 * Dropout on the attention weights (p_a in the paper's hyper-parameter tables, which give the
 * rate and no formula): inverted dropout after the softmax.  With rate p the output is
 * out_u = sum_e keep_e p_e v_v / (1 - p); lse is that of the full softmax; the backward uses the
 * same mask (pass the same dropout_p and dropout_seed to forward and backward).  keep_e is a
 * counter-based hash, so that no mask is stored and every kernel that meets an edge can form it:
 *   mix(z): z ^= z >> 16; z *= 0x7FEB352D; z ^= z >> 15; z *= 0x846CA68B; z ^= z >> 16  (32 bit)
 *   keep_e = mix(mix(mix(seed ^ 0x9E3779B9 * bh) + u) + x_e) >= floor(p * 2^32),
 * bh = b * H + h, u = query node, x_e = relative-position id of the edge for a token row and
 * 2^31 + key node for a span row.  Use a fresh seed per layer and step.
 *
 * Sequences shorter than n (batches of sequences of different lengths).  The paper
 * states the tree for n a power of two (Sec. 3.2.1).  A batch entry b with
 * len = seq_len[b] < n tokens lives on the same node ids and keeps the nodes that hold
 * at least one of its tokens: node (l, m) is kept iff m * 2^l < len, so level l keeps
 * its first ceil(len / 2^l) nodes, the last one possibly cut short.  An edge of the
 * graph counts iff both of its nodes are kept; this is what Algorithm 1 gives when its
 * runs are clipped to the kept nodes of each level.  Rows of nodes that are not kept
 * produce zeros in every output (out, lse, dQ, dK, dV) -- or are left unwritten, see
 * bpt_shape_t.leave_unkept -- and add nothing to d_rel; their input rows are never used but
 * must hold finite values.  Values of seq_len outside [0, n] are clamped.
 */
#ifndef BPT_H_
#define BPT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bpt_graph bpt_graph_t; /* opaque; device-resident; owned by the library */

typedef enum { BPT_F32 = 0, BPT_BF16 = 1 } bpt_dtype_t;

typedef enum {
    BPT_OK = 0,
    BPT_ERR_INVALID_ARG = 1, /* null pointer, k < 1, n < 2, bad stride, small workspace */
    BPT_ERR_UNSUPPORTED = 2, /* n not a power of two, n > 2^22, k > 2^20, D != 64, dtype; attention calls also:
                                a graph of 2^29 edges or more, a (batch, head) slab (N * stride_n elements) of
                                2 GiB or more, a row stride of 16 MiB or more -- see bpt_attn_fwd */
    BPT_ERR_ALLOC = 3,       /* device or host allocation failed */
    BPT_ERR_LAUNCH = 4,      /* a HIP call or kernel launch failed */
    BPT_ERR_OVERFLOW = 5,    /* the graph has more than INT32_MAX edges */
    BPT_ERR_SCRATCH = 6      /* bpt_attn_fwd_static: the shape needs more than BPT_STATIC_SCRATCH_BYTES of scratch */
} bpt_status_t;

typedef struct {
    int32_t B, H, D;     /* batch, heads, head width (D must be 64) */
    int32_t dtype;       /* bpt_dtype_t of Q, K, V, rel, out, dout */
    int64_t stride_b, stride_h, stride_n; /* in elements; stride_n >= D, multiples of 8 */
    float scale;         /* softmax scale; <= 0 selects 1/sqrt(D) (Sec. 3.1 eq. (6)) */
    const int32_t* seq_len; /* device pointer to B token counts, or NULL: every sequence has n
                              tokens.  See "Sequences shorter than n" above. */
    float dropout_p;     /* dropout rate on the attention weights, 0 <= p < 1; 0: none.  See below. */
    uint32_t dropout_seed;
    int32_t leave_unkept; /* with seq_len, nonzero: the rows of out, lse, dQ, dK, dV of nodes that a sequence does
                             not keep are left unwritten (they hold whatever the buffers held) instead of being
                             zero-filled, so that the time and the bytes written follow the tokens that exist
                             rather than the padded size.  Rows of kept nodes and d_rel are the same either way. */
    int32_t grad_dtype;   /* bpt_dtype_t of dQ, dK, dV: BPT_F32 (0, the default) or, with dtype = BPT_BF16, BPT_BF16:
                             the backward then writes the three gradients rounded to bf16 (round to nearest even,
                             from the same fp32 sums), with the tensor strides counted in bf16 elements -- half
                             the bytes written, and gradients that feed a bf16 GEMM need no cast.  d_rel stays
                             fp32.  Any other combination: BPT_ERR_INVALID_ARG. */
} bpt_shape_t;

/* Sec. 3.2 + Algorithm 1.  Builds, on the current device, the graph of a
 * sequence of n tokens (power of two, 2 <= n <= 2^22) with density k
 * (1 <= k <= 2^20): CSR by query node, its transposed adjacency, and the launch
 * schedules the attention kernels use.  causal != 0 drops every token's right
 * context (left contexts only).  All edges are produced by GPU kernels; the
 * result is bit-identical to a sequential CPU construction.  *out is owned by
 * the library until bpt_graph_destroy.  Synchronises `stream`. */
int bpt_build_graph(int32_t n, int32_t k, int32_t causal, void* stream, bpt_graph_t** out);

/* Sec. 4.1 (batches of sequences of different lengths; the appendix on implementation
 * details: the graphs of a batch are joined into one).  Builds, on the current device, ONE
 * graph for a batch of `batch` sequences, sequence b holding lengths[b] tokens (host array,
 * 0 <= lengths[b] <= n, at least one token in all; 1 <= batch <= 65536): the disjoint union
 * of the graphs that "Sequences shorter than n" above defines for each length on the tree
 * over n (n, k, causal as for bpt_build_graph).  Only kept nodes get a row, so tensors,
 * workspaces and work follow the tokens that exist instead of batch * (2n-1).
 * Row numbering ("packed", see bpt_graph_layout): level-major over the batch -- the tokens of
 * sequence 0, of sequence 1, ..., then the level-1 nodes of sequence 0, of sequence 1, ... up
 * to the root level; node (level l, index m) of sequence b is row first_row[l][b] + m and
 * level l of that sequence has ceil(lengths[b] / 2^l) rows.  col / t_src hold packed rows;
 * rel ids and the canonical order within a row are those of the single-sequence graph, and
 * the relative-position table is shared by all sequences (Sec. 3.4).
 * The attention calls (and bpt_layer_fwd / bpt_layer_bwd) take such a graph like any other,
 * with N = its row count, B = 1 (or B independent batches of the same length mix) and
 * seq_len = NULL (BPT_ERR_INVALID_ARG otherwise).  bf16 tensors with B = 1 run the matrix-core
 * kernels (they walk the tree of one sequence once per sequence and head and address the packed
 * rows through the per-level offsets; n >= 32 and at most 512 relative-position ids in use),
 * anything else the gather kernels; the results are the same rows either way.  Dropout on the
 * attention weights is refused on it (BPT_ERR_UNSUPPORTED).
 * More than 2^23 rows: BPT_ERR_UNSUPPORTED.  Synchronises `stream`. */
int bpt_build_batch_graph(int32_t n, int32_t k, int32_t causal, const int32_t* lengths, int32_t batch,
                          void* stream, bpt_graph_t** out);

/* The same for callers that build a graph for every batch they see (training on sentences): on an
 * existing graph `tree` of bpt_build_graph(n, k, causal), which the new graph shares instead of
 * building its own (the caller keeps `tree` alive until the new graph is destroyed; both on the
 * current device), and, with with_edges == 0, without the batch's own CSR, transposed adjacency and
 * gather schedules: only the row layout and the small tables the matrix-core kernels need are made
 * (host arithmetic and four small copies).  Such a graph serves every call that runs on the
 * matrix-core kernels (see above; also the layer and stack calls); the graph accessors and calls
 * that would need the gather kernels return BPT_ERR_UNSUPPORTED (workspace queries SIZE_MAX), and
 * bpt_graph_info reports 0 edges. */
int bpt_build_batch_graph_on(const bpt_graph_t* tree, const int32_t* lengths, int32_t batch,
                             int32_t with_edges, void* stream, bpt_graph_t** out);

/* Row layout of a graph: *batch = sequences in it (1 for bpt_build_graph), *n_tokens = token
 * rows (they come first), and, into host arrays of num_levels * batch entries indexed
 * [level * batch + b], first_row = row of node (level, 0) of sequence b and row_count = nodes
 * of that level the sequence keeps.  NULL skips an output. */
int bpt_graph_layout(const bpt_graph_t* g, int32_t* batch, int32_t* n_tokens, int32_t* first_row,
                     int32_t* row_count);

/* Any output pointer may be NULL.  num_levels = log2(n)+1, rel_width = W,
 * ctx_levels = number of levels on which some token has contextual nodes. */
int bpt_graph_info(const bpt_graph_t* g, int32_t* n, int32_t* k, int32_t* causal,
                   int32_t* num_nodes, int64_t* num_edges, int32_t* num_levels,
                   int32_t* rel_width, int32_t* ctx_levels);

/* Device pointers into the graph, valid until destroy: row_ptr[N+1], col[E], rel[E]. */
int bpt_graph_csr(const bpt_graph_t* g, const int32_t** row_ptr, const int32_t** col,
                  const int32_t** rel);

/* Transposed adjacency (device pointers): for each key node v, t_ptr[v]..t_ptr[v+1]
 * lists the edges that point at it in ascending edge index: t_src = query node,
 * t_eid = index of the edge in col/rel. */
int bpt_graph_transposed(const bpt_graph_t* g, const int32_t** t_ptr, const int32_t** t_src,
                         const int32_t** t_eid);

/* Copies to host arrays the caller allocated (sizes as above); NULL skips one. */
int bpt_graph_to_host(const bpt_graph_t* g, int32_t* row_ptr, int32_t* col, int32_t* rel);
int bpt_graph_transposed_to_host(const bpt_graph_t* g, int32_t* t_ptr, int32_t* t_src,
                                 int32_t* t_eid);

void bpt_graph_destroy(bpt_graph_t* g);

/* Bytes of device scratch the forward / backward need for this graph and shape
 * (0 is possible).  The caller allocates it (256-byte aligned) and may reuse it
 * between calls on the same stream.  SIZE_MAX ((size_t)-1) if the attention calls
 * would refuse this graph and shape (see the limits at bpt_attn_fwd). */
size_t bpt_attn_fwd_workspace(const bpt_graph_t* g, const bpt_shape_t* s);
size_t bpt_attn_bwd_workspace(const bpt_graph_t* g, const bpt_shape_t* s);

/* Sec. 3.4 eq. (8), for every node u of every (batch, head):
 *   s_e   = scale * q_u . (k_v + rel[id_e])        over the edges e = (u <- v) of row u
 *   lse_u = log sum_e exp(s_e)                      (natural log)
 *   out_u = sum_e exp(s_e - lse_u) * v_v
 * Arithmetic is fp32 whatever the storage dtype.  Q, K, V, rel: device, read only.
 * out (tensor dtype) and lse (fp32): device, written.  workspace: device scratch
 * of at least bpt_attn_fwd_workspace bytes (may be NULL when that is 0).
 * Limits of every attention call (the kernels address the edge arrays and one (batch,
 * head) slab of a tensor with 32-bit byte offsets), BPT_ERR_UNSUPPORTED beyond them: the
 * graph has fewer than 2^29 edges (bpt_build_graph itself accepts up to INT32_MAX);
 * N * stride_n * element size < 2 GiB; stride_n * element size < 16 MiB;
 * B * H * N <= 2^40.  All tensor pointers start on a 16-byte boundary, else
 * BPT_ERR_INVALID_ARG. */
int bpt_attn_fwd(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K,
                 const void* V, const void* rel, void* out, float* lse, void* workspace,
                 size_t workspace_bytes, void* stream);

/* bpt_attn_fwd for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and kernels as bpt_attn_fwd, but the scratch (partial results of span rows that are cut over
 * several workgroups) lives in a buffer of BPT_STATIC_SCRATCH_BYTES that is part of the library's
 * device code: nothing is allocated or freed, by this call or by anything it calls, and no
 * workspace is passed.  Every device the library is loaded on holds the buffer until the process
 * ends.  A graph and shape whose bpt_attn_fwd_workspace exceeds the buffer is refused with
 * BPT_ERR_SCRATCH (e.g. n = 65536 with 8 heads; n = 8192 with 4 x 8 heads needs 17 MB and fits).
 * g must have been built on the current device (BPT_ERR_INVALID_ARG otherwise); the buffer's address
 * is looked up in bpt_build_graph, so a call under graph capture does no look-up either.  All calls
 * on one device share the one buffer: calls that may overlap on a device (different streams, or
 * host threads without an ordering between their streams) race on it and must be serialised by the
 * caller.  The buffer keeps the previous call's contents; the forward writes every partial before it
 * reads it, so nothing needs clearing. */
#define BPT_STATIC_SCRATCH_BYTES (32u << 20)
int bpt_attn_fwd_static(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K,
                        const void* V, const void* rel, void* out, float* lse, void* stream);

/* Gradient of eq. (8) given dout = dL/dout.  With p_e = exp(s_e - lse_u),
 * dP_e = dout_u . v_v, delta_u = sum_e p_e dP_e (= dout_u . out_u), dS_e = p_e (dP_e - delta_u):
 *   dQ_u = scale * sum_e dS_e (k_v + rel[id_e])
 *   dK_v = scale * sum_{e -> v} dS_e q_u        dV_v = sum_{e -> v} p_e dout_u
 *   d_rel[id] = scale * sum over batch, head and edges with id_e = id of dS_e q_u
 * lse is the forward's result; the forward's `out` is not needed (delta is
 * recomputed in fp32 from p and dP).  dQ, dK, dV (fp32, or bf16 with
 * bpt_shape_t.grad_dtype; the tensor strides, in elements) and
 * d_rel (fp32, contiguous [num_levels][W][D]) are overwritten.  No atomics are
 * used anywhere: dK and dV are reduced over the transposed adjacency and d_rel as
 * a dense contraction over blocks of token rows, so all four gradients are
 * run-to-run identical.  workspace: device scratch of at least
 * bpt_attn_bwd_workspace bytes. */
int bpt_attn_bwd(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q, const void* K,
                 const void* V, const void* rel, const float* lse, const void* dout, void* dQ,
                 void* dK, void* dV, float* d_rel, void* workspace, size_t workspace_bytes,
                 void* stream);

/* The two stages of bpt_attn_bwd, callable on their own (same workspace, same
 * stream order): the query side walks the CSR rows and produces dQ, d_rel and,
 * in the workspace, delta; the key side walks the transposed adjacency, reads that
 * delta and produces dK and dV.  bpt_attn_bwd is exactly the first followed by the
 * second. */
int bpt_attn_bwd_query_side(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q,
                            const void* K, const void* V, const void* rel, const float* lse,
                            const void* dout, void* dQ, float* d_rel, void* workspace,
                            size_t workspace_bytes, void* stream);
int bpt_attn_bwd_key_side(const bpt_graph_t* g, const bpt_shape_t* s, const void* Q,
                          const void* K, const void* V, const void* rel, const float* lse,
                          const void* dout, void* dK, void* dV, void* workspace,
                          size_t workspace_bytes, void* stream);

/* For benchmarks and tuning (not part of the paper's method): while enabled, every
 * kernel the library launches is bracketed by two HIP events on the launch stream.
 * bpt_profile_enable(on != 0) starts a fresh record, bpt_profile_enable(0) drops it.
 * bpt_profile_report waits for the recorded events and writes one line per kernel,
 * "name launches total_ms", NUL-terminated and truncated to `capacity`, into the host
 * buffer `buf` (may be NULL); it returns the bytes the full text needs, or -1 on a
 * HIP error.  Enabling creates events (allocations) on every launch and the state is
 * global and not thread-safe: leave it off outside measurements.  Launches on a stream
 * that is being captured are not recorded. */
int bpt_profile_enable(int on);
int64_t bpt_profile_report(char* buf, size_t capacity);

/* For measurements (not part of the paper's method): a gather of known HBM traffic, against which
 * hardware counters of the attention kernels' row gathers can be scaled.  Row perm[i] (128 bytes)
 * of src is copied to row i of dst for i < rows, with the request shape of the attention kernels (8
 * consecutive lanes fetch one row, 16 bytes each).  With perm a permutation of 0..rows-1 and the
 * tensors much larger than the caches, the call reads rows * 128 bytes of rows once, rows * 4
 * bytes of indices, and writes rows * 128 bytes.  src, dst: device, 16-byte aligned, rows * 128
 * bytes each; perm: device, rows entries in [0, rows).  rows < 2^31. */
int bpt_calibrate_gather(const void* src, const int32_t* perm, void* dst, int64_t rows, void* stream);

/* Parameters of one graph layer (Sec. 3.1, Sec. 3.3): all device pointers, owned by the caller.
 * d = H * 64.  A map is stored row-major as [inputs][outputs] and applied as y = x W; head i of
 * Q, K, V is columns [64 i, 64 i + 64) of the projected features.  The paper writes the
 * projections without a bias; the position-wise FFN and the layer normalisation carry theirs. */
typedef struct {
    const void *Wq, *Wk, *Wv, *Wo; /* [d][d] bf16 */
    const void* W1;                /* [d][d_ff] bf16 */
    const void* W2;                /* [d_ff][d] bf16 */
    const float *b1, *b2;          /* [d_ff], [d] */
    const float *g1, *beta1;       /* [d] gain and bias of the normalisation after attention */
    const float *g2, *beta2;       /* [d] the same after the FFN */
    int32_t d_ff;                  /* a multiple of 8 */
    float eps;                     /* <= 0 selects 1e-5 */
} bpt_layer_params_t;

/* Sec. 3.1 (Transformer layer) and Sec. 3.3 (the update of the graph, one iteration of its
 * loop), forward, bf16:  Z = norm(X + GSA(G, X)),  Y = norm(Z + FFN(Z)),  with
 * GSA(G, X) = [head_1 .. head_H] Wo, the heads being eq. (8) on Q = X Wq, K = X Wk, V = X Wv,
 * FFN(z) = max(0, z W1 + b1) W2 + b2, norm = layer normalisation over the d features (biased
 * variance).  X and Y are [B][N][d] bf16, contiguous, N = 2n-1 rows per batch entry in node-id
 * order (span rows of the first layer are zero, Sec. 3.3); all nodes are updated from the same
 * X.  rel, scale and seq_len as for bpt_attn_fwd (with seq_len, rows of nodes that are not
 * kept hold unspecified values).  The dense maps run as library GEMMs with fp32 accumulation
 * (hipBLASLt, with b1 and the ReLU applied to the fp32 sums in the product's epilogue; rocBLAS for
 * the weight gradients and for any product hipBLASLt has no algorithm for);
 * Q, K, V, the attention output, Z and the hidden FFN activations are stored in bf16 and stay
 * in the workspace for bpt_layer_bwd.
 * workspace: device memory of at least bpt_layer_fwd_workspace bytes; nothing is allocated
 * except, once per host thread and device, the two libraries' handles and 32 MiB of scratch
 * memory for hipBLASLt, and the first call with a new shape times that library's candidate
 * kernels on the caller's buffers (it synchronises with the stream, which therefore must not be
 * capturing; later calls can be captured).  H * 64 <= 2048.  Every tensor
 * of the layer and stack calls (parameters and gradients included) starts on a 16-byte
 * boundary, else BPT_ERR_INVALID_ARG.  The layer and stack workspace queries return SIZE_MAX when
 * the attention calls would refuse the graph and shape, and the calls then BPT_ERR_UNSUPPORTED. */
size_t bpt_layer_fwd_workspace(const bpt_graph_t* g, int32_t B, int32_t H, int32_t d_ff);
int bpt_layer_fwd(const bpt_graph_t* g, int32_t B, int32_t H, float scale, const int32_t* seq_len, const void* rel,
                  const void* X, const bpt_layer_params_t* p, void* Y, void* workspace, size_t workspace_bytes,
                  void* stream);

/* Gradients of the parameters of one layer, device arrays in fp32 with the shapes of the
 * parameters they belong to; every array is overwritten, none may be NULL. */
typedef struct {
    float *dWq, *dWk, *dWv, *dWo;  /* [d][d] */
    float *dW1, *db1;              /* [d][d_ff], [d_ff] */
    float *dW2, *db2;              /* [d_ff][d], [d] */
    float *dg1, *dbeta1;           /* [d] */
    float *dg2, *dbeta2;           /* [d] */
} bpt_layer_grads_t;

/* Backward of bpt_layer_fwd (the chain rule through the steps of Sec. 3.1 / Sec. 3.3 listed
 * there, in reverse): given dY = the gradient of a scalar with respect to Y, [B][N][d] bf16,
 * writes dX [B][N][d] bf16, d_rel [levels][rel_width][64] fp32 (as bpt_attn_bwd) and the
 * gradients of all parameters.  g, B, H, scale, seq_len, rel, X and p must be those of the
 * forward call, and fwd_workspace its workspace, unchanged since that call returned: it
 * holds the activations the backward reads (Q, K, V, the attention output and lse, the two
 * pre-normalisation sums with their means and reciprocal deviations, Z, the hidden FFN
 * activations).  With seq_len, rows of dY of nodes that are not kept are taken as zero and
 * the same rows of dX are zero.  The dense maps run as library GEMMs as in the forward (bf16
 * operands: the attention's backward writes its gradients rounded to bf16; fp32
 * accumulation); sums over rows (biases, gains) are formed in a fixed order, so results are
 * run-to-run identical as far as the GEMM library's are.  workspace: at least
 * bpt_layer_bwd_workspace bytes of device memory; nothing is allocated.  d_ff <= 8192. */
size_t bpt_layer_bwd_workspace(const bpt_graph_t* g, int32_t B, int32_t H, int32_t d_ff);
int bpt_layer_bwd(const bpt_graph_t* g, int32_t B, int32_t H, float scale, const int32_t* seq_len, const void* rel,
                  const void* X, const bpt_layer_params_t* p, const void* fwd_workspace, size_t fwd_workspace_bytes,
                  const void* dY, void* dX, float* d_rel, const bpt_layer_grads_t* grads, void* workspace,
                  size_t workspace_bytes, void* stream);

/* Sec. 3.3, the update of the graph from its initial states to its output, bf16: the states before
 * the first layer are the embeddings E [B][n][d] on the token rows and zero on the span rows;
 * layer l = 0 .. num_layers-1 is bpt_layer_fwd with its own parameters p[l] and its own
 * relative-position table rel[l] (p and rel are host arrays of num_layers entries; every
 * p[l].d_ff must be the same); the output is the root's row of the last states, root [B][d],
 * and / or their token rows, tokens [B][n][d] (one of the two may be NULL).  With seq_len, the
 * root is still node 2n-2 (it is kept by every sequence with a token) and token rows past a
 * sequence's end hold unspecified values.  The workspace (bpt_stack_fwd_workspace bytes of
 * device memory) keeps every layer's input states and activations for bpt_stack_bwd; nothing
 * is allocated beyond what bpt_layer_fwd states, so after one call outside a capture the call
 * (and bpt_stack_bwd) can be captured into a HIP graph.  num_layers <= 256.
 * On the graph of a packed batch (bpt_build_batch_graph): B = 1 and seq_len = NULL
 * (BPT_ERR_INVALID_ARG otherwise), E and tokens are [T][d] with T = the tokens of all sequences in
 * row order, and root is [batch][d], one row per sequence (zero for a sequence without tokens);
 * bpt_stack_bwd takes d_root [batch][d] and d_tokens [T][d] and writes dE [T][d]. */
size_t bpt_stack_fwd_workspace(const bpt_graph_t* g, int32_t B, int32_t H, int32_t d_ff, int32_t num_layers);
int bpt_stack_fwd(const bpt_graph_t* g, int32_t B, int32_t H, int32_t num_layers, float scale, const int32_t* seq_len,
                  const void* const* rel, const void* E, const bpt_layer_params_t* p, void* root, void* tokens,
                  void* workspace, size_t workspace_bytes, void* stream);

/* Backward of bpt_stack_fwd: given the gradient of a scalar with respect to the outputs, d_root
 * [B][d] and / or d_tokens [B][n][d] in bf16 (a NULL one counts as zero; not both), runs
 * bpt_layer_bwd from the last layer to the first and writes dE [B][n][d] bf16 (the gradient
 * with respect to the embeddings), d_rel[l] and grads[l] for every layer (host arrays of
 * num_layers entries, each as for bpt_layer_bwd).  The other arguments must be those of the
 * forward call and fwd_workspace its workspace, unchanged.  workspace: at least
 * bpt_stack_bwd_workspace bytes of device memory (it does not grow with num_layers); nothing
 * is allocated. */
size_t bpt_stack_bwd_workspace(const bpt_graph_t* g, int32_t B, int32_t H, int32_t d_ff);
int bpt_stack_bwd(const bpt_graph_t* g, int32_t B, int32_t H, int32_t num_layers, float scale, const int32_t* seq_len,
                  const void* const* rel, const bpt_layer_params_t* p, const void* fwd_workspace,
                  size_t fwd_workspace_bytes, const void* d_root, const void* d_tokens, void* dE, float* const* d_rel,
                  const bpt_layer_grads_t* grads, void* workspace, size_t workspace_bytes, void* stream);

/* Sec. 3.2 with the rule for shorter sequences stated at the top of this header: the number
 * of edges of the graph over n tokens with density k that a sequence of len tokens keeps
 * (0 <= len <= n; len == n gives the graph's own edge count).  Host arithmetic only, no
 * device is touched; O(len log n).  The throughput of a batch of sequences of different
 * lengths is counted in these edges.  BPT_ERR_INVALID_ARG / BPT_ERR_UNSUPPORTED as for
 * bpt_build_graph, or if len is out of range. */
int bpt_count_edges(int32_t n, int32_t k, int32_t causal, int32_t len, int64_t* edges);

/* Static, never NULL. */
const char* bpt_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* BPT_H_ */
