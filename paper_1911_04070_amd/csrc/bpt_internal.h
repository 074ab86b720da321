// Internal definitions shared by the library's translation units (not installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "bpt.h"

namespace bpt {

constexpr int kD = 64;            // head width the kernels are written for
constexpr int kSeg = 512;         // most edges one wavefront handles for one row
constexpr int kTileWork = 4096;   // target work (edges + per-row cost) of one workgroup tile
constexpr int kRowCost = 24;      // per-row overhead, in edge equivalents, for tile balancing
constexpr int kPartSpan8 = -2;    // seg_part of a group of 8 equal-degree span rows handled one per 8-lane group
constexpr int kSpan8MaxDeg = 64;
constexpr int kPartStride = 66;   // forward partial: 64 accumulators, running max, running sum

// A launch schedule over one adjacency (by query node, or transposed by key
// node).  Rows are cut into segments of at most kSeg edges; a wavefront
// processes one segment.  Rows with several segments write partial results that
// a merge kernel combines.  Segments are grouped into tiles of about equal work.
struct Schedule {
    int32_t num_segs = 0, num_tiles = 0, num_multi = 0, num_part = 0;
    int32_t* seg_row = nullptr;    // [num_segs]   row (node id) of the segment
    int32_t* seg_begin = nullptr;  // [num_segs]   first edge of the segment
    int32_t* seg_part = nullptr;   // [num_segs]   partial slot, -1 if the row has one segment, kPartSpan8 for a row group
    int32_t* tile_ptr = nullptr;   // [num_tiles+1] segments of a tile
    int32_t* multi_row = nullptr;  // [num_multi]  rows that have several segments
    int32_t* multi_ptr = nullptr;  // [num_multi+1] their partial slots
};

// Dense tiles over the token rows, for the matrix-core forward.  A tile is 16
// consecutive token rows; its columns are the union of the rows' key nodes in
// ascending node id, cut into chunks of 16 (an even number of chunks per tile;
// padding slots repeat a real node and are masked).
struct TokenTiles {
    int32_t num_tiles = 0;   // n / 16; 0 when the tile path is not built
    int32_t num_chunks = 0;  // chunks of all tiles together
    int32_t num_cids = 0;    // relative-position ids used by token rows (compact numbering)
    int32_t* chunk_ptr = nullptr;  // [num_tiles+1] first chunk of a tile
    int32_t* cols = nullptr;       // [chunks][16] node id of a column
    int16_t* map = nullptr;        // [chunks][16 rows][16 columns] compact id of the edge, or -1
    int32_t* cid_to_id = nullptr;  // [num_cids] compact id -> row of the relative-position table
    int32_t* id_to_cid = nullptr;  // [rows of the table] the inverse, -1 for ids no token row uses
};

// Dense tiles over the key nodes, for the matrix-core key-side backward.  A tile is up
// to 16 consecutive nodes of one level; its columns are the nodes that attend to any
// of them (tokens on either side, and for token keys their ancestor spans), in
// ascending node id, in chunks of 16 (an even number per tile).  A tile's chunk list
// is cut into tasks of at most key_task_chunks(n) chunks; tiles with several tasks are
// summed by a merge kernel in task order.  Tiles with few chunks (the fine levels: a key of level l is read
// by about (k + 1) 2^l tokens) are chained instead: one task walks several consecutive tiles of a level, so
// that the software pipeline of the kernel runs through them instead of starting up for every tile.
// Longer tasks mean fewer partial sums to write and
// merge (n = 65536: key side 0.67 -> 0.60 ms) but, when a (batch, head) has few tiles, waves
// that wait for the one with the longest task (n = 512: 0.12 -> 0.29 ms).
inline int key_task_chunks(int n) { return n >= 16384 ? 64 : 32; }
struct KeyTiles {
    int32_t num_tasks = 0, num_multi = 0, num_part = 0;
    int32_t num_chunks = 0;         // chunks of all tiles together
    int32_t nb_pad = 0;             // relative-position ids a tile can meet, padded to 16
    int32_t first_uncovered = 0;    // nodes from here on have no in-edges (levels without contextual edges)
    int32_t* chunk_ptr = nullptr;   // [tiles+1] first chunk of a tile
    int32_t* tile_node0 = nullptr;  // [tiles] first key node
    int32_t* tile_info = nullptr;   // [tiles] level | valid keys << 8
    int32_t* cols = nullptr;        // [chunks][16] query node of a column
    int16_t* map = nullptr;         // [chunks][16 keys][16 columns] tile-local relative-position id, or -1
    int32_t* task_tile = nullptr;   // [tasks]
    int32_t* task_c0 = nullptr;     // [tasks] first chunk
    int32_t* task_nch = nullptr;    // [tasks] chunks (even)
    int32_t* task_part = nullptr;   // [tasks] partial slot, or -1 if the tile has one task
    int32_t* task_ntiles = nullptr; // [tasks] consecutive tiles of one level the task walks (1 unless chained)
    int32_t* multi_tile = nullptr;  // [num_multi] tiles with several tasks
    int32_t* multi_ptr = nullptr;   // [num_multi+1] their partial slots
};

}  // namespace bpt

struct bpt_graph {
    int32_t n = 0, k = 0, causal = 0;
    int32_t num_nodes = 0, num_levels = 0, rel_width = 0, ctx_levels = 0;
    int32_t n_tokens = 0;         // token rows (they come first): n, or the tokens of all sequences of a batch graph
    int32_t batch = 0;            // sequences packed into this graph (bpt_build_batch_graph); 0: the graph of one sequence
    std::vector<int32_t> first_row, row_count;   // batch graph: [level][sequence] first node row and node count
    // batch graph, for the matrix-core kernels: the graph of one sequence of n tokens (their tile metadata), and on the
    // device the lengths [sequence] and delta[level][sequence] = first_row - first id of the level in that tree
    bpt_graph* tree = nullptr;
    bool owns_tree = false;       // built by this graph (else shared with the caller, who keeps it alive)
    int32_t *d_lengths = nullptr, *d_delta = nullptr;
    // batch graph, for the stack's readout: the row of every sequence's root (-1: the sequence is empty), and for
    // the rows from first_root on (the root level) the sequence they belong to
    int32_t *d_root_row = nullptr, *d_root_seq = nullptr;
    int32_t first_root = 0;
    int64_t num_edges = 0;
    int64_t num_token_edges = 0;  // edges of token rows: they come first in the CSR
    int device = 0;
    int num_cus = 0;
    // CSR by query node
    int32_t *row_ptr = nullptr, *col = nullptr, *rel = nullptr;
    // transposed adjacency by key node
    int32_t *t_ptr = nullptr, *t_src = nullptr, *t_eid = nullptr, *t_rel = nullptr;
    bpt::Schedule fwd, tr;
    bpt::Schedule fwd_span;   // span rows only (used with the token tiles)
    bpt::TokenTiles tiles;
    bpt::KeyTiles ktiles;
};

namespace bpt {
// bpt_attn.hip: address of the current device's copy of the library's static scratch, resolved on first use
int static_scratch(int device, void** out);
// bpt_tiles.hip: token tiles and key tiles of a graph whose CSR is on the device
int build_tile_metadata(bpt_graph* g, const int32_t* cnt_l, const int32_t* min_l, const int32_t* cnt_r,
                        const int32_t* min_r, hipStream_t st);
}  // namespace bpt

// Optional per-kernel timing: when enabled, every kernel launch of the library is
// bracketed by two HIP events on the launch stream (see bpt_profile_enable).
namespace bpt {
namespace prof {
bool enabled();
void begin(const char* name, hipStream_t st);
void end(hipStream_t st);
}  // namespace prof
}  // namespace bpt

#define BPT_LAUNCH(name, kernel, grid, block, lds, st, ...)          \
    do {                                                             \
        const bool prof__ = bpt::prof::enabled();                    \
        if (prof__) bpt::prof::begin(name, st);                      \
        hipLaunchKernelGGL(kernel, grid, block, lds, st, __VA_ARGS__); \
        if (prof__) bpt::prof::end(st);                              \
    } while (0)

#define BPT_HIP(expr)                                  \
    do {                                               \
        hipError_t e__ = (expr);                       \
        if (e__ != hipSuccess) {                       \
            (void)hipGetLastError();                   \
            return e__ == hipErrorOutOfMemory ? BPT_ERR_ALLOC : BPT_ERR_LAUNCH; \
        }                                              \
    } while (0)
