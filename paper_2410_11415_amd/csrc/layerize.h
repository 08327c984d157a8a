// Host-side layerization and tensorization of a circuit DAG (paper Section 3.1 Eq. 2,
// Section 3.2, Appendix C Alg. 2 and Alg. 3).  Pure C++, no device code: the result is a set
// of plain index arrays that the evaluator uploads once.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

namespace klay {

struct Options {
    bool no_reorder = false;
    int32_t heavy_fan = 48;     // rows with more sources than this are evaluated in split passes
    int32_t min_segment = 24;   // smallest segment of a split row, in edges
    bool no_tail = false;       // never use the persistent kernels for the narrow top layers
    bool alias_chains = false;  // no unary chain nodes below the narrow top of the circuit: edges index the rows of any lower layer
    bool no_merge = false;      // keep structurally identical gates apart
    int32_t tail_rows_cap = 0;  // > 0: layers with more nodes than this are no candidates for the persistent kernels
                                // (at most kTailRowsCap; for tests of the boundary between the two parts)
    bool small_batch_edges = false;   // evaluator option (not used by the layerizer): lanes = edges kernel for B <= 32
    bool no_fusion = false;     // build no fused plans (LayerPlan::fwd2): every forward sweep writes every AND node's value
};

// Layers at the top of the circuit with at most this many nodes are candidates for the persistent
// kernels, which keep two layers of one batch column in LDS (values forward, adjoints in the reverse sweep):
// 20000 rows is what two arrays in 160 KB hold.  In those kernels a lane walks a whole row, so a candidate
// layer has no row with more sources than kTailFanCap (the reverse plan: no node with more parents).
constexpr int64_t kTailRowsCap = 20000;
constexpr int64_t kTailFanCap = 64;

// Index vectors of one layer for the persistent kernels.  Rows are taken in chunks of 64 consecutive
// rows (one per lane of a wave); a chunk has as many steps as its longest row, and step i of a chunk
// is one line of 64 words: lane j holds the i-th source of row 64 * chunk + j, or a padding word when
// that row is shorter or does not exist.  A padding word names source n_src, one past the last source
// row: the kernels keep the identity of the layer's operation in that slot, so padding needs no test.
// In the reverse plan the word that a lane holds in the last line of a chunk carries kRowFlag when the lane's row
// is an OR node with more than one child (its adjoint is stored in the one-gather form).
// The 16 waves of the workgroup take the chunks round-robin, and the lines of the chunks of one wave
// are stored back to back in the order the wave walks them, so a wave streams through one contiguous
// run of lines and can fetch them far ahead.  Every word of the last line of a chunk carries
// kLastEdge: the wave then closes the 64 rows of the chunk and moves on to its next one (16 chunks
// further).  Runs are padded with lines of padding words to a multiple of kSlabBlock lines, the unit
// the kernels fetch.
constexpr int kSlabWaves = 16;
constexpr int kSlabBlock = 8;
struct SlabPlan {
    int32_t wave_line[kSlabWaves + 1] = {};   // first line of each wave's run (wave_line[16] = all lines)
    std::vector<uint32_t> ent;                // 64 words per line: source row | flags
};

// One gather-reduce pass set over a CSR whose rows are the outputs.
//   rows [0, n_main)                 write output row i; a split row holds the single entry kSkip
//   rows [n_main, n_main + n_seg)    are segments of split rows, writing scratch row (i - n_main)
//   combine: output row comb_row[h] reduces scratch rows comb_idx[comb_ptr[h] .. comb_ptr[h+1])
// Index entries carry the source row in bits 0..28, "last edge of its row" in bit 31, in the
// reverse sweep "weighted edge" in bit 30 (the parent is an OR node with more than one child), and on
// the last entry of a row bit 29 may flag the output row itself (reverse sweep into an OR layer: the row
// is an OR node with more than one child, whose adjoint is stored in the one-gather form).
// tasks: runs of consecutive main rows with a bounded edge count, as (first row, first edge)
// pairs with a closing (n_main, main edge count) pair: the unit of work of one wave.
constexpr uint32_t kLastEdge = 0x80000000u, kWeightedEdge = 0x40000000u, kRowFlag = 0x20000000u, kSkipRow = 0xFFFFFFFFu;
// In the fused plans (LayerPlan::fwd2) that bit means something else: kGroupEnd on the last entry of a group.  The
// entries of a group are combined by the AND operation, the group results are the children of the OR row.
constexpr uint32_t kGroupEnd = kWeightedEdge;
// The OR rows that read through fused AND rows have at most this many entries (and at most half of
// Options::heavy_fan), so they are never split.  (Measured with 48 and the split threshold to match: 95% instead
// of 75% of the AND rows of the layered circuits fused, and the forward pass 3% slower: the long rows cost the
// fused launches more than the shorter AND launches save.)
constexpr int64_t kFusedRowMax = 24;
constexpr int64_t kMaxRows = (int64_t)1 << 29;      // row ids fit the 29-bit source field
constexpr int kIdxPad = 16;
struct PassPlan {
    int32_t n_main = 0;
    int32_t n_seg = 0;
    int32_t n_heavy = 0;
    int64_t edges = 0;
    std::vector<int32_t> ptr;        // [n_main + n_seg + 1]
    std::vector<uint32_t> idx;       // entries of all rows, zero padded by kIdxPad for chunked reads
    std::vector<int32_t> tasks;      // [2 * (n_tasks + 1)]
    int32_t n_tasks = 0;
    std::vector<int32_t> seg_tasks;  // same for the segment rows n_main .. n_main + n_seg - 1
    int32_t n_seg_tasks = 0;
    bool has_weighted = false;       // some entry carries kWeightedEdge
    std::vector<int32_t> seg_owner;  // [n_seg] output row each segment belongs to
    std::vector<int32_t> comb_ptr;   // [n_heavy + 1]
    std::vector<uint32_t> comb_idx;  // [n_seg + kIdxPad] scratch rows per split row, zero padded
    std::vector<int32_t> comb_row;   // [n_heavy]
};

struct LayerPlan {
    int64_t n = 0;                   // nodes in this layer
    int64_t e = 0;                   // edges from this layer down to layer - 1
    std::vector<int32_t> row_ptr;    // [n + 1] plain CSR by parent (Alg. 3: R_l implicit)
    std::vector<int32_t> child;      // [e]    S_l: position of the child in layer - 1
    std::vector<int32_t> origin;     // [n] input node id the row stands for
    std::vector<uint8_t> is_pad;     // [n] 1 for unary chain nodes
    std::vector<uint32_t> multi;     // [(n + 31) / 32] bit i: row i has more than one child (OR layers: the rows
                                     // whose edges carry a softmax weight in the reverse sweep)
    bool tail_fwd_ok = false;        // slab_fwd is built: the layer may run in the persistent forward kernel
    bool tail_bwd_ok = false;        // slab_bwd is built as well
    SlabPlan slab_fwd;               // rows = nodes of this layer, sources = positions in layer - 1
    SlabPlan slab_bwd;               // rows = nodes of layer - 1, sources = parents in this layer (| kWeightedEdge)
    PassPlan fwd;                    // outputs = nodes of this layer, sources = layer - 1
    PassPlan bwd;                    // outputs = nodes of layer - 1, sources = this layer
    // Fused AND rows (padding-free part only).  An AND node below layer alias_top that has at most one child
    // which is not a leaf and only OR parents whose rows stay short when they read its children instead of
    // it, is "fused": the forward plans below never read its value, so a forward sweep that uses them does not
    // have to write it.
    int64_t n_fused = 0;             // AND layers: so many of the rows are fused
    PassPlan fwd_kept;               // AND layers with fused rows: fwd with those rows left out (kSkipRow entries)
    PassPlan fwd2;                   // OR layers that read fused rows: every child is a group of entries (kGroupEnd),
                                     // a fused AND child being replaced by its own children
};

struct CircuitPlan {
    int32_t num_vars = 0, num_roots = 0, num_layers = 0;
    std::vector<LayerPlan> layers;       // 0 .. num_layers
    std::vector<int32_t> leaf_code;      // layer 0: +(v+1), -(v+1), INT32_MAX (TRUE), INT32_MIN (FALSE)
    std::vector<int32_t> pos_row, neg_row;   // [V] layer-0 row of each literal or -1
    std::vector<int32_t> root_pos;       // [R] position of each root in the top layer
    std::vector<int32_t> top_ptr, top_root;  // top-layer node -> root columns that read it
    int64_t num_nodes = 0, num_edges = 0, dag_nodes = 0, dag_edges = 0, num_pad_nodes = 0;
    int64_t max_layer_nodes = 0, max_fan_in = 0, max_fan_out = 0, num_split_rows = 0;
    int64_t num_merged = 0;              // input gates identified with an identical gate
    int64_t max_fwd_seg = 0, max_bwd_seg = 0;   // scratch rows needed by split passes
    int32_t tail_first = 0;              // layers tail_first..num_layers may run in the persistent forward kernel (0: none)
    int32_t tail_bwd_first = 0;          // layers tail_bwd_first..num_layers also in the reverse one (>= tail_first; 0: none)
    // Padding-free lower part (Options::alias_chains): layers 1 .. alias_top hold no chain nodes, except
    // that layer alias_top holds a stand-in for every node read from above it.  Their child entries are
    // rows of the whole activation buffer (row0[l] = first row of layer l), and layers[l].bwd for
    // l <= alias_top gathers the adjoints of layer l-1 from parents in any layer up to alias_top (adjoint
    // rows numbered like activation rows).  Layers above alias_top are as in the paper: child entries and
    // reverse-sweep sources are positions in the neighbouring layer.  0: the paper's layerization
    // throughout; num_layers: no chain nodes except the stand-ins of roots in the top layer.
    int32_t alias_top = 0;
    bool alias = false;                  // alias_top > 0
    int64_t num_fused = 0;               // AND rows whose values the fused plans do not need
    std::vector<int64_t> row0;
};

// Status codes mirror klay_status (0 ok, 1 invalid, 2 cycle, 3 no memory).
int layerize(int32_t num_vars, int64_t num_nodes, const uint8_t* node_type, const int32_t* node_lit,
             const int64_t* child_ptr, const int32_t* child_idx, int32_t num_roots,
             const int32_t* roots, const Options& opt, CircuitPlan& plan, std::string& err);

// Split a CSR (n rows, ptr[n+1], idx) into main rows, segments and combine rows.
// `flags` (optional, one per edge) is OR-ed into the entries.
// `row_bits` (optional, a bit per output row) puts kRowFlag on the last entry of the flagged rows (for a
// split row: on the last entry of its combine list).
// `skip` (optional, a byte per row): rows to leave out; like a split row such a row is one kSkipRow entry.
void make_pass_plan(int64_t n, const int32_t* ptr, const int32_t* idx, const Options& opt, PassPlan& out,
                    const uint32_t* flags = nullptr, const uint32_t* row_bits = nullptr, const uint8_t* skip = nullptr);

}  // namespace klay
