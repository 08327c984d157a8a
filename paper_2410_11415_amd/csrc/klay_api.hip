// C ABI of the layered circuit evaluator (see include/klay.h): handle management, workspace,
// and the launch sequences of the forward sweep (paper Section 4, Alg. 1 / Appendix C, Alg. 4)
// and of the reverse sweep that yields the derivative with respect to the leaf weights.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/klay.h"
#include "klay_kernels.hip.h"
#include "klay_kernels_f64.hip.h"
#include "layerize.h"

// Workspace of klay_forward_static, the entry point that allocates nothing: a fixed array in device
// memory.  Every GPU the library runs on holds its own copy at its own address until the process
// ends.  In host code the name below is only a handle for hipGetSymbolAddress; the kernels get the
// address that call returned (kept per device in g_static_ws).
constexpr size_t kStaticWorkspaceBytes = KLAY_STATIC_WORKSPACE_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticWorkspaceBytes];

// Layers with split rows and at most this many index entries run main rows and segments in one generic
// launch (measured at B = 64 on the two power-law workloads, ms per step: this threshold 0.69 / 0.76, ten times
// larger 0.66 / 0.80, every layer 0.68 / 0.92; with the layerization of unary chains throughout 60000 and
// 150000 both gave 0.73 against 0.81 without the rule).
constexpr int64_t kSmallPassEntries = 100000;
constexpr size_t kTailLdsMax = 160 * 1024;     // LDS of a gfx950 compute unit: the most a workgroup of the persistent kernels gets

namespace {

thread_local std::string g_err;

constexpr int kMaxDevices = 64;
std::mutex g_static_mu;
float* g_static_ws[kMaxDevices] = {};      // device address of `scratch` on each device

// Looks the array's address up once per device; `device` must be the current device.
hipError_t static_workspace(int device, float** out) {
    if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_static_mu);
    if (!g_static_ws[device]) {
        void* ptr = nullptr;
        hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_static_ws[device] = static_cast<float*>(ptr);
    }
    *out = g_static_ws[device];
    return hipSuccess;
}

klay_status fail(klay_status s, const std::string& msg) {
    g_err = msg;
    return s;
}

#define KLAY_HIP(call)                                                                         \
    do {                                                                                       \
        hipError_t e__ = (call);                                                               \
        if (e__ != hipSuccess)                                                                 \
            return fail(KLAY_EHIP, std::string(#call) + ": " + hipGetErrorString(e__));        \
    } while (0)

constexpr size_t kAlignInts = 64;   // 256-byte alignment of every uploaded array

struct DevPass {
    const int32_t *ptr = nullptr, *seg_owner = nullptr, *comb_ptr = nullptr, *comb_row = nullptr, *tasks = nullptr,
                  *seg_tasks = nullptr;
    const uint32_t *idx = nullptr, *comb_idx = nullptr;
    int32_t n_main = 0, n_seg = 0, n_heavy = 0, n_tasks = 0, n_seg_tasks = 0;
    bool has_weighted = false;
    int64_t edges = 0;
    int64_t main_entries = 0, seg_entries = 0;   // index entries of light main rows / of segments
    int64_t n_src = 0;                           // distinct source rows the pass reads
};

// Log-semiring reverse sweep: adjoints of OR layers travel in the one-gather form (off: the two-gather step).
constexpr bool kOneGather = true;

struct DevLayer {
    int64_t n = 0, e = 0;
    int64_t row0 = 0;        // first row of this layer in the activation buffer
    DevPass fwd, bwd;
    // the fused plans (LayerPlan::fwd_kept, fwd2), where the layerizer built them
    DevPass fwd_kept, fwd2;
    bool has_fwd2 = false;
    int64_t n_fused = 0;     // AND layers: so many rows are fused (their values are not written when the fused plans run)
    bool has_fwd_kept = false;
    const uint32_t* multi = nullptr;   // OR layers: bit r = node r has more than one child
    bool has_multi = false;
};

struct Geometry {            // how a batch of B columns is mapped onto lanes
    int vec = 1, w = 64, ld = 0, tiles = 1;
};

Geometry geometry(int B) {
    Geometry g;
    if (B > 128) { g.vec = 4; g.w = 64; }
    else if (B > 64) { g.vec = 2; g.w = 64; }
    else if (B > 32) { g.vec = 1; g.w = 64; }
    else {
        g.vec = 1;
        g.w = 1;
        while (g.w < B) g.w *= 2;
    }
    g.ld = B > 32 ? (B + 3) / 4 * 4 : B;        // rows of wave-wide batches are float4-aligned
    const int tile = g.w * g.vec;
    g.tiles = (B + tile - 1) / tile;
    return g;
}

size_t align_floats(size_t n) { return (n + 63) / 64 * 64; }

struct Workspace {
    size_t act = 0, wT = 0, seg_rows = 0, g0 = 0, g1 = 0, g2 = 0, tb = 0, stage = 0, flags = 0, total = 0;   // offsets in floats
};

struct EventRec {
    int cls;
    hipEvent_t start, stop;
    double bytes, min_bytes;
};

}  // namespace

struct klay_circuit {
    klay::CircuitPlan plan;
    int device = -1;
    bool small_batch_edges = false;      // klay_options.small_batch_edges
    bool one_gather = false;             // the log reverse sweep may use the one-gather form (see upload)
    std::vector<DevLayer> dl;
    int32_t* d_index = nullptr;          // one allocation holding every index array
    size_t index_bytes = 0;
    const int32_t *d_pos_row = nullptr, *d_neg_row = nullptr, *d_root_pos = nullptr, *d_top_ptr = nullptr,
                  *d_top_root = nullptr;
    int32_t true_row = -1, false_row = -1;
    const klay::SlabLayer* d_tail = nullptr;   // descriptors of layers plan.tail_first .. L
    const int32_t* d_leaf_code = nullptr;      // layer 0: literal / constant code of every row
    size_t tail_lds_bytes = 0;                 // LDS a workgroup of the persistent kernels may use (0: kernels unusable)
    int64_t tail_rows = 0;                     // T: rows of all tail candidate layers (one column of the tail buffer)
    int32_t last_tail_first = 0;               // first layer the last forward ran in the persistent kernel (0: none)
    // real-semiring reverse sweep (built at its first use): per AND layer the plain by-parent index
    // vectors (for prod_parent_kernel); for the layers below alias_top also the by-child pass over the
    // parents in all higher layers up to alias_top, whose entries tell AND parents from plain adjoint rows
    struct RealLayer { const int32_t* ptr = nullptr; const int32_t* child = nullptr; DevPass by_child; };
    std::vector<RealLayer> real_layers;
    int32_t* d_real_index = nullptr;
    void* ws_own = nullptr;
    size_t ws_own_bytes = 0;
    void* ws_user = nullptr;
    size_t ws_user_bytes = 0;
    // state of the most recent forward
    bool no_fusion = false;                    // klay_options.no_fusion
    bool have_fwd = false;
    bool last_fused = false;                   // the forward pass ran the fused plans: the values of fused AND rows do not exist
    bool bwd_followed = false;                 // klay_backward was called after the most recent forward pass
    int32_t last_B = 0;
    int last_semiring = 0;
    bool last_neg_explicit = false;            // the negated literals had weights of their own
    bool last_ws_has_bwd = false;
    // double-precision evaluation (its own library-owned workspace)
    void* ws64 = nullptr;
    size_t ws64_bytes = 0;
    bool have_fwd64 = false;
    int32_t last64_B = 0;
    int last64_semiring = 0;
    bool last64_neg_explicit = false;
    // profiling
    bool profiling = false;
    std::vector<EventRec> ev_fwd, ev_bwd;
    std::vector<hipEvent_t> ev_pool;
};

namespace {

// widest layer above the padding-free part (1 if there is none): the size of the two adjoint buffers
// that the layer-by-layer part of the reverse sweep alternates between
int64_t top_layer_rows(const klay::CircuitPlan& p) {
    int64_t n = 1;
    for (int l = p.alias_top + 1; l <= p.num_layers; ++l) n = std::max(n, p.layers[(size_t)l].n);
    return n;
}

int64_t tail_stage_rows(const klay_circuit* c, int B);

Workspace workspace_layout(const klay_circuit* c, int B, bool need_bwd) {
    const Geometry g = geometry(B);
    const klay::CircuitPlan& p = c->plan;
    Workspace w;
    size_t off = 0;
    w.act = off; off += align_floats((size_t)p.num_nodes * g.ld);
    w.wT = off; off += align_floats((size_t)std::max(1, p.num_vars) * g.ld);
    const int64_t seg = std::max(p.max_fwd_seg, need_bwd ? p.max_bwd_seg : 0);
    w.seg_rows = off; off += align_floats((size_t)std::max<int64_t>(seg, 1) * g.ld);
    // values of the tail layers, one run of tail_rows floats per batch column
    w.tb = off; off += align_floats((size_t)c->tail_rows * (size_t)B);
    // the layer below the persistent forward kernel's first one, column-major, for that kernel to read
    w.stage = off; off += align_floats((size_t)tail_stage_rows(c, B) * (size_t)B);
    if (need_bwd) {
        // adjoints: one row per node of the layers 0 .. alias_top, and two buffers of the widest layer above
        // them that the layer-by-layer part of the sweep alternates between
        w.g0 = off; off += align_floats((size_t)p.row0[(size_t)p.alias_top + 1] * g.ld);
        w.g1 = off; off += align_floats((size_t)top_layer_rows(p) * g.ld);
        w.g2 = off; off += align_floats((size_t)top_layer_rows(p) * g.ld);
        // one word per layer: the real-semiring sweep's "a node value of this product layer is zero" flags
        w.flags = off; off += align_floats((size_t)p.num_layers + 1);
    }
    w.total = off;
    return w;
}

template <int OP, int VEC, int W>
void launch_one(const klay::PassArgs& a, dim3 grid, hipStream_t s) {
    hipLaunchKernelGGL((klay::pass_kernel<OP, VEC, W>), grid, dim3(256), 0, s, a);
}

template <int OP>
void launch_op(const klay::PassArgs& a, const Geometry& g, dim3 grid, hipStream_t s) {
    if (g.w == 64) {
        if (g.vec == 4) launch_one<OP, 4, 64>(a, grid, s);
        else if (g.vec == 2) launch_one<OP, 2, 64>(a, grid, s);
        else launch_one<OP, 1, 64>(a, grid, s);
        return;
    }
    switch (g.w) {                      // B <= 32: one column per lane, a lane group per row
    case 32: launch_one<OP, 1, 32>(a, grid, s); break;
    case 16: launch_one<OP, 1, 16>(a, grid, s); break;
    case 8: launch_one<OP, 1, 8>(a, grid, s); break;
    case 4: launch_one<OP, 1, 4>(a, grid, s); break;
    case 2: launch_one<OP, 1, 2>(a, grid, s); break;
    default: launch_one<OP, 1, 1>(a, grid, s); break;
    }
}

// Launch one gather-reduce pass over `n_total` rows.
void launch_pass(int op, klay::PassArgs a, const Geometry& g, hipStream_t s) {
    const int64_t rows = (int64_t)a.n_total - a.row_begin;
    if (rows <= 0) return;
    const int rpw = 64 / g.w;
    const int64_t groups = (rows + rpw - 1) / rpw;                    // row groups = wave work items
    // enough waves to fill 256 CUs several times over before a wave takes more than one group
    int iters = (int)std::min<int64_t>(8, std::max<int64_t>(1, groups / 32768));
    a.iters = iters;
    int64_t blocks = (groups + (int64_t)4 * iters - 1) / ((int64_t)4 * iters);
    blocks = (blocks + 7) / 8 * 8;
    dim3 grid((unsigned)blocks, (unsigned)g.tiles);
    switch (op) {
    case klay::OP_SUM: launch_op<klay::OP_SUM>(a, g, grid, s); break;
    case klay::OP_PROD: launch_op<klay::OP_PROD>(a, g, grid, s); break;
    case klay::OP_LSE: launch_op<klay::OP_LSE>(a, g, grid, s); break;
    case klay::OP_MAX: launch_op<klay::OP_MAX>(a, g, grid, s); break;
    case klay::OP_PROD_BWD: launch_op<klay::OP_PROD_BWD>(a, g, grid, s); break;
    case klay::OP_SUM_H: launch_op<klay::OP_SUM_H>(a, g, grid, s); break;
    case klay::OP_SOFTMAX_H: launch_op<klay::OP_SOFTMAX_H>(a, g, grid, s); break;
    case klay::OP_SUM_P: launch_op<klay::OP_SUM_P>(a, g, grid, s); break;
    case klay::OP_PROD_BWD_P: launch_op<klay::OP_PROD_BWD_P>(a, g, grid, s); break;
    default: launch_op<klay::OP_SOFTMAX_BWD>(a, g, grid, s); break;
    }
}

// Small batches (B <= 32): the lanes = edges kernel over the main rows and the segments of a pass.
template <int OP, int LPR>
void launch_edge_one(const DevPass& dp, const float* src, const float* src2, const float* own, float* dst,
                     float* dst_seg, int B, int ld, hipStream_t s, int* zf) {
    constexpr int EPW = 64 / LPR, CH = EPW >= 16 ? 4 : 8;
    const int64_t entries = dp.main_entries + dp.n_heavy;
    // a wave takes about two rounds of its gathers: CH steps of EPW entries each
    const double per_task = dp.n_tasks > 0 ? (double)entries / dp.n_tasks : 16.0;
    int span = (int)(2.0 * CH * EPW / std::max(1.0, per_task) + 0.5);
    span = std::max(1, span);
    const int64_t waves = ((int64_t)dp.n_tasks + span - 1) / span + ((int64_t)dp.n_seg_tasks + span - 1) / span;
    if (waves <= 0) return;
    dim3 grid((unsigned)((waves + 3) / 4));
    hipLaunchKernelGGL((klay::edge_kernel<OP, LPR>), grid, dim3(256), 0, s, reinterpret_cast<const int2*>(dp.tasks),
                       dp.n_tasks, span, dp.idx, src, src2, own, dst, B, ld, reinterpret_cast<const int2*>(dp.seg_tasks),
                       dp.n_seg_tasks, dp.seg_owner, dp.n_main, dst_seg, zf);
}

template <int OP>
void launch_edge_op(const DevPass& dp, const Geometry& g, const float* src, const float* src2, const float* own,
                    float* dst, float* dst_seg, int B, hipStream_t s, int* zf) {
    switch (g.w) {
    case 32: launch_edge_one<OP, 32>(dp, src, src2, own, dst, dst_seg, B, g.ld, s, zf); break;
    case 16: launch_edge_one<OP, 16>(dp, src, src2, own, dst, dst_seg, B, g.ld, s, zf); break;
    case 8: launch_edge_one<OP, 8>(dp, src, src2, own, dst, dst_seg, B, g.ld, s, zf); break;
    case 4: launch_edge_one<OP, 4>(dp, src, src2, own, dst, dst_seg, B, g.ld, s, zf); break;
    case 2: launch_edge_one<OP, 2>(dp, src, src2, own, dst, dst_seg, B, g.ld, s, zf); break;
    default: launch_edge_one<OP, 1>(dp, src, src2, own, dst, dst_seg, B, g.ld, s, zf); break;
    }
}

void launch_edge(int op, const DevPass& dp, const Geometry& g, const float* src, const float* src2, const float* own,
                 float* dst, float* dst_seg, int B, hipStream_t s, int* zf) {
    switch (op) {
    case klay::OP_SUM: launch_edge_op<klay::OP_SUM>(dp, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_PROD: launch_edge_op<klay::OP_PROD>(dp, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_LSE: launch_edge_op<klay::OP_LSE>(dp, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_MAX: launch_edge_op<klay::OP_MAX>(dp, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_PROD_BWD: launch_edge_op<klay::OP_PROD_BWD>(dp, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_SUM_H: launch_edge_op<klay::OP_SUM_H>(dp, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_SOFTMAX_H: launch_edge_op<klay::OP_SOFTMAX_H>(dp, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_SUM_P: launch_edge_op<klay::OP_SUM_P>(dp, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_PROD_BWD_P: launch_edge_op<klay::OP_PROD_BWD_P>(dp, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    default: launch_edge_op<klay::OP_SOFTMAX_BWD>(dp, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    }
}

// Streaming kernel over the main rows of a pass and / or the segments of its split rows (batch
// tiles of one wave: B > 32).  dst_seg is the base of the partial rows shifted by -n_main rows: segment rows are
// numbered after the main rows.
template <int OP>
void launch_stream_op(const DevPass& dp, bool main_rows, bool segments, const Geometry& g, const float* src,
                      const float* src2, const float* own, float* dst, float* dst_seg, int B, hipStream_t s, int* zf) {
    const int2* tasks = reinterpret_cast<const int2*>(dp.tasks);
    const int2* seg_tasks = reinterpret_cast<const int2*>(dp.seg_tasks);
    int n_tasks = main_rows ? dp.n_tasks : 0;
    int n_seg_tasks = segments ? dp.n_seg_tasks : 0;
    int64_t blocks = ((int64_t)n_tasks + n_seg_tasks + 3) / 4;
    blocks = (blocks + 7) / 8 * 8;
    // outputs larger than the L2s together (8 x 4 MB) are written with streaming stores
    const int nt = (int64_t)dp.n_main * g.ld * 4 > (int64_t)64 << 20 ? 1 : 0;
    dim3 grid((unsigned)blocks, (unsigned)g.tiles);
    if (g.vec == 4)
        hipLaunchKernelGGL((klay::stream_kernel<OP, 4>), grid, dim3(256), 0, s, tasks, n_tasks, dp.idx, src, src2, own, dst, B, g.ld, nt, seg_tasks, n_seg_tasks, dst_seg, dp.seg_owner, dp.n_main, zf);
    else if (g.vec == 2)
        hipLaunchKernelGGL((klay::stream_kernel<OP, 2>), grid, dim3(256), 0, s, tasks, n_tasks, dp.idx, src, src2, own, dst, B, g.ld, nt, seg_tasks, n_seg_tasks, dst_seg, dp.seg_owner, dp.n_main, zf);
    else
        hipLaunchKernelGGL((klay::stream_kernel<OP, 1>), grid, dim3(256), 0, s, tasks, n_tasks, dp.idx, src, src2, own, dst, B, g.ld, nt, seg_tasks, n_seg_tasks, dst_seg, dp.seg_owner, dp.n_main, zf);
}

void launch_stream(int op, const DevPass& dp, bool main_rows, bool segments, const Geometry& g, const float* src,
                   const float* src2, const float* own, float* dst, float* dst_seg, int B, hipStream_t s, int* zf) {
    if ((main_rows ? dp.n_tasks : 0) + (segments ? dp.n_seg_tasks : 0) <= 0) return;
    switch (op) {
    case klay::OP_SUM: launch_stream_op<klay::OP_SUM>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_PROD: launch_stream_op<klay::OP_PROD>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_LSE: launch_stream_op<klay::OP_LSE>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_MAX: launch_stream_op<klay::OP_MAX>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_PROD_BWD: launch_stream_op<klay::OP_PROD_BWD>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_SUM_H: launch_stream_op<klay::OP_SUM_H>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_SOFTMAX_H: launch_stream_op<klay::OP_SOFTMAX_H>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_SUM_P: launch_stream_op<klay::OP_SUM_P>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_PROD_BWD_P: launch_stream_op<klay::OP_PROD_BWD_P>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_LSE2: launch_stream_op<klay::OP_LSE2>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_MAX2: launch_stream_op<klay::OP_MAX2>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    case klay::OP_SUMPROD2: launch_stream_op<klay::OP_SUMPROD2>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    default: launch_stream_op<klay::OP_SOFTMAX_BWD>(dp, main_rows, segments, g, src, src2, own, dst, dst_seg, B, s, zf); break;
    }
}

struct Profiler {
    klay_circuit* c;
    std::vector<EventRec>* recs;
    hipStream_t s;
    size_t next = 0;
    bool on;
    Profiler(klay_circuit* c_, std::vector<EventRec>* r, hipStream_t s_, bool enable = true)
        : c(c_), recs(r), s(s_), on(enable && c_->profiling) {
        if (on) recs->clear();
    }
    hipEvent_t get() {
        // events of the previous forward stay referenced by ev_fwd while backward records its own
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        c->ev_pool.push_back(e);
        return e;
    }
    // bytes: no-reuse model; min_bytes: compulsory bytes (every distinct row once); < 0: same as bytes
    void begin(int cls, double bytes, double min_bytes = -1.0) {
        if (!on) return;
        EventRec r{cls, get(), get(), bytes, min_bytes < 0 ? bytes : min_bytes};
        if (r.start) (void)hipEventRecord(r.start, s);
        recs->push_back(r);
    }
    void end() {
        if (!on || recs->empty()) return;
        if (recs->back().stop) (void)hipEventRecord(recs->back().stop, s);
    }
};

void release_events(klay_circuit* c) {
    for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
    c->ev_pool.clear();
    c->ev_fwd.clear();
    c->ev_bwd.clear();
}

klay_status get_workspace(klay_circuit* c, int B, bool need_bwd, float** base, Workspace* lay) {
    *lay = workspace_layout(c, B, need_bwd);
    const size_t bytes = lay->total * sizeof(float);
    if (c->ws_user) {
        if (bytes > c->ws_user_bytes)
            return fail(KLAY_ENOMEM, "caller workspace too small: need " + std::to_string(bytes) + " bytes");
        *base = static_cast<float*>(c->ws_user);
        return KLAY_OK;
    }
    if (bytes > c->ws_own_bytes) {
        if (c->ws_own) { KLAY_HIP(hipFree(c->ws_own)); c->ws_own = nullptr; c->ws_own_bytes = 0; }
        if (hipMalloc(&c->ws_own, bytes) != hipSuccess) {
            (void)hipGetLastError();
            return fail(KLAY_ENOMEM, "hipMalloc of " + std::to_string(bytes) + " workspace bytes failed");
        }
        c->ws_own_bytes = bytes;
    }
    *base = static_cast<float*>(c->ws_own);
    return KLAY_OK;
}

// Packs host arrays into one buffer with 256-byte aligned starts; returns offsets in ints.
struct Packer {
    std::vector<int32_t> buf;
    size_t add(const std::vector<int32_t>& v) { return add(v.data(), v.size()); }
    size_t add(const std::vector<uint32_t>& v) { return add(reinterpret_cast<const int32_t*>(v.data()), v.size()); }
    size_t add(const int32_t* p, size_t n) {
        size_t off = (buf.size() + kAlignInts - 1) / kAlignInts * kAlignInts;
        buf.resize(off + std::max<size_t>(n, 1), 0);
        if (n) std::memcpy(buf.data() + off, p, n * sizeof(int32_t));
        return off;
    }
};

struct PassOffsets { size_t ptr, idx, seg_owner, comb_ptr, comb_idx, comb_row, tasks, seg_tasks; };

PassOffsets pack_pass(Packer& pk, const klay::PassPlan& p) {
    PassOffsets o;
    o.ptr = pk.add(p.ptr);
    o.idx = pk.add(p.idx);
    o.seg_owner = pk.add(p.seg_owner);
    o.comb_ptr = pk.add(p.comb_ptr);
    o.comb_idx = pk.add(p.comb_idx);
    o.comb_row = pk.add(p.comb_row);
    o.tasks = pk.add(p.tasks);
    o.seg_tasks = pk.add(p.seg_tasks);
    return o;
}

void bind_pass(DevPass& d, const klay::PassPlan& p, const PassOffsets& o, const int32_t* base) {
    d.ptr = base + o.ptr;
    d.idx = reinterpret_cast<const uint32_t*>(base + o.idx);
    d.seg_owner = base + o.seg_owner;
    d.comb_ptr = base + o.comb_ptr;
    d.comb_idx = reinterpret_cast<const uint32_t*>(base + o.comb_idx);
    d.comb_row = base + o.comb_row;
    d.tasks = base + o.tasks;
    d.n_tasks = p.n_tasks;
    d.seg_tasks = base + o.seg_tasks;
    d.n_seg_tasks = p.n_seg_tasks;
    d.has_weighted = p.has_weighted;
    d.main_entries = (int64_t)p.ptr[(size_t)p.n_main] - p.n_heavy;
    d.seg_entries = (int64_t)p.ptr[(size_t)p.n_main + (size_t)p.n_seg] - p.ptr[(size_t)p.n_main];
    d.n_main = p.n_main;
    d.n_seg = p.n_seg;
    d.n_heavy = p.n_heavy;
    d.edges = p.edges;
    // distinct source rows (for the compulsory-byte count of the profile)
    uint32_t max_id = 0;
    const size_t n_entries = (size_t)p.ptr[(size_t)p.n_main + (size_t)p.n_seg];
    for (size_t j = 0; j < n_entries; ++j)
        if (p.idx[j] != klay::kSkipRow) max_id = std::max(max_id, p.idx[j] & klay::kIdMask);
    std::vector<uint8_t> seen((size_t)max_id + 1, 0);
    for (size_t j = 0; j < n_entries; ++j)
        if (p.idx[j] != klay::kSkipRow && !seen[p.idx[j] & klay::kIdMask]) { seen[p.idx[j] & klay::kIdMask] = 1; ++d.n_src; }
}

klay_status upload(klay_circuit* c) {
    const klay::CircuitPlan& p = c->plan;
    Packer pk;
    const int L = p.num_layers;
    // tail candidates first (their descriptors hold 32-bit offsets, and these arrays are small):
    // plain index vectors by parent and by child, then the descriptor array
    size_t o_tail = 0;
    if (p.tail_first > 0) {
        std::vector<klay::SlabLayer> descs;
        int64_t row0 = 0, tb_off = 0;
        for (int l = 0; l < p.tail_first; ++l) row0 += p.layers[(size_t)l].n;
        for (int l = p.tail_first; l <= L; ++l) {
            const klay::LayerPlan& lay = p.layers[(size_t)l];
            klay::SlabLayer t{};
            t.n = (int32_t)lay.n;
            t.n_below = (int32_t)p.layers[(size_t)l - 1].n;
            t.row0 = row0;
            t.row0_below = row0 - t.n_below;
            t.tb_off = (int32_t)tb_off;
            tb_off += lay.n;
            row0 += lay.n;
            descs.push_back(t);
        }
        // One stream of lines per wave and direction: the wave's runs of all candidate layers back to
        // back, in the order the sweep visits them, closed by a block of padding lines (the kernels fetch
        // one block ahead of the one they work on).
        auto add_streams = [&](bool backward) {
            const int lo = backward ? p.tail_bwd_first : p.tail_first;
            if (lo <= 0) return;
            std::vector<uint32_t> stream;
            std::vector<int64_t> start((size_t)(L + 1) * klay::kSlabWaves, 0);
            for (int w = 0; w < klay::kSlabWaves; ++w) {
                for (int step = 0; step <= L - lo; ++step) {
                    const int l = backward ? L - step : lo + step;
                    const klay::SlabPlan& sp = backward ? p.layers[(size_t)l].slab_bwd : p.layers[(size_t)l].slab_fwd;
                    start[(size_t)l * klay::kSlabWaves + w] = (int64_t)stream.size();
                    stream.insert(stream.end(), sp.ent.begin() + (size_t)sp.wave_line[w] * 64,
                                  sp.ent.begin() + (size_t)sp.wave_line[w + 1] * 64);
                }
                stream.insert(stream.end(), (size_t)klay::kSlabBlock * 64, 0u);
            }
            const size_t base_off = pk.add(stream);
            for (int l = lo; l <= L; ++l) {
                klay::SlabLayer& t = descs[(size_t)(l - p.tail_first)];
                const klay::SlabPlan& sp = backward ? p.layers[(size_t)l].slab_bwd : p.layers[(size_t)l].slab_fwd;
                for (int w = 0; w < klay::kSlabWaves; ++w) {
                    const int32_t at = (int32_t)(base_off + (size_t)start[(size_t)l * klay::kSlabWaves + w]);
                    const int32_t cnt = sp.wave_line[w + 1] - sp.wave_line[w];
                    if (backward) { t.bwd_start[w] = at; t.bwd_count[w] = cnt; }
                    else { t.fwd_start[w] = at; t.fwd_count[w] = cnt; }
                }
            }
        };
        add_streams(false);
        add_streams(true);
        static_assert(sizeof(klay::SlabLayer) % sizeof(int32_t) == 0, "descriptor must pack into ints");
        o_tail = pk.add(reinterpret_cast<const int32_t*>(descs.data()), descs.size() * sizeof(klay::SlabLayer) / sizeof(int32_t));
    }
    const size_t o_leaf_code = pk.add(p.leaf_code);
    std::vector<PassOffsets> fo((size_t)L + 1), bo((size_t)L + 1), fko((size_t)L + 1), f2o((size_t)L + 1);
    for (int l = 1; l <= L; ++l) {
        fo[(size_t)l] = pack_pass(pk, p.layers[(size_t)l].fwd);
        bo[(size_t)l] = pack_pass(pk, p.layers[(size_t)l].bwd);
        if (!p.layers[(size_t)l].fwd_kept.ptr.empty()) fko[(size_t)l] = pack_pass(pk, p.layers[(size_t)l].fwd_kept);
        if (!p.layers[(size_t)l].fwd2.ptr.empty()) f2o[(size_t)l] = pack_pass(pk, p.layers[(size_t)l].fwd2);
    }
    std::vector<size_t> mo((size_t)L + 1, 0);
    for (int l = 2; l <= L; l += 2) mo[(size_t)l] = pk.add(p.layers[(size_t)l].multi);
    const size_t o_pos = pk.add(p.pos_row), o_neg = pk.add(p.neg_row), o_root = pk.add(p.root_pos);
    const size_t o_tptr = pk.add(p.top_ptr), o_troot = pk.add(p.top_root);

    KLAY_HIP(hipSetDevice(c->device));
    {
        float* static_ws = nullptr;      // klay_forward_static's workspace on this device
        KLAY_HIP(static_workspace(c->device, &static_ws));
    }
    c->index_bytes = pk.buf.size() * sizeof(int32_t);
    if (hipMalloc(reinterpret_cast<void**>(&c->d_index), c->index_bytes) != hipSuccess) {
        (void)hipGetLastError();
        return fail(KLAY_ENOMEM, "hipMalloc of " + std::to_string(c->index_bytes) + " index bytes failed");
    }
    KLAY_HIP(hipMemcpy(c->d_index, pk.buf.data(), c->index_bytes, hipMemcpyHostToDevice));
    const int32_t* base = c->d_index;
    c->dl.resize((size_t)L + 1);
    int64_t row0 = 0;
    for (int l = 0; l <= L; ++l) {
        DevLayer& d = c->dl[(size_t)l];
        d.n = p.layers[(size_t)l].n;
        d.e = p.layers[(size_t)l].e;
        d.row0 = row0;
        row0 += d.n;
        if (l >= 1) {
            bind_pass(d.fwd, p.layers[(size_t)l].fwd, fo[(size_t)l], base);
            bind_pass(d.bwd, p.layers[(size_t)l].bwd, bo[(size_t)l], base);
            const klay::LayerPlan& lp = p.layers[(size_t)l];
            d.n_fused = lp.n_fused;
            if (!lp.fwd_kept.ptr.empty()) { bind_pass(d.fwd_kept, lp.fwd_kept, fko[(size_t)l], base); d.has_fwd_kept = true; }
            if (!lp.fwd2.ptr.empty()) { bind_pass(d.fwd2, lp.fwd2, f2o[(size_t)l], base); d.has_fwd2 = true; }
            if ((l & 1) == 0) {
                d.multi = reinterpret_cast<const uint32_t*>(base + mo[(size_t)l]);
                for (uint32_t w : p.layers[(size_t)l].multi) d.has_multi = d.has_multi || w != 0;
            }
        }
    }
    // The one-gather form needs every layer below alias_top to either store encoded rows or read weighted
    // edges, not both: OR rows have AND parents only, so this holds for every circuit the layerizer accepts.
    c->one_gather = true;
    for (int l = 2; l < p.alias_top; l += 2)
        if (c->dl[(size_t)l].has_multi && c->dl[(size_t)l + 1].bwd.has_weighted) c->one_gather = false;
    c->d_pos_row = base + o_pos;
    c->d_neg_row = base + o_neg;
    c->d_root_pos = base + o_root;
    c->d_top_ptr = base + o_tptr;
    c->d_top_root = base + o_troot;
    if (p.tail_first > 0) c->d_tail = reinterpret_cast<const klay::SlabLayer*>(base + o_tail);
    c->d_leaf_code = base + o_leaf_code;
    return KLAY_OK;
}

// Algorithmic bytes (no-reuse model) of a gather-reduce over `rows` output rows with `entries` index
// entries: every entry gathers one row (two in the two-gather softmax adjoint), every output row is written
// once (and, in the reverse-sweep ops other than the plain sum, reads its own value row), plus the index
// entries themselves.
double pass_bytes(int op, double entries, double rows, int B) {
    const double per_entry = op == klay::OP_SOFTMAX_BWD ? 2.0 : 1.0;
    const double per_row = (op == klay::OP_SUM || op == klay::OP_PROD || op == klay::OP_LSE || op == klay::OP_MAX ||
                            op == klay::OP_LSE2 || op == klay::OP_MAX2 || op == klay::OP_SUMPROD2) ? 1.0 : 2.0;
    return 4.0 * B * (per_entry * entries + per_row * rows) + 4.0 * (entries + rows);
}

// Compulsory bytes of the same pass: every distinct source row and every output row moves once.
double pass_min_bytes(int op, double entries, double rows, double n_src, int B) {
    const double f = op == klay::OP_SOFTMAX_BWD ? 2.0 : 1.0;
    return 4.0 * B * f * (n_src + rows) + 4.0 * (entries + rows);
}

// Combine pass of the split rows: a workgroup per split row for batches wider than 32 columns
// (combine_kernel), the generic kernel otherwise.
template <int OP>
void launch_combine_op(const klay::PassArgs& a, const Geometry& g, hipStream_t s) {
    constexpr int NW = 8;
    dim3 grid((unsigned)a.n_main, (unsigned)g.tiles);
    if (g.vec == 4) hipLaunchKernelGGL((klay::combine_kernel<OP, 4, NW>), grid, dim3(NW * 64), 0, s, a);
    else if (g.vec == 2) hipLaunchKernelGGL((klay::combine_kernel<OP, 2, NW>), grid, dim3(NW * 64), 0, s, a);
    else hipLaunchKernelGGL((klay::combine_kernel<OP, 1, NW>), grid, dim3(NW * 64), 0, s, a);
}

void launch_combine(int op, const klay::PassArgs& a, const Geometry& g, hipStream_t s) {
    if (a.n_main <= 0) return;
    if (g.w != 64) { launch_pass(op, a, g, s); return; }
    switch (op) {
    case klay::OP_SUM: launch_combine_op<klay::OP_SUM>(a, g, s); break;
    case klay::OP_PROD: launch_combine_op<klay::OP_PROD>(a, g, s); break;
    case klay::OP_LSE: launch_combine_op<klay::OP_LSE>(a, g, s); break;
    case klay::OP_MAX: launch_combine_op<klay::OP_MAX>(a, g, s); break;
    case klay::OP_SUM_H: launch_combine_op<klay::OP_SUM_H>(a, g, s); break;
    case klay::OP_SUM_P: launch_combine_op<klay::OP_SUM_P>(a, g, s); break;
    default: launch_pass(op, a, g, s); break;
    }
}

// Main rows and combine rows in one launch (one column per lane; the segments have run in a launch before it).
template <int OP, int COP>
void launch_stream_combine_op(const DevPass& dp, const Geometry& g, const float* src, const float* src2, const float* own,
                              float* dst, int B, hipStream_t s, int* zf, const klay::PassArgs& cmb) {
    const int2* tasks = reinterpret_cast<const int2*>(dp.tasks);
    int64_t blocks = ((int64_t)dp.n_tasks + 3) / 4;
    blocks = (blocks + 7) / 8 * 8;
    const int n_comb_blocks = (cmb.n_main + 7) / 8 * 8;
    const int nt = (int64_t)dp.n_main * g.ld * 4 > (int64_t)64 << 20 ? 1 : 0;
    dim3 grid((unsigned)(blocks + n_comb_blocks), (unsigned)g.tiles);
    hipLaunchKernelGGL((klay::stream_combine_kernel<OP, COP, 1>), grid, dim3(256), 0, s, tasks, dp.n_tasks, dp.idx, src, src2,
                       own, dst, B, g.ld, nt, dp.n_main, zf, n_comb_blocks, cmb);
}

// false: no such kernel for this pair of operations
bool launch_stream_combine(int op, int combine_op, const DevPass& dp, const Geometry& g, const float* src,
                           const float* src2, const float* own, float* dst, int B, hipStream_t s, int* zf,
                           const klay::PassArgs& cmb) {
    using namespace klay;
#define KLAY_SC(A, C) \
    if (op == A && combine_op == C) { launch_stream_combine_op<A, C>(dp, g, src, src2, own, dst, B, s, zf, cmb); return true; }
    KLAY_SC(OP_SUM, OP_SUM)
    KLAY_SC(OP_PROD, OP_PROD)
    KLAY_SC(OP_LSE, OP_LSE)
    KLAY_SC(OP_MAX, OP_MAX)
    KLAY_SC(OP_SUM_H, OP_SUM_H)
    KLAY_SC(OP_SOFTMAX_H, OP_SUM)
    KLAY_SC(OP_SUM_P, OP_SUM_P)
    KLAY_SC(OP_PROD_BWD, OP_SUM)
    KLAY_SC(OP_PROD_BWD_P, OP_SUM_P)
#undef KLAY_SC
    return false;
}

klay::PassArgs combine_args(const DevPass& dp, const float* seg_rows, const float* own, float* dst, const Geometry& g,
                            int B, int* zero_flag) {
    klay::PassArgs cmb{};
    cmb.ptr = dp.comb_ptr;
    cmb.idx = dp.comb_idx;
    cmb.src = seg_rows;
    cmb.own = own;               // OP_SUM_H, OP_SUM_P: the value rows of the nodes the combine pass writes
    cmb.zero_flag = zero_flag;
    cmb.out_row = dp.comb_row;
    cmb.dst = dst;
    cmb.dst_seg = nullptr;
    cmb.row_begin = 0;
    cmb.n_main = dp.n_heavy;
    cmb.n_total = dp.n_heavy;
    cmb.B = B;
    cmb.ld = g.ld;
    return cmb;
}

bool stream_combine_pair(int op, int combine_op) {
    using namespace klay;
    return (op == combine_op && (op == OP_SUM || op == OP_PROD || op == OP_LSE || op == OP_MAX || op == OP_SUM_H || op == OP_SUM_P)) ||
           (op == OP_SOFTMAX_H && combine_op == OP_SUM) || (op == OP_PROD_BWD && combine_op == OP_SUM) ||
           (op == OP_PROD_BWD_P && combine_op == OP_SUM_P);
}

// One layer-level gather-reduce: main rows, segments of split rows, then the combine pass.  The main
// launch is timed under `cls`, a separate segment launch under KLAY_K_SPLIT, the combine launch under KLAY_K_COMBINE.
void run_pass_set(int op, int combine_op, const DevPass& dp, const float* src, const float* src2,
                  const float* own, float* dst, float* seg_rows, const Geometry& g, int B, hipStream_t s,
                  Profiler& prof, int cls, int* zero_flag = nullptr) {
    const bool edges = prof.c->small_batch_edges;
    klay::PassArgs a{};
    a.zero_flag = zero_flag;
    a.ptr = dp.ptr;
    a.idx = dp.idx;
    a.src = src;
    a.src2 = src2;
    a.own = own;
    a.seg_owner = dp.seg_owner;
    a.out_row = nullptr;
    a.dst = dst;
    a.dst_seg = seg_rows;
    a.n_main = dp.n_main;
    a.n_total = dp.n_main + dp.n_seg;
    a.B = B;
    a.ld = g.ld;
    const double light_rows = (double)dp.n_main - dp.n_heavy;
    if (g.w == 64) {
        // Tiles of two or four columns per lane: the segments of split rows ride in the same launch as
        // the main rows (same streaming walk, output to partial rows).  One-column tiles (B <= 64) measured
        // 9% faster through the generic kernel: separate launch.
        const bool merged = dp.n_seg > 0 && g.vec >= 2;
        float* seg_base = seg_rows - (ptrdiff_t)dp.n_main * g.ld;     // only indexed with rows >= n_main
        if (!merged && dp.n_seg > 0 && dp.main_entries + dp.seg_entries <= kSmallPassEntries) {
            // A small layer with split rows whose segments cannot ride in the streaming launch: main rows
            // and segments in one launch of the generic kernel (a wave per row) instead of two launches.
            // Such layers are bound by their launches, not by what the kernels move.
            prof.begin(cls, pass_bytes(op, (double)(dp.main_entries + dp.seg_entries), light_rows + dp.n_seg, B),
                       pass_min_bytes(op, (double)(dp.main_entries + dp.seg_entries), light_rows + dp.n_seg, (double)dp.n_src, B));
            a.row_begin = 0;
            launch_pass(op, a, g, s);
            prof.end();
        } else if (!merged && dp.n_seg > 0 && dp.n_heavy > 0 && dp.n_tasks > 0 && stream_combine_pair(op, combine_op)) {
            // One column per lane and a layer too large for one generic launch: the segments first, then the
            // main rows together with the combine rows (two launches instead of three).
            prof.begin(KLAY_K_SPLIT, pass_bytes(op, (double)dp.seg_entries, (double)dp.n_seg, B),
                       pass_min_bytes(op, (double)dp.seg_entries, (double)dp.n_seg, 0.0, B));
            a.row_begin = dp.n_main;
            launch_pass(op, a, g, s);
            prof.end();
            prof.begin(KLAY_K_MAIN_COMBINE,
                       pass_bytes(op, (double)dp.main_entries, light_rows, B) + pass_bytes(combine_op, (double)dp.n_seg, (double)dp.n_heavy, B),
                       pass_min_bytes(op, (double)dp.main_entries, light_rows, (double)dp.n_src, B) +
                           pass_bytes(combine_op, (double)dp.n_seg, (double)dp.n_heavy, B));
            launch_stream_combine(op, combine_op, dp, g, src, src2, own, dst, B, s, zero_flag,
                                  combine_args(dp, seg_rows, own, dst, g, B, zero_flag));
            prof.end();
            return;
        } else {
        double bytes = pass_bytes(op, (double)dp.main_entries, light_rows, B);
        if (merged) bytes += pass_bytes(op, (double)dp.seg_entries, (double)dp.n_seg, B);
        // the distinct source rows are charged to the main launch, a separate segment launch only
        // adds its index entries and the partial rows it writes
        double min_bytes = pass_min_bytes(op, (double)dp.main_entries, light_rows, (double)dp.n_src, B);
        if (merged) min_bytes += pass_min_bytes(op, (double)dp.seg_entries, (double)dp.n_seg, 0.0, B);
        prof.begin(cls, bytes, min_bytes);
        launch_stream(op, dp, true, merged, g, src, src2, own, dst, seg_base, B, s, zero_flag);
        prof.end();
        if (dp.n_seg > 0 && !merged) {
            prof.begin(KLAY_K_SPLIT, pass_bytes(op, (double)dp.seg_entries, (double)dp.n_seg, B),
                       pass_min_bytes(op, (double)dp.seg_entries, (double)dp.n_seg, 0.0, B));
            a.row_begin = dp.n_main;
            launch_pass(op, a, g, s);
            prof.end();
        }
        }
    } else {
        // small batches: main rows and segments in one launch (a lane group per row, or lanes = edges)
        prof.begin(cls, pass_bytes(op, (double)(dp.main_entries + dp.seg_entries), light_rows + dp.n_seg, B),
                   pass_min_bytes(op, (double)(dp.main_entries + dp.seg_entries), light_rows + dp.n_seg, (double)dp.n_src, B));
        if (edges) {
            launch_edge(op, dp, g, src, src2, own, dst, seg_rows - (ptrdiff_t)dp.n_main * g.ld, B, s, zero_flag);
        } else {
            a.row_begin = 0;
            launch_pass(op, a, g, s);
        }
        prof.end();
    }
    if (dp.n_heavy > 0) {
        const klay::PassArgs cmb = combine_args(dp, seg_rows, own, dst, g, B, zero_flag);
        prof.begin(KLAY_K_COMBINE, pass_bytes(combine_op, (double)dp.n_seg, (double)dp.n_heavy, B));
        launch_combine(combine_op, cmb, g, s);
        prof.end();
    }
}

// ---- persistent kernels for the top layers -----------------------------------------------------
struct TailChoice {
    int first = 0;       // first layer run by the persistent kernel (0: not used)
    int ct = 1;          // batch columns per workgroup
    int nmax = 0;        // LDS rows per buffer
};

// Batch columns per workgroup: one column per workgroup until the batch needs more workgroups
// than the chip has compute units; few columns mean few rows per lane and a short layer time.
int tail_ct(int B) {
    int ct = 1;
    while (ct < 8 && (B + ct - 1) / ct > 256) ct *= 2;
    return ct;
}

// Largest suffix of the candidate layers, not starting below `lowest`, whose `buffers` value arrays of
// CT columns fit the LDS of a workgroup.  The arrays hold the layers first .. L, and layer 0 as well
// when the kernel starts at layer 1 and evaluates the leaf layer itself.  At least two layers,
// otherwise a kernel of its own is not worth it.
TailChoice choose_tail(const klay_circuit* c, int B, int buffers, int lowest) {
    TailChoice t;
    const klay::CircuitPlan& p = c->plan;
    if (lowest <= 0 || c->tail_lds_bytes == 0) return t;
    t.ct = tail_ct(B);
    const int L = p.num_layers;
    const int64_t words = (int64_t)(c->tail_lds_bytes / sizeof(float));
    int64_t nmax = 0;
    int first = 0;
    for (int l = L; l >= lowest; --l) {
        int64_t n2 = std::max(nmax, p.layers[(size_t)l].n);
        if (l == 1) n2 = std::max(n2, p.layers[0].n);
        if ((int64_t)buffers * (n2 + 1) * t.ct > words) break;      // + 1: the padding slot of every array
        nmax = n2;
        first = l;
    }
    if (first == 0 || L - first + 1 < 2) return t;
    t.first = first;
    t.nmax = (int)nmax;
    return t;
}

// the layers the forward sweep runs in the persistent kernel ...
TailChoice choose_tail_fwd(const klay_circuit* c, int B) { return choose_tail(c, B, 2, c->plan.tail_first); }

// Rows of the layer below the forward kernel's first one if the kernel reads that layer from the column-major
// stage buffer: it then has to fit an LDS array (the arrays are made as long as it, if the LDS has the room).
// 0: no stage buffer (the kernel evaluates the leaf layer itself, or gathers from the rows).
int64_t tail_stage_rows(const klay_circuit* c, const TailChoice& t) {
    if (t.first < 2) return 0;
    const int64_t nb = c->plan.layers[(size_t)t.first - 1].n;
    const int64_t rows = std::max<int64_t>(nb, t.nmax);
    return (size_t)2 * (size_t)(rows + 1) * t.ct * sizeof(float) <= c->tail_lds_bytes ? nb : 0;
}
int64_t tail_stage_rows(const klay_circuit* c, int B) { return tail_stage_rows(c, choose_tail_fwd(c, B)); }
// ... and the layers the reverse sweep does, given the forward choice (fewer where a layer has a node with more
// than kTailFanCap parents)
TailChoice choose_tail_bwd(const klay_circuit* c, int B, int fwd_first) {
    if (fwd_first <= 0 || c->plan.tail_bwd_first <= 0) return TailChoice();
    return choose_tail(c, B, 2, std::max(fwd_first, c->plan.tail_bwd_first));
}

template <int CT>
hipError_t tail_attr(int bytes) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&klay::slab_fwd_kernel<CT>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(&klay::slab_bwd_kernel<CT>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

// LDS bytes a workgroup of the persistent kernels may use: the largest of 160, 128 and 64 KB that the
// runtime accepts for all of them (gfx950 has 160 KB per compute unit), 0 if none.
size_t enable_tail_lds() {
    static_assert(kTailLdsMax == 160 * 1024, "the first size tried is the largest");
    for (int kb : {160, 128, 64}) {
        const int bytes = kb * 1024;
        hipError_t e = tail_attr<8>(bytes);
        if (e == hipSuccess) e = tail_attr<4>(bytes);
        if (e == hipSuccess) e = tail_attr<2>(bytes);
        if (e == hipSuccess) e = tail_attr<1>(bytes);
        if (e == hipSuccess) return (size_t)bytes;
        (void)hipGetLastError();
    }
    return 0;
}

// `stage`: room for the layer below the kernel's first one in column-major form.  When that layer fits an LDS
// array (the arrays are made as long as it, if the LDS has the room) it is transposed there first, so that a
// workgroup reads its column as one run instead of one float per row.
void launch_tail_fwd(const klay_circuit* c, const TailChoice& t, const float* act, float* tb, float* stage, int B, int ld,
                     int semiring, const klay::SlabLeaf& leaf, float* out, hipStream_t s) {
    const klay::CircuitPlan& p = c->plan;
    const float* staged = nullptr;
    int nmax = t.nmax;
    if (!leaf.w) {
        const int64_t nb = tail_stage_rows(c, t);
        if (nb > 0) {
            nmax = (int)std::max<int64_t>(nb, t.nmax);
            dim3 tg((unsigned)((nb + 31) / 32), (unsigned)((B + 31) / 32));
            hipLaunchKernelGGL(klay::rows_to_cols_kernel, tg, dim3(256), 0, s,
                               act + (size_t)c->dl[(size_t)t.first - 1].row0 * ld, (int)nb, B, ld, stage);
            staged = stage;
        }
    }
    const klay::SlabLayer* descs = c->d_tail + (t.first - p.tail_first);
    const int n_layers = p.num_layers - t.first + 1;
    const int first_is_and = t.first & 1;
    const size_t lds = (size_t)2 * (nmax + 1) * t.ct * sizeof(float);
    dim3 grid((unsigned)((B + t.ct - 1) / t.ct));
#define KLAY_TAIL_FWD(CT)                                                                              \
    hipLaunchKernelGGL((klay::slab_fwd_kernel<CT>), grid, dim3(klay::kSlabThreads), lds, s, descs,     \
                       n_layers, first_is_and, c->d_index, act, B, ld, semiring, nmax, tb, (int)c->tail_rows, leaf, \
                       c->d_root_pos, p.num_roots, out, staged)
    switch (t.ct) {
    case 8: KLAY_TAIL_FWD(8); break;
    case 4: KLAY_TAIL_FWD(4); break;
    case 2: KLAY_TAIL_FWD(2); break;
    default: KLAY_TAIL_FWD(1); break;
    }
#undef KLAY_TAIL_FWD
}

// The kernel leaves the adjoints of its first layer column-major in `g_cols` (B runs of n_first floats); they are
// transposed into the rows of g_out afterwards.
void launch_tail_bwd(const klay_circuit* c, const TailChoice& t, const float* tb, const float* dout,
                     float* g_cols, float* g_out, const uint32_t* top_multi, int B, int ld, hipStream_t s) {
    const klay::CircuitPlan& p = c->plan;
    const klay::SlabLayer* descs = c->d_tail + (t.first - p.tail_first);
    const int n_layers = p.num_layers - t.first + 1;
    const int first_is_and = t.first & 1;
    const size_t lds = (size_t)2 * (t.nmax + 1) * t.ct * sizeof(float);
    dim3 grid((unsigned)((B + t.ct - 1) / t.ct));
#define KLAY_TAIL_BWD(CT)                                                                              \
    hipLaunchKernelGGL((klay::slab_bwd_kernel<CT>), grid, dim3(klay::kSlabThreads), lds, s, descs,     \
                       n_layers, first_is_and, c->d_index, dout, c->d_top_ptr, c->d_top_root,          \
                       p.num_roots, g_cols, B, t.nmax, tb, (int)c->tail_rows, top_multi)
    switch (t.ct) {
    case 8: KLAY_TAIL_BWD(8); break;
    case 4: KLAY_TAIL_BWD(4); break;
    case 2: KLAY_TAIL_BWD(2); break;
    default: KLAY_TAIL_BWD(1); break;
    }
#undef KLAY_TAIL_BWD
    const int n_first = (int)p.layers[(size_t)t.first].n;
    dim3 tgrid((unsigned)((n_first + 31) / 32), (unsigned)((ld + 31) / 32));
    hipLaunchKernelGGL(klay::tb_to_rows_kernel, tgrid, dim3(256), 0, s, g_cols, n_first, 0, n_first, B, ld, g_out);
}

// Values of layers first .. last (all run by the persistent forward kernel) from the column-major
// buffer into their rows of the activation buffer, for the ordinary launches of a reverse sweep.
void launch_tb_to_rows(const klay_circuit* c, int first, int last, const float* tb, float* act, int B, int ld, hipStream_t s) {
    const klay::CircuitPlan& p = c->plan;
    int64_t tb_first = 0, n_rows = 0;
    for (int l = p.tail_first; l < first; ++l) tb_first += p.layers[(size_t)l].n;
    for (int l = first; l <= last; ++l) n_rows += p.layers[(size_t)l].n;
    if (n_rows <= 0) return;
    dim3 grid((unsigned)((n_rows + 31) / 32), (unsigned)((ld + 31) / 32));
    hipLaunchKernelGGL(klay::tb_to_rows_kernel, grid, dim3(256), 0, s, tb, (int)c->tail_rows, (int)tb_first, (int)n_rows, B,
                       ld, act + (size_t)c->dl[(size_t)first].row0 * ld);
}

double tail_alg_bytes(const klay_circuit* c, int first, int B, bool backward) {
    double bytes = 0;
    for (int l = first; l <= c->plan.num_layers; ++l) {
        const klay::LayerPlan& lay = c->plan.layers[(size_t)l];
        const double below = (double)c->plan.layers[(size_t)l - 1].n;
        if (!backward) bytes += 4.0 * B * ((double)lay.e + (double)lay.n) + 4.0 * ((double)lay.e + (double)lay.n);
        else if (l > first) {
            const bool is_and = (l & 1) != 0;
            bytes += 4.0 * B * ((is_and ? 1.0 : 2.0) * (double)lay.e + (is_and ? 1.0 : 2.0) * below) +
                     4.0 * ((double)lay.e + below);
        }
    }
    return bytes;
}

// what a persistent launch has to move through memory: the values it writes (forward) or reads (reverse)
// once, its index vectors, the rows it reads from or leaves in the activation buffer
double tail_min_bytes(const klay_circuit* c, int first, int B, bool backward) {
    double bytes = 0;
    for (int l = first; l <= c->plan.num_layers; ++l) {
        const klay::LayerPlan& lay = c->plan.layers[(size_t)l];
        bytes += 4.0 * B * (double)lay.n + 4.0 * (double)(backward ? lay.slab_bwd.ent.size() : lay.slab_fwd.ent.size());
    }
    bytes += 4.0 * B * (double)(backward ? c->plan.layers[(size_t)first].n : c->plan.layers[(size_t)first - 1].n);
    return bytes;
}


// ---- real-semiring reverse sweep -----------------------------------------------------------------
klay_status ensure_real_bwd(klay_circuit* c) {
    const klay::CircuitPlan& p = c->plan;
    const int L = p.num_layers;
    if (!c->real_layers.empty()) return KLAY_OK;
    Packer pk;
    struct Off { size_t ptr = 0, child = 0; PassOffsets pass{}; klay::PassPlan plan; };
    std::vector<Off> offs((size_t)L + 1);
    klay::Options opt;
    for (int l = 1; l <= L; l += 2) {           // AND layers: plain index vectors by parent
        offs[(size_t)l].ptr = pk.add(p.layers[(size_t)l].row_ptr);
        offs[(size_t)l].child = pk.add(p.layers[(size_t)l].child);
    }
    const int B0 = p.alias_top;
    if (B0 > 0) {
        // Every row below layer B0 gathers from its parents in any higher layer up to B0.  An AND parent's
        // row holds P (see prod_parent_kernel); a sum node's row holds plain adjoints: those entries carry
        // the weighted bit, which OP_PROD_BWD reads as "add as it is".
        const int64_t NR = p.row0[(size_t)B0];
        std::vector<int32_t> gptr((size_t)NR + 1, 0);
        for (int l = 1; l <= B0; ++l)
            for (int32_t ch : p.layers[(size_t)l].child) ++gptr[(size_t)ch + 1];
        for (int64_t i = 0; i < NR; ++i) gptr[(size_t)i + 1] += gptr[(size_t)i];
        std::vector<int32_t> gsrc((size_t)gptr[(size_t)NR]);
        std::vector<uint32_t> gflag((size_t)gptr[(size_t)NR], 0u);
        {
            std::vector<int32_t> fill(gptr.begin(), gptr.end() - 1);
            for (int l = 1; l <= B0; ++l) {
                const klay::LayerPlan& lay = p.layers[(size_t)l];
                for (int64_t r = 0; r < lay.n; ++r)
                    for (int32_t j = lay.row_ptr[(size_t)r]; j < lay.row_ptr[(size_t)r + 1]; ++j) {
                        const int32_t slot = fill[(size_t)lay.child[(size_t)j]]++;
                        gsrc[(size_t)slot] = (int32_t)(p.row0[(size_t)l] + r);
                        if ((l & 1) == 0) gflag[(size_t)slot] = klay::kWeightedEdge;
                    }
            }
        }
        for (int l = 0; l < B0; ++l) {
            const klay::LayerPlan& lay = p.layers[(size_t)l];
            Off& o = offs[(size_t)l];
            const int64_t a = p.row0[(size_t)l];
            std::vector<int32_t> lptr((size_t)lay.n + 1);
            for (int64_t i = 0; i <= lay.n; ++i) lptr[(size_t)i] = gptr[(size_t)(a + i)] - gptr[(size_t)a];
            klay::make_pass_plan(lay.n, lptr.data(), gsrc.data() + gptr[(size_t)a], opt, o.plan, gflag.data() + gptr[(size_t)a]);
            if (o.plan.n_seg > p.max_bwd_seg)
                return fail(KLAY_EINVAL, "klay_backward: split plan of the real-semiring sweep exceeds the workspace");
            o.pass = pack_pass(pk, o.plan);
        }
    }
    const size_t bytes = pk.buf.size() * sizeof(int32_t);
    if (hipMalloc(reinterpret_cast<void**>(&c->d_real_index), bytes) != hipSuccess) {
        (void)hipGetLastError();
        return fail(KLAY_ENOMEM, "klay_backward: hipMalloc of the real-semiring index arrays failed");
    }
    if (hipError_t e = hipMemcpy(c->d_real_index, pk.buf.data(), bytes, hipMemcpyHostToDevice); e != hipSuccess) {
        (void)hipFree(c->d_real_index);
        c->d_real_index = nullptr;
        return fail(KLAY_EHIP, std::string("klay_backward: upload of the real-semiring index arrays: ") +
                                   hipGetErrorString(e));
    }
    c->real_layers.resize((size_t)L + 1);
    for (int l = 0; l <= L; ++l) {
        klay_circuit::RealLayer& r = c->real_layers[(size_t)l];
        if (l & 1) {
            r.ptr = c->d_real_index + offs[(size_t)l].ptr;
            r.child = c->d_real_index + offs[(size_t)l].child;
        }
        if (l < B0) bind_pass(r.by_child, offs[(size_t)l].plan, offs[(size_t)l].pass, c->d_real_index);
    }
    return KLAY_OK;
}

// adjoint rows of an AND layer -> P rows, in place (see prod_parent_kernel)
void launch_prod_parent(const klay_circuit::RealLayer& r, int n, const float* below, float* gl, const float* own,
                        const int* zero_flag, const Geometry& g, int B, hipStream_t s) {
    if (n <= 0) return;                               // a layer without chain nodes can be empty
    const int rpw = 64 / g.w;
    int64_t blocks = ((int64_t)n + 4 * rpw - 1) / (4 * rpw);
    // with the values of the nodes given the kernel mostly finds nothing to do: a small grid that strides
    if (own) blocks = std::min<int64_t>(blocks, std::max<int64_t>(256, 2048 / g.tiles));
    dim3 grid((unsigned)blocks, (unsigned)g.tiles);
#define KLAY_PP(VEC, W) \
    hipLaunchKernelGGL((klay::prod_parent_kernel<VEC, W>), grid, dim3(256), 0, s, r.ptr, r.child, below, gl, n, B, g.ld, own, zero_flag)
    if (g.w == 64) {
        if (g.vec == 4) KLAY_PP(4, 64);
        else if (g.vec == 2) KLAY_PP(2, 64);
        else KLAY_PP(1, 64);
    } else {
        switch (g.w) {
        case 32: KLAY_PP(1, 32); break;
        case 16: KLAY_PP(1, 16); break;
        case 8: KLAY_PP(1, 8); break;
        case 4: KLAY_PP(1, 4); break;
        case 2: KLAY_PP(1, 2); break;
        default: KLAY_PP(1, 1); break;
        }
    }
#undef KLAY_PP
}

// ---- double-precision evaluation ---------------------------------------------------------------
struct Workspace64 {
    size_t act = 0, wT = 0, seg_rows = 0, g0 = 0, g1 = 0, g2 = 0, total = 0;   // offsets in doubles
};

Workspace64 workspace_layout64(const klay_circuit* c, int ld) {
    const klay::CircuitPlan& p = c->plan;
    Workspace64 w;
    size_t off = 0;
    auto take = [&](size_t n) { const size_t o = off; off += (n + 31) / 32 * 32; return o; };
    w.act = take((size_t)p.num_nodes * ld);
    w.wT = take((size_t)std::max(1, p.num_vars) * ld);
    w.seg_rows = take((size_t)std::max<int64_t>(std::max(p.max_fwd_seg, p.max_bwd_seg), 1) * ld);
    // adjoints: one row per node of the layers 0 .. alias_top, two sets of rows for the layers above
    w.g0 = take((size_t)p.row0[(size_t)p.alias_top + 1] * ld);
    w.g1 = take((size_t)top_layer_rows(p) * ld);
    w.g2 = take((size_t)top_layer_rows(p) * ld);
    w.total = off;
    return w;
}

// two columns per lane (16-byte loads) once the batch is wider than a wave; ld is even then
template <int OP>
void launch_pass64(const klay::f64::PassArgs& a, hipStream_t s) {
    if (a.n_total <= 0) return;
    const unsigned rows = (unsigned)(((int64_t)a.n_total + 3) / 4);
    if (a.B > 64) {
        hipLaunchKernelGGL((klay::f64::pass_kernel<OP, 2>), dim3(rows, (unsigned)((a.B + 127) / 128)), dim3(256), 0, s, a);
    } else {
        hipLaunchKernelGGL((klay::f64::pass_kernel<OP, 1>), dim3(rows, 1), dim3(256), 0, s, a);
    }
}

void launch_pass64(int op, const klay::f64::PassArgs& a, hipStream_t s) {
    switch (op) {
    case klay::OP_SUM: launch_pass64<klay::OP_SUM>(a, s); break;
    case klay::OP_PROD: launch_pass64<klay::OP_PROD>(a, s); break;
    case klay::OP_LSE: launch_pass64<klay::OP_LSE>(a, s); break;
    case klay::OP_MAX: launch_pass64<klay::OP_MAX>(a, s); break;
    case klay::OP_PROD_BWD: launch_pass64<klay::OP_PROD_BWD>(a, s); break;
    default: launch_pass64<klay::OP_SOFTMAX_BWD>(a, s); break;
    }
}

// main rows and segments in one launch, then the combine rows of split rows
void run_pass_set64(int op, int combine_op, const DevPass& dp, const double* src, const double* src2,
                    const double* own, double* dst, double* seg_rows, int B, int ld, hipStream_t s) {
    klay::f64::PassArgs a{};
    a.ptr = dp.ptr;
    a.idx = dp.idx;
    a.src = src;
    a.src2 = src2;
    a.own = own;
    a.seg_owner = dp.seg_owner;
    a.out_row = nullptr;
    a.dst = dst;
    a.dst_seg = seg_rows;
    a.n_main = dp.n_main;
    a.n_total = dp.n_main + dp.n_seg;
    a.B = B;
    a.ld = ld;
    launch_pass64(op, a, s);
    if (dp.n_heavy > 0) {
        klay::f64::PassArgs cmb{};
        cmb.ptr = dp.comb_ptr;
        cmb.idx = dp.comb_idx;
        cmb.src = seg_rows;
        cmb.out_row = dp.comb_row;
        cmb.dst = dst;
        cmb.n_main = dp.n_heavy;
        cmb.n_total = dp.n_heavy;
        cmb.B = B;
        cmb.ld = ld;
        launch_pass64(combine_op, cmb, s);
    }
}

klay_status forward64_impl(klay_circuit* c, const double* w, const double* wneg, int32_t B, double* out,
                           klay_semiring semiring, void* stream) {
    if (!c || !w || !out) return fail(KLAY_EINVAL, "klay_forward_f64: null argument");
    if (c->device < 0) return fail(KLAY_ESTATE, "klay_forward_f64: host-only handle (built with device = -1)");
    if (B < 1) return fail(KLAY_EINVAL, "klay_forward_f64: B must be >= 1");
    if (semiring != KLAY_REAL && semiring != KLAY_LOG && semiring != KLAY_MAXLOG)
        return fail(KLAY_EINVAL, "klay_forward_f64: unknown semiring");
    KLAY_HIP(hipSetDevice(c->device));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const klay::CircuitPlan& p = c->plan;
    const int ld = B > 64 ? (B + 1) / 2 * 2 : B;       // even rows for two columns per lane
    c->have_fwd64 = false;
    const Workspace64 lay = workspace_layout64(c, ld);
    const size_t bytes = lay.total * sizeof(double);
    if (bytes > c->ws64_bytes) {
        if (c->ws64) { KLAY_HIP(hipFree(c->ws64)); c->ws64 = nullptr; c->ws64_bytes = 0; }
        if (hipMalloc(&c->ws64, bytes) != hipSuccess) {
            (void)hipGetLastError();
            return fail(KLAY_ENOMEM, "hipMalloc of " + std::to_string(bytes) + " workspace bytes failed");
        }
        c->ws64_bytes = bytes;
    }
    double* ws = static_cast<double*>(c->ws64);
    double* act = ws + lay.act;
    double* wT = ws + lay.wT;
    double* seg_rows = ws + lay.seg_rows;
    const int L = p.num_layers, V = p.num_vars;
    const bool log_domain = semiring != KLAY_REAL;
    const dim3 row_grid((unsigned)((ld + 255) / 256));
    if (V > 0)
        hipLaunchKernelGGL(klay::f64::leaf_fwd_kernel, dim3((unsigned)V, (unsigned)((ld + 255) / 256)), dim3(256), 0, s, w,
                           wneg, (int)B, V, ld, c->d_pos_row, c->d_neg_row, wT, act, log_domain ? 1 : 0);
    if (c->true_row >= 0)
        hipLaunchKernelGGL(klay::f64::fill_row_kernel, row_grid, dim3(256), 0, s, act + (size_t)c->true_row * ld, ld,
                           log_domain ? 0.0 : 1.0);
    if (c->false_row >= 0)
        hipLaunchKernelGGL(klay::f64::fill_row_kernel, row_grid, dim3(256), 0, s, act + (size_t)c->false_row * ld, ld,
                           log_domain ? (double)-INFINITY : 0.0);
    for (int l = 1; l <= L; ++l) {
        const DevLayer& d = c->dl[(size_t)l];
        const bool is_and = (l & 1) != 0;
        const int or_op = semiring == KLAY_MAXLOG ? klay::OP_MAX : klay::OP_LSE;
        const int op = log_domain ? (is_and ? klay::OP_SUM : or_op) : (is_and ? klay::OP_PROD : klay::OP_SUM);
        // up to alias_top child entries are rows of the whole buffer, above it of the layer below
        const double* below = l <= p.alias_top ? act : act + (size_t)c->dl[(size_t)l - 1].row0 * ld;
        run_pass_set64(op, op, d.fwd, below, nullptr, nullptr, act + (size_t)d.row0 * ld, seg_rows, B, ld, s);
    }
    hipLaunchKernelGGL(klay::f64::root_out_kernel, dim3((unsigned)p.num_roots), dim3(256), 0, s,
                       act + (size_t)c->dl[(size_t)L].row0 * ld, c->d_root_pos, (int)B, p.num_roots, ld, out);
    KLAY_HIP(hipGetLastError());
    c->have_fwd64 = true;
    c->last64_B = B;
    c->last64_semiring = semiring;
    c->last64_neg_explicit = wneg != nullptr;
    return KLAY_OK;
}

klay_status backward64_impl(klay_circuit* c, const double* dout, double* dleaf, double* dneg, void* stream) {
    if (!c || !dout || !dleaf) return fail(KLAY_EINVAL, "klay_backward_f64: null argument");
    if (c->device < 0) return fail(KLAY_ESTATE, "klay_backward_f64: host-only handle");
    if (!c->have_fwd64) return fail(KLAY_ESTATE, "klay_backward_f64: no double-precision forward pass to differentiate");
    if (c->last64_semiring == KLAY_MAXLOG)
        return fail(KLAY_EINVAL, "klay_backward_f64: the (max, +) semiring is not differentiated");
    const bool real = c->last64_semiring == KLAY_REAL;
    if (dneg && !c->last64_neg_explicit)
        return fail(KLAY_ESTATE, "klay_backward_f64: dneg given, but the forward pass had no weights for the negated literals");
    KLAY_HIP(hipSetDevice(c->device));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const klay::CircuitPlan& p = c->plan;
    const int B = c->last64_B, ld = B > 64 ? (B + 1) / 2 * 2 : B;
    const Workspace64 lay = workspace_layout64(c, ld);
    double* ws = static_cast<double*>(c->ws64);
    double* act = ws + lay.act;
    double* wT = ws + lay.wT;
    double* seg_rows = ws + lay.seg_rows;
    double* G = ws + lay.g0;
    double* gcur = ws + lay.g1;
    double* gnext = ws + lay.g2;
    const int L = p.num_layers, V = p.num_vars, R = p.num_roots, B0 = p.alias_top;
    const int leaf_mode = c->last64_neg_explicit ? 2 : (real ? 0 : 1);
    const dim3 leaf_grid((unsigned)std::max(V, 1), (unsigned)((B + 255) / 256));
    auto grow = [&](int l) { return G + (size_t)c->dl[(size_t)l].row0 * ld; };   // adjoint rows of a layer <= B0
    // Same course as the fp32 sweep (see klay_backward's implementation): the layers above B0 one by one,
    // alternating between two buffers, the last of these steps writing the rows of layer B0 into G; then
    // the rows of the layers below B0, each gathering from its parents anywhere in G.
    if (real) {
        klay_status rs = ensure_real_bwd(c);
        if (rs != KLAY_OK) return rs;
        const dim3 pp_block(256);
        auto prod_parent = [&](int l, const double* below, double* gl) {
            const DevLayer& d = c->dl[(size_t)l];
            if (d.n <= 0) return;
            const klay_circuit::RealLayer& r = c->real_layers[(size_t)l];
            hipLaunchKernelGGL(klay::f64::prod_parent_kernel, dim3((unsigned)((d.n + 3) / 4), (unsigned)((B + 63) / 64)),
                               pp_block, 0, s, r.ptr, r.child, below, gl, (int)d.n, B, ld);
        };
        hipLaunchKernelGGL(klay::f64::seed_kernel, dim3((unsigned)c->dl[(size_t)L].n), dim3(256), 0, s, dout, c->d_top_ptr,
                           c->d_top_root, B, R, ld, L == B0 ? grow(L) : gcur);
        for (int l = L; l > B0; --l) {
            const DevLayer& d = c->dl[(size_t)l];
            const DevLayer& below = c->dl[(size_t)l - 1];
            double* dst = l - 1 == B0 ? grow(B0) : gnext;
            if ((l & 1) == 0) {
                run_pass_set64(klay::OP_SUM, klay::OP_SUM, d.bwd, gcur, nullptr, nullptr, dst, seg_rows, B, ld, s);
            } else {
                prod_parent(l, act + (size_t)below.row0 * ld, gcur);
                run_pass_set64(klay::OP_PROD_BWD, klay::OP_SUM, d.bwd, gcur, nullptr, act + (size_t)below.row0 * ld, dst,
                               seg_rows, B, ld, s);
            }
            std::swap(gcur, gnext);
        }
        if (B0 > 0 && (B0 & 1)) prod_parent(B0, act, grow(B0));
        for (int l = B0 - 1; l >= 0; --l) {
            run_pass_set64(klay::OP_PROD_BWD, klay::OP_SUM, c->real_layers[(size_t)l].by_child, G, nullptr,
                           act + (size_t)c->dl[(size_t)l].row0 * ld, grow(l), seg_rows, B, ld, s);
            if (l & 1) prod_parent(l, act, grow(l));
        }
    } else {
        hipLaunchKernelGGL(klay::f64::seed_kernel, dim3((unsigned)c->dl[(size_t)L].n), dim3(256), 0, s, dout, c->d_top_ptr,
                           c->d_top_root, B, R, ld, L == B0 ? grow(L) : gcur);
        for (int l = L; l > B0; --l) {
            const DevLayer& d = c->dl[(size_t)l];
            const DevLayer& below = c->dl[(size_t)l - 1];
            double* dst = l - 1 == B0 ? grow(B0) : gnext;
            if ((l & 1) != 0 || !d.bwd.has_weighted)
                run_pass_set64(klay::OP_SUM, klay::OP_SUM, d.bwd, gcur, nullptr, nullptr, dst, seg_rows, B, ld, s);
            else
                run_pass_set64(klay::OP_SOFTMAX_BWD, klay::OP_SUM, d.bwd, gcur, act + (size_t)d.row0 * ld,
                               act + (size_t)below.row0 * ld, dst, seg_rows, B, ld, s);
            std::swap(gcur, gnext);
        }
        for (int l = B0 - 1; l >= 0; --l) {
            const DevPass& dp = c->dl[(size_t)l + 1].bwd;
            run_pass_set64(dp.has_weighted ? klay::OP_SOFTMAX_BWD : klay::OP_SUM, klay::OP_SUM, dp, G, act,
                           act + (size_t)c->dl[(size_t)l].row0 * ld, grow(l), seg_rows, B, ld, s);
        }
    }
    if (V > 0)
        hipLaunchKernelGGL(klay::f64::leaf_bwd_kernel, leaf_grid, dim3(256), 0, s, G, wT, c->d_pos_row, c->d_neg_row, B, V,
                           ld, leaf_mode, dleaf, dneg);
    KLAY_HIP(hipGetLastError());
    return KLAY_OK;
}

}  // namespace

// Circuits collected for a joint layerization: node arrays concatenated, ids shifted.
struct klay_builder {
    int32_t num_vars = 0;
    std::vector<uint8_t> type;
    std::vector<int32_t> lit;
    std::vector<int64_t> ptr{0};
    std::vector<int32_t> idx;
    std::vector<int32_t> roots;
};

extern "C" {

const char* klay_last_error(void) { return g_err.c_str(); }

klay_status klay_build_ex(int32_t num_vars, int64_t num_nodes, const uint8_t* node_type,
                          const int32_t* node_lit, const int64_t* child_ptr, const int32_t* child_idx,
                          int32_t num_roots, const int32_t* roots, int32_t device,
                          const klay_options* opts, klay_circuit** out) {
    if (!out) return fail(KLAY_EINVAL, "klay_build: out is null");
    *out = nullptr;
    klay::Options o;
    o.alias_chains = true;                    // the default: padding-free below the narrow top
    if (opts) {
        o.no_reorder = opts->no_reorder != 0;
        if (opts->heavy_fan > 0) o.heavy_fan = opts->heavy_fan;
        if (opts->min_segment > 0) o.min_segment = opts->min_segment;
        o.no_tail = opts->no_tail != 0;
        o.alias_chains = opts->unary_chains == 0;
        if (opts->tail_rows_cap > 0) o.tail_rows_cap = opts->tail_rows_cap;
        o.no_merge = opts->no_merge != 0;
        o.small_batch_edges = opts->small_batch_edges != 0;
        o.no_fusion = opts->no_fusion != 0;
    }
    std::unique_ptr<klay_circuit> c;
    try {
        c.reset(new klay_circuit());
        std::string err;
        int st = klay::layerize(num_vars, num_nodes, node_type, node_lit, child_ptr, child_idx, num_roots,
                                roots, o, c->plan, err);
        if (st != 0) return fail(static_cast<klay_status>(st), err);
    } catch (const std::bad_alloc&) {
        return fail(KLAY_ENOMEM, "klay_build: out of host memory");
    }
    for (int64_t i = 0; i < c->plan.layers[0].n; ++i) {
        if (c->plan.leaf_code[(size_t)i] == INT32_MAX) c->true_row = (int32_t)i;
        if (c->plan.leaf_code[(size_t)i] == INT32_MIN) c->false_row = (int32_t)i;
    }
    c->device = device;
    c->small_batch_edges = o.small_batch_edges;
    c->no_fusion = o.no_fusion;
    if (c->plan.tail_first > 0) {
        // sizes of the persistent kernels' buffers (part of the workspace, so host-only handles know them too)
        const klay::CircuitPlan& p = c->plan;
        for (int l = p.tail_first; l <= p.num_layers; ++l) c->tail_rows += p.layers[(size_t)l].n;
    }
    if (device >= 0) {
        int ndev = 0;
        if (hipGetDeviceCount(&ndev) != hipSuccess || device >= ndev) {
            (void)hipGetLastError();
            return fail(KLAY_EHIP, "klay_build: HIP device " + std::to_string(device) + " not available");
        }
        klay_status st;
        try {
            st = upload(c.get());
        } catch (const std::bad_alloc&) {
            st = fail(KLAY_ENOMEM, "klay_build: out of host memory");
        }
        if (st != KLAY_OK) {
            if (c->d_index) (void)hipFree(c->d_index);
            return st;
        }
        c->tail_lds_bytes = c->plan.tail_first > 0 ? enable_tail_lds() : 0;
    } else {
        // a host-only handle sizes workspaces for a device that grants the whole LDS of a compute unit
        c->tail_lds_bytes = c->plan.tail_first > 0 ? kTailLdsMax : 0;
    }
    *out = c.release();
    return KLAY_OK;
}

klay_status klay_build(int32_t num_vars, int64_t num_nodes, const uint8_t* node_type,
                       const int32_t* node_lit, const int64_t* child_ptr, const int32_t* child_idx,
                       int32_t num_roots, const int32_t* roots, int32_t device, klay_circuit** out) {
    return klay_build_ex(num_vars, num_nodes, node_type, node_lit, child_ptr, child_idx, num_roots, roots,
                         device, nullptr, out);
}

klay_status klay_builder_create(int32_t num_vars, klay_builder** out) {
    if (!out) return fail(KLAY_EINVAL, "klay_builder_create: out is null");
    *out = nullptr;
    if (num_vars < 0) return fail(KLAY_EINVAL, "klay_builder_create: negative num_vars");
    try {
        *out = new klay_builder();
    } catch (const std::bad_alloc&) {
        return fail(KLAY_ENOMEM, "klay_builder_create: out of host memory");
    }
    (*out)->num_vars = num_vars;
    return KLAY_OK;
}

klay_status klay_builder_add(klay_builder* b, int64_t num_nodes, const uint8_t* node_type,
                             const int32_t* node_lit, const int64_t* child_ptr, const int32_t* child_idx,
                             int32_t num_roots, const int32_t* roots, int32_t* first_root) {
    if (!b) return fail(KLAY_EINVAL, "klay_builder_add: null builder");
    if (num_nodes <= 0 || num_roots <= 0 || !node_type || !node_lit || !child_ptr || !roots)
        return fail(KLAY_EINVAL, "klay_builder_add: empty circuit or null array");
    const int64_t base = (int64_t)b->type.size();
    if (base + num_nodes > (int64_t)INT32_MAX || (int64_t)b->roots.size() + num_roots > (int64_t)INT32_MAX)
        return fail(KLAY_EINVAL, "klay_builder_add: more than 2^31-1 nodes or roots in total");
    if (child_ptr[0] != 0) return fail(KLAY_EINVAL, "klay_builder_add: child_ptr[0] must be 0");
    for (int64_t i = 0; i < num_nodes; ++i)
        if (child_ptr[i + 1] < child_ptr[i]) return fail(KLAY_EINVAL, "klay_builder_add: child_ptr not monotone");
    const int64_t ne = child_ptr[num_nodes];
    if (ne > 0 && !child_idx) return fail(KLAY_EINVAL, "klay_builder_add: child_idx is null");
    for (int64_t j = 0; j < ne; ++j)
        if (child_idx[j] < 0 || child_idx[j] >= num_nodes)
            return fail(KLAY_EINVAL, "klay_builder_add: child index out of range");
    for (int32_t r = 0; r < num_roots; ++r)
        if (roots[r] < 0 || roots[r] >= num_nodes) return fail(KLAY_EINVAL, "klay_builder_add: root out of range");
    try {
        const size_t e0 = b->idx.size();
        b->type.reserve(b->type.size() + (size_t)num_nodes);
        b->lit.reserve(b->lit.size() + (size_t)num_nodes);
        b->ptr.reserve(b->ptr.size() + (size_t)num_nodes);
        b->idx.reserve(e0 + (size_t)ne);
        b->roots.reserve(b->roots.size() + (size_t)num_roots);
        // nothing below can throw: capacity is reserved
        b->type.insert(b->type.end(), node_type, node_type + num_nodes);
        b->lit.insert(b->lit.end(), node_lit, node_lit + num_nodes);
        for (int64_t i = 0; i < num_nodes; ++i) b->ptr.push_back((int64_t)e0 + child_ptr[i + 1]);
        for (int64_t j = 0; j < ne; ++j) b->idx.push_back((int32_t)(base + child_idx[j]));
        if (first_root) *first_root = (int32_t)b->roots.size();
        for (int32_t r = 0; r < num_roots; ++r) b->roots.push_back((int32_t)(base + roots[r]));
    } catch (const std::bad_alloc&) {
        return fail(KLAY_ENOMEM, "klay_builder_add: out of host memory");
    }
    return KLAY_OK;
}

klay_status klay_builder_finish(const klay_builder* b, int32_t device, const klay_options* opts,
                                klay_circuit** out) {
    if (!b) return fail(KLAY_EINVAL, "klay_builder_finish: null builder");
    if (b->type.empty()) return fail(KLAY_ESTATE, "klay_builder_finish: no circuit was added");
    return klay_build_ex(b->num_vars, (int64_t)b->type.size(), b->type.data(), b->lit.data(), b->ptr.data(),
                         b->idx.data(), (int32_t)b->roots.size(), b->roots.data(), device, opts, out);
}

void klay_builder_destroy(klay_builder* b) { delete b; }

void klay_destroy(klay_circuit* c) {
    if (!c) return;
    if (c->device >= 0) {
        (void)hipSetDevice(c->device);
        release_events(c);
        if (c->d_index) (void)hipFree(c->d_index);
        if (c->ws_own) (void)hipFree(c->ws_own);
        if (c->d_real_index) (void)hipFree(c->d_real_index);
        if (c->ws64) (void)hipFree(c->ws64);
    }
    delete c;
}

klay_status klay_info(const klay_circuit* c, klay_info_t* info) {
    if (!c || !info) return fail(KLAY_EINVAL, "klay_info: null argument");
    const klay::CircuitPlan& p = c->plan;
    std::memset(info, 0, sizeof(*info));
    info->num_vars = p.num_vars;
    info->num_roots = p.num_roots;
    info->num_layers = p.num_layers;
    info->device = c->device;
    info->num_nodes = p.num_nodes;
    info->num_edges = p.num_edges;
    info->dag_nodes = p.dag_nodes;
    info->dag_edges = p.dag_edges;
    info->num_pad_nodes = p.num_pad_nodes;
    info->max_layer_nodes = p.max_layer_nodes;
    info->max_fan_in = p.max_fan_in;
    info->max_fan_out = p.max_fan_out;
    info->num_split_rows = p.num_split_rows;
    info->index_bytes = (int64_t)c->index_bytes;
    info->tail_first_layer = p.tail_first;
    info->num_merged_nodes = p.num_merged;
    info->alias_top_layer = p.alias_top;
    info->num_fused_rows = p.num_fused;
    return KLAY_OK;
}

klay_status klay_layer_sizes(const klay_circuit* c, int64_t* nodes, int64_t* edges) {
    if (!c || !nodes || !edges) return fail(KLAY_EINVAL, "klay_layer_sizes: null argument");
    for (int l = 0; l <= c->plan.num_layers; ++l) {
        nodes[l] = c->plan.layers[(size_t)l].n;
        edges[l] = c->plan.layers[(size_t)l].e;
    }
    return KLAY_OK;
}

klay_status klay_layer_csr(const klay_circuit* c, int32_t layer, int64_t* row_ptr, int32_t* child) {
    if (!c || !row_ptr || !child) return fail(KLAY_EINVAL, "klay_layer_csr: null argument");
    if (layer < 1 || layer > c->plan.num_layers) return fail(KLAY_EINVAL, "klay_layer_csr: layer out of range");
    const klay::LayerPlan& l = c->plan.layers[(size_t)layer];
    for (int64_t i = 0; i <= l.n; ++i) row_ptr[i] = l.row_ptr[(size_t)i];
    std::copy(l.child.begin(), l.child.end(), child);
    return KLAY_OK;
}

klay_status klay_layer_nodes(const klay_circuit* c, int32_t layer, int32_t* origin, uint8_t* is_pad) {
    if (!c || !origin || !is_pad) return fail(KLAY_EINVAL, "klay_layer_nodes: null argument");
    if (layer < 0 || layer > c->plan.num_layers) return fail(KLAY_EINVAL, "klay_layer_nodes: layer out of range");
    const klay::LayerPlan& l = c->plan.layers[(size_t)layer];
    std::copy(l.origin.begin(), l.origin.end(), origin);
    std::copy(l.is_pad.begin(), l.is_pad.end(), is_pad);
    return KLAY_OK;
}

klay_status klay_root_positions(const klay_circuit* c, int32_t* position) {
    if (!c || !position) return fail(KLAY_EINVAL, "klay_root_positions: null argument");
    std::copy(c->plan.root_pos.begin(), c->plan.root_pos.end(), position);
    return KLAY_OK;
}

size_t klay_workspace_bytes(const klay_circuit* c, int32_t B, int need_backward) {
    if (!c || B < 1) return 0;
    return workspace_layout(c, B, need_backward != 0).total * sizeof(float);
}

klay_status klay_set_workspace(klay_circuit* c, void* dev_ptr, size_t bytes) {
    if (!c) return fail(KLAY_EINVAL, "klay_set_workspace: null handle");
    if (dev_ptr && (reinterpret_cast<uintptr_t>(dev_ptr) & 255u))
        return fail(KLAY_EINVAL, "klay_set_workspace: pointer must be 256-byte aligned");
    c->ws_user = dev_ptr;
    c->ws_user_bytes = dev_ptr ? bytes : 0;
    c->have_fwd = false;
    return KLAY_OK;
}

klay_status klay_set_profiling(klay_circuit* c, int32_t enable) {
    if (!c) return fail(KLAY_EINVAL, "klay_set_profiling: null handle");
    if (c->device < 0) return fail(KLAY_ESTATE, "klay_set_profiling: host-only handle");
    KLAY_HIP(hipSetDevice(c->device));
    c->profiling = enable != 0;
    if (!c->profiling) release_events(c);
    return KLAY_OK;
}

klay_status klay_get_profile(klay_circuit* c, klay_profile_t* prof) {
    if (!c || !prof) return fail(KLAY_EINVAL, "klay_get_profile: null argument");
    std::memset(prof, 0, sizeof(*prof));
    for (const std::vector<EventRec>* recs : {&c->ev_fwd, &c->ev_bwd})
        for (const EventRec& r : *recs) {
            if (!r.start || !r.stop) continue;
            KLAY_HIP(hipEventSynchronize(r.stop));
            float ms = 0.f;
            KLAY_HIP(hipEventElapsedTime(&ms, r.start, r.stop));
            prof->ms[r.cls] += ms;
            prof->launches[r.cls] += 1;
            prof->alg_bytes[r.cls] += r.bytes;
            prof->min_bytes[r.cls] += r.min_bytes;
        }
    return KLAY_OK;
}

// static_ws: run in the fixed device array instead of the handle's workspace (klay_forward_static):
// no allocation, no event, nothing kept for a backward pass.
static klay_status forward_impl(klay_circuit* c, const float* leaf_weights, const float* neg_weights, int32_t B,
                                float* out, klay_semiring semiring, void* stream, bool static_ws = false) {
    if (!c || !leaf_weights || !out) return fail(KLAY_EINVAL, "klay_forward: null argument");
    if (c->device < 0) return fail(KLAY_ESTATE, "klay_forward: host-only handle (built with device = -1)");
    if (B < 1) return fail(KLAY_EINVAL, "klay_forward: B must be >= 1");
    if (semiring != KLAY_REAL && semiring != KLAY_LOG && semiring != KLAY_MAXLOG)
        return fail(KLAY_EINVAL, "klay_forward: unknown semiring");
    KLAY_HIP(hipSetDevice(c->device));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const klay::CircuitPlan& p = c->plan;
    const Geometry g = geometry(B);
    const bool log_domain = semiring != KLAY_REAL;      // leaf weights are log p in both log-domain semirings
    if (!static_ws && c->profiling && !c->ev_pool.empty()) release_events(c);

    float* ws = nullptr;
    Workspace lay;
    if (!static_ws) c->have_fwd = false;     // a static call leaves the handle's own forward state alone
    // the backward regions are part of the layout whenever the workspace can hold them
    bool with_bwd = true;
    if (static_ws) {
        with_bwd = false;
        lay = workspace_layout(c, B, false);
        if (lay.total * sizeof(float) > kStaticWorkspaceBytes)
            return fail(KLAY_ENOMEM, "klay_forward_static: this circuit at B = " + std::to_string(B) + " needs " +
                                         std::to_string(lay.total * sizeof(float)) + " workspace bytes, the fixed buffer holds " +
                                         std::to_string(kStaticWorkspaceBytes));
        KLAY_HIP(static_workspace(c->device, &ws));
    } else {
        if (c->ws_user && workspace_layout(c, B, true).total * sizeof(float) > c->ws_user_bytes) with_bwd = false;
        klay_status st = get_workspace(c, B, with_bwd, &ws, &lay);
        if (st != KLAY_OK) return st;
    }

    float* act = ws + lay.act;
    float* wT = ws + lay.wT;
    float* seg_rows = ws + lay.seg_rows;
    const int L = p.num_layers;
    const int V = p.num_vars;
    Profiler prof(c, &c->ev_fwd, s, !static_ws);

    // the top layers run in one persistent kernel; when that kernel starts at layer 1 it evaluates the
    // leaf layer itself (a workgroup reads its own rows of the weight arrays)
    const TailChoice tail = choose_tail_fwd(c, B);
    const bool fused_leaf = tail.first == 1;

    // leaf layer
    if (!fused_leaf) {
        prof.begin(KLAY_K_LEAF, 4.0 * B * V + 4.0 * B * (double)(V + p.layers[0].n));
        if (V > 0 && g.ld == B && B <= 32) {
            hipLaunchKernelGGL(klay::leaf_fwd_small_kernel, dim3((unsigned)(((int64_t)V * B + 255) / 256)), dim3(256), 0, s,
                               leaf_weights, neg_weights, (int)B, V, c->d_pos_row, c->d_neg_row, wT, act, log_domain ? 1 : 0);
        } else if (V > 0) {
            dim3 grid((unsigned)((V + 31) / 32), (unsigned)((g.ld + 63) / 64));
            hipLaunchKernelGGL(klay::leaf_fwd_kernel, grid, dim3(256), 0, s, leaf_weights, neg_weights, (int)B, V, g.ld,
                               c->d_pos_row, c->d_neg_row, wT, act, log_domain ? 1 : 0);
        }
        if (c->true_row >= 0)
            hipLaunchKernelGGL(klay::fill_row_kernel, dim3((unsigned)((g.ld + 255) / 256)), dim3(256), 0, s,
                               act + (size_t)c->true_row * g.ld, g.ld, log_domain ? 0.0f : 1.0f);
        if (c->false_row >= 0)
            hipLaunchKernelGGL(klay::fill_row_kernel, dim3((unsigned)((g.ld + 255) / 256)), dim3(256), 0, s,
                               act + (size_t)c->false_row * g.ld, g.ld, log_domain ? -INFINITY : 0.0f);
        prof.end();
    }

    // gate layers: odd = AND, even = OR (Alg. 1 / Alg. 4)
    // The fused plans run where the streaming kernel takes main rows and segments in one launch (two or four
    // columns per lane).
    // A handle whose previous forward pass was followed by klay_backward is in a training loop: the reverse sweep
    // needs every value, so this pass writes them all (klay_backward would otherwise evaluate the fused rows first).
    const bool fused = g.w == 64 && g.vec >= 2 && p.num_fused > 0 && !c->no_fusion &&
                       (static_ws || !c->bwd_followed);
    const int last_regular = tail.first > 0 ? tail.first - 1 : L;
    for (int l = 1; l <= last_regular; ++l) {
        const DevLayer& d = c->dl[(size_t)l];
        const bool is_and = (l & 1) != 0;
        const int or_op = semiring == KLAY_MAXLOG ? klay::OP_MAX : klay::OP_LSE;
        const int op = log_domain ? (is_and ? klay::OP_SUM : or_op) : (is_and ? klay::OP_PROD : klay::OP_SUM);
        const int cls = op == klay::OP_SUM ? KLAY_K_FWD_SUM
                        : op == klay::OP_PROD ? KLAY_K_FWD_PROD
                        : op == klay::OP_MAX ? KLAY_K_FWD_MAX : KLAY_K_FWD_LSE;
        // up to alias_top child entries are rows of the whole buffer, above it of the layer below
        const float* below = l <= p.alias_top ? act : act + (size_t)c->dl[(size_t)l - 1].row0 * g.ld;
        if (fused && is_and && d.n_fused > 0) {
            // the fused rows are not evaluated: the OR rows above read their children
            if (d.has_fwd_kept) run_pass_set(op, op, d.fwd_kept, below, nullptr, nullptr, act + (size_t)d.row0 * g.ld, seg_rows, g, B, s, prof, cls);
        } else if (fused && !is_and && d.has_fwd2) {
            run_pass_set(!log_domain ? klay::OP_SUMPROD2 : semiring == KLAY_MAXLOG ? klay::OP_MAX2 : klay::OP_LSE2, op, d.fwd2, below, nullptr, nullptr,
                         act + (size_t)d.row0 * g.ld, seg_rows, g, B, s, prof, KLAY_K_FWD_OR_FUSED);
        } else {
            run_pass_set(op, op, d.fwd, below, nullptr, nullptr, act + (size_t)d.row0 * g.ld, seg_rows, g, B, s, prof, cls);
        }
    }

    if (tail.first > 0) {
        // the persistent kernel also writes out[B, R]: the top layer is in its LDS
        klay::SlabLeaf leaf{};
        if (fused_leaf) {
            leaf.w = leaf_weights;
            leaf.wneg = neg_weights;
            leaf.leaf_code = c->d_leaf_code;
            leaf.wT = wT;
            leaf.act0 = act;
            leaf.V = V;
            leaf.n0 = (int32_t)p.layers[0].n;
        }
        prof.begin(KLAY_K_TAIL_FWD, tail_alg_bytes(c, tail.first, B, false) + 8.0 * B * p.num_roots,
                   tail_min_bytes(c, tail.first, B, false) + 4.0 * B * p.num_roots);
        launch_tail_fwd(c, tail, act, ws + lay.tb, ws + lay.stage, B, g.ld, (int)semiring, leaf, out, s);
        prof.end();
    } else {
        prof.begin(KLAY_K_ROOT, 8.0 * B * p.num_roots);
        dim3 grid((unsigned)p.num_roots);
        hipLaunchKernelGGL(klay::root_out_kernel, grid, dim3(256), 0, s,
                           act + (size_t)c->dl[(size_t)L].row0 * g.ld, c->d_root_pos, (int)B, p.num_roots, g.ld, out);
        prof.end();
    }
    KLAY_HIP(hipGetLastError());
    if (static_ws) return KLAY_OK;       // the values live in the shared array: nothing to differentiate later
    c->have_fwd = true;
    c->last_fused = fused;
    c->bwd_followed = false;
    c->last_B = B;
    c->last_semiring = semiring;
    c->last_neg_explicit = neg_weights != nullptr;
    c->last_ws_has_bwd = with_bwd;
    c->last_tail_first = tail.first;
    return KLAY_OK;
}

static klay_status backward_impl(klay_circuit* c, const float* dout, float* dleaf, float* dneg, bool lits,
                                 void* stream) {
    if (!c || !dout || !dleaf) return fail(KLAY_EINVAL, "klay_backward: null argument");
    if (c->device < 0) return fail(KLAY_ESTATE, "klay_backward: host-only handle");
    if (!c->have_fwd) return fail(KLAY_ESTATE, "klay_backward: no forward pass to differentiate");
    if (lits != c->last_neg_explicit)
        return fail(KLAY_ESTATE, lits ? "klay_backward_lits: the forward pass was not run by klay_forward_lits with neg_weights"
                                      : "klay_backward: the forward pass had weights for the negated literals; use klay_backward_lits");
    if (c->last_semiring == KLAY_MAXLOG)
        return fail(KLAY_EINVAL, "klay_backward: the (max, +) semiring is not differentiated");
    const bool real = c->last_semiring == KLAY_REAL;
    if (!c->last_ws_has_bwd) return fail(KLAY_ENOMEM, "klay_backward: caller workspace has no room for adjoints");
    KLAY_HIP(hipSetDevice(c->device));
    hipStream_t s = static_cast<hipStream_t>(stream);
    const klay::CircuitPlan& p = c->plan;
    const int B = c->last_B;
    const Geometry g = geometry(B);
    float* ws = nullptr;
    Workspace lay;
    klay_status st = get_workspace(c, B, true, &ws, &lay);
    if (st != KLAY_OK) return st;
    float* act = ws + lay.act;
    float* wT = ws + lay.wT;
    float* seg_rows = ws + lay.seg_rows;
    float* G = ws + lay.g0;
    float* gcur = ws + lay.g1;
    float* gnext = ws + lay.g2;
    const int L = p.num_layers, V = p.num_vars, R = p.num_roots, B0 = p.alias_top;
    Profiler prof(c, &c->ev_bwd, s);
    // Course of the sweep.  The layers above B0 = alias_top are taken one by one, every step gathering the
    // adjoints of layer l - 1 from those of layer l, alternating between two buffers; the step into layer
    // B0 writes into G, which holds one adjoint row per node of the layers 0 .. B0, numbered like the rows
    // of the activation buffer.  Below B0 a layer's rows gather from their parents anywhere in G (all
    // final by then).  The leaf kernel reads the rows of layer 0 at the start of G.
    auto grow = [&](int l) { return G + (size_t)c->dl[(size_t)l].row0 * g.ld; };
    auto values = [&](int l) { return act + (size_t)c->dl[(size_t)l].row0 * g.ld; };

    c->bwd_followed = true;
    if (c->last_fused) {
        // The forward pass ran the fused plans: the values of the fused AND rows, which this sweep needs, were
        // never written.  Evaluate those layers now (all their rows; the others come out the same again).
        for (int l = 1; l < B0; l += 2) {
            const DevLayer& d = c->dl[(size_t)l];
            if (d.n_fused > 0)
                run_pass_set(real ? klay::OP_PROD : klay::OP_SUM, real ? klay::OP_PROD : klay::OP_SUM, d.fwd, act, nullptr, nullptr,
                             values(l), seg_rows, g, B, s, prof, real ? KLAY_K_FWD_PROD : KLAY_K_FWD_SUM);
        }
        c->last_fused = false;
    }

    if (real) {
        // Real semiring: a sum layer passes adjoints through (plain by-child sums).  For a product layer
        // the adjoint rows of its nodes are first turned, in place, into P rows (adjoint times the product
        // of the non-zero children, prod_parent_kernel), and the by-child pass OP_PROD_BWD hands every
        // child its share, using the child's own value.  Nothing is stored per edge.
        klay_status rs = ensure_real_bwd(c);
        if (rs != KLAY_OK) return rs;
        // this sweep runs layer by layer on rows of the activation buffer: bring back the values the
        // persistent forward kernel kept column-major
        if (c->last_tail_first > 0) launch_tb_to_rows(c, c->last_tail_first, L, ws + lay.tb, act, B, g.ld, s);
        // `pre`: the rows arrive premultiplied by the pass that produced them (OP_SUM_P, OP_PROD_BWD_P), and the
        // kernel only repairs the columns whose node value is zero; the seed's rows are plain adjoints
        // flags[l]: raised by the pass that writes the rows of product layer l when it meets a node value of zero
        int* flags = reinterpret_cast<int*>(ws + lay.flags);
        hipLaunchKernelGGL(klay::fill_row_kernel, dim3((unsigned)((L + 256) / 256)), dim3(256), 0, s, ws + lay.flags, L + 1, 0.0f);
        auto prod_parent = [&](int l, const float* below, float* gl, bool pre) {
            const DevLayer& d = c->dl[(size_t)l];
            prof.begin(KLAY_K_PROD_EDGES, pre ? 4.0 : 4.0 * B * ((double)d.e + 2.0 * (double)d.n));
            launch_prod_parent(c->real_layers[(size_t)l], (int)d.n, below, gl, pre ? values(l) : nullptr, flags + l, g, B, s);
            prof.end();
        };
        prof.begin(KLAY_K_SEED, 4.0 * B * R + 4.0 * B * (double)c->dl[(size_t)L].n);
        hipLaunchKernelGGL(klay::seed_kernel, dim3((unsigned)c->dl[(size_t)L].n), dim3(256), 0, s, dout, c->d_top_ptr,
                           c->d_top_root, B, R, g.ld, L == B0 ? grow(L) : gcur, (const uint32_t*)nullptr,
                           (const float*)nullptr);
        prof.end();
        for (int l = L; l > B0; --l) {
            const DevLayer& d = c->dl[(size_t)l];
            float* dst = l - 1 == B0 ? grow(B0) : gnext;
            if ((l & 1) == 0) {
                // into an AND layer: plain sums, leaving premultiplied by the nodes' own values
                run_pass_set(klay::OP_SUM_P, klay::OP_SUM_P, d.bwd, gcur, nullptr, values(l - 1), dst, seg_rows, g, B, s,
                             prof, KLAY_K_BWD_SUM_MUL, flags + (l - 1));
            } else {
                prod_parent(l, values(l - 1), gcur, l != L);
                // the by-child plan of an AND layer carries no weighted bit: every entry is a P row
                run_pass_set(klay::OP_PROD_BWD, klay::OP_SUM, d.bwd, gcur, nullptr, values(l - 1), dst, seg_rows, g, B, s,
                             prof, KLAY_K_BWD_PROD);
            }
            std::swap(gcur, gnext);
        }
        // below B0 the entries of a by-child plan tell P rows (AND parents) from plain adjoint rows
        if (B0 > 0 && (B0 & 1)) prod_parent(B0, act, grow(B0), B0 != L);
        for (int l = B0 - 1; l >= 0; --l) {
            const bool and_rows = (l & 1) != 0;
            run_pass_set(and_rows ? klay::OP_PROD_BWD_P : klay::OP_PROD_BWD, and_rows ? klay::OP_SUM_P : klay::OP_SUM,
                         c->real_layers[(size_t)l].by_child, G, nullptr, values(l), grow(l), seg_rows, g, B, s, prof,
                         and_rows ? KLAY_K_BWD_PROD_MUL : KLAY_K_BWD_PROD, and_rows ? flags + l : nullptr);
            if (and_rows) prod_parent(l, act, grow(l), true);
        }
    } else {
        // The adjoint rows of an OR layer with weighted edges travel in the one-gather form (encode_h): the
        // step that produces them (OP_SUM_H, the seed, or the persistent kernel's last write) folds the
        // node's own value in, and the step through the OR layer (OP_SOFTMAX_H) gathers that one row per
        // edge instead of the adjoint row and the parent's value row.
        const bool one = kOneGather && c->one_gather;
        auto encoded = [&](int l) { return one && l >= 2 && (l & 1) == 0 && c->dl[(size_t)l].has_multi; };

        // the layers the forward pass ran in the persistent kernel are swept by its reverse counterpart,
        // which seeds the adjoints itself and leaves those of its first layer in gcur
        int top = L;
        // (its adjoints of OR nodes are in the one-gather form throughout, so it needs that form to be in use)
        const TailChoice tail = one ? choose_tail_bwd(c, B, c->last_tail_first) : TailChoice();
        if (c->last_tail_first > 0) {
            // the ordinary launches below read values of layers last_tail_first .. top as rows of the
            // activation buffer; the persistent forward kernel kept them column-major
            const int last_needed = tail.first > 0 ? tail.first : L;
            launch_tb_to_rows(c, c->last_tail_first, last_needed, ws + lay.tb, act, B, g.ld, s);
        }
        if (tail.first > 0) {
            prof.begin(KLAY_K_TAIL_BWD, tail_alg_bytes(c, tail.first, B, true) + 4.0 * B * R,
                       tail_min_bytes(c, tail.first, B, true) + 4.0 * B * R);
            launch_tail_bwd(c, tail, ws + lay.tb, dout, gnext, gcur, encoded(L) ? c->dl[(size_t)L].multi : nullptr, B, g.ld, s);
            prof.end();
            top = tail.first;
        } else {
            const bool enc = encoded(L);
            prof.begin(KLAY_K_SEED, 4.0 * B * R + 4.0 * B * (double)c->dl[(size_t)L].n * (enc ? 2.0 : 1.0));
            dim3 grid((unsigned)c->dl[(size_t)L].n);
            hipLaunchKernelGGL(klay::seed_kernel, grid, dim3(256), 0, s, dout, c->d_top_ptr, c->d_top_root, B, R, g.ld,
                               L == B0 ? grow(L) : gcur, enc ? c->dl[(size_t)L].multi : (const uint32_t*)nullptr,
                               enc ? values(L) : (const float*)nullptr);
            prof.end();
        }
        for (int l = top; l > B0; --l) {
            const DevLayer& d = c->dl[(size_t)l];
            float* dst = l - 1 == B0 ? grow(B0) : gnext;
            const bool is_and = (l & 1) != 0 || !d.bwd.has_weighted;   // no weighted edge: plain sums
            if (is_and) {
                const bool enc = encoded(l - 1);
                run_pass_set(enc ? klay::OP_SUM_H : klay::OP_SUM, enc ? klay::OP_SUM_H : klay::OP_SUM, d.bwd, gcur, nullptr,
                             enc ? values(l - 1) : nullptr, dst, seg_rows, g, B, s, prof,
                             enc ? KLAY_K_BWD_SUM_ENC : KLAY_K_BWD_SUM);
            } else if (one) {
                run_pass_set(klay::OP_SOFTMAX_H, klay::OP_SUM, d.bwd, gcur, nullptr, values(l - 1), dst, seg_rows, g, B, s,
                             prof, KLAY_K_BWD_SOFTMAX_ONE);
            } else {
                run_pass_set(klay::OP_SOFTMAX_BWD, klay::OP_SUM, d.bwd, gcur, values(l), values(l - 1), dst, seg_rows, g, B,
                             s, prof, KLAY_K_BWD_SOFTMAX);
            }
            std::swap(gcur, gnext);
        }
        for (int l = B0 - 1; l >= 0; --l) {
            // rows of even layers are OR nodes, whose parents are AND nodes (plain sums; encoded on the way
            // out where the node has more than one child); rows of odd layers and leaves read weighted edges
            const DevPass& dp = c->dl[(size_t)l + 1].bwd;
            const bool enc = encoded(l);
            if (one && (enc || dp.has_weighted))
                run_pass_set(enc ? klay::OP_SUM_H : klay::OP_SOFTMAX_H, enc ? klay::OP_SUM_H : klay::OP_SUM, dp, G, nullptr,
                             values(l), grow(l), seg_rows, g, B, s, prof, enc ? KLAY_K_BWD_SUM_ENC : KLAY_K_BWD_SOFTMAX_ONE);
            else if (dp.has_weighted)
                run_pass_set(klay::OP_SOFTMAX_BWD, klay::OP_SUM, dp, G, act, values(l), grow(l), seg_rows, g, B, s, prof,
                             KLAY_K_BWD_SOFTMAX);
            else
                run_pass_set(klay::OP_SUM, klay::OP_SUM, dp, G, nullptr, nullptr, grow(l), seg_rows, g, B, s, prof,
                             KLAY_K_BWD_SUM);
        }
    }

    prof.begin(KLAY_K_BWD_LEAF, 4.0 * B * (3.0 * V));
    if (V > 0) {
        dim3 grid((unsigned)((V + 31) / 32), (unsigned)((B + 63) / 64));
        hipLaunchKernelGGL(klay::leaf_bwd_kernel, grid, dim3(256), 0, s, G, wT, c->d_pos_row, c->d_neg_row, B, V, g.ld,
                           lits ? 2 : (real ? 0 : 1), dleaf, dneg);
    }
    prof.end();
    KLAY_HIP(hipGetLastError());
    return KLAY_OK;
}

// No C++ exception crosses the C boundary: host allocations of the launch sequences (event records,
// the index arrays of the real-semiring reverse sweep) report KLAY_ENOMEM instead.
klay_status klay_forward(klay_circuit* c, const float* leaf_weights, int32_t B, float* out,
                         klay_semiring semiring, void* stream) {
    return klay_forward_lits(c, leaf_weights, nullptr, B, out, semiring, stream);
}

klay_status klay_forward_lits(klay_circuit* c, const float* pos_weights, const float* neg_weights, int32_t B,
                              float* out, klay_semiring semiring, void* stream) {
    try {
        return forward_impl(c, pos_weights, neg_weights, B, out, semiring, stream);
    } catch (const std::bad_alloc&) {
        if (c) c->have_fwd = false;
        return fail(KLAY_ENOMEM, "klay_forward: out of host memory");
    }
}

klay_status klay_forward_static(klay_circuit* c, const float* leaf_weights, int32_t B, float* out,
                                klay_semiring semiring, void* stream) {
    try {
        return forward_impl(c, leaf_weights, nullptr, B, out, semiring, stream, true);
    } catch (const std::bad_alloc&) {
        return fail(KLAY_ENOMEM, "klay_forward_static: out of host memory");
    }
}

klay_status klay_backward(klay_circuit* c, const float* dout, float* dleaf, void* stream) {
    try {
        return backward_impl(c, dout, dleaf, nullptr, false, stream);
    } catch (const std::bad_alloc&) {
        return fail(KLAY_ENOMEM, "klay_backward: out of host memory");
    }
}

klay_status klay_backward_lits(klay_circuit* c, const float* dout, float* dpos, float* dneg, void* stream) {
    try {
        return backward_impl(c, dout, dpos, dneg, true, stream);
    } catch (const std::bad_alloc&) {
        return fail(KLAY_ENOMEM, "klay_backward_lits: out of host memory");
    }
}

klay_status klay_forward_f64(klay_circuit* c, const double* pos_weights, const double* neg_weights, int32_t B,
                             double* out, klay_semiring semiring, void* stream) {
    try {
        return forward64_impl(c, pos_weights, neg_weights, B, out, semiring, stream);
    } catch (const std::bad_alloc&) {
        if (c) c->have_fwd64 = false;
        return fail(KLAY_ENOMEM, "klay_forward_f64: out of host memory");
    }
}

klay_status klay_backward_f64(klay_circuit* c, const double* dout, double* dpos, double* dneg, void* stream) {
    try {
        return backward64_impl(c, dout, dpos, dneg, stream);
    } catch (const std::bad_alloc&) {
        return fail(KLAY_ENOMEM, "klay_backward_f64: out of host memory");
    }
}

}  // extern "C"
