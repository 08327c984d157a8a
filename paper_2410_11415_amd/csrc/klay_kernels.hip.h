// Device kernels of the layered circuit evaluator for gfx950 (wave64).
//
// Data layout: every layer's node values live in one activation buffer, row = node,
// `ld` consecutive floats per row = the batch (batch-inner), so the gather of one edge
// (paper Section 4: E_l = N_{l-1}[S_l]) is one contiguous read of B floats.  A layer is
// evaluated by a fused gather + segment-reduce (Alg. 1 / Alg. 4 without materialising E_l,
// M or T): a lane group of W lanes owns one parent row and VEC consecutive batch columns per
// lane, loops over the row's CSR range and keeps the reduction in registers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "layerize.h"

namespace klay {

enum PassOp : int { OP_SUM = 0, OP_PROD = 1, OP_LSE = 2, OP_SOFTMAX_BWD = 3, OP_MAX = 4, OP_PROD_BWD = 5, OP_SUM_H = 6, OP_SOFTMAX_H = 7,
                    OP_SUM_P = 8, OP_PROD_BWD_P = 9,
                    // over the fused plans (see LayerPlan::fwd2): an OR row whose children are groups of entries
                    // (sum within a group, then logsumexp / max over the groups; real semiring: product within a
                    // group, then the sum of the groups)
                    OP_LSE2 = 10, OP_MAX2 = 11, OP_SUMPROD2 = 12 };
// what the ops have in common: `own` = the walk needs the value of the output row itself, `additive` = partial
// results add up
template <int OP> struct OpTraits {
    static constexpr bool own = OP == OP_SOFTMAX_BWD || OP == OP_PROD_BWD || OP == OP_SUM_H || OP == OP_SOFTMAX_H ||
                                OP == OP_SUM_P || OP == OP_PROD_BWD_P;
    static constexpr bool additive = OP == OP_SUM || own;
    static constexpr bool premul = OP == OP_SUM_P || OP == OP_PROD_BWD_P;      // the row leaves multiplied by its own value
    static constexpr bool shares = OP == OP_PROD_BWD || OP == OP_PROD_BWD_P;   // entries are P rows of AND parents
    // a segment of a split row needs the value of the row that owns it (the others only use it to finish a row)
    static constexpr bool seg_own = OP == OP_SOFTMAX_BWD || OP == OP_SOFTMAX_H || shares;
};

// Index entries: bits 0..28 = source row, bit 31 = last edge of its output row, bit 30 = weighted
// edge (reverse sweep only: the parent is an OR node with more than one child, so the adjoint
// passes through the softmax weight exp(child - parent); an unweighted edge passes it unchanged),
// bit 29 (on the last entry of a row only) = the output row is an OR node with more than one child, whose
// adjoint is stored in the one-gather form (see encode_h).
// kSkip (all ones) stands for a whole output row that this pass leaves untouched (a split row).
constexpr uint32_t kLast = kLastEdge, kWeighted = kWeightedEdge, kSkip = kSkipRow, kIdMask = kRowFlag - 1u;

struct PassArgs {
    const int32_t* ptr;        // [n_total + 1] CSR offsets into idx
    const uint32_t* idx;       // index entries (readable up to 16 entries past the end)
    const float* src;          // [*, ld] source rows (values of the layer below, adjoints, or partials)
    const float* src2;         // OP_SOFTMAX_BWD: values N_l of the parents, same row index as src
    const float* own;          // ops with OpTraits::own: values of the output rows themselves
    const int32_t* seg_owner;  // output row owning segment i (rows >= n_main), may be null
    const int32_t* out_row;    // optional output row map for rows < n_main (combine pass)
    float* dst;                // output rows for rows < n_main
    float* dst_seg;            // scratch rows for rows >= n_main
    int32_t row_begin;         // first row this launch evaluates
    int32_t n_main;
    int32_t n_total;
    int32_t B;
    int32_t ld;
    int32_t iters;             // row groups per wave
    int* zero_flag;            // OP_SUM_P, OP_PROD_BWD_P: set to 1 when an output row's own value is zero in some column
};

// s_waitcnt immediate (gfx9 encoding: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8) that waits
// for vmcnt = 0 only: expcnt and lgkmcnt keep their maxima (7 and 15), so scalar loads stay in flight.
constexpr int kWaitVmcnt0 = 0x0F70;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// exp and log on the transcendental unit (v_exp_f32 / v_log_f32 are base 2).  Arguments of
// fexp are <= 0 here, so the rounding of x*log2(e) costs at most |x| e^x 2^-24 absolute.
__device__ __forceinline__ float fexp(float x) { return __builtin_amdgcn_exp2f(x * kLog2e); }
__device__ __forceinline__ float flog(float x) { return __builtin_amdgcn_logf(x) * kLn2; }

template <int VEC> struct Pack;
template <> struct Pack<1> { using T = float; };
template <> struct Pack<2> { using T = float2; };
template <> struct Pack<4> { using T = float4; };

template <int VEC>
__device__ __forceinline__ void load_vec(float (&x)[VEC], const float* p) {
    using T = typename Pack<VEC>::T;
    T t = *reinterpret_cast<const T*>(p);
    const float* f = reinterpret_cast<const float*>(&t);
#pragma unroll
    for (int v = 0; v < VEC; ++v) x[v] = f[v];
}

// Streaming store: the rows of a wide layer are written once and next read by another kernel,
// long after they have left the 4 MB L2, so they are marked non-temporal to leave the L2 to the
// gathers.  Narrow layers keep ordinary stores: their rows are still in L2 when the next layer reads.
template <int VEC>
__device__ __forceinline__ void store_vec_stream(float* p, const float (&x)[VEC]) {
    typedef float vf __attribute__((ext_vector_type(VEC)));
    vf t;
#pragma unroll
    for (int v = 0; v < VEC; ++v) t[v] = x[v];
    __builtin_nontemporal_store(t, reinterpret_cast<vf*>(p));
}
template <>
__device__ __forceinline__ void store_vec_stream<1>(float* p, const float (&x)[1]) {
    __builtin_nontemporal_store(x[0], p);
}

template <int VEC>
__device__ __forceinline__ void store_vec(float* p, const float (&x)[VEC]) {
    using T = typename Pack<VEC>::T;
    T t;
    float* f = reinterpret_cast<float*>(&t);
#pragma unroll
    for (int v = 0; v < VEC; ++v) f[v] = x[v];
    *reinterpret_cast<T*>(p) = t;
}

// Workgroups are handed to the 8 XCDs round-robin; give each XCD a contiguous eighth of the
// rows so that neighbouring rows (which read neighbouring children) share one L2.  The grid's
// x extent is a multiple of 8.  (Measured on the headline workload: 4% of the step, and 28% of
// the time of the split-row segments, which are ordered by the rows they read.)
__device__ __forceinline__ int xcd_block(int bid, int nblocks) { return (bid & 7) * (nblocks >> 3) + (bid >> 3); }

// One step of the streaming reductions.  acc/mx carry the state of the current output row:
//   OP_SUM / OP_PROD  acc = running sum / product
//   OP_MAX            acc = running maximum (OR layers of the (max, +) semiring)
//   OP_LSE            (mx, acc) = (running max, sum of exp(x - mx)); one exp per element:
//                     a new maximum rescales the sum by exp(mx - x), otherwise exp(x - mx) is added
//   OP_SOFTMAX_BWD    acc += g * exp(own - parent value) on weighted edges (a parent at -inf
//                     passes nothing down), acc += g on unweighted ones
//   OP_PROD_BWD       real-semiring reverse sweep: x is the row that prod_parent_kernel left for an AND
//                     parent r, P_r = G_r * (product of r's non-zero children), with the lowest mantissa
//                     bit telling whether r has exactly one zero child (rows with more are all zero).
//                     The child with value `own` gets P_r / own when r has no zero child, P_r when the
//                     child is r's one zero, nothing otherwise.  A weighted entry is a plain adjoint row
//                     (a sum node above, or a root's dout row) and is added as it is.
//   OP_SUM_P, OP_PROD_BWD_P   OP_SUM / OP_PROD_BWD whose output rows are AND nodes: the finished adjoint G
//                     leaves as G * (the node's own value), lowest mantissa bit clear, which is the row P
//                     above whenever the node has no zero child; where the own value is zero G is left
//                     as it is for prod_parent_kernel to deal with (see there).
// One-gather form of the softmax adjoint (log semiring, reverse sweep through an OR layer).  The adjoint
// G_r of an OR node r with more than one child only ever reaches its children as G_r exp(N_c - N_r), so
// the pass that produces G_r (OP_SUM_H: a plain sum, finished with the node's own value N_r) stores
//   H_r = log|G_r| - N_r, with the sign of G_r in the lowest mantissa bit (-inf when G_r = 0 or N_r = -inf),
// and the pass through the OR layer (OP_SOFTMAX_H) gathers that one row per edge and adds
// +-exp(H_r + N_c): N_c <= N_r, so nothing overflows.  Rows of single-child OR nodes (and chain nodes)
// keep the plain adjoint; their edges are the unweighted ones and pass it unchanged.
__device__ __forceinline__ float encode_h(float g, float n) {
    const bool none = g == 0.0f || n == -INFINITY;
    const float h = none ? -INFINITY : flog(fabsf(g)) - n;
    return __uint_as_float((__float_as_uint(h) & ~1u) | ((g < 0.0f && !none) ? 1u : 0u));
}
__device__ __forceinline__ float decode_h(float hbits, float nc) {
    const uint32_t b = __float_as_uint(hbits);
    const float v = fexp(__uint_as_float(b & ~1u) + nc);
    return __uint_as_float(__float_as_uint(v) | (b << 31));      // v >= 0: the stored sign bit goes on with one shift-or
}

__device__ __forceinline__ float premultiply(float g, float n) {
    return n != 0.0f ? __uint_as_float(__float_as_uint(g * n) & ~1u) : g;
}

// one element of a running logsumexp: (mx, acc) = (maximum so far, sum of exp(x - mx)), one exp per element
__device__ __forceinline__ void lse_step(float& acc, float& mx, float x) {
    // d is +inf on the first finite element (e = 0, acc = 1), -inf for an impossible child under a finite
    // maximum (e = 0), and NaN only for -inf - -inf, where the maximum of NaN and 0 is 0 and the comparison fails
    const float d = x - mx;
    const float e = fmaxf(fexp(-fabsf(d)), 0.0f);
    const bool up = d > 0.0f;                                 // the same as x > mx
    acc = up ? fmaf(acc, e, 1.0f) : acc + e;
    mx = up ? x : mx;
}

// nc: the value of the output row itself where the operation needs it; OP_LSE2 / OP_MAX2 keep the sum of the
// group in hand there (weighted = the entry closes its group).
template <int OP>
__device__ __forceinline__ void accumulate(float& acc, float& mx, float x, float y, float& nc, bool weighted = true) {
    if (OP == OP_SUM_H || OP == OP_SUM_P) { acc += x; return; }
    if (OP == OP_SOFTMAX_H) { acc += weighted ? decode_h(x, nc) : x; return; }
    if (OP == OP_SUMPROD2) {
        nc *= x;
        if (weighted) { acc += nc; nc = 1.0f; }
        return;
    }
    if (OP == OP_LSE2 || OP == OP_MAX2) {
        nc += x;
        if (weighted) {
            if (OP == OP_LSE2) lse_step(acc, mx, nc);
            else acc = nc > acc ? nc : acc;
            nc = 0.0f;
        }
        return;
    }
    if (OpTraits<OP>::shares) {
        const uint32_t bits = __float_as_uint(x);
        const float val = __uint_as_float(bits & ~1u);
        const bool one_zero = (bits & 1u) != 0;
        const float part = one_zero ? (nc == 0.0f ? val : 0.0f) : (nc != 0.0f ? val / nc : 0.0f);
        acc += weighted ? x : part;
        return;
    }
    if (OP == OP_SUM) acc += x;
    else if (OP == OP_PROD) acc *= x;
    else if (OP == OP_MAX) acc = x > acc ? x : acc;               // no NaN reaches here: two instructions, fmaxf takes three
    else if (OP == OP_LSE) lse_step(acc, mx, x);
    else {
        const float wgt = !weighted ? 1.0f : ((y == -INFINITY) ? 0.0f : fexp(nc - y));
        acc = fmaf(x, wgt, acc);
    }
}

template <int OP>
__device__ __forceinline__ float finish(float acc, float mx) {
    if (OP == OP_LSE || OP == OP_LSE2) return (mx == -INFINITY) ? -INFINITY : mx + flog(acc);
    return acc;
}

template <int OP>
__device__ __forceinline__ float identity() { return OP == OP_PROD ? 1.0f : ((OP == OP_MAX || OP == OP_MAX2) ? -INFINITY : 0.0f); }

// what an index entry that is not part of the row contributes: nothing
template <int OP>
__device__ __forceinline__ float dead_value() {
    return (OP == OP_PROD || OP == OP_SUMPROD2) ? 1.0f : ((OP == OP_LSE || OP == OP_MAX) ? -INFINITY : 0.0f);
}

// ---------------------------------------------------------------------------------------------
// Streaming segmented gather-reduce for B > 32 (one wave spans the batch tile, VEC columns per
// lane).  A task is a run of consecutive output rows with a bounded number of edges, fixed at
// build time; the wave walks the task's edges in chunks of CH, keeps CH row gathers in flight,
// prefetches the next chunk's index entries while they fly, and closes an output row whenever
// an entry carries the end-of-row bit.  Everything that steers control flow is wave-uniform.
// Index entries past a task's end are valid entries of later rows (or zero padding).
// ---------------------------------------------------------------------------------------------
// bx of nbx: the workgroup's place among the workgroups that walk tasks (nbx a multiple of 8, bx mod 8 the XCD
// the workgroup runs on).
template <int OP, int VEC>
__device__ __forceinline__ void stream_body(int bx, int nbx, const int2* __restrict__ tasks, int n_tasks,
                                            const uint32_t* __restrict__ idx, const float* __restrict__ src,
                                            const float* __restrict__ src2, const float* __restrict__ own,
                                            float* __restrict__ dst, int B, int ld, int stream_stores,
                                            const int2* __restrict__ seg_tasks, int n_seg_tasks,
                                            float* __restrict__ dst_seg, const int32_t* __restrict__ seg_owner,
                                            int n_main, int* __restrict__ zero_flag) {
    // entries per chunk: measured on the headline workload, 4 (2 for the softmax adjoint, which loads
    // three rows per entry) beat 8 / 4 by 2%: the kernel is bandwidth-bound, fewer registers per wave
    // buy more resident waves
    // With one column per lane (B <= 64) a row is 256 bytes and twice as many have to be in flight:
    // 8 (4) measured 3% faster on the power-law workload at B = 64, 4% on the headline circuit at B = 64.
    constexpr int CH = (OP == OP_SOFTMAX_BWD) ? (VEC == 1 ? 4 : 2) : (VEC == 1 ? 8 : 4);
    static_assert(kGroupEnd == kWeighted, "the fused plans reuse this bit");
    // the walk needs the output row's own value
    constexpr bool OWN = OpTraits<OP>::own;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = ((int)blockIdx.y * 64 + lane) * VEC;
    if (col >= B) return;
    int t = xcd_block(bx, nbx) * 4 + wave;
    if (t >= n_tasks + n_seg_tasks) return;
    // tasks past the main list are segments of split rows: same walk, output rows go to scratch
    // (dst_seg is shifted so that segment row numbers, which continue after the main rows, index it)
    const bool seg = t >= n_tasks;
    if (seg) { t -= n_tasks; tasks = seg_tasks; dst = dst_seg; stream_stores = 0; }
    const int2 t0 = tasks[t], t1 = tasks[t + 1];
    int row = t0.x;
    int j = t0.y;
    const int e1 = t1.y;
    const int last_row = t1.x - 1;
    const float* srcc = src + col;
    const float* src2c = src2 + col;
    const float* ownc = own + col;
    float* dstc = dst + col;

    float acc[VEC], mx[VEC], nc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) { acc[v] = identity<OP>(); mx[v] = -INFINITY; nc[v] = OP == OP_SUMPROD2 ? 1.0f : 0.0f; }
    bool fresh = true;                       // the next edge opens a new output row
    uint32_t ids[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) ids[i] = idx[j + i];

    while (j < e1) {
        const int n = e1 - j;
        int rws[CH];
        bool first[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            rws[i] = row;
            first[i] = fresh;
            if (i < n) {
                fresh = (ids[i] & kLast) != 0;
                row += fresh ? 1 : 0;
            }
        }
        // All CH gathers are issued unconditionally (entries past the task's end or kSkip are
        // redirected to valid rows and their data ignored): loads under wave-uniform branches
        // would make the compiler drain the memory pipeline before each of them.
        float x[CH][VEC], y[CH][VEC], z[CH][VEC];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const uint32_t srow = (ids[i] == kSkip) ? 0u : (ids[i] & kIdMask);
            const size_t off = (size_t)srow * (size_t)ld;
            load_vec<VEC>(x[i], srcc + off);
            if (OP == OP_SOFTMAX_BWD) {
                // an unweighted edge needs no parent value: re-read the row just requested (an L1 hit)
                load_vec<VEC>(y[i], ((ids[i] & kWeighted) && ids[i] != kSkip ? src2c : srcc) + off);
            }
            if (OWN) {
                // (a segment of a split row works with the value of the row that owns it, if with any)
                int orow = rws[i] < last_row ? rws[i] : last_row;
                if (seg) orow = OpTraits<OP>::seg_own ? seg_owner[orow - n_main] : 0;
                load_vec<VEC>(z[i], ownc + (size_t)orow * (size_t)ld);
            }
        }
        uint32_t nxt[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) nxt[i] = idx[j + CH + i];       // padded: always readable
        // s_waitcnt vmcnt(0) (scalar prefetch left in flight): the gathers are complete on every
        // path from here on, so no later register reuse has to wait on them again.
        __builtin_amdgcn_s_waitcnt(kWaitVmcnt0);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            // branch-free accumulation: a dead entry contributes the identity
            const bool live = (i < n) && (ids[i] != kSkip);
            if (OWN) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) nc[v] = (live && first[i]) ? z[i][v] : nc[v];
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const float xv = live ? x[i][v] : dead_value<OP>();
                const float yv = OP == OP_SOFTMAX_BWD ? (live ? y[i][v] : -INFINITY) : 0.0f;
                accumulate<OP>(acc[v], mx[v], xv, yv, nc[v], live && (ids[i] & kWeighted) != 0);
            }
            if (live && (ids[i] & kLast)) {
                float o[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    o[v] = finish<OP>(acc[v], mx[v]);
                    // the adjoint of an OR node with more than one child leaves in the one-gather form
                    if (OP == OP_SUM_H && !seg && (ids[i] & kRowFlag)) o[v] = encode_h(o[v], nc[v]);
                    if (OpTraits<OP>::premul && !seg) {
                        if (nc[v] == 0.0f && zero_flag) *zero_flag = 1;          // this layer needs prod_parent_kernel's repair
                        o[v] = premultiply(o[v], nc[v]);
                    }
                    acc[v] = identity<OP>();
                    mx[v] = -INFINITY;
                }
                if (stream_stores) store_vec_stream<VEC>(dstc + (size_t)rws[i] * (size_t)ld, o);
                else store_vec<VEC>(dstc + (size_t)rws[i] * (size_t)ld, o);
            }
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) ids[i] = nxt[i];
        j += CH;
    }
}

template <int OP, int VEC>
__global__ __launch_bounds__(256) void stream_kernel(const int2* __restrict__ tasks, int n_tasks,
                                                     const uint32_t* __restrict__ idx,
                                                     const float* __restrict__ src,
                                                     const float* __restrict__ src2,
                                                     const float* __restrict__ own, float* __restrict__ dst,
                                                     int B, int ld, int stream_stores,
                                                     const int2* __restrict__ seg_tasks, int n_seg_tasks,
                                                     float* __restrict__ dst_seg,
                                                     const int32_t* __restrict__ seg_owner, int n_main,
                                                     int* __restrict__ zero_flag) {
    stream_body<OP, VEC>((int)blockIdx.x, (int)gridDim.x, tasks, n_tasks, idx, src, src2, own, dst, B, ld, stream_stores,
                         seg_tasks, n_seg_tasks, dst_seg, seg_owner, n_main, zero_flag);
}

// ---------------------------------------------------------------------------------------------
// Small batches (B <= 32): lanes = edges.  A lane group of LPR lanes (B rounded up to a power of two)
// holds one index entry, its lanes the batch columns, so a wave takes EPW = 64 / LPR consecutive entries
// per step (all 64 at B = 1): one coalesced read of the entries, one gather of their rows, and the
// entries of an output row, which sit in neighbouring lane groups, are reduced across the wave:
//   - a step in which no row ends only accumulates, every lane group into a partial of its own;
//   - a step in which rows end folds those partials into one (butterfly over the lane groups), adds
//     it to the first lane group, and runs a segmented inclusive scan over the lane groups (wave
//     shuffles; a lane knows its segment's start from the ballot of the end-of-row bits, so only values
//     travel); the lane groups that hold a row's last entry store the row, the part of a row that is
//     still open stays behind as the last lane group's partial.
// Same task lists and index entries as the streaming kernel (a wave takes `span` consecutive tasks);
// tasks past the main list are the segments of split rows.  The log-domain OR reduction travels as
// (maximum, sum of exp(x - maximum)) pairs.
// ---------------------------------------------------------------------------------------------
template <int OP>
__device__ __forceinline__ void edge_combine(float& am, float& as, float bm, float bs) {
    if (OpTraits<OP>::additive) am += bm;
    else if (OP == OP_PROD) am *= bm;
    else if (OP == OP_MAX) am = fmaxf(am, bm);
    else {
        const float M = fmaxf(am, bm);
        const float ea = (am == -INFINITY) ? 0.0f : fexp(am - M);
        const float eb = (bm == -INFINITY) ? 0.0f : fexp(bm - M);
        as = as * ea + bs * eb;
        am = M;
    }
}

template <int OP, int LPR>
__global__ __launch_bounds__(256) void edge_kernel(const int2* __restrict__ tasks, int n_tasks, int span,
                                                   const uint32_t* __restrict__ idx, const float* __restrict__ src,
                                                   const float* __restrict__ src2, const float* __restrict__ own,
                                                   float* __restrict__ dst, int B, int ld,
                                                   const int2* __restrict__ seg_tasks, int n_seg_tasks,
                                                   const int32_t* __restrict__ seg_owner, int n_main,
                                                   float* __restrict__ dst_seg, int* __restrict__ zero_flag) {
    constexpr int EPW = 64 / LPR;                 // entries per step
    constexpr int CH = EPW >= 16 ? 4 : 8;         // steps whose gathers are in flight together
    constexpr bool LSE = OP == OP_LSE;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int sub = lane / LPR, c = lane % LPR;
    const bool active = c < B;
    const int cc = active ? c : B - 1;            // lanes past the batch re-read its last column and store nothing
    const int n_main_waves = (n_tasks + span - 1) / span;
    int wt = (int)blockIdx.x * 4 + wave;
    bool seg = false;
    if (wt >= n_main_waves) {
        wt -= n_main_waves;
        seg = true;
        tasks = seg_tasks;
        n_tasks = n_seg_tasks;
        dst = dst_seg;
    }
    const int t0 = wt * span;
    if (t0 >= n_tasks) return;
    const int t1 = t0 + span < n_tasks ? t0 + span : n_tasks;
    const int2 ta = tasks[t0], tb = tasks[t1];
    int row = ta.x;
    const int e1 = tb.y;
    float accm = identity<OP>(), accs = 0.0f;     // this lane group's partial of the open row
    if (LSE) accm = -INFINITY;
    int state = 0;     // partials: 0 none holds anything, 1 only the last lane group's does, 2 any may
    for (int j = ta.y; j < e1; j += CH * EPW) {
        uint32_t id[CH];
        bool in[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int pos = j + i * EPW + sub;
            in[i] = pos < e1;
            id[i] = idx[in[i] ? pos : e1 - 1];
        }
        // rows of the entries: the open row plus the rows that end before them
        unsigned long long lm[CH], below[CH];
        int rowidx[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const bool last = in[i] && (id[i] & kLast) != 0;
            lm[i] = __builtin_amdgcn_ballot_w64(last && c == 0);
            below[i] = lm[i] & ((1ull << (sub * LPR)) - 1ull);
            rowidx[i] = row + __builtin_popcountll(below[i]);
            row += __builtin_popcountll(lm[i]);
        }
        float x[CH], y[CH], z[CH];
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const bool live = in[i] && id[i] != kSkip;
            const size_t off = (size_t)(live ? (id[i] & kIdMask) : 0u) * (size_t)ld + cc;
            x[i] = src[off];
            y[i] = 0.0f;
            z[i] = 0.0f;
            if (OpTraits<OP>::own) {
                const bool weighted = live && (id[i] & kWeighted) != 0;
                // value of the parent, and of the row the entry belongs to (a segment: of its owner)
                if (OP == OP_SOFTMAX_BWD) y[i] = (weighted ? src2 : src)[off];
                int orow = live ? rowidx[i] : (seg ? n_main : 0);      // an entry past the task's end has no row
                if (seg) orow = seg_owner[orow - n_main];
                z[i] = own[(size_t)orow * (size_t)ld + cc];
            }
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const bool live = in[i] && id[i] != kSkip;
            const bool last = in[i] && (id[i] & kLast) != 0;
            float vm, vs = 0.0f;
            if (OP == OP_SOFTMAX_BWD) {
                const bool weighted = live && (id[i] & kWeighted) != 0;
                const float wgt = !weighted ? 1.0f : ((y[i] == -INFINITY) ? 0.0f : fexp(z[i] - y[i]));
                vm = live ? x[i] * wgt : 0.0f;
            } else if (OP == OP_SOFTMAX_H) {
                vm = live ? ((id[i] & kWeighted) ? decode_h(x[i], z[i]) : x[i]) : 0.0f;
            } else if (OpTraits<OP>::shares) {
                float part = 0.0f, unused = 0.0f;
                accumulate<OP_PROD_BWD>(part, unused, x[i], 0.0f, z[i], (id[i] & kWeighted) != 0);
                vm = live ? part : 0.0f;
            } else if (LSE) {
                vm = live ? x[i] : -INFINITY;
                vs = live ? 1.0f : 0.0f;
            } else {
                vm = live ? x[i] : dead_value<OP>();
            }
            if (lm[i] == 0ull) {                      // no row ends in this step
                edge_combine<OP>(accm, accs, vm, vs);
                state = 2;
                continue;
            }
            if (state == 2) {                         // fold the partials of all lane groups
#pragma unroll
                for (int d = LPR; d < 64; d <<= 1) {
                    const float om = __shfl_xor(accm, d), os = LSE ? __shfl_xor(accs, d) : 0.0f;
                    edge_combine<OP>(accm, accs, om, os);
                }
            } else if (state == 1) {                  // only the last lane group holds one
                accm = __shfl(accm, (EPW - 1) * LPR + c);
                if (LSE) accs = __shfl(accs, (EPW - 1) * LPR + c);
            }
            if (sub == 0) edge_combine<OP>(vm, vs, accm, accs);
            // segmented inclusive scan over the lane groups: a segment starts after every end of row
            const int start = below[i] ? (63 - __builtin_clzll(below[i])) / LPR + 1 : 0;
            const int dist = sub - start;
#pragma unroll
            for (int d = 1; d < EPW; d <<= 1) {
                const float om = __shfl_up(vm, d * LPR), os = LSE ? __shfl_up(vs, d * LPR) : 0.0f;
                if (dist >= d) edge_combine<OP>(vm, vs, om, os);
            }
            if (last && live && active) {
                float o = vm;
                if (LSE) o = (vm == -INFINITY) ? -INFINITY : vm + flog(vs);
                if (OP == OP_SUM_H && !seg && (id[i] & kRowFlag)) o = encode_h(o, z[i]);
                if (OpTraits<OP>::premul && !seg) {
                    if (z[i] == 0.0f && zero_flag) *zero_flag = 1;
                    o = premultiply(o, z[i]);
                }
                dst[(size_t)rowidx[i] * (size_t)ld + c] = o;
            }
            // the open row's part stays with the last lane group
            const bool tail_last = ((lm[i] >> ((EPW - 1) * LPR)) & 1ull) != 0ull;
            const bool keep = sub == EPW - 1 && !tail_last;
            accm = keep ? vm : (LSE ? -INFINITY : identity<OP>());
            accs = keep ? vs : 0.0f;
            state = tail_last ? 0 : 1;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Generic gather-reduce: a lane group of W lanes owns one output row (W < 64: several rows per
// wave, for small batches).  Also evaluates the segments of split rows (rows >= n_main, written
// to scratch rows) and the combine pass (out_row map).
// ---------------------------------------------------------------------------------------------
template <int OP, int VEC, int W>
__global__ __launch_bounds__(256) void pass_kernel(PassArgs a) {
    constexpr int RPW = 64 / W;                       // rows per wave
    constexpr int CH = (OP == OP_SOFTMAX_BWD) ? 4 : 8;    // sources in flight per lane
    constexpr bool OWN = OpTraits<OP>::own;
    const int lane = threadIdx.x & 63;
    int wave = threadIdx.x >> 6;
    if (W == 64) wave = __builtin_amdgcn_readfirstlane(wave);
    const int sub = (W == 64) ? 0 : lane / W;
    const int col = ((int)blockIdx.y * W + (lane % W)) * VEC;
    if (col >= a.B) return;
    const int blk = xcd_block((int)blockIdx.x, (int)gridDim.x);
    const int64_t first_group = ((int64_t)blk * 4 + wave) * a.iters;

    for (int it = 0; it < a.iters; ++it) {
        const int64_t row64 = (first_group + it) * RPW + sub + a.row_begin;
        if (row64 >= a.n_total) break;
        const int row = (int)row64;
        const int beg = a.ptr[row], end = a.ptr[row + 1];
        if (a.idx[beg] == kSkip) continue;            // split row: evaluated by segments + combine

        float nc[VEC];                                // OP_SOFTMAX_BWD: own value
#pragma unroll
        for (int v = 0; v < VEC; ++v) nc[v] = 0.0f;
        if (OWN) {
            // the row whose value this output belongs to: itself, the row a combine pass writes, or a segment's owner
            const int owner = row < a.n_main ? (a.out_row ? a.out_row[row] : row) : a.seg_owner[row - a.n_main];
            load_vec<VEC>(nc, a.own + (size_t)owner * a.ld + col);
        }
        float acc[VEC], mx[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) { acc[v] = identity<OP>(); mx[v] = -INFINITY; }

        for (int j = beg; j < end; j += CH) {
            const int n = end - j;
            uint32_t id[CH];
            bool wt[CH];
#pragma unroll
            for (int i = 0; i < CH; ++i) {                                    // padded array: always in bounds
                const uint32_t raw = a.idx[j + i];
                id[i] = raw == kSkip ? 0u : (raw & kIdMask);
                wt[i] = (raw & kWeighted) != 0;
            }
            // all gathers are issued unconditionally: entries past the row's end are valid entries of
            // later rows (or zero padding); their data is ignored below
            float x[CH][VEC], y[CH][VEC];
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                load_vec<VEC>(x[i], a.src + (size_t)id[i] * a.ld + col);
                if (OP == OP_SOFTMAX_BWD) load_vec<VEC>(y[i], (wt[i] ? a.src2 : a.src) + (size_t)id[i] * a.ld + col);
            }
            // branch-free accumulation (a conditional use would let the compiler sink each load into
            // its branch and serialise the gathers): a dead entry contributes the identity
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const bool live = i < n;
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const float dead = OP == OP_PROD ? 1.0f : ((OP == OP_LSE || OP == OP_MAX) ? -INFINITY : 0.0f);
                    const float xv = live ? x[i][v] : dead;
                    const float yv = OP == OP_SOFTMAX_BWD ? (live ? y[i][v] : -INFINITY) : 0.0f;
                    accumulate<OP>(acc[v], mx[v], xv, yv, nc[v], live && wt[i]);
                }
            }
        }
        float o[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) o[v] = finish<OP>(acc[v], mx[v]);
        if (OP == OP_SUM_H && row < a.n_main && (a.idx[end - 1] & kRowFlag)) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) o[v] = encode_h(o[v], nc[v]);
        }
        if (OpTraits<OP>::premul && row < a.n_main) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                if (nc[v] == 0.0f && a.zero_flag) *a.zero_flag = 1;
                o[v] = premultiply(o[v], nc[v]);
            }
        }
        float* out;
        if (row < a.n_main) out = a.dst + (size_t)(a.out_row ? a.out_row[row] : row) * a.ld + col;
        else out = a.dst_seg + (size_t)(row - a.n_main) * a.ld + col;
        store_vec<VEC>(out, o);
    }
}

// ---------------------------------------------------------------------------------------------
// Combine pass of split rows for B > 32: one workgroup of NW waves per split row.  The partial rows of a
// split row (up to a few hundred for the widest rows) are dealt to the waves in chunks of 8, every wave
// reduces its share with all its gathers of a chunk in flight, and wave 0 folds the NW states in wave
// order (so the result does not depend on timing) and finishes the row like pass_kernel does.  A single
// wave would walk the widest row 8 partial rows at a time, and the launch lasts as long as that walk.
// Arguments as for pass_kernel's combine use: ptr / idx = combine lists, src = partial rows, out_row = the
// rows to write, n_main = number of split rows.
// ---------------------------------------------------------------------------------------------
template <int OP, int VEC, int NW>
__device__ __forceinline__ void combine_body(int row, const PassArgs& a) {
    constexpr int CH = 8;
    constexpr bool LSE = OP == OP_LSE;
    __shared__ float part_v[NW][64 * VEC];
    __shared__ float part_m[LSE ? NW : 1][LSE ? 64 * VEC : 1];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int colu = ((int)blockIdx.y * 64 + lane) * VEC;
    const int col = colu < a.B ? colu : 0;                 // lanes past the batch work on column 0 and store nothing
    const int beg = a.ptr[row], end = a.ptr[row + 1];
    float acc[VEC], mx[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) { acc[v] = identity<OP>(); mx[v] = -INFINITY; }
    for (int j = beg + wave * CH; j < end; j += NW * CH) {
        float x[CH][VEC];
#pragma unroll
        for (int i = 0; i < CH; ++i)                         // padded list: always in bounds
            load_vec<VEC>(x[i], a.src + (size_t)(a.idx[j + i] & kIdMask) * a.ld + col);
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const bool live = j + i < end;
#pragma unroll
            for (int v = 0; v < VEC; ++v) { float none = 0.0f; accumulate<OP>(acc[v], mx[v], live ? x[i][v] : dead_value<OP>(), 0.0f, none, false); }
        }
    }
    if (wave > 0) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            part_v[wave][lane * VEC + v] = acc[v];
            if (LSE) part_m[wave][lane * VEC + v] = mx[v];
        }
    }
    __syncthreads();
    if (wave > 0 || colu >= a.B) return;
    for (int w = 1; w < NW; ++w) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const float ov = part_v[w][lane * VEC + v];
            if (LSE) {
                const float om = part_m[w][lane * VEC + v];
                edge_combine<OP>(mx[v], acc[v], om, ov);
            } else {
                float unused = 0.0f;
                edge_combine<OP>(acc[v], unused, ov, 0.0f);
            }
        }
    }
    const int out_row = a.out_row[row];
    float o[VEC], nc[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) { o[v] = finish<OP>(acc[v], mx[v]); nc[v] = 0.0f; }
    if (OP == OP_SUM_H || OP == OP_SUM_P) load_vec<VEC>(nc, a.own + (size_t)out_row * a.ld + col);
    if (OP == OP_SUM_H && (a.idx[end - 1] & kRowFlag)) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) o[v] = encode_h(o[v], nc[v]);
    }
    if (OP == OP_SUM_P) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            if (nc[v] == 0.0f && a.zero_flag) *a.zero_flag = 1;
            o[v] = premultiply(o[v], nc[v]);
        }
    }
    store_vec<VEC>(a.dst + (size_t)out_row * a.ld + col, o);
}

template <int OP, int VEC, int NW>
__global__ __launch_bounds__(NW * 64) void combine_kernel(PassArgs a) {
    combine_body<OP, VEC, NW>((int)blockIdx.x, a);
}

// The main rows of a layer and the combine rows of its split rows in one launch, for the tiles whose segments
// run in a launch of their own beforehand (one column per lane): the first n_comb_blocks workgroups (a multiple
// of 8, so that the others keep their XCDs) take one combine row each, four waves per row, the rest walk the
// tasks of the main rows.  One launch less per layer where the launches, not the bytes, set the time.
template <int OP, int COP, int VEC>
__global__ __launch_bounds__(256) void stream_combine_kernel(const int2* __restrict__ tasks, int n_tasks,
                                                             const uint32_t* __restrict__ idx,
                                                             const float* __restrict__ src,
                                                             const float* __restrict__ src2,
                                                             const float* __restrict__ own, float* __restrict__ dst,
                                                             int B, int ld, int stream_stores, int n_main,
                                                             int* __restrict__ zero_flag, int n_comb_blocks,
                                                             PassArgs cmb) {
    if ((int)blockIdx.x < n_comb_blocks) {
        if ((int)blockIdx.x < cmb.n_main) combine_body<COP, VEC, 4>((int)blockIdx.x, cmb);
    } else {
        stream_body<OP, VEC>((int)blockIdx.x - n_comb_blocks, (int)gridDim.x - n_comb_blocks, tasks, n_tasks, idx, src,
                             src2, own, dst, B, ld, stream_stores, nullptr, 0, nullptr, nullptr, n_main, zero_flag);
    }
}

// ---------------------------------------------------------------------------------------------
// Persistent kernels for the top of the circuit (the layers that taper to the roots; for a small
// circuit every layer): instead of one launch per layer, a workgroup owns CT batch columns, keeps
// the values (forward) or the adjoints (reverse) of the current and the previous layer in LDS and
// walks the layers with a barrier in between.  Batch columns are independent, so no grid-wide
// barrier is needed.
//   Index vectors stay in global memory, in the form the host builds for these layers: rows in chunks
// of 64 (one row per lane), a chunk as long as its longest row, and the lines of 64 words that make
// up the chunks of one wave stored back to back.  A wave therefore streams through one contiguous
// run of lines per layer, a block of kSlabBlock lines at a time, fetches the next block (at the end
// of a run: the first block of the next layer's run, so the fetch is in flight across the barrier)
// before it works on the one in hand, and learns from the end-of-chunk bit of a line, which is the
// same in all its words, when to close the 64 rows it is working on.  Padding words name the slot one
// past the last source row, where the identity of the layer's operation is kept, so the inner loop has
// no test for them.  The rows of these layers are stored sorted by fan-in group, so the rows of a
// chunk have similar lengths; the 16 waves take the chunks round-robin.
//   One compute unit evaluates a whole column, so the instruction count per line, not memory, bounds
// these kernels: a line costs its fetch, one LDS gather and the accumulation.
//   A lane owns rows of one batch column, so writing values into the row-major activation buffer
// would cost one cache line per lane.  The values go to a column-major buffer tb[column][T] instead
// (T = rows of all candidate layers), where consecutive lanes write consecutive floats; the reverse
// kernel reads it the same way, and rows that an ordinary launch needs are transposed back on demand
// (tb_to_rows_kernel).
//   LDS (floats): forward 2 * (nmax + 1) * CT, reverse 4 * (nmax + 1) * CT.
// ---------------------------------------------------------------------------------------------
constexpr int kSlabThreads = 64 * kSlabWaves;      // kSlabWaves, kSlabBlock: the plan's format constants (layerize.h)
constexpr int kSlabD = kSlabBlock;

struct SlabLayer {
    int32_t n, n_below;            // nodes of this layer and of the layer below
    int32_t tb_off;                // first entry of this layer in a column of tb
    int32_t reserved;
    // Per wave: where its run of lines for this layer starts (offset in ints into the index buffer) and
    // how many lines it has (a multiple of kSlabD).  The runs of one wave for consecutive layers are
    // stored back to back, bottom-up for the forward sweep and top-down for the reverse one, with a
    // block of padding lines after the last, so a wave fetches ahead through one contiguous stream.
    int32_t fwd_start[kSlabWaves], fwd_count[kSlabWaves];
    int32_t bwd_start[kSlabWaves], bwd_count[kSlabWaves];
    int64_t row0, row0_below;      // first activation rows
};

// identity of a layer's forward operation: the value kept in the padding slot of its source array
__device__ __forceinline__ float slab_identity(int semiring, bool is_and) {
    if (semiring == 0) return is_and ? 1.0f : 0.0f;
    return is_and ? 0.0f : -INFINITY;
}

// one block of lines starting at p (this lane's word of the first of them)
__device__ __forceinline__ void slab_fetch(uint32_t (&a)[kSlabD], const uint32_t* p) {
#pragma unroll
    for (int u = 0; u < kSlabD; ++u) a[u] = p[u * 64];
}

// One block of one layer, forward: works on the lines in `a` while the block at `fetch` travels into `b`.
template <int OP, int CT, bool FG>
__device__ __forceinline__ void slab_fwd_block(const uint32_t (&a)[kSlabD], uint32_t (&b)[kSlabD], const uint32_t* fetch,
                                               int n_rows, int n_below, int& q, float (&acc)[CT], float (&mx)[CT],
                                               const float* prev, float* cur, const float* __restrict__ below, int ld,
                                               int nact, float* __restrict__ tb_col, int T) {
    slab_fetch(b, fetch);
    float x[kSlabD][CT];
#pragma unroll
    for (int u = 0; u < kSlabD; ++u) {
        const int ch = (int)(a[u] & kIdMask);
#pragma unroll
        for (int k = 0; k < CT; ++k) {
            if (FG) {
                // sources in global memory: a padding word (source n_below) must not be followed
                const bool live = ch != n_below && k < nact;
                const float v = below[(size_t)(live ? ch : 0) * ld + (live ? k : 0)];
                x[u][k] = live ? v : dead_value<OP>();
            } else {
                // byte offset of the source's CT values: the shift drops the end-of-chunk bit, the only flag
                // of a forward stream (CT = 1, 2, 4, 8: at least the top two bits go)
                constexpr int kShift = CT == 1 ? 2 : (CT == 2 ? 3 : (CT == 4 ? 4 : 5));
                x[u][k] = *reinterpret_cast<const float*>(reinterpret_cast<const char*>(prev) + (a[u] << kShift) + 4 * k);
            }
        }
    }
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int u = 0; u < kSlabD; ++u) {
#pragma unroll
        for (int k = 0; k < CT; ++k) { float none = 0.0f; accumulate<OP>(acc[k], mx[k], x[u][k], 0.0f, none); }
        // the end-of-chunk bit is the same in all words of a line
        if (__builtin_amdgcn_readfirstlane((int)a[u]) & (int)kLast) {
            const int r = q * 64 + lane;
            if (r < n_rows) {
#pragma unroll
                for (int k = 0; k < CT; ++k) {
                    const float o = finish<OP>(acc[k], mx[k]);
                    cur[r * CT + k] = o;
                    if (k < nact) tb_col[(size_t)k * T + r] = o;
                }
            }
#pragma unroll
            for (int k = 0; k < CT; ++k) { acc[k] = identity<OP>(); mx[k] = -INFINITY; }
            q += kSlabWaves;
        }
    }
}

// One layer, forward: the `lines` lines at sp (this wave's run).  `a` holds the first block on entry and
// the block that follows the run (the next layer's first, or padding) on exit.  FG: the sources are rows
// of the activation buffer in global memory (the layer below the first persistent one), otherwise the
// previous layer's values in LDS.
template <int OP, int CT, bool FG>
__device__ __forceinline__ void slab_fwd_rows(int n_rows, int n_below, const uint32_t* sp, int lines,
                                              uint32_t (&a)[kSlabD], const float* prev, float* cur,
                                              const float* __restrict__ below, int ld, int nact,
                                              float* __restrict__ tb_col, int T) {
    if (lines <= 0) return;
    int q = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));      // chunk in hand
    float acc[CT], mx[CT];
#pragma unroll
    for (int k = 0; k < CT; ++k) { acc[k] = identity<OP>(); mx[k] = -INFINITY; }
    uint32_t b[kSlabD];
    for (int i = 0;;) {       // two blocks per turn, the two register sets change roles
        slab_fwd_block<OP, CT, FG>(a, b, sp + (size_t)(i + kSlabD) * 64, n_rows, n_below, q, acc, mx, prev, cur, below, ld, nact, tb_col, T);
        i += kSlabD;
        if (i >= lines) {
#pragma unroll
            for (int u = 0; u < kSlabD; ++u) a[u] = b[u];
            break;
        }
        slab_fwd_block<OP, CT, FG>(b, a, sp + (size_t)(i + kSlabD) * 64, n_rows, n_below, q, acc, mx, prev, cur, below, ld, nact, tb_col, T);
        i += kSlabD;
        if (i >= lines) break;
    }
}

template <int CT, bool FG>
__device__ __forceinline__ void slab_fwd_layer(int semiring, bool is_and, int n_rows, int n_below, const uint32_t* sp,
                                               int lines, uint32_t (&a)[kSlabD], const float* prev, float* cur,
                                               const float* __restrict__ below, int ld, int nact,
                                               float* __restrict__ tb_col, int T) {
    if (semiring == 2) {           // (max, +) on log weights
        if (is_and) slab_fwd_rows<OP_SUM, CT, FG>(n_rows, n_below, sp, lines, a, prev, cur, below, ld, nact, tb_col, T);
        else slab_fwd_rows<OP_MAX, CT, FG>(n_rows, n_below, sp, lines, a, prev, cur, below, ld, nact, tb_col, T);
    } else if (semiring == 1) {    // (logsumexp, +)
        if (is_and) slab_fwd_rows<OP_SUM, CT, FG>(n_rows, n_below, sp, lines, a, prev, cur, below, ld, nact, tb_col, T);
        else slab_fwd_rows<OP_LSE, CT, FG>(n_rows, n_below, sp, lines, a, prev, cur, below, ld, nact, tb_col, T);
    } else {
        if (is_and) slab_fwd_rows<OP_PROD, CT, FG>(n_rows, n_below, sp, lines, a, prev, cur, below, ld, nact, tb_col, T);
        else slab_fwd_rows<OP_SUM, CT, FG>(n_rows, n_below, sp, lines, a, prev, cur, below, ld, nact, tb_col, T);
    }
}

__device__ __forceinline__ float log1mexp_f(float x) {
    return x > -0.69314718f ? logf(-expm1f(x)) : log1pf(-expf(x));
}

// Arguments of the leaf layer when the persistent kernel evaluates it itself (its first layer is
// layer 1): a workgroup reads its own rows of the leaf-weight arrays, which are contiguous.
struct SlabLeaf {
    const float* w;             // [B, V] leaf weights (null: the leaf layer was evaluated by leaf_fwd_kernel)
    const float* wneg;          // [B, V] weights of the negated literals, or null
    const int32_t* leaf_code;   // [n_0] +(v+1), -(v+1), INT32_MAX (true), INT32_MIN (false)
    float* wT;                  // [V, ld] transposed leaf weights kept for the reverse sweep
    float* act0;                // [n_0, ld] rows of layer 0 in the activation buffer
    int32_t V, n0;
};

template <int CT>
__global__ __launch_bounds__(kSlabThreads) void slab_fwd_kernel(const SlabLayer* __restrict__ layers, int n_layers,
                                                                int first_is_and, const int32_t* __restrict__ ibase,
                                                                const float* __restrict__ act, int B, int ld,
                                                                int semiring, int nmax, float* __restrict__ tb, int T,
                                                                SlabLeaf leaf, const int32_t* __restrict__ root_pos,
                                                                int R, float* __restrict__ out,
                                                                const float* __restrict__ stage) {
    extern __shared__ float smem[];
    float* prev = smem;
    float* cur = smem + (size_t)(nmax + 1) * CT;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int col0 = (int)blockIdx.x * CT;
    const int nact = B - col0 < CT ? B - col0 : CT;          // active columns of this workgroup (>= 1)
    float* tb0 = tb + (size_t)col0 * T;
    const bool log_domain = semiring != 0;
    // this wave's stream of lines; its first block is on its way while the leaf layer is evaluated
    const uint32_t* sp = reinterpret_cast<const uint32_t*>(ibase) + layers[0].fwd_start[wave] + lane;
    uint32_t a[kSlabD];
    slab_fetch(a, sp);
    if (leaf.w) {
        // leaf layer into LDS; the transposed weights and the rows of layer 0 also go to global memory
        // for the reverse sweep (every column of [0, ld): the last workgroup zeroes the padding columns)
        for (int i = threadIdx.x; i < leaf.n0; i += kSlabThreads) {
            const int code = leaf.leaf_code[i];
#pragma unroll
            for (int k = 0; k < CT; ++k) {
                float v = 0.0f;
                if (k < nact) {
                    if (code == INT32_MAX) v = log_domain ? 0.0f : 1.0f;
                    else if (code == INT32_MIN) v = log_domain ? -INFINITY : 0.0f;
                    else {
                        const int var = (code > 0 ? code : -code) - 1;
                        const size_t at = (size_t)(col0 + k) * leaf.V + var;
                        if (code > 0) v = leaf.w[at];
                        else if (leaf.wneg) v = leaf.wneg[at];
                        else v = log_domain ? log1mexp_f(leaf.w[at]) : 1.0f - leaf.w[at];
                    }
                    leaf.act0[(size_t)i * ld + col0 + k] = v;
                }
                prev[i * CT + k] = v;
            }
            if (blockIdx.x == gridDim.x - 1)
                for (int b = B; b < ld; ++b) leaf.act0[(size_t)i * ld + b] = 0.0f;
        }
        for (int v = threadIdx.x; v < leaf.V; v += kSlabThreads) {
            for (int k = 0; k < nact; ++k) leaf.wT[(size_t)v * ld + col0 + k] = leaf.w[(size_t)(col0 + k) * leaf.V + v];
            if (blockIdx.x == gridDim.x - 1)
                for (int b = B; b < ld; ++b) leaf.wT[(size_t)v * ld + b] = 0.0f;
        }
        if (threadIdx.x < CT) prev[leaf.n0 * CT + threadIdx.x] = slab_identity(semiring, first_is_and != 0);
        __syncthreads();
    }
    if (!leaf.w && stage) {
        // the layer below the first one, column-major in `stage` (B runs of n_below floats, written by
        // rows_to_cols_kernel): into LDS with consecutive lanes reading consecutive floats
        const int nb0 = layers[0].n_below;
        for (int i = threadIdx.x; i < nb0; i += kSlabThreads)
#pragma unroll
            for (int k = 0; k < CT; ++k) prev[i * CT + k] = k < nact ? stage[(size_t)(col0 + k) * nb0 + i] : 0.0f;
        if (threadIdx.x < CT) prev[nb0 * CT + threadIdx.x] = slab_identity(semiring, first_is_and != 0);
        __syncthreads();
    }
    // the few numbers a layer needs are read a layer ahead
    int lines = layers[0].fwd_count[wave], n_rows = layers[0].n, n_below = layers[0].n_below, tb_off = layers[0].tb_off;
    for (int t = 0; t < n_layers; ++t) {
        const bool is_and = ((t & 1) == 0) == (first_is_and != 0);
        const int tn = t + 1 < n_layers ? t + 1 : t;
        const int lines2 = layers[tn].fwd_count[wave], n_rows2 = layers[tn].n, n_below2 = layers[tn].n_below,
                  tb_off2 = layers[tn].tb_off;
        float* tb_col = tb0 + tb_off;
        // the padding slot of this layer's values, for the layer above (the other operation)
        if (threadIdx.x < CT) cur[n_rows * CT + threadIdx.x] = slab_identity(semiring, !is_and);
        if (t == 0 && !leaf.w && !stage)
            slab_fwd_layer<CT, true>(semiring, is_and, n_rows, n_below, sp, lines, a, prev, cur,
                                     act + (size_t)layers[0].row0_below * ld + col0, ld, nact, tb_col, T);
        else
            slab_fwd_layer<CT, false>(semiring, is_and, n_rows, n_below, sp, lines, a, prev, cur, nullptr, ld, nact, tb_col, T);
        sp += (size_t)lines * 64;
        lines = lines2; n_rows = n_rows2; n_below = n_below2; tb_off = tb_off2;
        __syncthreads();
        float* tmp = prev; prev = cur; cur = tmp;
    }
    // roots: the top layer is in LDS
    for (int i = threadIdx.x; i < R * CT; i += kSlabThreads) {
        const int r = i / CT, k = i % CT;
        if (k < nact) out[(size_t)(col0 + k) * R + r] = prev[root_pos[r] * CT + k];
    }
}

// One block of one step of the reverse sweep.  OR: the step goes through an OR layer; its weighted edges read the
// parent's adjoint in the one-gather form (see encode_h) and need the value of the row they belong to.
// Otherwise every edge passes the adjoint on, and a row that is an OR node with more than one child (kRowFlag
// on the word the lane holds when the chunk closes) is stored in that form, again with the row's own value.
// `own` is that value for the row in hand, read from the column-major value buffer (consecutive lanes,
// consecutive floats) when a chunk opens.
template <int CT, bool OR>
__device__ __forceinline__ void slab_bwd_block(const uint32_t (&a)[kSlabD], uint32_t (&b)[kSlabD], const uint32_t* fetch,
                                               int n_below, int& q, float (&acc)[CT], float (&own)[CT],
                                               const float* cur, float* nxt, const float* __restrict__ tb_below, int T,
                                               int nact) {
    slab_fetch(b, fetch);
    float g[kSlabD][CT];
#pragma unroll
    for (int u = 0; u < kSlabD; ++u) {
        const int p = (int)(a[u] & kIdMask);          // a padding word names the slot past the last parent: adjoint 0
#pragma unroll
        for (int k = 0; k < CT; ++k) g[u][k] = cur[p * CT + k];
    }
    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int u = 0; u < kSlabD; ++u) {
        // an unweighted edge (chain node or single-child OR above) passes the adjoint unchanged
        const bool weighted = OR && (a[u] & kWeighted) != 0;
#pragma unroll
        for (int k = 0; k < CT; ++k) acc[k] += weighted ? decode_h(g[u][k], own[k]) : g[u][k];
        if (__builtin_amdgcn_readfirstlane((int)a[u]) & (int)kLast) {
            const int r = q * 64 + lane;
            if (r < n_below) {
                const bool enc = !OR && (a[u] & kRowFlag) != 0;
#pragma unroll
                for (int k = 0; k < CT; ++k) nxt[r * CT + k] = enc ? encode_h(acc[k], own[k]) : acc[k];
            }
            q += kSlabWaves;
            const int r2 = q * 64 + lane;
#pragma unroll
            for (int k = 0; k < CT; ++k) {
                acc[k] = 0.0f;
                own[k] = (r2 < n_below && k < nact) ? tb_below[(size_t)k * T + r2] : 0.0f;
            }
        }
    }
}

template <int CT, bool OR>
__device__ __forceinline__ void slab_bwd_rows(int n_below, const uint32_t* sp, int lines, uint32_t (&a)[kSlabD],
                                              const float* cur, float* nxt, const float* __restrict__ tb_below, int T,
                                              int nact) {
    if (lines <= 0) return;
    int q = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = threadIdx.x & 63;
    float acc[CT], own[CT];
#pragma unroll
    for (int k = 0; k < CT; ++k) {
        acc[k] = 0.0f;
        const int r = q * 64 + lane;
        own[k] = (r < n_below && k < nact) ? tb_below[(size_t)k * T + r] : 0.0f;
    }
    uint32_t b[kSlabD];
    for (int i = 0;;) {
        slab_bwd_block<CT, OR>(a, b, sp + (size_t)(i + kSlabD) * 64, n_below, q, acc, own, cur, nxt, tb_below, T, nact);
        i += kSlabD;
        if (i >= lines) {
#pragma unroll
            for (int u = 0; u < kSlabD; ++u) a[u] = b[u];
            break;
        }
        slab_bwd_block<CT, OR>(b, a, sp + (size_t)(i + kSlabD) * 64, n_below, q, acc, own, cur, nxt, tb_below, T, nact);
        i += kSlabD;
        if (i >= lines) break;
    }
}

// Reverse sweep over the same layers (log semiring): seeds the top layer's adjoints from dout, walks
// down to the first layer of the launch and leaves that layer's adjoints in g_out[B][n_first] (column-major).
// LDS: the adjoints of the layer in hand and of the one below (two arrays, as in the forward kernel, so both
// kernels take the same layers); node values come from the column-major buffer tb, once per row.  The adjoints
// of OR nodes with more than one child are kept in the one-gather form throughout, also in g_out; top_multi
// (or null) flags such nodes of the top layer for the seed.
template <int CT>
__global__ __launch_bounds__(kSlabThreads) void slab_bwd_kernel(const SlabLayer* __restrict__ layers, int n_layers,
                                                                int first_is_and, const int32_t* __restrict__ ibase,
                                                                const float* __restrict__ dout,
                                                                const int32_t* __restrict__ top_ptr,
                                                                const int32_t* __restrict__ top_root, int R,
                                                                float* __restrict__ g_out, int B, int nmax,
                                                                const float* __restrict__ tb, int T,
                                                                const uint32_t* __restrict__ top_multi) {
    extern __shared__ float smem[];
    const size_t stride = (size_t)(nmax + 1) * CT;
    float* cur = smem;
    float* nxt = smem + stride;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int col0 = (int)blockIdx.x * CT;
    const int nact = B - col0 < CT ? B - col0 : CT;
    const float* tb0 = tb + (size_t)col0 * T;
    // this wave's stream of lines, from the top layer's step downwards
    const uint32_t* sp = reinterpret_cast<const uint32_t*>(ibase) + layers[n_layers - 1].bwd_start[wave] + lane;
    uint32_t a[kSlabD];
    slab_fetch(a, sp);
    {   // adjoint seed of the top layer
        const SlabLayer& L = layers[n_layers - 1];
        for (int i = threadIdx.x; i < L.n; i += kSlabThreads) {
            const bool enc = top_multi && ((top_multi[i >> 5] >> (i & 31)) & 1u);
#pragma unroll
            for (int k = 0; k < CT; ++k) {
                float acc = 0.0f;
                if (k < nact) {
                    for (int t = top_ptr[i]; t < top_ptr[i + 1]; ++t) acc += dout[(size_t)(col0 + k) * R + top_root[t]];
                    if (enc) acc = encode_h(acc, tb0[(size_t)k * T + L.tb_off + i]);
                }
                cur[i * CT + k] = acc;
            }
        }
        if (threadIdx.x < CT) cur[L.n * CT + threadIdx.x] = 0.0f;       // padding slot: adjoint 0
    }
    for (int t = n_layers - 1; t >= 1; --t) {      // adjoints of layer t -> layer t - 1
        const SlabLayer& L = layers[t];
        const bool is_and = ((t & 1) == 0) == (first_is_and != 0);
        const int lines = L.bwd_count[wave];
        const float* tb_below = tb0 + layers[t - 1].tb_off;
        __syncthreads();
        if (is_and) slab_bwd_rows<CT, false>(L.n_below, sp, lines, a, cur, nxt, tb_below, T, nact);
        else slab_bwd_rows<CT, true>(L.n_below, sp, lines, a, cur, nxt, tb_below, T, nact);
        sp += (size_t)lines * 64;
        if (threadIdx.x < CT) nxt[L.n_below * CT + threadIdx.x] = 0.0f;  // padding slot of the next step
        __syncthreads();
        float* tmp = cur; cur = nxt; nxt = tmp;
    }
    // column-major, like tb: a lane owns rows of one column, so row-major stores would be 4 bytes per cache line
    // (measured: 40 us of 163 on the headline workload); tb_to_rows_kernel transposes afterwards
    const int n_first = layers[0].n;
    for (int r = threadIdx.x; r < n_first; r += kSlabThreads)
#pragma unroll
        for (int k = 0; k < CT; ++k)
            if (k < nact) g_out[(size_t)(col0 + k) * n_first + r] = cur[r * CT + k];
}

// cols[b, r] = rows[r, b] for r < n_rows, b < B: the rows of a layer of the activation buffer into the column-major
// form in which a workgroup of the persistent forward kernel reads its column (32 x 32 tiles through LDS).
__global__ __launch_bounds__(256) void rows_to_cols_kernel(const float* __restrict__ rows, int n_rows, int B, int ld,
                                                           float* __restrict__ cols) {
    __shared__ float tile[32][33];
    const int r0 = blockIdx.x * 32, b0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;       // 32 x 8
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = r0 + ty + 8 * j, b = b0 + tx;
        tile[ty + 8 * j][tx] = (r < n_rows && b < B) ? rows[(size_t)r * ld + b] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int b = b0 + ty + 8 * j, r = r0 + tx;
        if (b < B && r < n_rows) cols[(size_t)b * n_rows + r] = tile[tx][ty + 8 * j];
    }
}

// rows[r, b] = tb[b, first + r] for r < n_rows: values that the persistent forward kernel left in the
// column-major buffer, transposed into rows of the activation buffer through a 32 x 33 LDS tile.
__global__ __launch_bounds__(256) void tb_to_rows_kernel(const float* __restrict__ tb, int T, int first, int n_rows,
                                                         int B, int ld, float* __restrict__ rows) {
    __shared__ float tile[32][33];
    const int r0 = blockIdx.x * 32, b0 = blockIdx.y * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;       // 32 x 8
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int b = b0 + ty + 8 * j, r = r0 + tx;
        tile[ty + 8 * j][tx] = (b < B && r < n_rows) ? tb[(size_t)b * T + first + r] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int r = r0 + ty + 8 * j, b = b0 + tx;
        if (r < n_rows && b < ld) rows[(size_t)r * ld + b] = tile[tx][ty + 8 * j];
    }
}

// ---------------------------------------------------------------------------------------------
// Reverse sweep of a product (AND) layer in the real semiring, first half.  The adjoint of child c of
// parent r is G[r] times the product of r's other children.  Per parent the kernel forms, per batch
// column, the product q of the non-zero children and the number z of zero ones, and replaces the
// parent's adjoint row in place by
//   P[r] = G[r] * q  (0 when z >= 2),  lowest mantissa bit = (z == 1),
// from which the by-child pass (OP_PROD_BWD) gives every child its share: P / value for a parent
// without zero children, P itself for the one zero child of a parent with z = 1.  Exact also when
// children are zero (leaves with p = 0 or p = 1); nothing is stored per edge.  A lane group of W lanes
// owns one parent row.
//   With `own` (the values of the parents themselves) the rows arrive premultiplied (OP_SUM_P,
// OP_PROD_BWD_P): G * value where the value is not zero, which is P already, and plain G where it is
// zero.  Then only the waves that hold a zero value walk the children, and only those columns change; that pass
// also raises zero_flag when it meets a zero value, and a launch that finds it down returns at once.
// ---------------------------------------------------------------------------------------------
template <int VEC, int W>
__global__ __launch_bounds__(256) void prod_parent_kernel(const int32_t* __restrict__ ptr,
                                                          const int32_t* __restrict__ child,
                                                          const float* __restrict__ below, float* __restrict__ g, int n,
                                                          int B, int ld, const float* __restrict__ own,
                                                          const int* __restrict__ zero_flag) {
    constexpr int RPW = 64 / W;
    const int lane = threadIdx.x & 63;
    const int col = ((int)blockIdx.y * W + (lane % W)) * VEC;
    if (col >= B) return;
    if (own && zero_flag && *zero_flag == 0) return;          // the pass that wrote the rows met no zero value: nothing to repair
    // the grid is capped (the launch that finds the flag down should cost as little as a launch can): a
    // workgroup takes every gridDim.x-th group of rows
    for (int64_t blk = blockIdx.x; blk * (4 * RPW) < n; blk += gridDim.x) {
    const int64_t row64 = (blk * 4 + (threadIdx.x >> 6)) * RPW + lane / W;
    if (row64 >= n) continue;
    const int row = (int)row64;
    float nv[VEC];
    if (own) {
        load_vec<VEC>(nv, own + (size_t)row * ld + col);
        bool zero_here = false;
#pragma unroll
        for (int v = 0; v < VEC; ++v) zero_here = zero_here || nv[v] == 0.0f;
        if (!__any(zero_here)) continue;
    }
    const int beg = ptr[row], end = ptr[row + 1];
    float q[VEC], z[VEC], gr[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) { q[v] = 1.0f; z[v] = 0.0f; }
    load_vec<VEC>(gr, g + (size_t)row * ld + col);
    constexpr int CH = 8;
    float x[CH][VEC];
    // 8 gathers in flight (entries past the row's end re-read its last child)
    for (int j = beg; j < end; j += CH) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int jj = j + i < end ? j + i : end - 1;
            load_vec<VEC>(x[i], below + (size_t)child[jj] * ld + col);
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const bool live = j + i < end;
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const bool zero = x[i][v] == 0.0f;
                z[v] += (live && zero) ? 1.0f : 0.0f;
                q[v] *= (live && !zero) ? x[i][v] : 1.0f;
            }
        }
    }
    float p[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        const float val = z[v] >= 2.0f ? 0.0f : gr[v] * q[v];
        p[v] = __uint_as_float((__float_as_uint(val) & ~1u) | (z[v] == 1.0f ? 1u : 0u));
        if (own && nv[v] != 0.0f) p[v] = gr[v];          // premultiplied already
    }
    store_vec<VEC>(g + (size_t)row * ld + col, p);
    }
}

// ---------------------------------------------------------------------------------------------
// Leaf layer: leaf_weights[B,V] (batch-outer) -> wT[V,ld] (kept for the backward pass) and the
// literal rows of layer 0, through an LDS tile of 32 variables x 64 batch columns.  The negated
// literal of v gets wneg[b, v] when the caller supplies weights of its own for the negated literals,
// otherwise 1 - w (real semiring) or log(1 - exp(w)) (log domain).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void leaf_fwd_kernel(const float* __restrict__ w, const float* __restrict__ wneg,
                                                       int B, int V, int ld,
                                                       const int32_t* __restrict__ pos_row,
                                                       const int32_t* __restrict__ neg_row,
                                                       float* __restrict__ wT, float* __restrict__ act0,
                                                       int log_domain) {
    __shared__ float tile[32][65];
    __shared__ float tile_neg[32][65];
    const int v0 = blockIdx.x * 32, b0 = blockIdx.y * 64;
    {
        const int vx = threadIdx.x & 31, by = threadIdx.x >> 5;
        for (int k = 0; k < 8; ++k) {
            const int b = b0 + by + 8 * k, v = v0 + vx;
            const bool in = b < B && v < V;
            tile[vx][by + 8 * k] = in ? w[(size_t)b * V + v] : 0.0f;
            if (wneg) tile_neg[vx][by + 8 * k] = in ? wneg[(size_t)b * V + v] : 0.0f;
        }
    }
    __syncthreads();
    const int bx = threadIdx.x & 63, vy = threadIdx.x >> 6;
    const int b = b0 + bx;
    if (b >= ld) return;
    for (int k = 0; k < 8; ++k) {
        const int v = v0 + vy + 4 * k;
        if (v >= V) break;
        const float x = tile[vy + 4 * k][bx];
        wT[(size_t)v * ld + b] = x;
        const int pr = pos_row[v], nr = neg_row[v];
        if (pr >= 0) act0[(size_t)pr * ld + b] = x;
        if (nr >= 0) {
            float y;
            if (b >= B) y = 0.0f;
            else if (wneg) y = tile_neg[vy + 4 * k][bx];
            else y = log_domain ? log1mexp_f(x) : 1.0f - x;
            act0[(size_t)nr * ld + b] = y;
        }
    }
}

// The same for small batches (ld = B <= 32), where the tile would be all but empty: a thread per (variable, column).
__global__ __launch_bounds__(256) void leaf_fwd_small_kernel(const float* __restrict__ w, const float* __restrict__ wneg,
                                                             int B, int V, const int32_t* __restrict__ pos_row,
                                                             const int32_t* __restrict__ neg_row,
                                                             float* __restrict__ wT, float* __restrict__ act0,
                                                             int log_domain) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= (int64_t)V * B) return;
    const int v = (int)(i / B), b = (int)(i % B);
    const float x = w[(size_t)b * V + v];
    wT[i] = x;
    const int pr = pos_row[v], nr = neg_row[v];
    if (pr >= 0) act0[(size_t)pr * B + b] = x;
    if (nr >= 0) act0[(size_t)nr * B + b] = wneg ? wneg[(size_t)b * V + v] : (log_domain ? log1mexp_f(x) : 1.0f - x);
}

__global__ void fill_row_kernel(float* row, int ld, float value) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < ld) row[b] = value;
}

// out[b, r] = top[root_pos[r], b]
__global__ void root_out_kernel(const float* __restrict__ top, const int32_t* __restrict__ root_pos,
                                int B, int R, int ld, float* __restrict__ out) {
    const int r = blockIdx.x;
    const float* row = top + (size_t)root_pos[r] * ld;
    for (int b = threadIdx.x; b < B; b += blockDim.x) out[(size_t)b * R + r] = row[b];
}

// G_top[i, b] = sum of dout[b, r] over the root columns r that read top-layer node i
// multi (or null) with the top layer's values: nodes flagged there leave in the one-gather form (encode_h)
__global__ void seed_kernel(const float* __restrict__ dout, const int32_t* __restrict__ top_ptr,
                            const int32_t* __restrict__ top_root, int B, int R, int ld,
                            float* __restrict__ g, const uint32_t* __restrict__ multi,
                            const float* __restrict__ top_values) {
    const int i = blockIdx.x;
    const bool enc = multi && ((multi[i >> 5] >> (i & 31)) & 1u);
    for (int b = threadIdx.x; b < ld; b += blockDim.x) {
        float acc = 0.0f;
        if (b < B)
            for (int t = top_ptr[i]; t < top_ptr[i + 1]; ++t) acc += dout[(size_t)b * R + top_root[t]];
        if (enc) acc = encode_h(acc, top_values[(size_t)i * ld + b]);
        g[(size_t)i * ld + b] = acc;
    }
}

// rows[r, b] = dout[b, r]: the adjoint seed as one row per root column
__global__ void seed_rows_kernel(const float* __restrict__ dout, int B, int R, int ld, float* __restrict__ rows) {
    const int r = blockIdx.x;
    for (int b = threadIdx.x; b < ld; b += blockDim.x) rows[(size_t)r * ld + b] = b < B ? dout[(size_t)b * R + r] : 0.0f;
}

// dleaf[b, v] = G0[+v, b] + G0[-v, b] * d(negated weight)/d(weight); tile transposed through LDS.
// mode 0: negated weight 1 - w, mode 1: log(1 - exp(w)), mode 2: the negated literals have weights
// of their own, so dleaf holds G0[+v, b] and dneg (may be null) receives G0[-v, b].
__global__ __launch_bounds__(256) void leaf_bwd_kernel(const float* __restrict__ g0, const float* __restrict__ wT,
                                                       const int32_t* __restrict__ pos_row,
                                                       const int32_t* __restrict__ neg_row, int B, int V,
                                                       int ld, int mode, float* __restrict__ dleaf,
                                                       float* __restrict__ dneg) {
    __shared__ float tile[32][65];
    __shared__ float tile_neg[32][65];
    const int v0 = blockIdx.x * 32, b0 = blockIdx.y * 64;
    {
        const int bx = threadIdx.x & 63, vy = threadIdx.x >> 6;
        const int b = b0 + bx;
        for (int k = 0; k < 8; ++k) {
            const int v = v0 + vy + 4 * k;
            float d = 0.0f, dn = 0.0f;
            if (v < V && b < B) {
                const int pr = pos_row[v], nr = neg_row[v];
                if (pr >= 0) d = g0[(size_t)pr * ld + b];
                if (nr >= 0) {
                    const float gn = g0[(size_t)nr * ld + b];
                    if (mode == 2) dn = gn;
                    else if (gn != 0.0f) d += mode == 1 ? -gn / expm1f(-wT[(size_t)v * ld + b]) : -gn;
                }
            }
            tile[vy + 4 * k][bx] = d;
            tile_neg[vy + 4 * k][bx] = dn;
        }
    }
    __syncthreads();
    const int vx = threadIdx.x & 31, by = threadIdx.x >> 5;
    for (int k = 0; k < 8; ++k) {
        const int b = b0 + by + 8 * k, v = v0 + vx;
        if (b < B && v < V) {
            dleaf[(size_t)b * V + v] = tile[vx][by + 8 * k];
            if (mode == 2 && dneg) dneg[(size_t)b * V + v] = tile_neg[vx][by + 8 * k];
        }
    }
}

}  // namespace klay
