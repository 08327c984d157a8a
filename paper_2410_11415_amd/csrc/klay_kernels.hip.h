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

namespace klay {

enum PassOp : int { OP_SUM = 0, OP_PROD = 1, OP_LSE = 2, OP_SOFTMAX_BWD = 3, OP_MAX = 4 };

// Index entries: bits 0..29 = source row, bit 31 = last edge of its output row, bit 30 = weighted
// edge (reverse sweep only: the parent is an OR node with more than one child, so the adjoint
// passes through the softmax weight exp(child - parent); an unweighted edge passes it unchanged).
// kSkip (all ones) stands for a whole output row that this pass leaves untouched (a split row).
constexpr uint32_t kLast = 0x80000000u, kWeighted = 0x40000000u, kSkip = 0xFFFFFFFFu, kIdMask = 0x3FFFFFFFu;

struct PassArgs {
    const int32_t* ptr;        // [n_total + 1] CSR offsets into idx
    const uint32_t* idx;       // index entries (readable up to 16 entries past the end)
    const float* src;          // [*, ld] source rows (values of the layer below, adjoints, or partials)
    const float* src2;         // OP_SOFTMAX_BWD: values N_l of the parents, same row index as src
    const float* own;          // OP_SOFTMAX_BWD: values N_{l-1} of the output rows
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
template <int OP>
__device__ __forceinline__ void accumulate(float& acc, float& mx, float x, float y, float nc, bool weighted = true) {
    if (OP == OP_SUM) acc += x;
    else if (OP == OP_PROD) acc *= x;
    else if (OP == OP_MAX) acc = fmaxf(acc, x);
    else if (OP == OP_LSE) {
        const float d = x - mx;                                   // +inf on the first finite element
        const float e = (x == -INFINITY) ? 0.0f : fexp(-fabsf(d));
        acc = (d > 0.0f) ? fmaf(acc, e, 1.0f) : acc + e;          // d is NaN only for -inf - -inf: e = 0
        mx = fmaxf(mx, x);
    } else {
        const float wgt = !weighted ? 1.0f : ((y == -INFINITY) ? 0.0f : fexp(nc - y));
        acc = fmaf(x, wgt, acc);
    }
}

template <int OP>
__device__ __forceinline__ float finish(float acc, float mx) {
    if (OP == OP_LSE) return (mx == -INFINITY) ? -INFINITY : mx + flog(acc);
    return acc;
}

template <int OP>
__device__ __forceinline__ float identity() { return OP == OP_PROD ? 1.0f : (OP == OP_MAX ? -INFINITY : 0.0f); }

// ---------------------------------------------------------------------------------------------
// Streaming segmented gather-reduce for B > 32 (one wave spans the batch tile, VEC columns per
// lane).  A task is a run of consecutive output rows with a bounded number of edges, fixed at
// build time; the wave walks the task's edges in chunks of CH, keeps CH row gathers in flight,
// prefetches the next chunk's index entries while they fly, and closes an output row whenever
// an entry carries the end-of-row bit.  Everything that steers control flow is wave-uniform.
// Index entries past a task's end are valid entries of later rows (or zero padding).
// ---------------------------------------------------------------------------------------------
template <int OP, int VEC>
__global__ __launch_bounds__(256) void stream_kernel(const int2* __restrict__ tasks, int n_tasks,
                                                     const uint32_t* __restrict__ idx,
                                                     const float* __restrict__ src,
                                                     const float* __restrict__ src2,
                                                     const float* __restrict__ own, float* __restrict__ dst,
                                                     int B, int ld, int stream_stores,
                                                     const int2* __restrict__ seg_tasks, int n_seg_tasks,
                                                     float* __restrict__ dst_seg) {
    // entries per chunk: measured on the headline workload, 4 (2 for the softmax adjoint, which loads
    // three rows per entry) beat 8 / 4 by 2%: the kernel is bandwidth-bound, fewer registers per wave
    // buy more resident waves
    constexpr int CH = (OP == OP_SOFTMAX_BWD) ? 2 : 4;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = ((int)blockIdx.y * 64 + lane) * VEC;
    if (col >= B) return;
    int t = xcd_block((int)blockIdx.x, (int)gridDim.x) * 4 + wave;
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
    for (int v = 0; v < VEC; ++v) { acc[v] = identity<OP>(); mx[v] = -INFINITY; nc[v] = 0.0f; }
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
                const int orow = rws[i] < last_row ? rws[i] : last_row;
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
            if (OP == OP_SOFTMAX_BWD) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) nc[v] = (live && first[i]) ? z[i][v] : nc[v];
            }
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const float dead = OP == OP_PROD ? 1.0f : ((OP == OP_LSE || OP == OP_MAX) ? -INFINITY : 0.0f);
                const float xv = live ? x[i][v] : dead;
                const float yv = OP == OP_SOFTMAX_BWD ? (live ? y[i][v] : -INFINITY) : 0.0f;
                accumulate<OP>(acc[v], mx[v], xv, yv, nc[v], (ids[i] & kWeighted) != 0);
            }
            if (live && (ids[i] & kLast)) {
                float o[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    o[v] = finish<OP>(acc[v], mx[v]);
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

// ---------------------------------------------------------------------------------------------
// Generic gather-reduce: a lane group of W lanes owns one output row (W < 64: several rows per
// wave, for small batches).  Also evaluates the segments of split rows (rows >= n_main, written
// to scratch rows) and the combine pass (out_row map).
// ---------------------------------------------------------------------------------------------
template <int OP, int VEC, int W>
__global__ __launch_bounds__(256) void pass_kernel(PassArgs a) {
    constexpr int RPW = 64 / W;                       // rows per wave
    constexpr int CH = (OP == OP_SOFTMAX_BWD) ? 4 : 8;    // sources in flight per lane
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
        if (OP == OP_SOFTMAX_BWD) {
            const int owner = row < a.n_main ? row : a.seg_owner[row - a.n_main];
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
                    accumulate<OP>(acc[v], mx[v], xv, yv, nc[v], wt[i]);
                }
            }
        }
        float o[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) o[v] = finish<OP>(acc[v], mx[v]);
        float* out;
        if (row < a.n_main) out = a.dst + (size_t)(a.out_row ? a.out_row[row] : row) * a.ld + col;
        else out = a.dst_seg + (size_t)(row - a.n_main) * a.ld + col;
        store_vec<VEC>(out, o);
    }
}

// ---------------------------------------------------------------------------------------------
// Persistent kernels for the narrow top of the circuit (layers that taper to the roots): instead
// of one launch per layer, a workgroup owns CT batch columns, keeps the values (forward) or the
// adjoints (backward) of the current and the previous layer in LDS and walks the layers with a
// barrier in between; batch columns are independent, so no grid-wide barrier is needed.  Each
// layer's index vectors are staged into LDS first.  Values are also written to the activation
// buffer, because the backward pass reads them.
//   LDS (floats): forward 2 * nmax * CT values, backward 3 * nmax * CT, then nmax + 1 + emax ints.
// A thread owns rows of one batch column, so writing the values into the row-major activation
// buffer costs one cache line per lane.  The values the reverse kernel needs therefore go to a
// tail value buffer tb[column][T] (T = rows of all tail layers), where consecutive threads write
// consecutive floats; only the first and the top tail layer (read by the regular reverse pass and
// by the root kernel) and, in the real semiring
// (whose reverse sweep runs layer by layer), every layer is also written to the activation buffer.
// ---------------------------------------------------------------------------------------------
struct TailLayer {
    int32_t n, e;          // nodes and edges of this layer
    int32_t n_below;       // nodes of the layer below
    int32_t fwd_off;       // [row_ptr (n+1) | child (e)] by parent, offset in ints into the index buffer
    int32_t bwd_off;       // [col_ptr (n_below+1) | parent (e)] by child
    int32_t tb_off;        // first entry of this layer in a column of the tail value buffer
    int64_t row0;          // first activation row of this layer
    int64_t row0_below;
};

constexpr int kTailThreads = 1024;
constexpr int kTailStash = 20;          // index entries per thread: covers rows + 1 + edges <= 20480

template <int OP, int CT>
__device__ __forceinline__ void tail_fwd_rows(const TailLayer& L, const int* ib, const float* prev, float* cur,
                                              const float* below, bool from_global, float* act_out, int ld,
                                              bool active, float* tb_out, bool write_act) {
    constexpr int RS = kTailThreads / CT;
    const int c = threadIdx.x % CT;
    for (int r = threadIdx.x / CT; r < L.n; r += RS) {
        const int beg = ib[r], end = ib[r + 1];
        float acc = identity<OP>(), mx = -INFINITY;
        const int* kids = ib + L.n + 1;
        int j = beg;
        for (; j + 4 <= end; j += 4) {                 // four independent reads in flight
            float x[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int ch = kids[j + u];
                if (from_global) x[u] = active ? below[(size_t)ch * ld] : identity<OP>();
                else x[u] = prev[ch * CT + c];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) accumulate<OP>(acc, mx, x[u], 0.0f, 0.0f);
        }
        for (; j < end; ++j) {
            const int ch = kids[j];
            float x;
            if (from_global) x = active ? below[(size_t)ch * ld] : identity<OP>();
            else x = prev[ch * CT + c];
            accumulate<OP>(acc, mx, x, 0.0f, 0.0f);
        }
        const float o = finish<OP>(acc, mx);
        cur[r * CT + c] = o;
        if (active) {
            tb_out[r] = o;
            if (write_act) act_out[(size_t)r * ld] = o;
        }
    }
}

template <int CT>
__global__ __launch_bounds__(kTailThreads) void tail_fwd_kernel(const TailLayer* __restrict__ layers, int n_layers,
                                                                int first_is_and, const int32_t* __restrict__ ibase,
                                                                float* act, int B, int ld, int semiring,
                                                                int nmax, float* __restrict__ tb, int T) {
    extern __shared__ float smem[];
    float* prev = smem;
    float* cur = smem + (size_t)nmax * CT;
    int* ib = reinterpret_cast<int*>(smem + (size_t)2 * nmax * CT);
    const int col = (int)blockIdx.x * CT + (int)(threadIdx.x % CT);
    const bool active = col < B;
    // The index vectors of a layer travel from global memory to registers two layers ahead (two
    // register stashes used in turn), so their latency is covered by two layers of evaluation.
    auto fetch = [&](int (&stash)[kTailStash], int t) {
        const TailLayer Lf = layers[t];
        const int32_t* g = ibase + Lf.fwd_off;
#pragma unroll
        for (int u = 0; u < kTailStash; ++u) {
            const int i = threadIdx.x + u * kTailThreads;
            stash[u] = i < Lf.n + 1 + Lf.e ? g[i] : 0;
        }
    };
    auto layer = [&](int (&stash)[kTailStash], int t) {
        const TailLayer L = layers[t];
#pragma unroll
        for (int u = 0; u < kTailStash; ++u) {
            const int i = threadIdx.x + u * kTailThreads;
            if (i < L.n + 1 + L.e) ib[i] = stash[u];
        }
        __syncthreads();
        if (t + 2 < n_layers) fetch(stash, t + 2);
        const bool is_and = ((t & 1) == 0) == (first_is_and != 0);
        const float* below = act + (size_t)L.row0_below * ld + col;
        float* out = act + (size_t)L.row0 * ld + col;
        const bool fg = t == 0;
        float* tbo = tb + (size_t)(active ? col : 0) * T + L.tb_off;
        // the first tail layer is read by the regular reverse pass below it, the top layer by the root kernel
        const bool wa = semiring == 0 || t == 0 || t == n_layers - 1;
        if (semiring == 2) {           // (max, +) on log weights
            if (is_and) tail_fwd_rows<OP_SUM, CT>(L, ib, prev, cur, below, fg, out, ld, active, tbo, wa);
            else tail_fwd_rows<OP_MAX, CT>(L, ib, prev, cur, below, fg, out, ld, active, tbo, wa);
        } else if (semiring == 1) {    // (logsumexp, +)
            if (is_and) tail_fwd_rows<OP_SUM, CT>(L, ib, prev, cur, below, fg, out, ld, active, tbo, wa);
            else tail_fwd_rows<OP_LSE, CT>(L, ib, prev, cur, below, fg, out, ld, active, tbo, wa);
        } else {
            if (is_and) tail_fwd_rows<OP_PROD, CT>(L, ib, prev, cur, below, fg, out, ld, active, tbo, wa);
            else tail_fwd_rows<OP_SUM, CT>(L, ib, prev, cur, below, fg, out, ld, active, tbo, wa);
        }
        __syncthreads();
        float* tmp = prev; prev = cur; cur = tmp;
    };
    int stash_a[kTailStash], stash_b[kTailStash];
    fetch(stash_a, 0);
    if (n_layers > 1) fetch(stash_b, 1);
    for (int t = 0; t < n_layers; t += 2) {
        layer(stash_a, t);
        if (t + 1 < n_layers) layer(stash_b, t + 1);
    }
}

// Reverse sweep over the same layers (log semiring): seeds the top layer's adjoints from dout,
// walks down to the first tail layer and leaves that layer's adjoints in g_out[n_first, ld].
template <int CT>
__global__ __launch_bounds__(kTailThreads) void tail_bwd_kernel(const TailLayer* __restrict__ layers, int n_layers,
                                                                int first_is_and, const int32_t* __restrict__ ibase,
                                                                const float* __restrict__ act,
                                                                const float* __restrict__ dout,
                                                                const int32_t* __restrict__ top_ptr,
                                                                const int32_t* __restrict__ top_root, int R,
                                                                float* __restrict__ g_out, int B, int ld, int nmax,
                                                                const float* __restrict__ tb, int T) {
    extern __shared__ float smem[];
    constexpr int RS = kTailThreads / CT;
    float* cur = smem;
    float* nxt = smem + (size_t)nmax * CT;
    float* nl = smem + (size_t)2 * nmax * CT;
    int* ib = reinterpret_cast<int*>(smem + (size_t)3 * nmax * CT);
    const int c = threadIdx.x % CT;
    const int col0 = (int)blockIdx.x * CT;
    const int col = col0 + c;
    const bool active = col < B;
    {   // adjoint seed of the top layer
        const TailLayer L = layers[n_layers - 1];
        for (int i = threadIdx.x / CT; i < L.n; i += RS) {
            float acc = 0.0f;
            if (active)
                for (int t = top_ptr[i]; t < top_ptr[i + 1]; ++t) acc += dout[(size_t)col * R + top_root[t]];
            cur[i * CT + c] = acc;
        }
    }
    // step t (adjoints of layer t -> layer t-1) uses the by-child index vectors of layer t; they are
    // fetched two steps ahead into two register stashes used in turn
    auto fetch = [&](int (&stash)[kTailStash], int t) {
        const TailLayer Lf = layers[t];
        const int32_t* g = ibase + Lf.bwd_off;
#pragma unroll
        for (int u = 0; u < kTailStash; ++u) {
            const int i = threadIdx.x + u * kTailThreads;
            stash[u] = i < Lf.n_below + 1 + Lf.e ? g[i] : 0;
        }
    };
    auto step = [&](int (&stash)[kTailStash], int t) {
        const TailLayer L = layers[t];
        const bool is_and = ((t & 1) == 0) == (first_is_and != 0);
#pragma unroll
        for (int u = 0; u < kTailStash; ++u) {
            const int i = threadIdx.x + u * kTailThreads;
            if (i < L.n_below + 1 + L.e) ib[i] = stash[u];
        }
        if (t - 2 >= 1) fetch(stash, t - 2);
        if (!is_and)
            for (int i = threadIdx.x; i < L.n * CT; i += kTailThreads) {
                const int cc = col0 + i % CT;
                nl[i] = cc < B ? tb[(size_t)cc * T + L.tb_off + i / CT] : 0.0f;
            }
        __syncthreads();
        const int off_below = layers[t - 1].tb_off;
        for (int r = threadIdx.x / CT; r < L.n_below; r += RS) {
            const int beg = ib[r], end = ib[r + 1];
            float acc = 0.0f, mx = 0.0f;
            if (is_and) {
                for (int j = beg; j < end; ++j) acc += cur[(ib[L.n_below + 1 + j] & (int)kIdMask) * CT + c];
            } else {
                const float own = active ? tb[(size_t)col * T + off_below + r] : 0.0f;
                for (int j = beg; j < end; ++j) {
                    // an unweighted edge (chain node or single-child OR above) passes the adjoint unchanged
                    const uint32_t pe = (uint32_t)ib[L.n_below + 1 + j];
                    const int p = (int)(pe & kIdMask);
                    accumulate<OP_SOFTMAX_BWD>(acc, mx, cur[p * CT + c], nl[p * CT + c], own, (pe & kWeighted) != 0);
                }
            }
            nxt[r * CT + c] = acc;
        }
        __syncthreads();
        float* tmp = cur; cur = nxt; nxt = tmp;
    };
    int stash_a[kTailStash], stash_b[kTailStash];
    if (n_layers - 1 >= 1) fetch(stash_a, n_layers - 1);
    if (n_layers - 2 >= 1) fetch(stash_b, n_layers - 2);
    for (int t = n_layers - 1; t >= 1; t -= 2) {
        step(stash_a, t);
        if (t - 1 >= 1) step(stash_b, t - 1);
    }
    const int n_first = layers[0].n;
    if (active)
        for (int r = threadIdx.x / CT; r < n_first; r += RS) g_out[(size_t)r * ld + col] = cur[r * CT + c];
}

// ---------------------------------------------------------------------------------------------
// Reverse sweep of a product (AND) layer in the real semiring.  The adjoint of child j of parent r
// is G[r] times the product of r's other children.  Per parent the kernel forms, per batch column,
// the product q of the non-zero children and the number z of zero children, and writes per edge
//   M[j] = G[r] * (x_j != 0 ? (z == 0 ? q / x_j : 0) : (z == 1 ? q : 0)),
// which is exact also when children are zero (p = 0 or p = 1 leaves).  A by-child sum over M then
// gives the adjoints of the layer below.  A lane group of W lanes owns one parent row.
// ---------------------------------------------------------------------------------------------
template <int VEC, int W>
__global__ __launch_bounds__(256) void prod_edge_kernel(const int32_t* __restrict__ ptr,
                                                        const int32_t* __restrict__ child,
                                                        const float* __restrict__ below,
                                                        const float* __restrict__ g, float* __restrict__ M, int n,
                                                        int B, int ld) {
    constexpr int RPW = 64 / W;
    const int lane = threadIdx.x & 63;
    const int col = ((int)blockIdx.y * W + (lane % W)) * VEC;
    if (col >= B) return;
    const int64_t row64 = ((int64_t)blockIdx.x * 4 + (threadIdx.x >> 6)) * RPW + lane / W;
    if (row64 >= n) return;
    const int row = (int)row64;
    const int beg = ptr[row], end = ptr[row + 1];
    float q[VEC], z[VEC], gr[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) { q[v] = 1.0f; z[v] = 0.0f; }
    load_vec<VEC>(gr, g + (size_t)row * ld + col);
    constexpr int CH = 8;
    float x[CH][VEC];
    // first pass: 8 gathers in flight (entries past the row's end re-read its last child), product of
    // the non-zero children and count of the zero ones
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
    // second pass: per-edge products; a row of at most 8 children still has them in registers
    const bool short_row = end - beg <= CH;
    for (int j = beg; j < end; j += CH) {
        if (!short_row) {
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                const int jj = j + i < end ? j + i : end - 1;
                load_vec<VEC>(x[i], below + (size_t)child[jj] * ld + col);
            }
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            if (j + i < end) {
                float m[VEC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const float xv = x[i][v];
                    const float others = xv != 0.0f ? (z[v] == 0.0f ? q[v] / xv : 0.0f) : (z[v] == 1.0f ? q[v] : 0.0f);
                    m[v] = gr[v] * others;
                }
                store_vec<VEC>(M + (size_t)(j + i) * ld + col, m);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Leaf layer: leaf_weights[B,V] (batch-outer) -> wT[V,ld] (kept for the backward pass) and the
// literal rows of layer 0; the negated literal gets 1-p (REAL) or log(1-exp(x)) (LOG).
// Tile = 32 variables x 64 batch columns through LDS.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float log1mexp_f(float x) {
    return x > -0.69314718f ? logf(-expm1f(x)) : log1pf(-expf(x));
}

// Leaf layer: transposes leaf weights [B, V] into rows [*, ld] through an LDS tile.  The negated
// literal of v gets wneg[b, v] when the caller supplies weights of its own for the negated literals,
// otherwise 1 - w (real semiring) or log(1 - exp(w)) (log domain).
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
__global__ void seed_kernel(const float* __restrict__ dout, const int32_t* __restrict__ top_ptr,
                            const int32_t* __restrict__ top_root, int B, int R, int ld,
                            float* __restrict__ g) {
    const int i = blockIdx.x;
    for (int b = threadIdx.x; b < ld; b += blockDim.x) {
        float acc = 0.0f;
        if (b < B)
            for (int t = top_ptr[i]; t < top_ptr[i + 1]; ++t) acc += dout[(size_t)b * R + top_root[t]];
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
