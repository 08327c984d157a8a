// Double-precision evaluation of the same launch plans (accuracy build): one generic gather-reduce
// kernel, a wave per output row and one or two batch columns per lane, plus the small leaf / root / seed
// kernels.  Same index arrays, same order of layers and the same split-row scheme as the fp32
// kernels (paper Section 4, Alg. 1 / Appendix C, Alg. 4); exp and log are the full-precision
// library routines.  Not tuned: the rows are twice as long and OR layers pay a double-precision
// exponential per edge.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "klay_kernels.hip.h"

namespace klay {
namespace f64 {

struct PassArgs {
    const int32_t* ptr;        // [n_total + 1] CSR offsets into idx
    const uint32_t* idx;       // index entries (readable up to 16 entries past the end)
    const double* src;         // [*, ld] source rows
    const double* src2;        // OP_SOFTMAX_BWD: values of the parents, same row index as src
    const double* own;         // OP_SOFTMAX_BWD: values of the output rows
    const int32_t* seg_owner;  // output row owning segment i (rows >= n_main), may be null
    const int32_t* out_row;    // optional output row map for rows < n_main (combine pass)
    double* dst;               // output rows for rows < n_main
    double* dst_seg;           // scratch rows for rows >= n_main
    int32_t n_main;
    int32_t n_total;
    int32_t B;
    int32_t ld;
};

template <int OP>
__device__ __forceinline__ double identity() { return OP == OP_PROD ? 1.0 : (OP == OP_MAX ? -INFINITY : 0.0); }

// same streaming forms as the fp32 accumulate: (mx, acc) = (running max, sum of exp(x - mx))
template <int OP>
__device__ __forceinline__ void accumulate(double& acc, double& mx, double x, double y, double nc, bool weighted) {
    if (OP == OP_PROD_BWD) {       // as the fp32 form: x is an AND parent's P row (lowest bit: one zero child)
        const unsigned long long bits = (unsigned long long)__double_as_longlong(x);
        const double val = __longlong_as_double((long long)(bits & ~1ull));
        const bool one_zero = (bits & 1ull) != 0;
        const double part = one_zero ? (nc == 0.0 ? val : 0.0) : (nc != 0.0 ? val / nc : 0.0);
        acc += weighted ? x : part;
        return;
    }
    if (OP == OP_SUM) acc += x;
    else if (OP == OP_PROD) acc *= x;
    else if (OP == OP_MAX) acc = fmax(acc, x);
    else if (OP == OP_LSE) {
        const double d = x - mx;
        const double e = (x == -INFINITY) ? 0.0 : exp(-fabs(d));
        acc = (d > 0.0) ? fma(acc, e, 1.0) : acc + e;
        mx = fmax(mx, x);
    } else {
        const double wgt = !weighted ? 1.0 : ((y == -INFINITY) ? 0.0 : exp(nc - y));
        acc = fma(x, wgt, acc);
    }
}

template <int OP>
__device__ __forceinline__ double finish(double acc, double mx) {
    if (OP == OP_LSE) return (mx == -INFINITY) ? -INFINITY : mx + log(acc);
    return acc;
}

template <int VEC>
__device__ __forceinline__ void load_vec(double (&x)[VEC], const double* p) {
    if (VEC == 2) {
        const double2 t = *reinterpret_cast<const double2*>(p);
        x[0] = t.x;
        x[VEC - 1] = t.y;
    } else {
        x[0] = *p;
    }
}

// VEC batch columns per lane (2 needs an even ld): a wave spans 64 * VEC columns of one row
template <int OP, int VEC>
__global__ __launch_bounds__(256) void pass_kernel(PassArgs a) {
    constexpr int CH = 4;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int col = ((int)blockIdx.y * 64 + lane) * VEC;
    if (col >= a.B) return;
    const int64_t row64 = (int64_t)blockIdx.x * 4 + wave;
    if (row64 >= a.n_total) return;
    const int row = (int)row64;
    const int beg = a.ptr[row], end = a.ptr[row + 1];
    if (a.idx[beg] == kSkip) return;                  // split row: evaluated by segments + combine
    double nc[VEC], acc[VEC], mx[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) { nc[v] = 0.0; acc[v] = identity<OP>(); mx[v] = -INFINITY; }
    if (OP == OP_SOFTMAX_BWD || OP == OP_PROD_BWD) {
        const int owner = row < a.n_main ? row : a.seg_owner[row - a.n_main];
        load_vec<VEC>(nc, a.own + (size_t)owner * a.ld + col);
    }
    for (int j = beg; j < end; j += CH) {
        const int n = end - j;
        double x[CH][VEC], y[CH][VEC];
        bool wt[CH];
        // entries past the row's end are valid entries of later rows (or zero padding): the gathers
        // are issued unconditionally and their data ignored
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const uint32_t raw = a.idx[j + i];
            const uint32_t id = raw == kSkip ? 0u : (raw & kIdMask);
            wt[i] = (raw & kWeighted) != 0;
            load_vec<VEC>(x[i], a.src + (size_t)id * a.ld + col);
            if (OP == OP_SOFTMAX_BWD) load_vec<VEC>(y[i], (wt[i] ? a.src2 : a.src) + (size_t)id * a.ld + col);
        }
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const bool live = i < n;
            const double dead = OP == OP_PROD ? 1.0 : ((OP == OP_LSE || OP == OP_MAX) ? -INFINITY : 0.0);
#pragma unroll
            for (int v = 0; v < VEC; ++v)
                accumulate<OP>(acc[v], mx[v], live ? x[i][v] : dead,
                               OP == OP_SOFTMAX_BWD ? (live ? y[i][v] : -INFINITY) : 0.0, nc[v], wt[i]);
        }
    }
    double* out;
    if (row < a.n_main) out = a.dst + (size_t)(a.out_row ? a.out_row[row] : row) * a.ld + col;
    else out = a.dst_seg + (size_t)(row - a.n_main) * a.ld + col;
    if (VEC == 2) *reinterpret_cast<double2*>(out) = make_double2(finish<OP>(acc[0], mx[0]), finish<OP>(acc[VEC - 1], mx[VEC - 1]));
    else *out = finish<OP>(acc[0], mx[0]);
}

__device__ __forceinline__ double log1mexp(double x) {
    return x > -0.6931471805599453 ? log(-expm1(x)) : log1p(-exp(x));
}

// leaf layer: thread per (variable, batch column); negated literal as in the fp32 kernel
__global__ void leaf_fwd_kernel(const double* __restrict__ w, const double* __restrict__ wneg, int B, int V, int ld,
                                const int32_t* __restrict__ pos_row, const int32_t* __restrict__ neg_row,
                                double* __restrict__ wT, double* __restrict__ act0, int log_domain) {
    const int b = blockIdx.y * blockDim.x + threadIdx.x;
    const int v = blockIdx.x;
    if (b >= ld) return;
    const double x = b < B ? w[(size_t)b * V + v] : 0.0;
    wT[(size_t)v * ld + b] = x;
    const int pr = pos_row[v], nr = neg_row[v];
    if (pr >= 0) act0[(size_t)pr * ld + b] = x;
    if (nr >= 0) {
        double y;
        if (b >= B) y = 0.0;
        else if (wneg) y = wneg[(size_t)b * V + v];
        else y = log_domain ? log1mexp(x) : 1.0 - x;
        act0[(size_t)nr * ld + b] = y;
    }
}

__global__ void fill_row_kernel(double* row, int ld, double value) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < ld) row[b] = value;
}

__global__ void root_out_kernel(const double* __restrict__ top, const int32_t* __restrict__ root_pos, int B, int R,
                                int ld, double* __restrict__ out) {
    const int r = blockIdx.x;
    const double* row = top + (size_t)root_pos[r] * ld;
    for (int b = threadIdx.x; b < B; b += blockDim.x) out[(size_t)b * R + r] = row[b];
}

__global__ void seed_kernel(const double* __restrict__ dout, const int32_t* __restrict__ top_ptr,
                            const int32_t* __restrict__ top_root, int B, int R, int ld, double* __restrict__ g) {
    const int i = blockIdx.x;
    for (int b = threadIdx.x; b < ld; b += blockDim.x) {
        double acc = 0.0;
        if (b < B)
            for (int t = top_ptr[i]; t < top_ptr[i + 1]; ++t) acc += dout[(size_t)b * R + top_root[t]];
        g[(size_t)i * ld + b] = acc;
    }
}

__global__ void seed_rows_kernel(const double* __restrict__ dout, int B, int R, int ld, double* __restrict__ rows) {
    const int r = blockIdx.x;
    for (int b = threadIdx.x; b < ld; b += blockDim.x) rows[(size_t)r * ld + b] = b < B ? dout[(size_t)b * R + r] : 0.0;
}

// Real-semiring reverse sweep of a product layer, first half, as the fp32 kernel of the same name: the
// adjoint row of every AND parent is replaced in place by P = G * (product of the non-zero children),
// 0 with two or more zero children, lowest mantissa bit = exactly one zero child.  A wave per parent
// row, a lane per batch column.
__global__ __launch_bounds__(256) void prod_parent_kernel(const int32_t* __restrict__ ptr, const int32_t* __restrict__ child,
                                                          const double* __restrict__ below, double* __restrict__ g,
                                                          int n, int B, int ld) {
    const int lane = threadIdx.x & 63;
    const int col = (int)blockIdx.y * 64 + lane;
    if (col >= B) return;
    const int64_t row64 = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row64 >= n) return;
    const int row = (int)row64;
    const int beg = ptr[row], end = ptr[row + 1];
    double q = 1.0;
    int z = 0;
    for (int j = beg; j < end; ++j) {
        const double x = below[(size_t)child[j] * ld + col];
        if (x == 0.0) ++z;
        else q *= x;
    }
    const double val = z >= 2 ? 0.0 : g[(size_t)row * ld + col] * q;
    const unsigned long long bits = ((unsigned long long)__double_as_longlong(val) & ~1ull) | (z == 1 ? 1ull : 0ull);
    g[(size_t)row * ld + col] = __longlong_as_double((long long)bits);
}

// mode 0: negated weight 1 - w; mode 1: log(1 - exp(w)); mode 2: the negated literals have weights of their own
__global__ void leaf_bwd_kernel(const double* __restrict__ g0, const double* __restrict__ wT,
                                const int32_t* __restrict__ pos_row, const int32_t* __restrict__ neg_row, int B,
                                int V, int ld, int mode, double* __restrict__ dleaf, double* __restrict__ dneg) {
    const int b = blockIdx.y * blockDim.x + threadIdx.x;
    const int v = blockIdx.x;
    if (b >= B) return;
    const int pr = pos_row[v], nr = neg_row[v];
    double d = 0.0, dn = 0.0;
    if (pr >= 0) d = g0[(size_t)pr * ld + b];
    if (nr >= 0) {
        const double gn = g0[(size_t)nr * ld + b];
        if (mode == 2) dn = gn;
        else if (gn != 0.0) d += mode == 1 ? -gn / expm1(-wT[(size_t)v * ld + b]) : -gn;
    }
    dleaf[(size_t)b * V + v] = d;
    if (mode == 2 && dneg) dneg[(size_t)b * V + v] = dn;
}

}  // namespace f64
}  // namespace klay
