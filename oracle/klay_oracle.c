/*
 * fp64 CPU oracle for arithmetic-circuit evaluation.  TEST INFRASTRUCTURE ONLY:
 * it exists so that the GPU library can be checked against something that is
 * obviously right.  It shares no code with the GPU library and must never be
 * called from the product path.
 *
 * What it computes is the node-value definition of the paper (Section 2, Eq. 1,
 * and the arithmetic-circuit reading that follows it): leaves carry weights,
 * AND gates multiply, OR gates add, children before parents.  The circuit is
 * the ORIGINAL linked-node DAG; nothing here knows about layers, unary padding
 * nodes, hashing or index vectors.  The log-domain variant follows Section 4 /
 * Appendix C (Alg. 4): AND adds, OR is a max-shifted logsumexp, with epsilon
 * read as 0 (an all -inf OR gives -inf).  Section 4 closes with the remark that any
 * pair of operations forming a semiring may be used; S_MAXLOG is the (max, +) semiring
 * on log weights (AND adds, OR takes the maximum: the log weight of the heaviest proof
 * tree, i.e. of the most probable model for a smooth d-DNNF), forward only.
 *
 * The backward pass is plain reverse-mode differentiation of exactly that
 * traversal (the paper delegates it to autograd, Section 6).
 *
 * Pins (see tests): closed forms of the paper's worked circuits, brute-force
 * weighted model counting, the tautology invariant, finite differences,
 * cross-semiring identities, scipy's logsumexp; for (max, +): enumeration of all
 * proof trees and of all models of a smooth d-DNNF.  Parity unpinned: nothing.
 *
 * Circuit encoding (all host memory, read-only):
 *   node_type[n]  0 literal, 1 AND, 2 OR, 3 TRUE, 4 FALSE
 *   node_lit[n]   for literals +(v+1) / -(v+1), v in [0,V)
 *   child_ptr[n+1], child_idx[]  children of gate i are child_idx[child_ptr[i]..child_ptr[i+1])
 *   roots[R]
 * Leaf weights: w[b*V+v] is p_v (REAL) or log p_v (LOG); the negative literal
 * gets 1-p resp. log(1-exp(x)), unless a second array wneg[b*V+v] gives the negative
 * literals weights of their own (weighted model counting with arbitrary literal weights;
 * the two arrays are then independent inputs with a gradient each).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { T_LIT = 0, T_AND = 1, T_OR = 2, T_TRUE = 3, T_FALSE = 4 };
enum { S_REAL = 0, S_LOG = 1, S_MAXLOG = 2 };

/* log(1 - exp(x)) for x <= 0, the usual two-branch form. */
static double log1mexp(double x) {
    if (x > -0.6931471805599453) return log(-expm1(x));
    return log1p(-exp(x));
}

/*
 * Post-order (children before parents) of every node reachable from the roots,
 * by an explicit-stack depth-first search.  Returns the number of nodes written
 * to order[], or -1 if a cycle is met, -2 on allocation failure.
 */
int64_t klay_oracle_postorder(int64_t num_nodes, const int64_t* child_ptr,
                              const int32_t* child_idx, int32_t num_roots,
                              const int32_t* roots, int32_t* order) {
    /* state: 0 unseen, 1 on stack (open), 2 done */
    uint8_t* state = (uint8_t*)calloc((size_t)num_nodes + 1, 1);
    int32_t* stack = (int32_t*)malloc(sizeof(int32_t) * ((size_t)num_nodes + 1));
    int64_t* next = (int64_t*)malloc(sizeof(int64_t) * ((size_t)num_nodes + 1));
    if (!state || !stack || !next) { free(state); free(stack); free(next); return -2; }
    int64_t count = 0, sp = 0;
    for (int32_t r = 0; r < num_roots; ++r) {
        int32_t s = roots[r];
        if (state[s] == 2) continue;
        stack[sp++] = s; state[s] = 1; next[s] = child_ptr[s];
        while (sp > 0) {
            int32_t n = stack[sp - 1];
            if (next[n] < child_ptr[n + 1]) {
                int32_t c = child_idx[next[n]++];
                if (state[c] == 1) { free(state); free(stack); free(next); return -1; }
                if (state[c] == 0) { state[c] = 1; next[c] = child_ptr[c]; stack[sp++] = c; }
            } else {
                state[n] = 2; order[count++] = n; --sp;
            }
        }
    }
    free(state); free(stack); free(next);
    return count;
}

/* Value of every node in `order` for one batch column; w points at V weights. */
static void eval_column(int semiring, const uint8_t* node_type, const int32_t* node_lit,
                        const int64_t* child_ptr, const int32_t* child_idx,
                        const int32_t* order, int64_t n_order, const double* w, const double* wn,
                        double* val) {
    for (int64_t i = 0; i < n_order; ++i) {
        int32_t n = order[i];
        int64_t a = child_ptr[n], e = child_ptr[n + 1];
        double v;
        switch (node_type[n]) {
        case T_LIT: {
            int32_t l = node_lit[n];
            double x = w[(l > 0 ? l : -l) - 1];
            if (l < 0 && wn) v = wn[-l - 1];
            else if (semiring == S_REAL) v = l > 0 ? x : 1.0 - x;
            else v = l > 0 ? x : log1mexp(x);
            break;
        }
        case T_TRUE: v = semiring == S_REAL ? 1.0 : 0.0; break;
        case T_FALSE: v = semiring == S_REAL ? 0.0 : -INFINITY; break;
        case T_AND:
            if (semiring == S_REAL) { v = 1.0; for (int64_t j = a; j < e; ++j) v *= val[child_idx[j]]; }
            else { v = 0.0; for (int64_t j = a; j < e; ++j) v += val[child_idx[j]]; }
            break;
        default: /* T_OR */
            if (semiring == S_REAL) { v = 0.0; for (int64_t j = a; j < e; ++j) v += val[child_idx[j]]; }
            else if (semiring == S_MAXLOG) {
                v = -INFINITY;
                for (int64_t j = a; j < e; ++j) if (val[child_idx[j]] > v) v = val[child_idx[j]];
            } else {
                double m = -INFINITY;
                for (int64_t j = a; j < e; ++j) if (val[child_idx[j]] > m) m = val[child_idx[j]];
                if (m == -INFINITY) v = -INFINITY;
                else if (m == INFINITY) v = INFINITY;
                else {
                    double t = 0.0;
                    for (int64_t j = a; j < e; ++j) t += exp(val[child_idx[j]] - m);
                    v = log(t) + m;
                }
            }
            break;
        }
        val[n] = v;
    }
}

/*
 * Forward.  out[b*R+r] = value of roots[r] on column b.  node_vals (nullable) receives
 * every reachable node's value as node_vals[b*num_nodes+n] (unreachable nodes: NaN).
 * Returns 0, -1 cycle, -2 out of memory.
 */
int klay_oracle_forward(int32_t num_vars, int64_t num_nodes, const uint8_t* node_type,
                        const int32_t* node_lit, const int64_t* child_ptr,
                        const int32_t* child_idx, int32_t num_roots, const int32_t* roots,
                        int32_t B, const double* w, const double* wneg, int semiring, double* out,
                        double* node_vals, int nthreads) {
    int32_t* order = (int32_t*)malloc(sizeof(int32_t) * ((size_t)num_nodes + 1));
    if (!order) return -2;
    int64_t n_order = klay_oracle_postorder(num_nodes, child_ptr, child_idx, num_roots, roots, order);
    if (n_order < 0) { free(order); return (int)n_order; }
    int fail = 0;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel num_threads(nthreads)
    {
        double* val = (double*)malloc(sizeof(double) * ((size_t)num_nodes + 1));
        if (!val) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int32_t b = 0; b < B; ++b) {
            if (!val) continue;
            if (node_vals) for (int64_t i = 0; i < num_nodes; ++i) val[i] = NAN;
            eval_column(semiring, node_type, node_lit, child_ptr, child_idx, order, n_order,
                        w + (size_t)b * num_vars, wneg ? wneg + (size_t)b * num_vars : NULL, val);
            for (int32_t r = 0; r < num_roots; ++r) out[(size_t)b * num_roots + r] = val[roots[r]];
            if (node_vals) memcpy(node_vals + (size_t)b * num_nodes, val, sizeof(double) * (size_t)num_nodes);
        }
        free(val);
    }
    free(order);
    return fail ? -2 : 0;
}

/*
 * Backward: dleaf[b*V+v] = sum_r dout[b*R+r] * d out[b,r] / d w[b,v], by reverse-mode
 * accumulation over the same traversal (forward recomputed per column).
 *   AND-LOG, OR-REAL : adj(c) += adj(n)
 *   OR-LOG           : adj(c) += adj(n) * exp(val(c) - val(n)); nothing if val(n) = -inf
 *   AND-REAL         : adj(c) += adj(n) * prod of the other children (prefix/suffix products)
 *   OR gate (LOG)    : child += adj * exp(child value - gate value); a gate at -inf (every child
 *                      impossible, weights 0/0) passes nothing, except that a gate with a single child
 *                      is the identity and passes adj unchanged whatever its value: Section 3.1 builds
 *                      its chains out of exactly such unary gates, so an input gate with one child must
 *                      behave like a chain node, which is transparent.
 *   literal +v       : dleaf += adj
 *   literal -v       : dleaf += adj * d(neg weight)/dw = -adj (REAL), -adj / expm1(-x) (LOG);
 *                      a zero adjoint contributes 0 even where that derivative is infinite.
 *                      With wneg given: dneg += adj instead (dleaf then holds the positive literals only).
 * With abs_mode != 0 the same sweep runs on |dout| and adds |adj * d(neg weight)/dw| at negated
 * literals, so that dleaf becomes the sum over all root-to-leaf paths of |contribution|: the
 * scale against which a floating-point gradient's cancellation error has to be judged.
 */
int klay_oracle_backward(int32_t num_vars, int64_t num_nodes, const uint8_t* node_type,
                         const int32_t* node_lit, const int64_t* child_ptr,
                         const int32_t* child_idx, int32_t num_roots, const int32_t* roots,
                         int32_t B, const double* w, const double* wneg, int semiring, const double* dout,
                         double* dleaf, double* dneg, int nthreads, int abs_mode) {
    if ((wneg == NULL) != (dneg == NULL)) return -3;
    if (semiring != S_REAL && semiring != S_LOG) return -3;   /* (max, +) is not differentiated */
    int32_t* order = (int32_t*)malloc(sizeof(int32_t) * ((size_t)num_nodes + 1));
    if (!order) return -2;
    int64_t n_order = klay_oracle_postorder(num_nodes, child_ptr, child_idx, num_roots, roots, order);
    if (n_order < 0) { free(order); return (int)n_order; }
    int64_t max_fan = 1;
    for (int64_t n = 0; n < num_nodes; ++n)
        if (child_ptr[n + 1] - child_ptr[n] > max_fan) max_fan = child_ptr[n + 1] - child_ptr[n];
    int fail = 0;
    if (nthreads < 1) nthreads = 1;
#pragma omp parallel num_threads(nthreads)
    {
        double* val = (double*)malloc(sizeof(double) * ((size_t)num_nodes + 1));
        double* adj = (double*)malloc(sizeof(double) * ((size_t)num_nodes + 1));
        double* pre = (double*)malloc(sizeof(double) * ((size_t)max_fan + 1));
        if (!val || !adj || !pre) {
#pragma omp atomic write
            fail = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int32_t b = 0; b < B; ++b) {
            if (!val || !adj || !pre) continue;
            const double* wb = w + (size_t)b * num_vars;
            double* gb = dleaf + (size_t)b * num_vars;
            const double* wnb = wneg ? wneg + (size_t)b * num_vars : NULL;
            double* gnb = dneg ? dneg + (size_t)b * num_vars : NULL;
            eval_column(semiring, node_type, node_lit, child_ptr, child_idx, order, n_order, wb, wnb, val);
            for (int64_t i = 0; i < n_order; ++i) adj[order[i]] = 0.0;
            for (int32_t v = 0; v < num_vars; ++v) gb[v] = 0.0;
            if (gnb) for (int32_t v = 0; v < num_vars; ++v) gnb[v] = 0.0;
            for (int32_t r = 0; r < num_roots; ++r) {
                double d = dout[(size_t)b * num_roots + r];
                adj[roots[r]] += abs_mode ? fabs(d) : d;
            }
            for (int64_t i = n_order - 1; i >= 0; --i) {
                int32_t n = order[i];
                double g = adj[n];
                int64_t a = child_ptr[n], e = child_ptr[n + 1];
                switch (node_type[n]) {
                case T_LIT: {
                    int32_t l = node_lit[n];
                    int32_t v = (l > 0 ? l : -l) - 1;
                    if (l > 0) gb[v] += g;
                    else if (gnb) gnb[v] += g;          /* a weight of its own: adj passes straight through */
                    else if (g != 0.0) {
                        double t = semiring == S_REAL ? -g : -g / expm1(-wb[v]);
                        gb[v] += abs_mode ? fabs(t) : t;
                    }
                    break;
                }
                case T_AND:
                    if (semiring == S_LOG) { for (int64_t j = a; j < e; ++j) adj[child_idx[j]] += g; }
                    else {
                        int64_t k = e - a;
                        pre[0] = 1.0;
                        for (int64_t j = 0; j < k; ++j) pre[j + 1] = pre[j] * val[child_idx[a + j]];
                        double suf = 1.0;
                        for (int64_t j = k - 1; j >= 0; --j) {
                            adj[child_idx[a + j]] += g * pre[j] * suf;
                            suf *= val[child_idx[a + j]];
                        }
                    }
                    break;
                case T_OR:
                    if (semiring == S_REAL) { for (int64_t j = a; j < e; ++j) adj[child_idx[j]] += g; }
                    else if (e - a == 1) adj[child_idx[a]] += g;   /* a unary OR is the identity, also at -inf */
                    else if (val[n] != -INFINITY) {
                        for (int64_t j = a; j < e; ++j) adj[child_idx[j]] += g * exp(val[child_idx[j]] - val[n]);
                    }
                    break;
                default: break;
                }
            }
        }
        free(val); free(adj); free(pre);
    }
    free(order);
    return fail ? -2 : 0;
}

int klay_oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
