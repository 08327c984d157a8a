/* Plain C user of the C ABI: include/klay.h must compile as C, and the library must be usable
 * without Python.  Builds the circuit of the paper's Figure 1(b) as a host-only handle and checks the
 * layer sizes of Figure 2 (Section 3.1).  With the argument "gpu" it also evaluates the circuit on
 * device 0 and compares with the closed form of the figure:
 *   P = (1-a)(1 - b c (1-d)) + a (1 - (1-c) d). */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../include/klay.h"

/* tiny HIP runtime surface, declared here so that this file needs no HIP headers */
extern int hipMalloc(void** p, size_t n);
extern int hipFree(void* p);
extern int hipMemcpy(void* dst, const void* src, size_t n, int kind);
extern int hipDeviceSynchronize(void);

#define CHECK(x) do { if (!(x)) { printf("FAILED line %d: %s (%s)\n", __LINE__, #x, klay_last_error()); return 1; } } while (0)

int main(int argc, char** argv) {
    /* variables a b c d = 0..3; literals as +-(v+1) */
    enum { A = 1, B = 2, C = 3, D = 4 };
    /* nodes: 0..7 literals a -a b -b c -c d -d; 8 n30 = AND(c,d); 9 n20 = OR(n30,-c); 10 n21 = OR(n30,-d);
       11 n10 = AND(-b,-a); 12 n11 = AND(-a,b,n20); 13 n12 = AND(n21,a); 14 root = OR(n10,n11,n12) */
    const uint8_t type[15] = {0, 0, 0, 0, 0, 0, 0, 0, KLAY_AND, KLAY_OR, KLAY_OR, KLAY_AND, KLAY_AND, KLAY_AND, KLAY_OR};
    const int32_t lit[15] = {A, -A, B, -B, C, -C, D, -D, 0, 0, 0, 0, 0, 0, 0};
    const int64_t ptr[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 2, 4, 6, 8, 11, 13, 16};
    const int32_t idx[16] = {4, 6, 8, 5, 8, 7, 3, 1, 1, 2, 9, 10, 0, 11, 12, 13};
    const int32_t roots[1] = {14};
    klay_circuit* c = NULL;
    klay_options opt;
    memset(&opt, 0, sizeof(opt));
    CHECK(klay_build_ex(4, 15, type, lit, ptr, idx, 1, roots, -1, &opt, &c) == KLAY_OK);
    klay_info_t info;
    CHECK(klay_info(c, &info) == KLAY_OK);
    CHECK(info.num_layers == 4 && info.num_roots == 1 && info.device == -1);
    int64_t nodes[5], edges[5];
    CHECK(klay_layer_sizes(c, nodes, edges) == KLAY_OK);
    const int64_t want_nodes[5] = {8, 7, 6, 3, 1}, want_edges[5] = {0, 9, 8, 6, 3};
    for (int l = 0; l <= 4; ++l) CHECK(nodes[l] == want_nodes[l] && edges[l] == want_edges[l]);
    float dummy;
    CHECK(klay_forward(c, &dummy, 1, &dummy, KLAY_LOG, NULL) == KLAY_ESTATE);   /* host-only handle */
    CHECK(strlen(klay_last_error()) > 0);
    klay_destroy(c);
    /* errors are reported, not thrown */
    const int32_t bad_roots[1] = {99};
    CHECK(klay_build(4, 15, type, lit, ptr, idx, 1, bad_roots, -1, &c) == KLAY_EINVAL && c == NULL);

    if (argc > 1 && strcmp(argv[1], "gpu") == 0) {
        CHECK(klay_build(4, 15, type, lit, ptr, idx, 1, roots, 0, &c) == KLAY_OK);
        const float p[2][4] = {{0.3f, 0.6f, 0.2f, 0.9f}, {0.5f, 0.5f, 0.5f, 0.5f}};
        float logp[2][4], out[2], dleaf[2][4];
        for (int b = 0; b < 2; ++b) for (int v = 0; v < 4; ++v) logp[b][v] = logf(p[b][v]);
        float *d_w = NULL, *d_out = NULL, *d_dout = NULL, *d_dleaf = NULL;
        CHECK(hipMalloc((void**)&d_w, sizeof(logp)) == 0 && hipMalloc((void**)&d_out, sizeof(out)) == 0);
        CHECK(hipMalloc((void**)&d_dout, sizeof(out)) == 0 && hipMalloc((void**)&d_dleaf, sizeof(dleaf)) == 0);
        const float ones[2] = {1.0f, 1.0f};
        CHECK(hipMemcpy(d_w, logp, sizeof(logp), 1) == 0 && hipMemcpy(d_dout, ones, sizeof(ones), 1) == 0);
        CHECK(klay_forward(c, d_w, 2, d_out, KLAY_LOG, NULL) == KLAY_OK);
        CHECK(klay_backward(c, d_dout, d_dleaf, NULL) == KLAY_OK);
        CHECK(hipDeviceSynchronize() == 0);
        CHECK(hipMemcpy(out, d_out, sizeof(out), 2) == 0 && hipMemcpy(dleaf, d_dleaf, sizeof(dleaf), 2) == 0);
        for (int b = 0; b < 2; ++b) {
            const double a = p[b][0], bb = p[b][1], cc = p[b][2], d = p[b][3];
            const double ref = (1 - a) * (1 - bb * cc * (1 - d)) + a * (1 - (1 - cc) * d);
            CHECK(fabs(out[b] - log(ref)) <= 1e-4);
            /* d log P / d log a = a dP/da / P */
            const double dPda = -(1 - bb * cc * (1 - d)) + (1 - (1 - cc) * d);
            CHECK(fabs(dleaf[b][0] - a * dPda / ref) <= 1e-4);
        }
        CHECK(fabs(exp(out[1]) - 13.0 / 16.0) <= 1e-4);     /* the value printed in the figure for p = 1/2 */
        hipFree(d_w); hipFree(d_out); hipFree(d_dout); hipFree(d_dleaf);
        klay_destroy(c);
        printf("gpu ok\n");
    }
    printf("ok\n");
    return 0;
}
