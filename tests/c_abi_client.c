/* A plain C99 client of include/mgwfbp.h: shows that the header is valid C and that the host half of the
 * library can be driven without any binding.  Reads "L a b" and then L lines "size_bytes t_backward" from
 * stdin, runs Algorithm 1, builds the host-side group / offset table for P = 2 binary32 workers, and
 * prints the plan, Eq. 8's t_iter - t_f, and the layout, one item per line, for the test to compare
 * with the oracle. */
#include <inttypes.h>
#include <stdio.h>
#include <stdlib.h>

#include "mgwfbp.h"

int main(void) {
    int L;
    double a, b;
    if (scanf("%d %lf %lf", &L, &a, &b) != 3 || L < 1) return 2;
    uint64_t* bytes = malloc(sizeof(uint64_t) * (size_t)L);
    uint64_t* elems = malloc(sizeof(uint64_t) * (size_t)L);
    double* tb = malloc(sizeof(double) * (size_t)L);
    uint8_t* merged = malloc((size_t)L);
    int32_t* first = malloc(sizeof(int32_t) * (size_t)(L + 1));
    uint64_t* off = malloc(sizeof(uint64_t) * (size_t)L);
    int32_t* grp = malloc(sizeof(int32_t) * (size_t)L);
    if (!bytes || !elems || !tb || !merged || !first || !off || !grp) return 2;
    for (int i = 0; i < L; ++i) {
        if (scanf("%" SCNu64 " %lf", &bytes[i], &tb[i]) != 2) return 2;
        elems[i] = bytes[i] / 4;
    }
    int32_t G = 0;
    int rc = mgwfbp_plan(bytes, tb, L, a, b, merged, first, &G);
    if (rc != MGWFBP_OK) return 3;
    double t = 0.0;
    rc = mgwfbp_eval(merged, bytes, tb, L, a, b, &t);
    if (rc != MGWFBP_OK) return 3;
    printf("groups %d\n", (int)G);
    printf("t_iter %.17g\n", t);
    for (int i = 0; i < L; ++i) printf("merged %d %d\n", i, (int)merged[i]);

    mgwfbp_ctx* ctx = NULL;
    rc = mgwfbp_ctx_create_host(&ctx, elems, L, merged, 2, MGWFBP_F32);
    if (rc != MGWFBP_OK) return 4;
    uint64_t* base = malloc(sizeof(uint64_t) * (size_t)G);
    uint64_t* ge = malloc(sizeof(uint64_t) * (size_t)G);
    if (!base || !ge) return 2;
    rc = mgwfbp_ctx_layout(ctx, off, grp, base, ge);
    if (rc != MGWFBP_OK) return 4;
    for (int i = 0; i < L; ++i) printf("tensor %d group %d off %" PRIu64 "\n", i, (int)grp[i], off[i]);
    for (int k = 0; k < G; ++k) printf("group %d elems %" PRIu64 "\n", k, ge[k]);
    /* a device call on a host-only context must be refused, not crash */
    rc = mgwfbp_pack(ctx, 0, (const void* const*)bytes, (void* const*)bytes, NULL);
    printf("device_call_on_host_ctx %d\n", rc);
    mgwfbp_ctx_destroy(ctx);
    /* invalid input: negative startup time */
    rc = mgwfbp_plan(bytes, tb, L, -1.0, b, merged, first, &G);
    printf("negative_a %d\n", rc);
    free(bytes); free(elems); free(tb); free(merged); free(first); free(off); free(grp); free(base); free(ge);
    return 0;
}
