/* The header is plain C: this file is compiled with gcc -std=c99 against libepp.so and run
 * without a GPU.  It only exercises argument checks that the library performs on the host. */
#include <stdio.h>
#include <string.h>

#include "epp.h"

#define CHECK(cond)                                             \
    do {                                                        \
        if (!(cond)) {                                          \
            printf("FAILED line %d: %s\n", __LINE__, #cond);    \
            return 1;                                           \
        }                                                       \
    } while (0)

int main(void) {
    epp_paths_t* paths = NULL;
    epp_path_t* full = NULL;
    epp_csr_t g;
    int32_t dummy = 0;
    float fdummy = 0.0f;
    epp_alloc_t no_alloc = {NULL, NULL, NULL}; /* alloc == NULL: the library's own hipMalloc */

    CHECK(epp_last_error() != NULL);
    CHECK(epp_prepare(NULL, NULL, 0, 2, NULL, NULL, &paths) == EPP_ERR_INVALID_ARG);
    CHECK(strlen(epp_last_error()) > 0);

    g.n = 10;
    g.nnz = 10;
    g.rowptr = &dummy; /* never dereferenced: the calls below fail before any GPU work */
    g.col = &dummy;
    g.val = &fdummy;
    CHECK(epp_prepare(&g, NULL, 0, 0, NULL, NULL, &paths) == EPP_ERR_INVALID_ARG);  /* L < 1 */
    CHECK(epp_prepare(&g, NULL, 3, 2, NULL, NULL, &paths) == EPP_ERR_INVALID_ARG);  /* ids NULL */
    g.n = (int64_t)1 << 29;
    CHECK(epp_prepare(&g, NULL, 0, 2, &no_alloc, NULL, &paths) == EPP_ERR_TOO_LARGE);
    CHECK(epp_prepare_full(&g, &no_alloc, NULL, &full) == EPP_ERR_TOO_LARGE);
    g.n = -1;
    CHECK(epp_prepare_full(&g, NULL, NULL, &full) == EPP_ERR_INVALID_ARG);

    CHECK(epp_paths_import(10, 1, NULL, 0, NULL, NULL, NULL, &paths) == EPP_ERR_INVALID_ARG);
    CHECK(epp_num_layers(NULL) == EPP_ERR_INVALID_ARG);
    CHECK(epp_get_path(NULL, 0) == NULL);
    CHECK(epp_select_group_size(NULL, 16) == EPP_ERR_INVALID_ARG);
    CHECK(epp_path_prepare_width(NULL, 16, NULL) == EPP_ERR_INVALID_ARG);
    CHECK(epp_backward_aggregate(NULL, &fdummy, &fdummy, 16, NULL) == EPP_ERR_INVALID_ARG);
    CHECK(epp_full_aggregate(NULL, &fdummy, &fdummy, 16, NULL) == EPP_ERR_INVALID_ARG);
    CHECK(epp_weight_gradient_workspace(NULL, 0, 16, 16) == EPP_ERR_INVALID_ARG);
    CHECK(epp_input_gradient(NULL, 0, &fdummy, 16, &fdummy, 16, &fdummy, NULL) == EPP_ERR_INVALID_ARG);
    CHECK(epp_paper_linreg_group_size(2708, 5278) == 2); /* Sec. 5 regression on the first row of Table 3 */
    epp_destroy_paths(NULL);
    epp_destroy_path(NULL);
    printf("ok\n");
    return 0;
}
