/* Compiled (not run) by tests/test_library_host.py as strict C99: the public header must be plain C. */
#include "../include/ivfpq.h"

int abi_smoke(void) {
    ivfpq_index_t* idx = 0;
    float x[8] = {0};
    int64_t n = 0;
    int32_t d = 0, lists = 0, s = 0, p = 0;
    int st = ivfpq_build_host(x, 2, 4, 1, 4, 8, 1, 0u, &idx);
    if (st != IVFPQ_OK) return (int)ivfpq_last_error()[0];
    st = ivfpq_index_info(idx, &n, &d, &lists, &s, &p);
    st |= ivfpq_set_fp8_encoding(idx, IVFPQ_LUT_FP8_E5M3, 15, IVFPQ_ROUND_NEAREST, 0);
    (void)ivfpq_search_workspace_bytes(idx, 1, 1, 1, IVFPQ_LUT_FP16);
    ivfpq_free(idx);
    return st + (int)(IVFPQ_MAX_K + IVFPQ_MAX_PROBES);
}
