/* The boundary seen from plain C: includes the public header as C99 (no C++ types may leak into
 * it), links against the library and calls the host-only entry points. Prints one line per call;
 * tests/test_host_api.py compares the lines with what the Python binding returns. */
#include <stdio.h>

#include "loza_ssa.h"

int main(void)
{
    int64_t a = -1, b = -1, c = -1;
    int rc = loza_ssa_live_ranges(10000, 128, 512, &a, &b, &c);
    printf("live_ranges %d %lld %lld %lld\n", rc, (long long)a, (long long)b, (long long)c);
    rc = loza_ssa_live_ranges_blocks(1000, 1, 7, 128, &a, &b, &c);
    printf("live_ranges_blocks %d %lld %lld %lld\n", rc, (long long)a, (long long)b, (long long)c);
    printf("live_pairs %lld\n", (long long)loza_ssa_live_pairs(131072, 128, 8192));
    printf("live_pairs_blocks %lld\n", (long long)loza_ssa_live_pairs_blocks(131072, 1, 7, 128));
    printf("decode_splits %d\n", loza_ssa_decode_num_splits(64, 64, 1, 262144, 128, 8192));
    printf("decode_ws %zu\n", loza_ssa_decode_workspace_bytes(64, 64, 1, 262144, 512, 128, 8192));
    printf("backward_ws %zu\n", loza_ssa_backward_workspace_bytes(1, 64, 1, 131072, 576, 512, 128, 8192, 1));
    printf("calibration_ws %zu\n", loza_ssa_calibration_workspace_bytes(1, 64, 4096, 512));
    printf("alpha_grad_ws %zu\n", loza_ssa_calibration_alpha_grad_workspace_bytes(4096));
    printf("status %s\n", loza_status_str(LOZA_ERR_WORKSPACE));
    /* validation happens before any device call: a NULL pointer is refused on any machine */
    printf("null_q %d\n", loza_ssa_prefill(NULL, NULL, NULL, NULL, NULL, 1, 1, 1, 16, 128, 128, 0, 1, 1.0f, NULL));
    return 0;
}
