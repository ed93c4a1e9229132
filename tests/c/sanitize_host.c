/* Driver for a build of the library whose HOST code is compiled under -fsanitize=address,undefined:
 * the host-only entry points and the argument validation of the launching ones (which returns
 * before any device call), on sizes at the edges of their ranges. The sanitizers abort on any
 * out-of-bounds access or undefined arithmetic (a signed overflow in the schedule arithmetic, say);
 * tests/test_sanitizers.py compares the printed values with the ordinary build's. */
#include <stdio.h>

#include "loza_ssa.h"

int main(void)
{
    int64_t a = -1, b = -1, c = -1;
    const int64_t big[] = {0, 1, 127, 128, 8192, 2147483518LL, 2147483519LL, INT64_MAX - 1, INT64_MAX};
    const int nb = (int)(sizeof big / sizeof big[0]);
    long long acc = 0;
    for (int x = 0; x < nb; ++x)
        for (int y = 0; y < nb; ++y)
            for (int z = 0; z < nb; ++z) {
                int rc = loza_ssa_live_ranges(big[x], big[y], big[z], &a, &b, &c);
                acc += rc + (rc == 0 ? (a % 1000) + (b % 1000) + (c % 1000) : 0);
                rc = loza_ssa_live_ranges_blocks(big[x], big[y], big[z], big[(x + y) % nb], &a, &b, &c);
                acc += rc + (rc == 0 ? (a % 1000) + (b % 1000) + (c % 1000) : 0);
                acc += loza_ssa_live_pairs(big[x] < 3000000 ? big[x] : 3000000, big[y], big[z]) % 1000;
                acc += loza_ssa_live_pairs_blocks(big[x] < 100000 ? big[x] : 100000, big[y], big[z], big[(x + z) % nb]) % 1000;
                acc += loza_ssa_decode_num_splits(64, 64, 1, big[x], big[y], big[z]);
                acc += (long long)(loza_ssa_decode_workspace_bytes(3, 16, 2, big[x], 512, big[y], big[z]) % 1000);
                acc += (long long)(loza_ssa_backward_workspace_bytes(1, 64, 1, big[x], 576, 512, big[y], big[z], 1) % 1000);
                acc += (long long)(loza_ssa_backward_workspace_bytes_blocks(2, 8, 2, big[x], 128, 128, big[y], big[z], big[(y + z) % nb], 0) % 1000);
            }
    printf("edges %lld\n", acc);
    printf("calibration_ws %zu %zu\n", loza_ssa_calibration_workspace_bytes(1, 64, 4096, 512),
           loza_ssa_calibration_workspace_bytes(1, 64, INT64_MAX, 512));
    printf("alpha_grad_ws %zu %zu\n", loza_ssa_calibration_alpha_grad_workspace_bytes(4096),
           loza_ssa_calibration_alpha_grad_workspace_bytes(INT64_MAX - 7));
    /* validation of the launching entry points: everything below is rejected before any device call */
    char buf[64];
    void *p = (void *)(((uintptr_t)buf + 15) & ~(uintptr_t)15);
    printf("rejected %d %d %d %d %d %d %d\n",
           loza_ssa_prefill(NULL, p, p, p, (float *)p, 1, 1, 1, 16, 128, 128, 0, 1, 1.0f, NULL),
           loza_ssa_prefill(p, p, p, p, (float *)p, 1, 3, 2, 16, 128, 128, 0, 1, 1.0f, NULL),
           loza_ssa_prefill(p, p, p, p, (float *)p, 1, 1, 1, INT64_MAX, 128, 128, 0, 1, 1.0f, NULL),
           loza_ssa_prefill(p, p, p, p, (float *)p, 1, 1, 1, 16, 96, 64, 0, 1, 1.0f, NULL),
           loza_ssa_prefill((char *)p + 2, p, p, p, (float *)p, 1, 1, 1, 16, 128, 128, 0, 1, 1.0f, NULL),
           loza_ssa_decode(p, p, p, (const int32_t *)p, p, (float *)p, 64, 64, 1, 262144, 576, 512, INT64_MAX, INT64_MAX, 0.07f, p, 16, NULL),
           loza_ssa_decode_static(p, p, p, (const int32_t *)p, p, (float *)p, 1000, 64, 1, 262144, 576, 512, 128, 8192, 0.07f, NULL));
    printf("status %s\n", loza_status_str(LOZA_ERR_ALIGN));
    return 0;
}
