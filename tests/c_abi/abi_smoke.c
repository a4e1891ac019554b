/* A plain C99 caller of the boundary: the header compiles as C, the library links without C++ or HIP on the
 * caller's side, and host-only calls work without a GPU.  Built and run by tests/test_wordset_host.py. */
#include "sig.h"
#include <stdio.h>

int main(void)
{
    sig_wordset* ws = 0;
    int rc = sig_wordset_build_truncated(3, 4, &ws);
    if (rc != SIG_OK) return 1;
    /* |W| = 3 + 9 + 27 + 81, d, longest word, multiply-adds per path and segment with shared Horner intermediates */
    printf("%lld %d %d %lld\n", (long long)sig_wordset_size(ws), sig_wordset_dim(ws), sig_wordset_max_len(ws),
           (long long)sig_wordset_min_fma_per_step(ws));
    /* a device call without a path is an argument error, not a crash */
    rc = sig_forward(ws, 0, 1, 5, 0, 0, 0, 0);
    printf("%d %s\n", rc, sig_strerror(rc));
    sig_wordset_free(ws);
    sig_wordset_free(0);
    return 0;
}
