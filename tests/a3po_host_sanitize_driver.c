/* Test driver: the host side of the library (micro-batch planner, workspace sizes, error strings, argument
 * validation of every entry point) under AddressSanitizer / UndefinedBehaviorSanitizer.  Nothing here reaches a
 * kernel launch: every call either is host-only or is refused by the argument checks. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "a3po.h"

static unsigned long long state = 88172645463325252ull;
static unsigned rnd(void)
{
    state ^= state << 13;
    state ^= state >> 7;
    state ^= state << 17;
    return (unsigned)(state >> 11);
}

int main(void)
{
    long planned = 0, refused = 0;
    for (int it = 0; it < 100000; ++it) {
        const int64_t S = rnd() % 40;
        const int32_t n = 1 + (int32_t)(rnd() % 6);
        const int64_t budget = 1 + rnd() % 50;
        const int64_t cap = rnd() % (S + n + 3);   /* exactly-sized arrays: an overrun is an ASan report */
        int64_t *len = malloc(sizeof(int64_t) * (size_t)(S ? S : 1));
        int64_t *first = malloc(sizeof(int64_t) * (size_t)(cap + 1));
        int32_t *owner = malloc(sizeof(int32_t) * (size_t)(cap ? cap : 1));
        int64_t nm = -7;
        for (int64_t i = 0; i < S; ++i) len[i] = rnd() % 5 == 0 ? 0 : rnd() % 70;
        if (a3po_plan_microbatches(len, S, n, budget, first, owner, cap, &nm) == A3PO_OK) {
            ++planned;
            if (nm < 0 || nm > cap || first[0] != 0 || first[nm] != S) return 1;
        } else {
            ++refused;
        }
        free(len);
        free(first);
        free(owner);
    }
    if (planned == 0 || refused == 0) return 2;
    for (int w = -1; w < 5; ++w)
        for (int64_t T = -1; T < 3; ++T) (void)a3po_workspace_bytes(w, T, 100, 64);
    for (int c = -12; c < 3; ++c)
        if (!a3po_strerror(c)) return 3;
    {
        char buf[64];
        int rc[12], k = 0;
        memset(buf, 0, sizeof buf);
        rc[k++] = a3po_token_logprobs(NULL, A3PO_BF16, 4, 64, 64, NULL, NULL, NULL, NULL, NULL);
        rc[k++] = a3po_token_logprobs(buf, (a3po_dtype)7, 4, 64, 64, (const int32_t *)buf, (float *)buf, NULL, NULL, NULL);
        rc[k++] = a3po_token_logprobs(buf, A3PO_F32, 4, 64, 8, (const int32_t *)buf, (float *)buf, NULL, NULL, NULL);
        rc[k++] = a3po_proximal_interp(NULL, NULL, NULL, 0, 4, NULL, NULL, NULL);
        rc[k++] = a3po_grpo_advantages(NULL, 8, 3, 1e-6f, NULL, 4, NULL, NULL);
        rc[k++] = a3po_histogram((const float *)buf, NULL, 4, (const float *)buf, 0, 0, (int64_t *)buf, NULL);
        rc[k++] = a3po_count_tokens(NULL, NULL, 4, 10, NULL, NULL, NULL);
        rc[k++] = a3po_shard_partials(NULL, A3PO_BF16, 4, 8, 8, NULL, 0, NULL, NULL);
        rc[k++] = a3po_shard_combine(NULL, 2, 4, NULL, 16, NULL, NULL, NULL, NULL);
        rc[k++] = a3po_fused_lmhead_logprob(NULL, NULL, 4, 64, 64, NULL, NULL, NULL, NULL, 0, NULL);
        rc[k++] = a3po_loss_fwd_bwd(buf, A3PO_F32, 4, 8, 8, (const int32_t *)buf, (const float *)buf, (const int32_t *)buf, 1,
                                    (const float *)buf, (const uint8_t *)buf, 0.2f, 0.0f, buf, (float *)buf, NULL,
                                    (float *)buf, NULL, buf, 16, NULL);
        for (int i = 0; i < k; ++i) {
            printf("%d ", rc[i]);
            if (rc[i] >= 0) return 4;   /* every one of these must have been refused */
        }
    }
    printf("ok\n");
    return 0;
}
