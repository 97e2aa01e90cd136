/* Drives every oracle function once over a small multi-layer input (empty layer, one-element
 * layer, ragged length); built with -fsanitize=address,undefined by tests/test_host_sanitizers.py. */
#include "tg_oracle.h"
#include <stdio.h>
#include <stdlib.h>
int main(void) {
    int64_t off[6] = {0, 5, 5, 1030, 1031, 5000};
    int64_t n = off[5], L = 5;
    float* g = malloc(n * 4); float tau[5], sl[5], ss[5];
    for (int64_t i = 0; i < n; ++i) g[i] = (float)((i * 2654435761u) % 2001) * 1e-4f - 0.1f;
    tgo_clip_stats(g, L, off, 2.5f, tau, sl);
    tgo_share_scalers(sl, 1, L, ss);
    uint8_t* c = malloc((n + 3) / 4);
    tgo_ternarize_pack(g, L, off, tau, ss, 77, 3, 1, c);
    const uint8_t* cs[2] = {c, c};
    float* avg = malloc(n * 4);
    tgo_unpack_average(cs, 2, L, off, ss, avg);
    tgo_unpack_update(cs, 2, L, off, ss, 0.1f, avg);
    uint8_t* k = malloc((n * 4 + 7) / 8);
    tgo_sum_pack(cs, 2, n, 4, k);
    tgo_decode_sum(k, 4, 2, L, off, ss, avg);
    const float* gs[2] = {g, g};
    tgo_average_float(gs, 2, n, avg);
    printf("ok %g\n", avg[n - 1]);
    free(g); free(c); free(avg); free(k);
    return 0;
}
