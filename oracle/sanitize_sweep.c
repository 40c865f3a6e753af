/*
 * Sanitizer sweep of the CPU oracle (TEST INFRASTRUCTURE ONLY, like comp_ams_oracle.c).
 *
 * Built by tests/test_sanitizers.py together with comp_ams_oracle.c into one executable with
 * -fsanitize=address,undefined and run once: every method (error feedback, CD-Adam, naive, none)
 * with every compressor (Top-k, scaled sign with uniform blocks and with a per-layer table,
 * Rand-k) on ragged sizes, a few steps each, so that an access out of bounds, a use after free, a
 * leak or undefined arithmetic anywhere in the oracle ends the run with a report.  Prints one
 * checksum line per case; it checks memory safety, not values (the pins do that).
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct oracle oracle_t;
oracle_t *oracle_create(int64_t d, int32_t n, int32_t compressor, int64_t k_or_block, float beta1, float beta2,
                        float eps, float lr);
void oracle_set_blocks(oracle_t *o, const int64_t *offsets, int32_t n_blocks);
void oracle_set_method(oracle_t *o, int32_t method);
void oracle_set_theta(oracle_t *o, const float *theta);
void oracle_set_lr(oracle_t *o, float lr);
void oracle_set_eps_mode(oracle_t *o, int32_t mode);
void oracle_set_rand(oracle_t *o, uint64_t seed, uint32_t draw);
void oracle_step(oracle_t *o, const float *g);
float *oracle_theta(oracle_t *o);
float *oracle_error(oracle_t *o);
float *oracle_gtilde(oracle_t *o);
uint32_t *oracle_selected(oracle_t *o);
float *oracle_scales(oracle_t *o);
int32_t oracle_n_blocks(oracle_t *o);
void oracle_destroy(oracle_t *o);

/* small deterministic generator for the inputs (no part of the method) */
static uint32_t lcg_state = 12345u;
static float next_value(void)
{
    lcg_state = lcg_state * 1664525u + 1013904223u;
    return (float)((int32_t)(lcg_state >> 8) - (1 << 23)) / (float)(1 << 20);
}

int main(void)
{
    static const int64_t sizes[] = {1, 2, 7, 64, 257, 1000};
    static const char *const mnames[] = {"ef", "cd", "naive", "none"};
    static const char *const cnames[] = {"topk", "sign", "randk", "layersign"};
    int cases = 0;
    for (int method = 0; method < 4; ++method)
        for (int comp = 0; comp < 4; ++comp)
            for (size_t q = 0; q < sizeof sizes / sizeof sizes[0]; ++q) {
                const int64_t d = sizes[q];
                const int32_t n = 1 + (int32_t)(q % 3);
                const int compressor = comp == 3 ? 1 : comp;
                const int64_t kb = compressor == 1 ? (d > 3 ? d / 3 : 1) : (d > 4 ? d / 4 : 1);
                oracle_t *o = oracle_create(d, n, compressor, kb, 0.9f, 0.999f, 1e-8f, 1e-3f);
                oracle_set_method(o, method);
                if (comp == 3) {
                    /* per-layer table: blocks of 1, 2, 3, ... coordinates, the last takes the rest */
                    int64_t off[64];
                    int32_t nb = 0;
                    int64_t at = 0;
                    off[0] = 0;
                    while (at < d && nb < 62) {
                        at += nb + 1;
                        if (at > d) at = d;
                        off[++nb] = at;
                    }
                    if (at < d) off[++nb] = d;
                    oracle_set_blocks(o, off, nb);
                }
                if (comp == 2) oracle_set_rand(o, 0x0123456789abcdefull, 3u);
                float *g = (float *)malloc((size_t)n * (size_t)d * sizeof(float));
                float *theta0 = (float *)malloc((size_t)d * sizeof(float));
                for (int64_t j = 0; j < d; ++j) theta0[j] = 0.01f * next_value();
                oracle_set_theta(o, theta0);
                oracle_set_eps_mode(o, method == 1);
                double sum = 0.0;
                for (int t = 0; t < 4; ++t) {
                    for (int64_t j = 0; j < (int64_t)n * d; ++j) g[j] = (j % 11 == 0) ? 0.0f : next_value();
                    if (t == 2) oracle_set_lr(o, 5e-4f);
                    oracle_step(o, g);
                    for (int64_t j = 0; j < d; ++j) sum += oracle_theta(o)[j];
                }
                if (method == 0) sum += oracle_error(o)[(size_t)n * (size_t)d - 1];
                if (method == 1) sum += oracle_gtilde(o)[d - 1];
                if (method != 3 && compressor != 1) sum += (double)oracle_selected(o)[(size_t)n * (size_t)kb - 1];
                if (method != 3 && compressor == 1) sum += oracle_scales(o)[(size_t)n * (size_t)oracle_n_blocks(o) - 1];
                printf("%s %s d=%lld n=%d checksum %.9g\n", mnames[method], cnames[comp], (long long)d, n, sum);
                free(g);
                free(theta0);
                oracle_destroy(o);
                ++cases;
            }
    printf("sanitize sweep: %d cases done\n", cases);
    return 0;
}
