/* Random inputs through the C oracle under AddressSanitizer + UBSan (tests/test_host_sanitizers.py). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
float kvo_half_to_float(uint16_t h);
uint16_t kvo_float_to_half(float x);
int kvo_reduce_key(const void* const* grads, int dtype, int W, int order, int64_t lo, int64_t hi, float* sum_out);
int kvo_step_key(const void* const* grads, int dtype, int W, int order, float rescale, float lr, float momentum, float wd,
                 float* w, float* m, float* sum_out, int64_t lo, int64_t hi);
static uint64_t s = 88172645463325252ull;
static uint64_t rnd(void) { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; }
int main(void) {
    for (int it = 0; it < 400; ++it) {
        int W = 1 + (int)(rnd() % 40), dtype = (int)(rnd() % 2), order = (int)(rnd() % 2);
        int64_t n = (int64_t)(rnd() % 3000);
        size_t isz = dtype ? 2 : 4;
        void** g = malloc(sizeof(void*) * (size_t)W);
        for (int r = 0; r < W; ++r) {
            g[r] = malloc(isz * (size_t)(n ? n : 1));
            for (int64_t i = 0; i < n; ++i) {
                if (dtype) ((uint16_t*)g[r])[i] = (uint16_t)rnd();            /* any bit pattern, NaN and Inf included */
                else { uint32_t b = (uint32_t)rnd(); memcpy((char*)g[r] + 4 * i, &b, 4); }
            }
        }
        float* w = malloc(4 * (size_t)(n ? n : 1)); float* m = malloc(4 * (size_t)(n ? n : 1)); float* su = malloc(4 * (size_t)(n ? n : 1));
        for (int64_t i = 0; i < n; ++i) { w[i] = (float)(rnd() % 1000) / 500.0f - 1.0f; m[i] = 0.0f; }
        int64_t lo = n ? (int64_t)(rnd() % (uint64_t)n) : 0, hi = n ? lo + (int64_t)(rnd() % (uint64_t)(n - lo + 1)) : 0;
        if (kvo_reduce_key((const void* const*)g, dtype, W, order, lo, hi, su) != 0) return 1;
        if (kvo_step_key((const void* const*)g, dtype, W, order, 0.125f, 0.1f, 0.9f, 1e-4f, w, m, (it & 1) ? su : NULL, lo, hi) != 0) return 1;
        if (kvo_step_key((const void* const*)g, dtype, 0, order, 1, 1, 1, 1, w, m, NULL, 0, n) != -1) return 1;   /* bad W */
        for (int r = 0; r < W; ++r) free(g[r]);
        free(g); free(w); free(m); free(su);
    }
    for (uint32_t h = 0; h < 65536; ++h) {
        float f = kvo_half_to_float((uint16_t)h);
        if (f == f && kvo_float_to_half(f) != (uint16_t)h) { printf("round trip %u\n", h); return 1; }
    }
    printf("oracle fuzz ok\n");
    return 0;
}
