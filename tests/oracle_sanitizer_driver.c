/* Runs every function of the CPU oracle on small heap buffers of exactly the sizes their
 * contracts state, so that AddressSanitizer / UBSan (the test builds this file together with
 * oracle/samo_oracle.c under -fsanitize=address,undefined) see any access outside them and any
 * undefined arithmetic.  Prints a checksum so that the work cannot be optimised away. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

uint16_t samo_oracle_f32_to_f16(float);
float samo_oracle_f16_to_f32(uint16_t);
uint16_t samo_oracle_f64_to_f16(double);
void samo_oracle_f32_to_f16_array(const float *, uint16_t *, int64_t);
void samo_oracle_f16_to_f32_array(const uint16_t *, float *, int64_t);
int64_t samo_oracle_build_index(const uint8_t *, int64_t, int32_t *);
void samo_oracle_decompress(const float *, const int32_t *, int64_t, uint16_t *, int64_t);
void samo_oracle_gather(const uint16_t *, const int32_t *, int64_t, float, float *);
void samo_oracle_compress_f16(const uint16_t *, const int32_t *, int64_t, uint16_t *);
void samo_oracle_accumulate_f16(const uint16_t *, const int32_t *, int64_t, uint16_t *);
void samo_oracle_upcast(const uint16_t *, int64_t, float, float *);
double samo_oracle_sum_squares(const float *, int64_t);
int32_t samo_oracle_has_nonfinite(const float *, int64_t);
void samo_oracle_scale(float *, int64_t, float);
void samo_oracle_sgd(float *, float *, const float *, int64_t, float, float, float);
void samo_oracle_adam(float *, float *, float *, const float *, int64_t, float, float, float, float, float, int32_t,
                      int32_t);
void samo_oracle_step(const uint16_t *, uint16_t *, int64_t, const int32_t *, int64_t, float *, float *, float *,
                      float *, float, float, float, float, float, float, int32_t, int32_t);
void samo_oracle_compress_f32(const float *, const int32_t *, int64_t, float, float *);
void samo_oracle_expand_f32(const float *, const int32_t *, int64_t, float *, int64_t);
void samo_oracle_step_fp32(const float *, float *, int64_t, const int32_t *, int64_t, float *, float *, float *,
                           float *, float, float, float, float, float, float, int32_t, int32_t);

static uint32_t lcg(uint32_t *s) { *s = *s * 1664525u + 1013904223u; return *s >> 8; }

int main(void)
{
    double check = 0.0;
    const int64_t sizes[] = {0, 1, 2, 63, 64, 1000};
    for (unsigned c = 0; c < sizeof(sizes) / sizeof(sizes[0]); ++c) {
        const int64_t n = sizes[c];
        uint32_t seed = 12345u + (uint32_t)n;
        uint8_t *mask = malloc((size_t)n + !n);
        for (int64_t j = 0; j < n; ++j) mask[j] = (lcg(&seed) % 3 == 0) ? (uint8_t)(1 + lcg(&seed) % 200) : 0;
        const int64_t nnz = samo_oracle_build_index(mask, n, NULL);
        int32_t *idx = malloc(sizeof(int32_t) * (size_t)nnz + !nnz);
        if (samo_oracle_build_index(mask, n, idx) != nnz) return 2;
        float *p = malloc(sizeof(float) * (size_t)nnz + !nnz), *m = calloc((size_t)nnz + !nnz, sizeof(float));
        float *v = calloc((size_t)nnz + !nnz, sizeof(float)), *gc = malloc(sizeof(float) * (size_t)nnz + !nnz);
        float *pc = malloc(sizeof(float) * (size_t)nnz + !nnz), *buf = calloc((size_t)nnz + !nnz, sizeof(float));
        uint16_t *g = malloc(sizeof(uint16_t) * (size_t)n + !n), *w = malloc(sizeof(uint16_t) * (size_t)n + !n);
        uint16_t *gc16 = malloc(sizeof(uint16_t) * (size_t)nnz + !nnz);
        float *g32 = malloc(sizeof(float) * (size_t)n + !n), *w32 = malloc(sizeof(float) * (size_t)n + !n);
        for (int64_t i = 0; i < nnz; ++i) p[i] = ((float)(lcg(&seed) % 2001) - 1000.0f) * 1e-4f;
        for (int64_t j = 0; j < n; ++j) {
            g[j] = (uint16_t)lcg(&seed);                               /* every half pattern, NaN and inf included */
            g32[j] = ((float)(lcg(&seed) % 2001) - 1000.0f) * 1e-6f;
            w32[j] = mask[j] ? ((float)(lcg(&seed) % 2001) - 1000.0f) * 1e-4f : 9.0f;
        }
        samo_oracle_decompress(p, idx, nnz, w, n);
        samo_oracle_gather(g, idx, nnz, 1.0f / 1024.0f, gc);
        samo_oracle_compress_f16(g, idx, nnz, gc16);
        samo_oracle_accumulate_f16(g, idx, nnz, gc16);
        samo_oracle_upcast(gc16, nnz, 1.0f / 1024.0f, gc);
        for (int64_t i = 0; i < nnz; ++i) if (!(gc[i] == gc[i]) || gc[i] > 1e30f || gc[i] < -1e30f) gc[i] = 0.5f;
        check += samo_oracle_sum_squares(gc, nnz) + samo_oracle_has_nonfinite(gc, nnz);
        samo_oracle_scale(gc, nnz, 0.5f);
        samo_oracle_sgd(p, buf, gc, nnz, 0.1f, 0.9f, 1e-4f);
        samo_oracle_adam(p, m, v, gc, nnz, 1e-3f, 0.9f, 0.999f, 1e-8f, 0.01f, 1, 1);
        for (int64_t j = 0; j < n; ++j) g[j] = samo_oracle_f32_to_f16(g32[j] * 1024.0f);
        samo_oracle_step(g, w, n, idx, nnz, p, m, v, gc, 1.0f / 1024.0f, 1e-3f, 0.9f, 0.999f, 1e-8f, 0.0f, 0, 2);
        samo_oracle_compress_f32(g32, idx, nnz, 1.0f, gc);
        samo_oracle_expand_f32(gc, idx, nnz, w32, n);
        samo_oracle_step_fp32(g32, w32, n, idx, nnz, m, v, gc, pc, 1.0f, 1e-3f, 0.9f, 0.999f, 1e-8f, 0.0f, 0, 3);
        float *f = malloc(sizeof(float) * (size_t)n + !n);
        samo_oracle_f16_to_f32_array(w, f, n);
        samo_oracle_f32_to_f16_array(f, w, n);
        for (int64_t j = 0; j < n; ++j) check += f[j] + w32[j];
        for (int64_t i = 0; i < nnz; ++i) check += p[i] + m[i] + v[i];
        free(f); free(g32); free(w32); free(gc16); free(w); free(g); free(buf); free(pc); free(gc); free(v); free(m);
        free(p); free(idx); free(mask);
    }
    for (uint32_t h = 0; h < 65536u; h += 7u) check += samo_oracle_f64_to_f16((double)samo_oracle_f16_to_f32((uint16_t)h)) == h;
    printf("checksum %.9g\n", check);
    return 0;
}
