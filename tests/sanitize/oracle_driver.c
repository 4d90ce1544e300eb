/* Runs every entry point of the CPU oracle on small inputs; built with -fsanitize=address,undefined
 * by tests/test_sanitizers_cpu.py, so an out-of-bounds access or undefined behaviour in the oracle
 * ends the run with a report instead of silently shaping an expected value. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int oracle_num_threads(void);
int64_t oracle_count_pairs(int T, int G, int grid_w, int block, int radius, const int32_t *coords_b);
int oracle_ns_attn(int B, int H, int T, int D, int G, int grid_h, int grid_w, int block, int radius, double scale,
                   const float *q, const float *k, const float *v, const int32_t *coords, const int32_t *rows,
                   int n_rows, double *out, double *prob);
int oracle_cls_scores(int B, int H, int T, int D, int G, double scale, const float *q, const float *k,
                      double *scores, double *logits, double *lse);
int oracle_topk(int B, int N, int k, const float *scores, int32_t *kept);
int oracle_gather(int B, int N, int k, int G, size_t row_bytes, const void *x, const int32_t *kept, void *y);

static float frand(uint32_t *s) {
  *s = *s * 1664525u + 1013904223u;
  return (float)((*s >> 8) & 0xffff) / 32768.0f - 1.0f;
}

int main(void) {
  uint32_t seed = 7;
  /* full grid, 7 x 5 patches (block 3 does not divide it), two global tokens */
  {
    const int B = 2, H = 3, D = 8, G = 2, gh = 7, gw = 5, T = G + gh * gw;
    const size_t n = (size_t)B * H * T * D;
    float *q = malloc(n * 4), *k = malloc(n * 4), *v = malloc(n * 4);
    for (size_t i = 0; i < n; i++) { q[i] = frand(&seed); k[i] = frand(&seed); v[i] = frand(&seed); }
    double *out = malloc(n * 8), *prob = malloc((size_t)B * H * T * T * 8);
    if (oracle_ns_attn(B, H, T, D, G, gh, gw, 3, 1, 0.35, q, k, v, NULL, NULL, 0, out, prob)) return 1;
    int32_t rows[4] = {0, 1, T - 1, G + gw};
    if (oracle_ns_attn(B, H, T, D, G, gh, gw, 3, 1, 0.35, q, k, v, NULL, rows, 4, out, NULL)) return 2;
    double *scores = malloc((size_t)B * (T - G) * 8), *logits = malloc((size_t)B * H * G * T * 8), *lse = malloc((size_t)B * H * G * 8);
    if (oracle_cls_scores(B, H, T, D, G, 0.35, q, k, scores, logits, lse)) return 3;
    if (oracle_count_pairs(T, G, gw, 3, 1, NULL) <= 0) return 4;
    /* a pruned sequence: every third patch survives */
    const int keep = (gh * gw + 2) / 3, Tp = G + keep;
    int32_t *coords = malloc((size_t)B * keep * 4);
    for (int b = 0; b < B; b++)
      for (int t = 0; t < keep; t++) coords[b * keep + t] = ((3 * t / gw) << 16) | (3 * t % gw);
    if (oracle_ns_attn(B, H, Tp, D, G, gh, gw, 3, 1, 0.35, q, k, v, coords, NULL, 0, out, NULL)) return 5;
    if (oracle_count_pairs(Tp, G, gw, 3, 1, coords) <= 0) return 6;
    free(q); free(k); free(v); free(out); free(prob); free(scores); free(logits); free(lse); free(coords);
  }
  /* selection with ties and compaction with several global rows */
  {
    const int B = 3, N = 37, k = 11, G = 3, C = 6;
    float *s = malloc((size_t)B * N * 4);
    for (int i = 0; i < B * N; i++) s[i] = (float)((i * 7) % 5);
    int32_t *kept = malloc((size_t)B * k * 4);
    if (oracle_topk(B, N, k, s, kept)) return 7;
    if (oracle_topk(B, N, N, s, kept = realloc(kept, (size_t)B * N * 4))) return 8;
    if (oracle_topk(B, N, k, s, kept)) return 9;
    uint16_t *x = malloc((size_t)B * (G + N) * C * 2), *y = malloc((size_t)B * (G + k) * C * 2);
    for (int i = 0; i < B * (G + N) * C; i++) x[i] = (uint16_t)i;
    if (oracle_gather(B, N, k, G, (size_t)C * 2, x, kept, y)) return 10;
    kept[0] = N;                       /* out of range: must be refused, not read */
    if (!oracle_gather(B, N, k, G, (size_t)C * 2, x, kept, y)) return 11;
    free(s); free(kept); free(x); free(y);
  }
  printf("oracle sanitizer run ok (%d threads)\n", oracle_num_threads());
  return 0;
}
