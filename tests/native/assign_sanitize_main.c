/* Test driver: runs the oracle's fixed-order fp32 assignment (oracle/assign_f32.c, compiled into
 * this program with -fsanitize=address,undefined) on inputs read from a file, and writes labels
 * and best scores. Heap buffers are sized exactly, so an out-of-bounds read or write in the
 * assignment loop is reported by the sanitizer and the program exits non-zero.
 * File format (little endian): int64 n, int32 d, int32 C, float x[n*d], float c[C*d].
 * Output: int32 labels[n], float best[n]. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

void svgear_oracle_assign_f32(const float* x, int64_t n, int d, const float* c, int C, int32_t* labels,
                              float* best_score);

int main(int argc, char** argv) {
  if (argc != 3) return 2;
  FILE* f = fopen(argv[1], "rb");
  if (!f) return 3;
  int64_t n;
  int32_t d, C;
  if (fread(&n, 8, 1, f) != 1 || fread(&d, 4, 1, f) != 1 || fread(&C, 4, 1, f) != 1) return 4;
  float* x = (float*)malloc((size_t)n * d * sizeof(float));
  float* c = (float*)malloc((size_t)C * d * sizeof(float));
  int32_t* labels = (int32_t*)malloc((size_t)n * sizeof(int32_t));
  float* best = (float*)malloc((size_t)n * sizeof(float));
  if (fread(x, sizeof(float), (size_t)n * d, f) != (size_t)n * d) return 5;
  if (fread(c, sizeof(float), (size_t)C * d, f) != (size_t)C * d) return 6;
  fclose(f);
  svgear_oracle_assign_f32(x, n, d, c, C, labels, best);
  svgear_oracle_assign_f32(x, n, d, c, C, labels, NULL); /* the optional output left out */
  FILE* g = fopen(argv[2], "wb");
  if (!g) return 7;
  fwrite(labels, sizeof(int32_t), (size_t)n, g);
  fwrite(best, sizeof(float), (size_t)n, g);
  fclose(g);
  free(x);
  free(c);
  free(labels);
  free(best);
  return 0;
}
