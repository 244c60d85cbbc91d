/* Test driver (CPU only, no GPU needed): calls every entry point of include/svgear.h with
 * arguments that the library must reject on the host, plus the host-only workspace queries at
 * ordinary and at extreme sizes. It is linked against a copy of the library whose host code was
 * compiled with -fsanitize=address,undefined, so a stray read of a caller array, an overflow in
 * a size computation or any other undefined behaviour on these paths ends the program with a
 * sanitizer report. Device pointers are fakes: a correct argument check never dereferences them.
 * Prints one line per check and returns the number of wrong status codes. */
#include <stdio.h>

#include "svgear.h"

static int failures = 0;
static void expect(const char* what, long long got, long long want) {
  printf("%-70s %lld%s\n", what, got, got == want ? "" : "   <-- WRONG");
  if (got != want) ++failures;
}

int main(void) {
  void* fake = (void*)0x1000;
  void* odd = (void*)0x1004;
  const size_t big = (size_t)1 << 40;
  int64_t st[3] = {128 * 16, 128 * 16, 128};
  int64_t st64[3] = {1024, 1024, 64};

  expect("version", svgear_version() >= 1, 1);
  /* workspace queries: ordinary, degenerate and extreme sizes (no overflow into undefined behaviour) */
  expect("kmeans_workspace(0 heads)", (long long)svgear_kmeans_workspace(0, 1, 10, 64, 2), 0);
  expect("kmeans_workspace(wan) > 0", svgear_kmeans_workspace(1, 40, 75600, 128, 500) > 0, 1);
  expect("kmeans_workspace(extreme) returns", svgear_kmeans_workspace(1 << 14, 1 << 14, (int64_t)1 << 30, 128, 8192) >= 0, 1);
  expect("permute_workspace(wan) > 0", svgear_permute_workspace(1, 40, 75600, 500) > 0, 1);
  expect("permute_workspace(extreme) returns", svgear_permute_workspace(1 << 14, 1 << 14, (int64_t)1 << 30, 8192) >= 0, 1);
  expect("probe_route_workspace(wan) > 0", svgear_probe_route_workspace(1, 40, 75600, 128, 100, 500) > 0, 1);
  expect("probe_route_workspace(extreme) returns",
         svgear_probe_route_workspace(1 << 14, 1 << 14, (int64_t)1 << 30, 128, 8192, 8192) >= 0, 1);
  expect("sparse_attn_comp_workspace(wan) > 0", svgear_sparse_attn_comp_workspace(1, 40, 75600, 75600, 128, 100, 500) > 0, 1);
  expect("sparse_attn_comp_workspace(extreme) returns",
         svgear_sparse_attn_comp_workspace(1 << 14, 1 << 14, (int64_t)1 << 30, (int64_t)1 << 30, 128, 8192, 8192) >= 0, 1);
  expect("two_stage_workspace(wan) > 0", svgear_sparse_attn_two_stage_workspace(1, 40, 75600, 75600, 128, 100, 500) > 0, 1);
  expect("permute_static_capacity", (long long)svgear_permute_static_capacity(), 8 << 20);

  /* k-means */
  expect("kmeans: null pointers",
         svgear_kmeans(NULL, NULL, SVGEAR_F32, 1, 1, 16, 0, 64, st64, 2, 1, NULL, NULL, NULL, NULL, NULL, 0, NULL), -1);
  expect("kmeans: C > N - n_tail",
         svgear_kmeans(fake, NULL, SVGEAR_F32, 1, 1, 16, 0, 64, st64, 17, 1, fake, NULL, fake, fake, fake, big, NULL), -1);
  expect("kmeans: d = 32",
         svgear_kmeans(fake, NULL, SVGEAR_F32, 1, 1, 16, 0, 32, st64, 2, 1, fake, NULL, fake, fake, fake, big, NULL), -1);
  expect("kmeans: bad dtype",
         svgear_kmeans(fake, NULL, (svgear_dtype)7, 1, 1, 16, 0, 64, st64, 2, 1, fake, NULL, fake, fake, fake, big, NULL), -1);
  expect("kmeans: iters = 0",
         svgear_kmeans(fake, NULL, SVGEAR_F32, 1, 1, 16, 0, 64, st64, 2, 0, fake, NULL, fake, fake, fake, big, NULL), -1);
  expect("kmeans: null strides",
         svgear_kmeans(fake, NULL, SVGEAR_F32, 1, 1, 16, 0, 64, NULL, 2, 1, fake, NULL, fake, fake, fake, big, NULL), -1);
  expect("kmeans: workspace too small",
         svgear_kmeans(fake, NULL, SVGEAR_F32, 1, 1, 16, 0, 64, st64, 2, 1, fake, NULL, fake, fake, fake, 8, NULL), -2);

  /* permute, its static-scratch form, permute_rows, unpermute */
  {
    const void* src[1] = {fake};
    void* dst[1] = {fake};
    const int64_t sst[1][3] = {{128 * 16, 128 * 16, 128}};
    expect("permute: null labels",
           svgear_permute(NULL, 1, 1, 16, 0, 2, fake, fake, 0, NULL, NULL, NULL, SVGEAR_BF16, 128, fake, big, NULL), -1);
    expect("permute: n_tensors = 5",
           svgear_permute(fake, 1, 1, 16, 0, 2, fake, fake, 5, src, sst, dst, SVGEAR_BF16, 128, fake, big, NULL), -1);
    expect("permute: tensors but null arrays",
           svgear_permute(fake, 1, 1, 16, 0, 2, fake, fake, 1, NULL, NULL, NULL, SVGEAR_BF16, 128, fake, big, NULL), -1);
    expect("permute: n_tail >= N",
           svgear_permute(fake, 1, 1, 16, 16, 2, fake, fake, 0, NULL, NULL, NULL, SVGEAR_BF16, 128, fake, big, NULL), -1);
    expect("permute: workspace too small",
           svgear_permute(fake, 1, 1, 16, 0, 2, fake, fake, 1, src, sst, dst, SVGEAR_BF16, 128, fake, 4, NULL), -2);
    expect("permute_static: beyond capacity",
           svgear_permute_static(fake, 1, 40, 75600, 0, 1500, fake, fake, 0, NULL, NULL, NULL, SVGEAR_BF16, 128, NULL), -2);
    expect("permute_static: B = 0",
           svgear_permute_static(fake, 0, 1, 16, 0, 2, fake, fake, 0, NULL, NULL, NULL, SVGEAR_BF16, 128, NULL), -1);
    expect("permute_rows: no tensors", svgear_permute_rows(fake, 1, 1, 16, 0, src, sst, dst, SVGEAR_BF16, 128, NULL), -1);
    expect("permute_rows: null perm", svgear_permute_rows(NULL, 1, 1, 16, 1, src, sst, dst, SVGEAR_BF16, 128, NULL), -1);
    expect("unpermute: null", svgear_unpermute(NULL, NULL, SVGEAR_F32, 1, 1, 16, 64, NULL, st64, NULL), -1);
    expect("unpermute: misaligned", svgear_unpermute(odd, fake, SVGEAR_F32, 1, 1, 16, 64, fake, st64, NULL), -1);
  }

  /* probe + route */
  expect("probe_route: negative budget",
         svgear_probe_route(fake, fake, fake, fake, fake, SVGEAR_F32, fake, fake, 1, 1, 16, 16, 64, 2, 2, -5, 0.125f, 0, fake,
                            fake, fake, fake, fake, fake, big, NULL), -1);
  expect("probe_route: unknown flag",
         svgear_probe_route(fake, fake, fake, fake, fake, SVGEAR_F32, fake, fake, 1, 1, 16, 16, 64, 2, 2, 5, 0.125f, 64, fake,
                            fake, fake, fake, fake, fake, big, NULL), -1);
  expect("probe_route: workspace too small",
         svgear_probe_route(fake, fake, fake, fake, fake, SVGEAR_F32, fake, fake, 1, 1, 16, 16, 64, 2, 2, 5, 0.125f, 0, fake,
                            fake, fake, fake, fake, fake, 8, NULL), -2);
  {
    const float ps[4] = {0.0f, -1.0f, 1.5f, 0.0f / 0.0f};
    for (int i = 0; i < 4; ++i)
      expect("probe_route_top_p: p outside (0, 1]",
             svgear_probe_route_top_p(fake, fake, fake, fake, fake, SVGEAR_BF16, fake, fake, 1, 1, 16, 16, 128, 2, 2, ps[i],
                                      0.1f, 0, fake, fake, fake, fake, fake, fake, fake, big, NULL), -1);
  }
  expect("probe_route_top_p: per-row flag set",
         svgear_probe_route_top_p(fake, fake, fake, fake, fake, SVGEAR_BF16, fake, fake, 1, 1, 16, 16, 128, 2, 2, 0.5f, 0.1f,
                                  SVGEAR_ROUTE_PER_ROW, fake, fake, fake, fake, fake, fake, fake, big, NULL), -1);
  expect("probe_route_top_p: null row_budget",
         svgear_probe_route_top_p(fake, fake, fake, fake, fake, SVGEAR_BF16, fake, fake, 1, 1, 16, 16, 128, 2, 2, 0.5f, 0.1f,
                                  0, fake, fake, fake, fake, fake, NULL, fake, big, NULL), -1);

  /* attention */
  expect("sparse_attn_comp: misaligned queries",
         svgear_sparse_attn_comp(odd, fake, fake, SVGEAR_BF16, fake, fake, fake, fake, fake, fake, fake, 1, 1, 16, 16, 64, 2,
                                 2, 0.125f, fake, NULL, fake, big, NULL), -1);
  expect("sparse_attn_comp: Ck beyond the LDS tables",
         svgear_sparse_attn_comp(fake, fake, fake, SVGEAR_BF16, fake, fake, fake, fake, fake, fake, fake, 1, 1, 4096, 4096,
                                 128, 2, 3000, 0.1f, fake, NULL, fake, big, NULL), -4);
  expect("sparse_attn_comp: more keys than 32-bit row offsets reach (bf16, d = 128)",
         svgear_sparse_attn_comp(fake, fake, fake, SVGEAR_BF16, fake, fake, fake, fake, fake, fake, fake, 1, 1, 4096,
                                 (int64_t)1 << 24, 128, 2, 2, 0.1f, fake, NULL, fake, big, NULL), -4);
  expect("sparse_attn_comp: workspace too small",
         svgear_sparse_attn_comp(fake, fake, fake, SVGEAR_BF16, fake, fake, fake, fake, fake, fake, fake, 1, 1, 16, 16, 128, 2,
                                 2, 0.1f, fake, NULL, fake, 8, NULL), -2);
  expect("token_order: null permutation",
         svgear_sparse_attn_comp_token_order(fake, st, fake, fake, SVGEAR_BF16, fake, fake, fake, fake, fake, fake, fake, NULL,
                                             1, 1, 16, 16, 128, 2, 2, 0.1f, fake, st, NULL, fake, big, NULL), -1);
  {
    int64_t bad[3] = {129 * 16, 129 * 16, 129};
    int64_t shrt[3] = {64 * 16, 64 * 16, 64};
    expect("token_order: output rows not 16-byte aligned",
           svgear_sparse_attn_comp_token_order(fake, st, fake, fake, SVGEAR_BF16, fake, fake, fake, fake, fake, fake, fake,
                                               fake, 1, 1, 16, 16, 128, 2, 2, 0.1f, fake, bad, NULL, fake, big, NULL), -1);
    expect("token_order: stride_n < d",
           svgear_sparse_attn_comp_token_order(fake, shrt, fake, fake, SVGEAR_BF16, fake, fake, fake, fake, fake, fake, fake,
                                               fake, 1, 1, 16, 16, 128, 2, 2, 0.1f, fake, st, NULL, fake, big, NULL), -1);
  }
  expect("two_stage: fp32 is unsupported",
         svgear_sparse_attn_two_stage(fake, fake, fake, SVGEAR_F32, fake, fake, fake, fake, fake, fake, fake, 1, 1, 16, 16, 128,
                                      2, 2, 0.1f, fake, NULL, fake, big, NULL), -4);
  expect("last_hip_error still 0", svgear_last_hip_error(), 0);
  printf("%d wrong status code(s)\n", failures);
  return failures;
}
