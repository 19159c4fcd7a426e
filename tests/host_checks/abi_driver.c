/* Host-side walk over the C ABI for the sanitizer build (AddressSanitizer +
 * UndefinedBehaviorSanitizer on the library's host code): every entry point is
 * called with arguments that its host checks must turn into a status code before
 * anything is enqueued - wrong dtypes, sizes, NULLs, misaligned pointers, short
 * workspaces, limits - and with empty batches, which return at once.  No GPU is
 * needed and none of the pointers is ever dereferenced.  Exit code 0 = every
 * status was the expected one; the sanitizers abort on their own findings. */
#include <stdint.h>
#include <stdio.h>

#include "../../include/sv.h"

static int failures = 0;
#define EXPECT(call, want)                                                                   \
  do {                                                                                       \
    const int got_ = (call);                                                                 \
    if (got_ != (want)) {                                                                    \
      printf("line %d: %s -> %d (%s), expected %d\n", __LINE__, #call, got_, sv_strerror(got_), (want)); \
      ++failures;                                                                            \
    }                                                                                        \
  } while (0)

int main(void) {
  void* p = (void*)(uintptr_t)(256 * 1024);        /* non-NULL, aligned, never dereferenced */
  void* odd = (void*)(uintptr_t)(256 * 1024 + 1);
  const size_t big = (size_t)1 << 30;
  int code;

  for (code = -9; code <= 1; ++code)
    if (!sv_strerror(code) || !sv_strerror(code)[0]) ++failures;

  /* workspace sizing over the whole range of shapes, including the largest ones */
  {
    const int Bs[] = {0, 1, 7, 64, 4096, 65535}, ks[] = {1, 8, 16, 64}, Vs[] = {1, 8191, 8192, 152064, 16777216};
    size_t last = 0;
    for (unsigned i = 0; i < sizeof Bs / sizeof *Bs; ++i)
      for (unsigned j = 0; j < sizeof ks / sizeof *ks; ++j)
        for (unsigned l = 0; l < sizeof Vs / sizeof *Vs; ++l) {
          const size_t w = sv_workspace_bytes(Bs[i], ks[j], Vs[l], SV_BF16);
          if (w == 0 || w % 256 != 0) { printf("workspace %d %d %d -> %zu\n", Bs[i], ks[j], Vs[l], w); ++failures; }
          last = w;
        }
    (void)last;
    if (sv_workspace_bytes(-1, 8, 100, SV_F32) != 0 || sv_workspace_bytes(4, 0, 100, SV_F32) != 0 ||
        sv_workspace_bytes(4, 8, 0, SV_F32) != 0 || sv_workspace_bytes(4, 8, 100, 9) != 0)
      ++failures;
  }

  /* sv_row_stats / _warped */
  EXPECT(sv_row_stats(p, p, p, 2, 2, 8, 7, p, p, p, p, 0, 0, 0, 0, p, big, 0), SV_ERR_DTYPE);
  EXPECT(sv_row_stats(p, p, p, 2, 0, 8, SV_BF16, p, p, p, p, 0, 0, 0, 0, p, big, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_row_stats(p, p, p, -1, 2, 8, SV_BF16, p, p, p, p, 0, 0, 0, 0, p, big, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_row_stats(0, p, p, 2, 2, 8, SV_BF16, p, p, p, p, 0, 0, 0, 0, p, big, 0), SV_ERR_NULL);
  EXPECT(sv_row_stats(odd, p, p, 2, 2, 8, SV_BF16, p, p, p, p, 0, 0, 0, 0, p, big, 0), SV_ERR_ALIGN);
  EXPECT(sv_row_stats(p, p, p, 2, 2, 8, SV_BF16, p, p, p, p, 0, 0, 0, 0, 0, big, 0), SV_ERR_WORKSPACE);
  EXPECT(sv_row_stats(p, p, p, 2, 2, 8, SV_BF16, p, p, p, p, 0, 0, 0, 0, p, 16, 0), SV_ERR_WORKSPACE);
  EXPECT(sv_row_stats(p, p, p, 0, 2, 8, SV_BF16, p, p, p, p, 0, 0, 0, 0, 0, 0, 0), SV_OK);
  EXPECT(sv_row_stats_warped(p, p, p, 2, 2, 8, SV_BF16, 0.0f, 0, 1.0f, 0, p, p, p, p, 0, 0, 0, 0, p, big, 0),
         SV_ERR_INVALID_ARG);
  EXPECT(sv_row_stats_warped(p, p, p, 2, 2, 8, SV_BF16, 1.0f, odd, 1.0f, 0, p, p, p, p, 0, 0, 0, 0, p, big, 0),
         SV_ERR_ALIGN);

  /* sv_accept_estimate */
  EXPECT(sv_accept_estimate(p, p, -1, p, 5, p, 5, p, p, 0, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_accept_estimate(p, p, 4, p, 0, p, 5, p, p, 0, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_accept_estimate(0, p, 4, p, 5, p, 5, p, p, 0, 0), SV_ERR_NULL);
  EXPECT(sv_accept_estimate(odd, p, 4, p, 5, p, 5, p, p, 0, 0), SV_ERR_ALIGN);

  /* sv_select_length */
  EXPECT(sv_select_length(p, 4, 4, p, 17, 2, p, p, p, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_select_length(p, 4, 4, p, 16, SV_BATCH_GREEDY, p, p, p, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_select_length(p, SV_SELECT_MAX_KEYS + 1, 1, p, 100000, SV_BATCH_GREEDY, p, p, p, 0), SV_ERR_TOO_LARGE);
  EXPECT(sv_select_length(p, 65536, 65536, p, 100000, SV_BATCH_GREEDY, p, p, p, 0), SV_ERR_TOO_LARGE);
  EXPECT(sv_select_length(0, 4, 4, p, 17, SV_BATCH_GREEDY, p, p, p, 0), SV_ERR_NULL);
  EXPECT(sv_select_length(0, 0, 4, 0, 0, SV_PER_SEQUENCE, 0, 0, 0, 0), SV_OK);

  EXPECT(sv_estimate_select(p, p, 4, 4, p, 5, p, 5, p, p, 17, 2, p, 0, p, p, p, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_estimate_select(p, p, 4, 4, p, 0, p, 5, p, p, 17, 0, p, 0, p, p, p, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_estimate_select(p, p, 4, 4, p, 5, p, 5, p, p, 16, 0, p, 0, p, p, p, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_estimate_select(0, p, 4, 4, p, 5, p, 5, p, p, 17, 0, p, 0, p, p, p, 0), SV_ERR_NULL);
  EXPECT(sv_estimate_select(p, p, 4, 4, p, 5, p, 5, p, p, 17, 0, 0, 0, p, p, p, 0), SV_ERR_NULL);
  EXPECT(sv_estimate_select(p, p, SV_SELECT_MAX_KEYS + 1, 1, p, 5, p, 5, p, p, 10000, 0, p, 0, p, p, p, 0), SV_ERR_TOO_LARGE);
  EXPECT(sv_estimate_select(0, 0, 0, 4, 0, 5, 0, 5, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0), SV_OK);
  EXPECT(sv_repetition_penalty(p, 0, 0, 2, 3, 8, -1, p, 4, 0, 0, 1.2f, 0), SV_ERR_DTYPE);
  EXPECT(sv_repetition_penalty(p, 0, 0, 2, 3, 8, SV_BF16, p, 4, 0, 0, 0.0f, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_repetition_penalty(p, 0, 0, 2, 0, 8, SV_BF16, p, 4, 0, 0, 1.2f, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_repetition_penalty(p, 0, 0, 2, 3, 8, SV_BF16, p, SV_PENALTY_MAX_TOKENS + 1, 0, 0, 1.2f, 0), SV_ERR_TOO_LARGE);
  EXPECT(sv_repetition_penalty(p, 0, 0, 2, 3, 8, SV_BF16, p, SV_PENALTY_MAX_TOKENS, p, 1, 1.2f, 0), SV_ERR_TOO_LARGE);
  EXPECT(sv_repetition_penalty(0, 0, 0, 2, 3, 8, SV_BF16, p, 4, 0, 0, 1.2f, 0), SV_ERR_NULL);
  EXPECT(sv_repetition_penalty(p, 0, 0, 2, 3, 8, SV_BF16, 0, 4, 0, 0, 1.2f, 0), SV_ERR_NULL);
  EXPECT(sv_repetition_penalty(p, 0, 0, 0, 3, 8, SV_BF16, 0, 4, 0, 0, 1.2f, 0), SV_OK);
  EXPECT(sv_repetition_penalty(p, 0, 0, 2, 3, 8, SV_BF16, 0, 0, 0, 0, 1.2f, 0), SV_OK);
  {
    void* zs[2] = {p, p};
    int rps[2] = {3, 4};
    EXPECT(sv_repetition_penalty_multi(0, zs, 0, 0, 2, rps, 8, SV_BF16, p, 4, 0, 0, 1.2f, 0), SV_ERR_INVALID_ARG);
    EXPECT(sv_repetition_penalty_multi(2, 0, 0, 0, 2, rps, 8, SV_BF16, p, 4, 0, 0, 1.2f, 0), SV_ERR_NULL);
    EXPECT(sv_repetition_penalty_multi(2, zs, 0, 0, 2, rps, 8, SV_BF16, p, 4, 0, 0, -1.0f, 0), SV_ERR_INVALID_ARG);
    EXPECT(sv_repetition_penalty_multi(2, zs, 0, 0, 0, rps, 8, SV_BF16, p, 4, 0, 0, 1.2f, 0), SV_OK);
  }
  /* sv_verify_sample and its variants */
  EXPECT(sv_verify_sample(p, 0, 0, p, p, 0, 2, 2, 8, -1, 0, 0, p, p, p, 0, p, big, 0), SV_ERR_DTYPE);
  EXPECT(sv_verify_sample(p, 0, 0, p, p, 0, 2, SV_MAX_K + 1, 8, SV_BF16, 0, 0, p, p, p, 0, p, big, 0), SV_ERR_TOO_LARGE);
  EXPECT(sv_verify_sample(p, 0, 0, p, p, 0, 65536, 2, 8, SV_BF16, 0, 0, p, p, p, 0, p, big, 0), SV_ERR_TOO_LARGE);
  EXPECT(sv_verify_sample(0, 0, 0, p, p, 0, 2, 2, 8, SV_BF16, 0, 0, p, p, p, 0, p, big, 0), SV_ERR_NULL);
  EXPECT(sv_verify_sample(p, p, -1, p, p, 0, 2, 2, 8, SV_BF16, 0, 0, p, p, p, 0, p, big, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_verify_sample(p, 0, 0, p, p, 0, 2, 2, 8, SV_BF16, 0, 0, p, p, p, 0, p, 0, 0), SV_ERR_WORKSPACE);
  EXPECT(sv_verify_sample(p, 0, 0, p, p, 0, 0, 2, 8, SV_BF16, 0, 0, 0, 0, 0, 0, 0, 0, 0), SV_OK);
  EXPECT(sv_verify_sample_warped(p, 0, 0, p, p, 0, 2, 2, 8, SV_BF16, 1e4f, 0, 1.0f, 0, 0, 0, p, p, p, 0, p, big, 0),
         SV_ERR_INVALID_ARG);
  EXPECT(sv_verify_sample_chained(p, 0, 0, p, p, 0, 2, 2, 8, SV_BF16, 0, 0, p, p, p, 0, p, 0, 0), SV_ERR_WORKSPACE);
  EXPECT(sv_verify_sample_chained(p, 0, 0, p, 0, 0, 2, 2, 8, SV_BF16, 0, 0, p, p, p, 0, p, big, 0), SV_ERR_NULL);
  EXPECT(sv_verify_sample_chained(p, 0, 0, p, p, 0, 0, 2, 8, SV_BF16, 0, 0, 0, 0, 0, 0, 0, 0, 0), SV_OK);
  EXPECT(sv_verify_sample_warped_chained(p, 0, 0, p, p, 0, 2, 2, 8, SV_BF16, 1.0f, 0, 0.0f, 0, 0, 0, p, p, p, 0, p, big,
                                         0),
         SV_ERR_INVALID_ARG);
  EXPECT(sv_verify_sample_static(p, 0, 0, p, p, 0, 4096, 64, 152064, SV_BF16, 0, 0, p, p, p, 0, 0), SV_ERR_TOO_LARGE);
  EXPECT(sv_verify_sample_static(p, 0, 0, p, p, 0, 0, 2, 8, SV_BF16, 0, 0, 0, 0, 0, 0, 0), SV_OK);
  EXPECT(sv_accept_ratio(p, 5, p, p, 2, 2, 8, SV_BF16, p, 0, p, big, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_accept_ratio(p, 3, p, p, 2, 2, 8, SV_BF16, 0, 0, p, big, 0), SV_ERR_NULL);
  EXPECT(sv_accept_ratio_warped(p, 3, p, p, 2, 2, 8, SV_BF16, 1.0f, 0, -1.0f, 0, p, 0, p, big, 0), SV_ERR_INVALID_ARG);

  /* profile pass */
  EXPECT(sv_quantile_edges(p, 9000, 4, 0.f, 1.f, p, 0), SV_ERR_TOO_LARGE);
  EXPECT(sv_quantile_edges(0, 10, 4, 0.f, 1.f, p, 0), SV_ERR_NULL);
  EXPECT(sv_profile_accumulate(p, p, p, 4, p, 5, p, 5, 2000, p, p, 0), SV_ERR_TOO_LARGE);
  EXPECT(sv_profile_accumulate(p, p, 0, 4, p, 5, p, 5, 8, p, p, 0), SV_ERR_NULL);
  EXPECT(sv_profile_finalize(0, p, 5, 5, 8, p, p, 0), SV_ERR_NULL);

  /* warps and compacted supports */
  EXPECT(sv_warp_cutoffs(p, 4, 100, SV_BF16, 0.0f, 0, 1.0f, p, 0, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_warp_cutoffs(p, 4, 100, SV_BF16, 1.0f, 0, 0.0f, p, 0, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_warp_cutoffs(0, 4, 100, SV_BF16, 1.0f, 0, 1.0f, p, 0, 0), SV_ERR_NULL);
  EXPECT(sv_warp_compact(p, 4, 100, SV_BF16, 1.0f, 0, 1.0f, SV_SUPPORT_MAX_CAP + 1, p, p, p, p, 0, 0, 0),
         SV_ERR_INVALID_ARG);
  EXPECT(sv_row_stats_sparse(0, p, p, p, p, p, p, p, 64, p, 2, 2, 100, p, p, p, p, 0, 0, 0, 0, 0), SV_ERR_NULL);
  EXPECT(sv_verify_sample_sparse(p, p, p, 0, 0, p, p, p, 64, p, 0, 2, SV_MAX_K + 1, 100, 0, 0, p, p, p, 0, 0),
         SV_ERR_TOO_LARGE);
  EXPECT(sv_accept_ratio_sparse(p, p, p, 7, p, p, p, 64, p, 2, 2, 100, p, 0, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_uniforms(0, 0, 2, 0, p, p, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_uniforms(0, 0, 2, 3, 0, p, 0), SV_ERR_NULL);
  EXPECT(sv_set_timing_events(99, 0, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_set_timing_events(SV_KERNEL_ROW_STATS, p, 0), SV_ERR_INVALID_ARG);
  EXPECT(sv_set_timing_events(SV_KERNEL_ROW_STATS, 0, 0), SV_OK);

  printf("%s (%d unexpected)\n", failures ? "FAILED" : "host ABI walk ok", failures);
  return failures ? 1 : 0;
}
