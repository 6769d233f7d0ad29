/* Host-side walk over the argument checks of every entry point of include/nat.h, for a build of the
 * library whose host code is instrumented with AddressSanitizer and UndefinedBehaviorSanitizer.
 * Every call below fails (or succeeds) before anything is launched, so no GPU is needed; pointers
 * named `fake` are never dereferenced.  Prints "host_abi_san OK" and exits 0 when every status is
 * the documented one. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <string.h>
#include "nat.h"

static int failures = 0;
#define EXPECT(call, want) do { nat_status got__ = (call); if (got__ != (want)) { ++failures; \
  fprintf(stderr, "line %d: %s = %d (%s), expected %d\n", __LINE__, #call, (int)got__, nat_status_string(got__), (int)(want)); } } while (0)

int main(void) {
  void* fake = (void*)(uintptr_t)256;
  nat_select_params ok;
  memset(&ok, 0, sizeof ok);
  ok.scheme = NAT_SCHEME_URS; ok.min_cut = 1; ok.p = 0.5; ok.trunc_frac = 0.5; ok.seed = 1;
  nat_select_params bad = ok;

  if (strcmp(nat_status_string(NAT_OK), "NAT_OK") || strcmp(nat_status_string(77), "NAT_UNKNOWN_STATUS")) ++failures;
  if (nat_mask_words(0) != 0 || nat_mask_words(65) != 4 || nat_mask_words(-5) != 0) ++failures;
  if (nat_compact_workspace_bytes(-1) != 0 || nat_compact_workspace_bytes(1 << 20) < 2052) ++failures;
  if (nat_loss_workspace_bytes(10, 100, 512, NAT_DTYPE_BF16) != 0) ++failures;
  if (nat_loss_workspace_min_bytes(100000, 4096, 151936, NAT_DTYPE_BF16) >= nat_loss_workspace_bytes(100000, 4096, 151936, NAT_DTYPE_BF16)) ++failures;
  if (nat_loss_workspace_bytes(2147483647, 4096, 151936, NAT_DTYPE_BF16) == 0) ++failures;     /* largest N_k: no overflow */
  if (nat_logp_workspace_bytes(-1, 64, 512, 0) != 0 || nat_logp_workspace_min_bytes(5, 64, 512, 7) != 0) ++failures;
  if (nat_probe_mfma_scratch_bytes() == 0 || nat_profile_num_classes() <= 0) ++failures;
  if (!nat_profile_class_name(0) || strcmp(nat_profile_class_name(-3), "unknown")) ++failures;

  EXPECT(nat_advantage(NULL, 2, 4, 1e-6f, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_advantage(fake, 0, 4, 1e-6f, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_advantage(fake, 2, 4, -1.f, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_advantage(fake, 2, 4, NAN, fake, NULL), NAT_INVALID_ARG);

  EXPECT(nat_select(NULL, fake, 4, 10, fake, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_select(&ok, NULL, 4, 10, fake, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_select(&ok, fake, 0, 10, fake, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_select(&ok, fake, 4, -1, fake, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_select(&ok, fake, 4, (int64_t)1 << 31, fake, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_select(&ok, fake, 4, 10, fake, NULL, NULL), NAT_INVALID_ARG);
  bad = ok; bad.p = 0.0;           EXPECT(nat_select(&bad, fake, 4, 10, fake, fake, NULL), NAT_INVALID_ARG);
  bad = ok; bad.p = NAN;           EXPECT(nat_select(&bad, fake, 4, 10, fake, fake, NULL), NAT_INVALID_ARG);
  bad = ok; bad.p = 1.5;           EXPECT(nat_select(&bad, fake, 4, 10, fake, fake, NULL), NAT_INVALID_ARG);
  bad = ok; bad.min_cut = 0;       EXPECT(nat_select(&bad, fake, 4, 10, fake, fake, NULL), NAT_INVALID_ARG);
  bad = ok; bad.trunc_frac = 2.0;  EXPECT(nat_select(&bad, fake, 4, 10, fake, fake, NULL), NAT_INVALID_ARG);
  bad = ok; bad.scheme = 4;        EXPECT(nat_select(&bad, fake, 4, 10, fake, fake, NULL), NAT_INVALID_ARG);
  bad = ok; bad.scheme = -1;       EXPECT(nat_select(&bad, fake, 4, 10, fake, fake, NULL), NAT_INVALID_ARG);

#define COMPACT(params, nroll, B, N, cap, idx, hid, hid_k, H, dt, ws, wsb) \
  nat_compact(params, nroll, fake, fake, B, N, cap, idx, fake, fake, fake, fake, NULL, hid, hid_k, H, dt, NULL, NULL, NULL, NULL, ws, wsb, NULL)
  EXPECT(COMPACT(NULL, 4, 4, 100, 100, fake, NULL, NULL, 0, 0, fake, 1 << 20), NAT_INVALID_ARG);
  EXPECT(COMPACT(&ok, 0, 4, 100, 100, fake, NULL, NULL, 0, 0, fake, 1 << 20), NAT_INVALID_ARG);
  EXPECT(COMPACT(&ok, 4, 0, 100, 100, fake, NULL, NULL, 0, 0, fake, 1 << 20), NAT_INVALID_ARG);
  EXPECT(COMPACT(&ok, 4, 4, 100, -1, fake, NULL, NULL, 0, 0, fake, 1 << 20), NAT_INVALID_ARG);
  EXPECT(COMPACT(&ok, 4, 4, 100, 100, NULL, NULL, NULL, 0, 0, fake, 1 << 20), NAT_INVALID_ARG);
  EXPECT(COMPACT(&ok, 4, 4, 100, 100, fake, fake, NULL, 64, 1, fake, 1 << 20), NAT_INVALID_ARG);
  EXPECT(COMPACT(&ok, 4, 4, 100, 100, fake, fake, fake, 3, 1, fake, 1 << 20), NAT_BAD_SHAPE);
  EXPECT(COMPACT(&ok, 4, 4, 100, 100, fake, fake, fake, 64, 5, fake, 1 << 20), NAT_UNSUPPORTED_DTYPE);
  EXPECT(COMPACT(&ok, 4, 4, 100, 100, fake, (void*)(uintptr_t)260, fake, 64, 1, fake, 1 << 20), NAT_INVALID_ARG);
  EXPECT(COMPACT(&ok, 4, 4, 100, 100, fake, NULL, NULL, 0, 0, fake, 8), NAT_WORKSPACE_TOO_SMALL);
  EXPECT(COMPACT(&ok, 4, 4, 100, 100, fake, NULL, NULL, 0, 0, NULL, 1 << 20), NAT_WORKSPACE_TOO_SMALL);
  EXPECT(nat_compact_static(&ok, 4, fake, fake, 4, (int64_t)NAT_COMPACT_STATIC_MAX_TOKENS + 1, 100, fake, fake, fake, fake, fake,
                            NULL, NULL, NULL, 0, 0, NULL, NULL, NULL, NULL, NULL), NAT_BAD_SHAPE);
  EXPECT(nat_compact_static(NULL, 4, fake, fake, 4, 100, 100, fake, fake, fake, fake, fake,
                            NULL, NULL, NULL, 0, 0, NULL, NULL, NULL, NULL, NULL), NAT_INVALID_ARG);
  EXPECT(nat_compact_pi(4, fake, NULL, fake, 4, 100, 100, fake, fake, fake, fake, fake, NULL, NULL, NULL, 0, 0, NULL, NULL,
                        NULL, NULL, fake, 1 << 20, NULL), NAT_INVALID_ARG);
  EXPECT(nat_compact_pi(4, fake, fake, fake, 4, 100, -5, fake, fake, fake, fake, fake, NULL, NULL, NULL, 0, 0, NULL, NULL,
                        NULL, NULL, fake, 1 << 20, NULL), NAT_INVALID_ARG);

  EXPECT(nat_select_schedule(NULL, fake, fake, 4, 10, fake, fake, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_select_schedule(&ok, NULL, fake, 4, 10, fake, fake, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_select_schedule(&ok, fake, fake, 4, (int64_t)1 << 31, fake, fake, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_select_schedule(&ok, fake, fake, 4, 10, fake, fake, NULL, NULL), NAT_INVALID_ARG);
  EXPECT(nat_select_poisson(&ok, NULL, fake, 4, 10, fake, NULL), NAT_INVALID_ARG);
  EXPECT(nat_select_poisson(&ok, fake, fake, 4, 10, NULL, NULL), NAT_INVALID_ARG);
  EXPECT(nat_select_poisson(&ok, fake, fake, 4, 0, NULL, NULL), NAT_OK);          /* nothing to draw */

  EXPECT(nat_prefix_pack(fake, NULL, fake, 4, 1, 100, 50, fake, fake, fake, fake, fake, fake, NULL, NULL, NULL, NULL), NAT_INVALID_ARG);
  EXPECT(nat_prefix_pack(fake, fake, fake, 4, 2, 100, 50, fake, fake, fake, fake, fake, fake, NULL, NULL, NULL, NULL), NAT_INVALID_ARG);
  EXPECT(nat_prefix_pack(NULL, fake, fake, 4, 1, 100, 50, fake, fake, fake, fake, fake, fake, NULL, NULL, NULL, NULL), NAT_INVALID_ARG);
  EXPECT(nat_prefix_pack(fake, fake, fake, 4, 1, -1, 50, fake, fake, fake, fake, fake, fake, NULL, NULL, NULL, NULL), NAT_INVALID_ARG);
  EXPECT(nat_prefix_pack(fake, fake, fake, 4, 1, (int64_t)1 << 31, 50, fake, fake, fake, fake, fake, fake, NULL, NULL, NULL, NULL), NAT_INVALID_ARG);
  EXPECT(nat_prefix_pack(fake, fake, fake, 4, 1, 100, 50, fake, fake, fake, fake, fake, fake, NULL, fake, NULL, NULL), NAT_INVALID_ARG);

#define LOSS(hid, W, Nk, H, V, dt, eps, ws, wsb) \
  nat_loss_fwd_bwd(hid, W, fake, fake, fake, fake, fake, Nk, H, V, dt, eps, eps, 1.f, fake, NULL, fake, fake, 0, ws, wsb, NULL)
  EXPECT(LOSS(fake, fake, 10, 64, 512, 7, 0.2f, fake, (size_t)1 << 34), NAT_UNSUPPORTED_DTYPE);
  EXPECT(LOSS(fake, fake, -1, 64, 512, 1, 0.2f, fake, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOSS(fake, fake, 10, 64, 512, 1, -0.1f, fake, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOSS(fake, fake, 10, 64, 512, 1, NAN, fake, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOSS(fake, fake, 10, 0, 512, 1, 0.2f, fake, (size_t)1 << 34), NAT_BAD_SHAPE);
  EXPECT(LOSS(fake, fake, 10, 100, 512, 1, 0.2f, fake, (size_t)1 << 34), NAT_BAD_SHAPE);
  EXPECT(LOSS(fake, NULL, 10, 64, 512, 1, 0.2f, fake, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOSS(NULL, fake, 10, 64, 512, 1, 0.2f, fake, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOSS(fake, fake, 10, 64, 512, 1, 0.2f, fake, 1024), NAT_WORKSPACE_TOO_SMALL);
  EXPECT(LOSS(fake, fake, 10, 64, 512, 1, 0.2f, NULL, (size_t)1 << 34), NAT_WORKSPACE_TOO_SMALL);
  EXPECT(LOSS(fake, fake, 10, 64, 512, 1, 0.2f, (void*)(uintptr_t)264, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOSS((void*)(uintptr_t)260, fake, 10, 64, 512, 1, 0.2f, fake, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOSS(fake, fake, 10, 64, 512, 0, 0.2f, fake, 64), NAT_WORKSPACE_TOO_SMALL);

#define LOSSKL(ref, beta, kind, dt, wsb) \
  nat_loss_fwd_bwd_kl(fake, fake, fake, fake, fake, fake, fake, 10, 64, 512, dt, 0.2f, 0.2f, 1.f, ref, beta, kind, fake, NULL, NULL, \
                      NULL, NULL, fake, fake, 0, fake, wsb, NULL)
  EXPECT(LOSSKL(fake, -0.5f, 0, 1, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOSSKL(fake, NAN, 0, 1, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOSSKL(fake, 0.1f, 2, 1, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOSSKL(NULL, 0.1f, 0, 1, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOSSKL(fake, 0.1f, 0, 9, (size_t)1 << 34), NAT_UNSUPPORTED_DTYPE);
  EXPECT(LOSSKL(fake, 0.1f, 0, 1, 64), NAT_WORKSPACE_TOO_SMALL);

#define LOGP(hid, W, Nk, H, V, dt, out, ws, wsb) nat_logp_fwd(hid, W, fake, Nk, H, V, dt, out, NULL, NULL, ws, wsb, NULL)
  EXPECT(LOGP(fake, fake, 10, 64, 512, 3, fake, fake, (size_t)1 << 34), NAT_UNSUPPORTED_DTYPE);
  EXPECT(LOGP(fake, fake, -1, 64, 512, 1, fake, fake, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOGP(fake, fake, 10, 100, 512, 1, fake, fake, (size_t)1 << 34), NAT_BAD_SHAPE);
  EXPECT(LOGP(NULL, fake, 10, 64, 512, 1, fake, fake, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOGP(fake, fake, 10, 64, 512, 1, NULL, fake, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOGP(fake, fake, 10, 64, 512, 1, fake, fake, 100), NAT_WORKSPACE_TOO_SMALL);
  EXPECT(LOGP(fake, (void*)(uintptr_t)264, 10, 64, 512, 1, fake, fake, (size_t)1 << 34), NAT_INVALID_ARG);
  EXPECT(LOGP(NULL, fake, 0, 64, 512, 1, NULL, NULL, 0), NAT_OK);                 /* nothing to do */

  EXPECT(nat_probe_mfma_bf16(1, 10, NULL, NULL, NULL), NAT_INVALID_ARG);
  EXPECT(nat_probe_mfma_bf16(1, 0, fake, NULL, NULL), NAT_INVALID_ARG);
  EXPECT(nat_probe_copy(fake, NULL, 1024, NULL), NAT_INVALID_ARG);
  EXPECT(nat_probe_copy(fake, fake, 1000, NULL), NAT_INVALID_ARG);
  EXPECT(nat_probe_copy(fake, (void*)(uintptr_t)260, 1024, NULL), NAT_INVALID_ARG);
  EXPECT(nat_probe_copy(fake, fake, 0, NULL), NAT_OK);

  {
    double ms[64];
    int64_t cnt[64];
    memset(ms, 0, sizeof ms); memset(cnt, 0, sizeof cnt);
    EXPECT(nat_profile_collect(ms, cnt, 1), NAT_INVALID_ARG);
    EXPECT(nat_profile_collect(NULL, cnt, 64), NAT_INVALID_ARG);
    EXPECT(nat_profile_collect(ms, cnt, nat_profile_num_classes()), NAT_OK);
  }
  if (failures) { fprintf(stderr, "host_abi_san: %d unexpected statuses\n", failures); return 1; }
  printf("host_abi_san OK\n");
  return 0;
}
