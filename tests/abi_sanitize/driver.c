/* Host-only exerciser of the argument checks of the spa2 C ABI, built with AddressSanitizer and
 * UndefinedBehaviorSanitizer on the host side (tests/test_abi_cpu.py compiles and runs it).  Every call below
 * must be rejected before anything is launched: the kernel launchers are replaced by stubs that abort. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "spa2.h"

static int failures = 0;
#define EXPECT(call, code)                                                                  \
  do {                                                                                      \
    int rc_ = (call);                                                                       \
    if (rc_ != (code)) { printf("line %d: got %d, expected %d\n", __LINE__, rc_, (code)); ++failures; } \
  } while (0)

static spa2_shape shape(int B, int H, int N, int d, int bq, int bkv, long long sn) {
  spa2_shape s;
  s.B = B; s.H = H; s.N = N; s.d = d; s.bq = bq; s.bkv = bkv;
  s.sn = sn ? sn : d; s.sh = (long long)N * s.sn; s.sb = (long long)H * s.sh;
  return s;
}

int main(void) {
  void* fake = (void*)0x1000;   /* 16-byte aligned, never dereferenced on a rejected call */
  void* odd = (void*)0x1004;
  spa2_pattern none = {0, 0, 0, 0, 0, 0, 0};
  spa2_pattern full = {(uint8_t*)fake, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, 0, 0};
  spa2_pattern half = {(uint8_t*)fake, (int32_t*)fake, (int32_t*)fake, (int32_t*)fake, 0, 0, 0};
  spa2_pattern rows_only = {(uint8_t*)fake, (int32_t*)fake, (int32_t*)fake, 0, 0, 0, 0};
  spa2_shape ok = shape(1, 2, 300, 128, 128, 64, 0);
  spa2_shape d96 = shape(1, 2, 300, 96, 128, 64, 0), bq64 = shape(1, 2, 300, 128, 64, 64, 0);
  spa2_shape n0 = shape(1, 2, 0, 128, 128, 64, 0), sn132 = shape(1, 2, 300, 128, 128, 64, 132);
  spa2_shape wide = shape(1, 1, 300, 128, 128, 64, (1 << 23) + 8);
  spa2_shape longrow = shape(1, 2, 64 * 8193, 64, 128, 64, 0);
  spa2_shape many = shape(1 << 12, 1 << 12, 20000, 64, 128, 64, 0);
  spa2_shape huge = shape(1, 1, 128, 128, 128, 64, 0);                /* B*H*N would overflow 64 bits if multiplied blindly */
  huge.B = huge.H = huge.N = 0x7fffffff;
  spa2_shape toolong = shape(1, 4, SPA2_STATIC_MAX_ROWS / 4 + 64, 128, 128, 64, 0);
  size_t big = (size_t)1 << 40;

  EXPECT(spa2_fwd(0, fake, fake, &ok, &full, 0.1f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_NULL);
  EXPECT(spa2_fwd(fake, fake, fake, 0, &full, 0.1f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_NULL);
  EXPECT(spa2_fwd(fake, fake, fake, &ok, &none, 0.1f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_NULL);
  EXPECT(spa2_fwd(odd, fake, fake, &ok, &full, 0.1f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_ALIGN);
  EXPECT(spa2_fwd(fake, fake, fake, &ok, &full, 0.0f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_RANGE);
  EXPECT(spa2_fwd(fake, fake, fake, &ok, &full, NAN, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_RANGE);
  EXPECT(spa2_fwd(fake, fake, fake, &d96, &full, 0.1f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_UNSUPPORTED);
  EXPECT(spa2_fwd(fake, fake, fake, &bq64, &full, 0.1f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_UNSUPPORTED);
  EXPECT(spa2_fwd(fake, fake, fake, &n0, &full, 0.1f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_SHAPE);
  EXPECT(spa2_fwd(fake, fake, fake, &sn132, &full, 0.1f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_ALIGN);
  EXPECT(spa2_fwd(fake, fake, fake, &wide, &full, 0.1f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_SHAPE);
  EXPECT(spa2_fwd(fake, fake, fake, &many, &full, 0.1f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_SHAPE);
  EXPECT(spa2_fwd(fake, fake, fake, &huge, &full, 0.1f, fake, 0, (float*)fake, 0, 0, 0), SPA2_ERR_SHAPE);

  EXPECT(spa2_fwd(fake, fake, fake, &ok, &full, 0.1f, fake, 0, (float*)fake, odd, big, 0), SPA2_ERR_ALIGN);
  EXPECT(spa2_mask(fake, fake, &ok, 1, 0.5f, 0.1f, &full, 0, 0, big, 0), SPA2_ERR_WORKSPACE);
  EXPECT(spa2_mask(fake, fake, &ok, 1, 0.5f, 0.1f, &full, 0, fake, 16, 0), SPA2_ERR_WORKSPACE);
  EXPECT(spa2_mask(fake, fake, &ok, 0, 0.0f, 0.1f, &full, 0, fake, big, 0), SPA2_ERR_RANGE);
  EXPECT(spa2_mask(fake, fake, &ok, 6, 0.5f, 0.1f, &full, 0, fake, big, 0), SPA2_ERR_RANGE);
  EXPECT(spa2_mask(fake, fake, &ok, -1, 0.5f, 0.1f, &full, 0, fake, big, 0), SPA2_ERR_RANGE);
  EXPECT(spa2_mask(fake, fake, &ok, 1, 1.5f, 0.1f, &full, 0, fake, big, 0), SPA2_ERR_RANGE);
  EXPECT(spa2_mask(fake, fake, &ok, 1, NAN, 0.1f, &full, 0, fake, big, 0), SPA2_ERR_RANGE);
  EXPECT(spa2_mask(fake, fake, &longrow, 1, 0.5f, 0.1f, &full, 0, fake, big, 0), SPA2_ERR_SHAPE);
  EXPECT(spa2_mask(fake, fake, &ok, 1, 0.5f, 0.1f, &half, 0, fake, big, 0), SPA2_ERR_NULL);
  EXPECT(spa2_mask_pool(fake, fake, &ok, fake, 16, 0), SPA2_ERR_WORKSPACE);
  EXPECT(spa2_mask_select(&ok, 1, 0.5f, 0.1f, &none, 0, fake, big, 0), SPA2_ERR_NULL);
  EXPECT(spa2_mask_columns(&longrow, &full, 0), SPA2_ERR_SHAPE);
  EXPECT(spa2_mask_columns(&many, &full, 0), SPA2_ERR_SHAPE);
  EXPECT(spa2_mask_columns(&ok, &rows_only, 0), SPA2_ERR_NULL);
  EXPECT(spa2_pattern_full(&ok, 0, 0), SPA2_ERR_NULL);

  EXPECT(spa2_bwd(fake, fake, fake, fake, 0, fake, (float*)fake, &ok, &rows_only, 0.1f, fake, fake, fake, fake, big, 0),
         SPA2_ERR_NULL);
  EXPECT(spa2_bwd(fake, fake, fake, fake, 0, fake, (float*)fake, &ok, &full, 0.1f, fake, fake, fake, fake, 8, 0),
         SPA2_ERR_WORKSPACE);
  EXPECT(spa2_bwd(fake, fake, fake, fake, odd, fake, (float*)fake, &ok, &full, 0.1f, fake, fake, fake, fake, big, 0),
         SPA2_ERR_ALIGN);
  EXPECT(spa2_bwd_delta(fake, 0, fake, &ok, fake, 8, 0), SPA2_ERR_WORKSPACE);
  EXPECT(spa2_bwd_dkdv(fake, fake, fake, fake, (float*)fake, &ok, &rows_only, 0.1f, fake, fake, fake, big, 0), SPA2_ERR_NULL);
  EXPECT(spa2_bwd_dq(fake, fake, fake, fake, (float*)fake, &ok, &full, -1.0f, fake, fake, big, 0), SPA2_ERR_RANGE);
  EXPECT(spa2_bwd_static(fake, fake, fake, fake, 0, fake, (float*)fake, 0, &full, 0.1f, fake, fake, fake, 0), SPA2_ERR_NULL);
  EXPECT(spa2_bwd_static(fake, fake, fake, fake, 0, fake, (float*)fake, &toolong, &full, 0.1f, fake, fake, fake, 0),
         SPA2_ERR_WORKSPACE);

  EXPECT(spa2_error_terms(fake, fake, (float*)fake, (float*)fake, &ok, 0, fake, big, 0), SPA2_ERR_NULL);
  EXPECT(spa2_error_terms(fake, fake, (float*)fake, (float*)fake, &ok, (double*)fake, fake, 8, 0), SPA2_ERR_WORKSPACE);
  EXPECT(spa2_vd_loss(0, fake, 8, SPA2_DTYPE_BF16, 1.0, (double*)fake, fake, big, 0), SPA2_ERR_NULL);
  EXPECT(spa2_vd_loss(fake, fake, 0, SPA2_DTYPE_BF16, 1.0, (double*)fake, fake, big, 0), SPA2_ERR_SHAPE);
  EXPECT(spa2_vd_loss(fake, fake, 8, 2, 1.0, (double*)fake, fake, big, 0), SPA2_ERR_UNSUPPORTED);
  EXPECT(spa2_vd_loss(odd, fake, 8, SPA2_DTYPE_F32, 1.0, (double*)fake, fake, big, 0), SPA2_ERR_ALIGN);
  EXPECT(spa2_vd_loss(fake, fake, 8, SPA2_DTYPE_F32, INFINITY, (double*)fake, fake, big, 0), SPA2_ERR_RANGE);
  EXPECT(spa2_vd_loss(fake, fake, 8, SPA2_DTYPE_F32, 1.0, (double*)fake, fake, 64, 0), SPA2_ERR_WORKSPACE);
  EXPECT(spa2_vd_loss_grad(fake, fake, 8, SPA2_DTYPE_F32, 1.0, 0, 0, 0), SPA2_ERR_NULL);

  /* host helpers and size queries over their whole argument range */
  if (spa2_topk_blocks(0.2, 10) != 2 || spa2_topk_blocks(0.0, 10) != 0 || spa2_topk_blocks(5.0, 10) != 10 ||
      spa2_topk_blocks(NAN, 10) != 0 || spa2_topk_blocks(0.5, -3) != 0 || spa2_topk_blocks(1e300, 0x7fffffff) != 0x7fffffff) {
    printf("spa2_topk_blocks\n"); ++failures;
  }
  if (spa2_mask_workspace_bytes(&huge) != 0 || spa2_bwd_workspace_bytes(&d96) != 0 || spa2_mask_workspace_bytes(0) != 0 ||
      spa2_error_workspace_bytes(&n0) != 0 || spa2_mask_workspace_bytes(&ok) == 0 || spa2_bwd_workspace_bytes(&ok) == 0 ||
      spa2_fwd_workspace_bytes(&ok) == 0 || spa2_fwd_workspace_bytes(&d96) != 0 ||
      spa2_bwd_workspace_min_bytes(&ok) == 0 || spa2_bwd_workspace_min_bytes(&ok) > spa2_bwd_workspace_bytes(&ok)) {
    printf("workspace sizes\n"); ++failures;
  }
  for (int c = 1; c >= -9; --c)
    if (!spa2_strerror(c) || !spa2_strerror(c)[0]) { printf("strerror %d\n", c); ++failures; }
  printf(failures ? "FAILED %d\n" : "all rejected before launch\n", failures);
  return failures ? 1 : 0;
}
