/* Plain C (C99) caller of libstc: the header compiles as C and the entry points link and
 * answer without a GPU (version, status strings, workspace sizes, argument errors). */
#include <stdio.h>
#include <string.h>

#include "stc.h"

int main(void) {
  stc_shape_t s;
  int fails = 0;
  memset(&s, 0, sizeof s);
  s.B = 2, s.Hq = 8, s.Hkv = 2, s.D = 128, s.N = 4096, s.P = 16, s.G = 8;
  s.v_cap_groups = 4096 * 8;
  if (stc_version() < 1) ++fails;
  if (strcmp(stc_status_string(STC_OK), "ok") != 0) ++fails;
  if (stc_status_string(STC_ERR_SHAPE)[0] == 0) ++fails;
  if (stc_workspace_bytes(&s, STC_WS_ROUTE, 0) == 0) ++fails;
  if (stc_workspace_bytes(&s, STC_WS_STEP, 64) <
      stc_workspace_bytes(&s, STC_WS_SELECT, 64) + stc_workspace_bytes(&s, STC_WS_ATTENTION, 64))
    ++fails;
  if (stc_bounds_bytes(&s) != (size_t)2 * 2 * 256 * 128 * 4) ++fails;
  if (stc_build_page_bounds(NULL, NULL, NULL, NULL) != STC_ERR_NULL) ++fails;
  if (stc_decode_step(&s, NULL, NULL, NULL, NULL, NULL, NULL, 64, NULL, NULL, NULL, 0, NULL) !=
      STC_ERR_NULL)
    ++fails;
  s.G = 5; /* not a power of two */
  if (stc_score_pages(&s, (const void *)16, (const void *)16, (float *)16, NULL) != STC_ERR_SHAPE)
    ++fails;
  printf("c_abi_check: %d failure(s)\n", fails);
  return fails;
}
