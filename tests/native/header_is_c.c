/* The boundary is a C ABI: this file must compile as C99 with nothing but the header. */
#include "avmp.h"

int use_types(void) {
  avmp_config_t cfg;
  avmp_step_t step;
  avmp_stats_t stats;
  avmp_policy_t pol;
  avmp_handle_t h = AVMP_INVALID_HANDLE;
  (void)cfg; (void)step; (void)stats; (void)pol;
  return (int)(h >> AVMP_PAGE_ID_BITS) + AVMP_OK + AVMP_POOL_SSM + AVMP_K_COUNT;
}
