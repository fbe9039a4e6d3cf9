/* Plain C99 user of the library: the header must compile as C and the entry points link
 * without any C++ or Python in between.  Built and run by tests/test_host_boundary.py. */
#include <stdio.h>
#include "hcache.h"
int main(void) {
  hc_model_desc d = {2, 256, 4, 4, 64, 16, 128, 0, 10000.0f, 1e-5f, HC_NORM_RMS};
  int32_t lh, lo, comp;
  if (hc_validate_desc(&d) != HC_OK) return 1;
  d.head_dim = 48;
  if (hc_validate_desc(&d) != HC_EINVAL) return 2;
  if (hc_partition_layers(32, 1.0, 2.0, 1.1, 10.0, &lh, &lo, &comp) != HC_OK || lh != 31 || lo != 1) return 3;
  printf("%s ok %s\n", hc_version(), hc_last_error());
  return 0;
}
