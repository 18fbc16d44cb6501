/* Error paths of libradial through the C ABI: no GPU work.  Compiled as strict C99 by the tests
 * (and once more under AddressSanitizer / UBSan). */
#include <stdio.h>
#include <string.h>
#include "radial.h"
int main(void) {
  radial_mask* m = (radial_mask*)0;
  radial_mask_params p = {4, 16, 100, 1, 0u, 1, 1, 0};      /* unsupported block size */
  if (radial_mask_build(&p, 0, &m) != RADIAL_EUNSUPPORTED || m) return 1;
  if (!strstr(radial_last_error(), "block")) return 2;
  p.block = 64; p.width_den = 0;                          /* bad sparsity knob */
  if (radial_mask_build(&p, 0, &m) != RADIAL_EINVAL) return 3;
  if (radial_mask_build_banded(4, 16, 64, 1, (const int32_t*)0, 0u, 0, &m) != RADIAL_EINVAL) return 4;
  if (radial_mask_info((const radial_mask*)0, 0, 0, 0, 0, 0) != RADIAL_EINVAL) return 5;
  radial_mask_free((radial_mask*)0);
  puts("ok");
  return 0;
}
