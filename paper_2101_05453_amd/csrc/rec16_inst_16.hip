// Instantiations of the 16-row recurrent kernel for k depth 16 (h rows up to 1024 bytes).
#include "rec16_kernel.inc.h"

namespace lstm_int {
rec_fn rec16_pick_16(int fl) { return rec16_pick_ks<16>(fl); }
}  // namespace lstm_int
