// Instantiations of the 16-row recurrent kernel for k depth 4 (h rows up to 256 bytes).
#include "rec16_kernel.inc.h"

namespace lstm_int {
rec_fn rec16_pick_4(int fl) { return rec16_pick_ks<4>(fl); }
}  // namespace lstm_int
