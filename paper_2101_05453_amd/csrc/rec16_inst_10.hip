// Instantiations of the 16-row recurrent kernel for k depth 10 (h rows up to 640 bytes).
#include "rec16_kernel.inc.h"

namespace lstm_int {
rec_fn rec16_pick_10(int fl) { return rec16_pick_ks<10>(fl); }
}  // namespace lstm_int
