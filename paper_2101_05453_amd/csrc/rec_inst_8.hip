// Instantiations of the persistent recurrent kernel for k depth 8 (h rows up to 256 bytes).
#include "rec_kernel.inc.h"

namespace lstm_int {
rec_fn rec_pick_8(int rt, int fl) { return rec_pick_ks<8>(rt, fl); }
}  // namespace lstm_int
