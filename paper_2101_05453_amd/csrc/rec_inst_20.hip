// Instantiations of the persistent recurrent kernel for k depth 20 (h rows up to 640 bytes).
#include "rec_kernel.inc.h"

namespace lstm_int {
rec_fn rec_pick_20(int rt, int fl) { return rec_pick_ks<20>(rt, fl); }
}  // namespace lstm_int
