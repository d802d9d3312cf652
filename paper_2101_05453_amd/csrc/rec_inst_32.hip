// Instantiations of the persistent recurrent kernel for k depth 32 (h rows up to 1024 bytes).
#include "rec_kernel.inc.h"

namespace lstm_int {
rec_fn rec_pick_32(int rt, int fl) { return rec_pick_ks<32>(rt, fl); }
}  // namespace lstm_int
