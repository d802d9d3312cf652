// Instantiations of the persistent recurrent kernel with 2:4 sparse recurrent weights, k depth 32.
#include "rec_kernel.inc.h"

namespace lstm_int {
rec_fn rec_pick_sparse_32(int fl) { return rec_pick_sparse_ks<32>(fl); }
}  // namespace lstm_int
