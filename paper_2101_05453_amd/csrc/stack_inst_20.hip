// Instantiations of the stacked recurrent kernel for k depth 20.
#include "stack_kernel.inc.h"

namespace lstm_int {
stack_fn stack_pick_20(int fl, bool one) {
  switch (fl) {
#define LSTM_STACK_CASE(F) case F: return one ? stack_kernel<20, F, true> : stack_kernel<20, F, false>;
    LSTM_STACK_CASE(0) LSTM_STACK_CASE(1) LSTM_STACK_CASE(2) LSTM_STACK_CASE(3)
    LSTM_STACK_CASE(4) LSTM_STACK_CASE(5) LSTM_STACK_CASE(6) LSTM_STACK_CASE(7)
    LSTM_STACK_CASE(8) LSTM_STACK_CASE(9) LSTM_STACK_CASE(10) LSTM_STACK_CASE(11)
    LSTM_STACK_CASE(12) LSTM_STACK_CASE(13) LSTM_STACK_CASE(14) LSTM_STACK_CASE(15)
#undef LSTM_STACK_CASE
  }
  return nullptr;
}
}  // namespace lstm_int
