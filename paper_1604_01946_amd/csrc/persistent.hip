#include "../../include/lstm.h"
#include "schedule.h"
namespace lstm {
bool persistent_supported(const Dims&, bool) { return false; }
int run_forward_persistent(const FwdArgs&) { return LSTM_UNSUPPORTED; }
int run_backward_persistent(const BwdArgs&) { return LSTM_UNSUPPORTED; }
}  // namespace lstm
