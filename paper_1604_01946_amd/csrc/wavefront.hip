// Placeholder schedules until the stream wavefront lands: run the layer-sequential step path.
#include "../../include/lstm.h"
#include "schedule.h"
namespace lstm {
int run_forward_wavefront(const FwdArgs& a) { return run_forward(a, LSTM_PATH_STEP); }
int run_backward_wavefront(const BwdArgs& a) { return run_backward(a, LSTM_PATH_STEP); }
void release_persistent();
void release_helpers() { release_persistent(); }
}  // namespace lstm
