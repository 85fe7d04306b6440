// 4-series forward LSTM kernel, last layer of a residual block: also writes block input + hidden state (see
// lstm_narrow_fwd.h).
#include "lstm_narrow_fwd.h"

namespace esrnn {

hipError_t launch_lstm_forward_narrow_residual(const Plan &pl, int layer, const int32_t *lengths, const float *weights,
                                               float *ws, hipStream_t st)
{
    return launch_narrow_fwd<true>(pl, layer, lengths, weights, ws, st);
}

}  // namespace esrnn
