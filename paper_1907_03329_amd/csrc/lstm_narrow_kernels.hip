// 4-series forward LSTM kernel, layers without a residual output (see lstm_narrow_fwd.h).
#include "lstm_narrow_fwd.h"

namespace esrnn {

hipError_t launch_lstm_forward_narrow(const Plan &pl, int layer, const int32_t *lengths, const float *weights,
                                      float *ws, hipStream_t st)
{
    if (pl.layer[layer].out) return launch_lstm_forward_narrow_residual(pl, layer, lengths, weights, ws, st);
    return launch_narrow_fwd<false>(pl, layer, lengths, weights, ws, st);
}

}  // namespace esrnn
