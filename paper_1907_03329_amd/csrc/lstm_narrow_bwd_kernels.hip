// 4-series reverse LSTM kernel, four waves per workgroup (see lstm_narrow_bwd.h).
#include "lstm_narrow_bwd.h"

namespace esrnn {

hipError_t launch_lstm_backward_narrow(const Plan &pl, int layer, const int32_t *lengths, float *ws, hipStream_t st)
{
    if (pl.layer[layer].split_bwd) return launch_lstm_backward_narrow_split(pl, layer, lengths, ws, st);
    return launch_narrow_bwd<false>(pl, layer, lengths, ws, st);
}

}  // namespace esrnn
