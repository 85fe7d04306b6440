// 4-series reverse LSTM kernel, eight waves per workgroup: the weight gradient on waves of its own (see
// lstm_narrow_bwd.h).
#include "lstm_narrow_bwd.h"

namespace esrnn {

hipError_t launch_lstm_backward_narrow_split(const Plan &pl, int layer, const int32_t *lengths, float *ws, hipStream_t st)
{
    return launch_narrow_bwd<true>(pl, layer, lengths, ws, st);
}

}  // namespace esrnn
