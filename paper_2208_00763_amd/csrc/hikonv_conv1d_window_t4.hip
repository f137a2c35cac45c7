// k_conv1d_window instantiated for kernels of 4 taps (one translation unit per tap count, so that the build runs in parallel)
#include "hikonv_conv1d_window.h"

namespace hikonv {
hipError_t launch_window_t4(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream)
{
    return launch_conv1d_window_taps<4>(a, a_signed, any_signed, stream);
}
} // namespace hikonv
