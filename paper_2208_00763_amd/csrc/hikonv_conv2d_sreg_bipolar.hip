// Instantiations of the scalar-register layer kernel: {-1,+1} data.
#include "hikonv_conv2d_sreg.h"

namespace hikonv {
hipError_t launch_conv2d_sreg_bipolar(const Conv2dArgs &a, int hi, dim3 g, hipStream_t stream)
{
    return launch_conv2d_sreg_sw<false, true>(a, hi, g, stream);
}
} // namespace hikonv
