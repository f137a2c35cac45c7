// Instantiations of the scalar-register layer kernel: unsigned data.
#include "hikonv_conv2d_sreg.h"

namespace hikonv {
hipError_t launch_conv2d_sreg_unsigned(const Conv2dArgs &a, int hi, dim3 g, hipStream_t stream)
{
    return launch_conv2d_sreg_sw<false>(a, hi, g, stream);
}
} // namespace hikonv
