// Instantiations of the packed layer kernel with the 32x32+64 multiply-accumulate.
#include <type_traits>
#include "hikonv_conv2d_kernel.h"

namespace hikonv {
hipError_t launch_conv2d_wide(const Conv2dArgs &a, bool any_signed, int co_tile, dim3 g, hipStream_t stream)
{
    return any_signed ? launch_conv2d_sw<true, true>(a, co_tile, g, stream)
                      : launch_conv2d_sw<false, true>(a, co_tile, g, stream);
}
} // namespace hikonv
