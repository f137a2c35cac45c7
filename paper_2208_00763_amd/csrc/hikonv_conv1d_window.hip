// Launcher of the packed 1-D window kernel (hikonv_conv1d_window.h); the kernels are
// instantiated per tap count in hikonv_conv1d_window_t*.hip.
#include "hikonv_conv1d_window.h"

namespace hikonv {

hipError_t launch_window_t1(const Conv1dArgs &, bool, bool, hipStream_t);
hipError_t launch_window_t2(const Conv1dArgs &, bool, bool, hipStream_t);
hipError_t launch_window_t3(const Conv1dArgs &, bool, bool, hipStream_t);
hipError_t launch_window_t4(const Conv1dArgs &, bool, bool, hipStream_t);
hipError_t launch_window_t5(const Conv1dArgs &, bool, bool, hipStream_t);
hipError_t launch_window_t6(const Conv1dArgs &, bool, bool, hipStream_t);
hipError_t launch_window_t7(const Conv1dArgs &, bool, bool, hipStream_t);

// Plans this form covers: up to 7 taps, K = min(taps, N) taps per B word (so that a kernel wider
// than one B word meets whole blocks), N one of the slice counts the planner produces for 32-bit
// words, a window of taps + 7 containers of up to 4 bits (taps + 3 of 8 bits, within 96 bits), positions inside a row within 32 bits.
bool conv1d_window_applicable(const Conv1dArgs &a)
{
    if (a.taps < 1 || a.taps > 7) return false;
    if (a.N != 2 && a.N != 3 && a.N != 4 && a.N != 5 && a.N != 6 && a.N != 8 && a.N != 11) return false;
    if (a.Kp != (a.taps < a.N ? a.taps : a.N) || a.chunks != (a.taps + a.Kp - 1) / a.Kp) return false;
    if (a.N * a.c > 32) return false;                        // a block's containers come out of one dword
    if (conv1d_window_group(a) == 8) return quad_stream_applicable(a, a.taps + 7);
    if ((a.taps + 3) * a.c > 64 && (a.c != 8 || a.N > 3)) return false;
    return quad_stream_applicable(a, a.taps + 3);
}

hipError_t launch_conv1d_window(const Conv1dArgs &a, bool a_signed, bool any_signed, hipStream_t stream)
{
    if (!conv1d_window_applicable(a)) return hipErrorNotSupported;
    switch (a.taps) {
    case 1: return launch_window_t1(a, a_signed, any_signed, stream);
    case 2: return launch_window_t2(a, a_signed, any_signed, stream);
    case 3: return launch_window_t3(a, a_signed, any_signed, stream);
    case 4: return launch_window_t4(a, a_signed, any_signed, stream);
    case 5: return launch_window_t5(a, a_signed, any_signed, stream);
    case 6: return launch_window_t6(a, a_signed, any_signed, stream);
    default: return launch_window_t7(a, a_signed, any_signed, stream);
    }
}

} // namespace hikonv
