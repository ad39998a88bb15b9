// Instantiations of the kernel: fp32 elements, 32 columns per lane.  See kernel.hpp.
#include "kernel.hpp"

namespace blink {

KernelFn kernel_f32_stream(int flavour) { return pick_kernel_of<float, kColumnsStream>(flavour); }

}  // namespace blink
