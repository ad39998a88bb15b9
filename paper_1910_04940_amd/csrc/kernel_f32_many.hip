// Instantiations of the kernel: fp32 elements, 16 columns per lane.  See kernel.hpp.
#include "kernel.hpp"

namespace blink {

KernelFn kernel_f32_many(int flavour) { return pick_kernel_of<float, kColumnsMany>(flavour); }

}  // namespace blink
