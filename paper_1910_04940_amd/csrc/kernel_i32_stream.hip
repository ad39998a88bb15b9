// Instantiations of the kernel: int32 elements (added as unsigned: wrap-around), 32 columns per lane.  See kernel.hpp.
#include "kernel.hpp"

namespace blink {

KernelFn kernel_i32_stream(int flavour) { return pick_kernel_of<unsigned, kColumnsStream>(flavour); }

}  // namespace blink
