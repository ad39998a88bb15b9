// Instantiations of the kernels for payloads that stream: wrap-around int32 elements.  See stream.hpp.
#include "stream.hpp"

namespace blink {

KernelFn kernel_i32_stream(int flavour, bool direct) { return pick_stream_kernel_of<unsigned>(flavour, direct); }

}  // namespace blink
