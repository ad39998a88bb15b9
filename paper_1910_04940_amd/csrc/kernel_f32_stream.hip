// Instantiations of the kernels for payloads that stream: fp32 elements.  See stream.hpp.
#include "stream.hpp"

namespace blink {

KernelFn kernel_f32_stream(int flavour, bool direct) { return pick_stream_kernel_of<float>(flavour, direct); }

}  // namespace blink
