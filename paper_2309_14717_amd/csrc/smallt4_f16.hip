// The one-column-per-lane streaming kernel reading 16-bit factors (fp16 alpha and beta packed
// into one word per group and column): its instantiations, compiled apart from the fp32 ones.
#include "smallt4_impl.hpp"

namespace qalora {

hipError_t launch_smallt4_f16(const SmallTArgs& a, hipStream_t st) { return launch_smallt4_impl<true>(a, st); }

}  // namespace qalora
