// Instantiates the single-launch decode step for bfloat16 hash weights (see step_small_kernel.h).
#include "step_small_kernel.h"

namespace spotlight {
namespace small {
template int launch_small<true, true>(spotlight_ctx*, const SmallArgs&, size_t);
template int launch_small<false, true>(spotlight_ctx*, const SmallArgs&, size_t);
}  // namespace small
}  // namespace spotlight
