// Instantiates the single-launch decode step for binary32 hash weights (see step_small_kernel.h).
#include "step_small_kernel.h"

namespace spotlight {
namespace small {
template int launch_small<true, false>(spotlight_ctx*, const SmallArgs&, size_t);
template int launch_small<false, false>(spotlight_ctx*, const SmallArgs&, size_t);
}  // namespace small
}  // namespace spotlight
