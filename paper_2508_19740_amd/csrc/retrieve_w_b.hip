// Instantiates the retrieval kernels for code lengths of 4, 5 words (see retrieve_kernels.h).
#include "retrieve_kernels.h"

namespace spotlight {
namespace retrieve_detail {
template int launch_w<4>(spotlight_ctx*, const RetrieveArgs&);
template int launch_w<5>(spotlight_ctx*, const RetrieveArgs&);
}  // namespace retrieve_detail
}  // namespace spotlight
