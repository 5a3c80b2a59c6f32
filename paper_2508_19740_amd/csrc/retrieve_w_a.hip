// Instantiates the retrieval kernels for code lengths of 1, 2, 3 words (see retrieve_kernels.h).
#include "retrieve_kernels.h"

namespace spotlight {
namespace retrieve_detail {
template int launch_w<1>(spotlight_ctx*, const RetrieveArgs&);
template int launch_w<2>(spotlight_ctx*, const RetrieveArgs&);
template int launch_w<3>(spotlight_ctx*, const RetrieveArgs&);
}  // namespace retrieve_detail
}  // namespace spotlight
