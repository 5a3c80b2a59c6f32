// Instantiates the retrieval kernels for code lengths of 13, 14, 15 words (see retrieve_kernels.h).
#include "retrieve_kernels.h"

namespace spotlight {
namespace retrieve_detail {
template int launch_w<13>(spotlight_ctx*, const RetrieveArgs&);
template int launch_w<14>(spotlight_ctx*, const RetrieveArgs&);
template int launch_w<15>(spotlight_ctx*, const RetrieveArgs&);
}  // namespace retrieve_detail
}  // namespace spotlight
