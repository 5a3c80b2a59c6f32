// Instantiates the retrieval kernels for code lengths of 10, 11, 12 words (see retrieve_kernels.h).
#include "retrieve_kernels.h"

namespace spotlight {
namespace retrieve_detail {
template int launch_w<10>(spotlight_ctx*, const RetrieveArgs&);
template int launch_w<11>(spotlight_ctx*, const RetrieveArgs&);
template int launch_w<12>(spotlight_ctx*, const RetrieveArgs&);
}  // namespace retrieve_detail
}  // namespace spotlight
