// Instantiates the retrieval kernels for code lengths of 32 words (see retrieve_kernels.h).
#include "retrieve_kernels.h"

namespace spotlight {
namespace retrieve_detail {
template int launch_w<32>(spotlight_ctx*, const RetrieveArgs&);
}  // namespace retrieve_detail
}  // namespace spotlight
