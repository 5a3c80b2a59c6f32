// Hamming scoring and per-head top-k: dispatch on the code length.  The kernels live in
// retrieve_kernels.h; retrieve_w*.hip instantiate them.
#include "retrieve_kernels.h"

namespace spotlight {
namespace retrieve_detail {
#define SPOTLIGHT_EXTERN_W(W) extern template int launch_w<W>(spotlight_ctx*, const RetrieveArgs&);
SPOTLIGHT_EXTERN_W(1) SPOTLIGHT_EXTERN_W(2) SPOTLIGHT_EXTERN_W(3) SPOTLIGHT_EXTERN_W(4)
SPOTLIGHT_EXTERN_W(5) SPOTLIGHT_EXTERN_W(6) SPOTLIGHT_EXTERN_W(7) SPOTLIGHT_EXTERN_W(8)
SPOTLIGHT_EXTERN_W(9) SPOTLIGHT_EXTERN_W(10) SPOTLIGHT_EXTERN_W(11) SPOTLIGHT_EXTERN_W(12)
SPOTLIGHT_EXTERN_W(13) SPOTLIGHT_EXTERN_W(14) SPOTLIGHT_EXTERN_W(15) SPOTLIGHT_EXTERN_W(16)
SPOTLIGHT_EXTERN_W(32)
#undef SPOTLIGHT_EXTERN_W
}  // namespace retrieve_detail
using namespace retrieve_detail;

int launch_retrieve(spotlight_ctx* ctx, const uint32_t* codes, int64_t n_tokens, int k, int n_sink, int n_local,
                    int32_t* out_idx, uint16_t* out_dist)
{
    RetrieveArgs a;
    a.codes = codes;
    a.n_tokens = n_tokens;
    a.n_sink = n_sink;
    a.local_begin = n_tokens - n_local;
    a.k = k;
    a.nblk = static_cast<int>((n_tokens + kTPB - 1) / kTPB);
    a.out_idx = out_idx;
    a.out_dist = out_dist;
    switch (ctx->plan.W) {
    case 1: return launch_w<1>(ctx, a);
    case 2: return launch_w<2>(ctx, a);
    case 3: return launch_w<3>(ctx, a);
    case 4: return launch_w<4>(ctx, a);
    case 5: return launch_w<5>(ctx, a);
    case 6: return launch_w<6>(ctx, a);
    case 7: return launch_w<7>(ctx, a);
    case 8: return launch_w<8>(ctx, a);
    case 9: return launch_w<9>(ctx, a);
    case 10: return launch_w<10>(ctx, a);
    case 11: return launch_w<11>(ctx, a);
    case 12: return launch_w<12>(ctx, a);
    case 13: return launch_w<13>(ctx, a);
    case 14: return launch_w<14>(ctx, a);
    case 15: return launch_w<15>(ctx, a);
    case 16: return launch_w<16>(ctx, a);
    case 32: return launch_w<32>(ctx, a);
    default: return SPOTLIGHT_ERR_UNSUPPORTED;
    }
}

}  // namespace spotlight
