// The decode step of a short context as one kernel launch: eligibility and dispatch.  The kernel
// is in step_small_kernel.h.
#include "step_small_kernel.h"

namespace spotlight {
namespace small {
extern template int launch_small<true, true>(spotlight_ctx*, const SmallArgs&, size_t);
extern template int launch_small<false, true>(spotlight_ctx*, const SmallArgs&, size_t);
extern template int launch_small<true, false>(spotlight_ctx*, const SmallArgs&, size_t);
extern template int launch_small<false, false>(spotlight_ctx*, const SmallArgs&, size_t);
}  // namespace small
using namespace small;

bool step_small_applies(const spotlight_ctx* ctx, int64_t n_tokens)
{
    const Plan& p = ctx->plan;
    if (!ctx->opt[SPOTLIGHT_OPT_STEP_SINGLE_LAUNCH]) return false;
    if (n_tokens > kSmMaxTokens || p.W > 8 || p.hidden % kHeadDim != 0 || p.hidden > kSmMaxHidden) return false;
    if (static_cast<int64_t>(p.B) * p.Hkv * n_tokens * p.W * 4 > kSmMaxCodeBytes) return false;
    return small_lds_bytes(p, n_tokens, false) <= static_cast<size_t>(ctx->max_lds);
}

int launch_step_small(spotlight_ctx* ctx, const HashLaunch& qjob, const HashLaunch& kjob, const void* q, const void* K,
                      const void* V, const uint32_t* codes, int64_t n_tokens, int k, int n_sink, int n_local,
                      float scale, int32_t* out_idx, float* out)
{
    const Plan& p = ctx->plan;
    SmallArgs a;
    a.job[0] = make_hash_args(qjob);
    a.job[1] = make_hash_args(kjob);
    a.job[0].zero = nullptr;   // no global histograms on this path
    a.q = q;
    a.K = K;
    a.V = V;
    a.codes = codes;
    a.out_idx = out_idx;
    a.out = out;
    a.n_tokens = n_tokens;
    a.Nmax = p.Nmax;
    a.n_sink = n_sink;
    a.local_begin = n_tokens - n_local;
    a.k = k;
    a.Hq = p.Hq;
    a.Hkv = p.Hkv;
    a.G = p.G;
    a.act_dim = p.hidden > 0 ? p.hidden : kHeadDim;
    a.chw = small_chw(n_tokens);
    a.packed = qjob.pack_out && (p.hidden == 0 || qjob.pack_w1) && kjob.pack_out == qjob.pack_out && kjob.pack_w1 == qjob.pack_w1;
    a.scale = scale;
    a.n_pad = small_n_pad(n_tokens);
    a.cache_bins = small_lds_bytes(p, n_tokens, true) <= static_cast<size_t>(ctx->max_lds) ? 1 : 0;
    const size_t lds = small_lds_bytes(p, n_tokens, a.cache_bins != 0);
    const bool kvb = p.kv_dtype == SPOTLIGHT_BF16, wb = p.w_dtype == SPOTLIGHT_BF16;
    if (kvb && wb) return launch_small<true, true>(ctx, a, lds);
    if (!kvb && wb) return launch_small<false, true>(ctx, a, lds);
    if (kvb && !wb) return launch_small<true, false>(ctx, a, lds);
    return launch_small<false, false>(ctx, a, lds);
}

}  // namespace spotlight
