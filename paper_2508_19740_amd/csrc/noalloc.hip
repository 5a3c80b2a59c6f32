// spotlight_decode_step_noalloc: the decode step for callers that cannot allocate.  The workspace
// is a fixed array in the library's code object instead of memory from hipMalloc; the context is a
// plain struct on the caller's stack.  Nothing here (or below it) allocates or frees.
#include <mutex>
#include <string.h>

#include "internal.h"

namespace {

// Each GPU holds its own copy of this array at its own address.  In host code the name is only a
// handle for hipGetSymbolAddress; kernels are given the address that call returns.
static __device__ __align__(256) unsigned char scratch[SPOTLIGHT_NOALLOC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
struct DeviceSlot {
    char* scratch_ptr;   // device address of `scratch` on this GPU (null: not asked yet)
    int max_lds, n_cus;
    // score workgroups resident at once, per kernel shape seen on this device
    struct { int W, G, resident; } shapes[8];
    int n_shapes;
};
DeviceSlot g_dev[kMaxDevices];
std::mutex g_mu;

// Set-up of the current device, once: the address of its copy of the array and two attributes.
int device_slot(int dev, DeviceSlot** out)
{
    if (dev < 0 || dev >= kMaxDevices) return SPOTLIGHT_ERR_UNSUPPORTED;
    DeviceSlot* s = &g_dev[dev];
    if (!s->scratch_ptr) {
        void* ptr = nullptr;
        int lds = 0, cus = 0;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return SPOTLIGHT_ERR_HIP;
        if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess ||
            hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
            return SPOTLIGHT_ERR_HIP;
        s->max_lds = lds;
        s->n_cus = cus;
        s->scratch_ptr = static_cast<char*>(ptr);
    }
    *out = s;
    return SPOTLIGHT_OK;
}

}  // namespace

extern "C" int spotlight_decode_step_noalloc(const spotlight_config* cfg, const void* q, const void* K, const void* V,
                                             const spotlight_hash_weights* w, uint32_t* codes, int64_t n_tokens,
                                             int32_t k, int32_t n_sink, int32_t n_local, float scale,
                                             int32_t* out_idx, float* out)
{
    using namespace spotlight;
    spotlight_ctx ctx;
    memset(&ctx, 0, sizeof(ctx));
    int rc = make_plan(cfg, &ctx.plan);   // host only
    if (rc != SPOTLIGHT_OK) return rc;
    // everything the step's kernels touch lies in front of the room for the packed weights
    if (ctx.plan.off_pack_w1 > sizeof(scratch)) return SPOTLIGHT_ERR_TOO_LARGE;
    ctx.cfg = *cfg;
    ctx.stream = static_cast<hipStream_t>(cfg->stream);
    rc = check_step_args(&ctx, q, K, V, w, codes, n_tokens, k, n_sink, n_local, out_idx, out);   // before any HIP call
    if (rc != SPOTLIGHT_OK) return rc;

    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return SPOTLIGHT_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mu);
    DeviceSlot* slot = nullptr;
    rc = device_slot(dev, &slot);
    if (rc != SPOTLIGHT_OK) return rc;
    ctx.workspace = slot->scratch_ptr;
    ctx.max_lds = slot->max_lds;
    ctx.n_cus = slot->n_cus;
    for (int i = 0; i < slot->n_shapes; ++i)
        if (slot->shapes[i].W == ctx.plan.W && slot->shapes[i].G == ctx.plan.G) ctx.score_resident = slot->shapes[i].resident;
    const bool known = ctx.score_resident != 0;

    rc = decode_step(&ctx, q, K, V, w, codes, n_tokens, k, n_sink, n_local, scale, out_idx, out);

    if (!known && ctx.score_resident != 0 && slot->n_shapes < 8) {
        slot->shapes[slot->n_shapes].W = ctx.plan.W;
        slot->shapes[slot->n_shapes].G = ctx.plan.G;
        slot->shapes[slot->n_shapes].resident = ctx.score_resident;
        slot->n_shapes += 1;
    }
    return rc;
}
