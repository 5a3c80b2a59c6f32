// Internal declarations shared by the HIP translation units of libspotlight (not installed).
#pragma once

#include <hip/hip_runtime.h>
#if defined(__HIPCC__)
#include <hip/hip_ext.h>
#endif
#include <stdint.h>

#include "spotlight.h"

namespace spotlight {

constexpr int kHeadDim = 128;
constexpr int kThreads = 256;       // 4 wavefronts of 64 lanes per workgroup (all kernels but the single-launch step)
constexpr int kMaxGroup = 8;        // query heads per key-value head
constexpr int kAttendMinRows = 32;  // smallest number of gathered rows one workgroup takes
constexpr int kTokensPerBlock = 4096;  // tokens one score / select workgroup covers (16 per thread)
constexpr int kCandCap = 1024;      // candidate-list entries per (query head, token block)
constexpr int kMaxProfile = 8192;

// Geometry derived once from the configuration.
struct Plan {
    int B, Hq, Hkv, G, L, W, hidden;
    int64_t Nmax;
    int max_topk;
    int kv_dtype, w_dtype;
    int max_blocks;        // ceil(Nmax / kTokensPerBlock)
    int max_splits;        // ceil(max_topk / kAttendMinRows)
    // workspace offsets in bytes
    size_t off_qcode;      // [B*Hq][W] query codes
    size_t off_gcum;       // [B*Hq][L+2] cumulative histogram of the head (bin 0: forced tokens, bin d+1: distance d)
    size_t off_blockcum;   // [B*Hq][max_blocks][L+2] cumulative histogram of each token block
    size_t off_blockmeta;  // [B*Hq][max_blocks] {candidate bound, four sub-list lengths}
    size_t off_cand;       // [B*Hq][max_blocks][4][kCandCap/4] candidates (distance << 16 | block offset)
    size_t off_part_ml;    // [B*Hq][max_splits] {max, sum} of each attention split
    size_t off_part_acc;   // [B*Hq][max_splits][128] weighted value sums of each split
    size_t off_wnorm;      // [Hkv][L] norms of the second hash layer's rows (bulk hashing on the matrix cores)
    size_t off_pack_w1;    // first hash layer in the single-vector kernel's read order (pack_w1_elems per kv head)
    size_t off_pack_out;   // output matrix of the hash (W2, or R of the linear hash) in that order
    size_t pack_w1_elems, pack_out_elems;   // elements per kv head; both 0 if the hash shape has no such copy
    size_t off_audit;      // AuditRec of the bulk hash (SPOTLIGHT_OPT_BULK_HASH_AUDIT)
    size_t total_bytes;
};

#if defined(__HIPCC__)
// Inclusive prefix sum of x over the 64 lanes of a wavefront, by data-parallel-primitive moves
// (shifts within rows of 16 lanes, then the last lane of a row broadcast to the rows behind it):
// six dependent vector instructions, no LDS round trips.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t x)
{
#define SPOTLIGHT_DPP_ADD(ctrl, rows) \
    x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), ctrl, rows, 0xf, true))
    SPOTLIGHT_DPP_ADD(0x111, 0xf);   // row_shr:1
    SPOTLIGHT_DPP_ADD(0x112, 0xf);   // row_shr:2
    SPOTLIGHT_DPP_ADD(0x114, 0xf);   // row_shr:4
    SPOTLIGHT_DPP_ADD(0x118, 0xf);   // row_shr:8
    SPOTLIGHT_DPP_ADD(0x142, 0xa);   // lane 15 of rows 0 and 2 to rows 1 and 3
    SPOTLIGHT_DPP_ADD(0x143, 0xc);   // lane 31 to rows 2 and 3
#undef SPOTLIGHT_DPP_ADD
    return x;
}

// Sum of x over the wavefront, in every lane.
__device__ __forceinline__ uint32_t wave_sum(uint32_t x)
{
    return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(wave_inclusive_scan(x)), 63));
}
#endif

int make_plan(const spotlight_config* cfg, Plan* plan);  // SPOTLIGHT_OK or an error code; host only

// What the audited bulk hash accumulates (device side), see spotlight_bulk_hash_audit_read.
struct AuditRec {
    unsigned long long outputs;    // hash outputs evaluated on the matrix cores
    unsigned long long listed;     // of those, the ones whose sign the bound did not settle (recomputed)
    unsigned long long wrong;      // outputs the bound settled whose sign differs from the chain's: must stay 0
    uint32_t max_ratio_bits;       // largest |y_matrix - y_chain| / (||W2[j]|| ||h||), as the bits of a non-negative float
    uint32_t pad;
};

struct ProfileRec {
    int stage;
    hipEvent_t start, stop;
};

}  // namespace spotlight

struct spotlight_ctx {
    spotlight_config cfg;
    spotlight::Plan plan;
    hipStream_t stream;
    char* workspace;
    int max_lds;                     // bytes of LDS one workgroup may use on this device
    int n_cus;                       // compute units of this device
    int score_resident;              // score workgroups the device holds at once (0: not asked yet)
    int opt[SPOTLIGHT_OPT_COUNT];    // spotlight_set_option
    const void* big_lds_kernels[16]; // kernels whose dynamic LDS limit has been raised already
    int n_big_lds_kernels;
    // the weights the packed copy in the workspace was made from (all null: no copy)
    const void* packed_w1;
    const void* packed_b1;
    const void* packed_w2;
    // profiling
    int profiling;
    int n_rec;                       // records in use since the last read
    int n_events;                    // event pairs created so far
    spotlight::ProfileRec* recs;     // kMaxProfile entries
    double stage_ms[SPOTLIGHT_STAGE_COUNT];
    int64_t stage_launches[SPOTLIGHT_STAGE_COUNT];
};

namespace spotlight {

// One timed kernel launch.  With profiling on, the launch carries a pair of events that the
// runtime stamps when the kernel starts and when it ends (so the difference is the kernel's own
// duration, without the gaps around it); with profiling off it is a plain launch.
struct StageTimer {
    spotlight_ctx* ctx;
    ProfileRec* rec;
    StageTimer(spotlight_ctx* c, int stage);
#if defined(__HIPCC__)
    template <typename F, typename... Args>
    void launch(F kernel, const dim3& grid, const dim3& block, size_t lds, Args... args)
    {
        if (rec) {
            hipExtLaunchKernelGGL(kernel, grid, block, static_cast<uint32_t>(lds), ctx->stream, rec->start, rec->stop, 0, args...);
            ctx->n_rec += 1;
            rec = nullptr;   // one launch per record
        } else {
            hipLaunchKernelGGL(kernel, grid, block, lds, ctx->stream, args...);
        }
    }
#endif
};

// Launchers (each returns SPOTLIGHT_OK or SPOTLIGHT_ERR_*).  All pointers are device pointers.
struct HashLaunch {
    const void* x;            // vectors to hash
    int x_dtype;
    int64_t x_head_stride;    // elements between consecutive x-heads
    int64_t x_row0;           // first row inside each x-head
    int64_t n_rows;           // rows per x-head
    int n_xheads;             // B * (heads on the x side)
    int heads_per_batch;      // heads on the x side per batch entry
    int group;                // x-heads per weight head
    const void* w1;
    const void* b1;
    const void* w2;
    int w_dtype, hidden, L;
    uint32_t* codes;
    int64_t code_head_stride; // words between consecutive x-heads
    int64_t code_row0;
    uint32_t* zero;           // if set: zero[xhead * zero_words ...) is cleared by the head's first tile
    int zero_words;
    float* wnorm;             // [weight heads][L] floats of scratch for the matrix-core path, or null
    AuditRec* audit;          // set: the matrix-core path also checks every output against the chain
    const void* pack_w1;      // packed copies of the weights (see launch_pack_weights), or null
    const void* pack_out;
};
int launch_hash(spotlight_ctx* ctx, const HashLaunch& a, int stage);
// Elements per weight head of the packed copies the single-vector hash kernel can read (0: none).
void pack_sizes(int hidden, int L, size_t* w1_elems, size_t* out_elems);
// Writes the packed copies of w1 and of the output matrix (w2, or w1 itself for the linear hash).
int launch_pack_weights(spotlight_ctx* ctx, const void* w1, const void* w2, int w_dtype, void* pack_w1, void* pack_out);
// Two hash jobs; one launch when both hash a single vector per head with the same network shape.
int launch_hash_pair(spotlight_ctx* ctx, const HashLaunch& a, const HashLaunch& b, int stage);

// The first n_sink and the last n_local tokens are always selected (0, 0: none).
int launch_retrieve(spotlight_ctx* ctx, const uint32_t* codes, int64_t n_tokens, int k, int n_sink, int n_local,
                    int32_t* out_idx, uint16_t* out_dist);

int launch_attend(spotlight_ctx* ctx, const void* q, const void* K, const void* V,
                  const int32_t* idx, int k, float scale, float* out);

// Error bound of the matrix-core second hash layer per unit of ||W2[j]|| * ||h||: `hidden` roundings
// of 2^-24 in the binary32 chain, at most 2 * hidden additions in the matrix core each taken to err
// by at most one unit in the last place, and the residue of the hi/lo split (2^-18, taken as 2^-17).
inline double bulk_hash_eps(int hidden) { return 1.01 * (hidden * (0x1p-24 + 1.01 * 0x1p-22) + 0x1p-17); }

// Raises a kernel's dynamic LDS limit (once per kernel and context).
int allow_dynamic_lds(spotlight_ctx* ctx, const void* kernel, size_t bytes);

// The decode step of a short context as one kernel (step_small.hip): whether it serves this call,
// and its launch with the two hash jobs of the step.
bool step_small_applies(const spotlight_ctx* ctx, int64_t n_tokens);
int launch_step_small(spotlight_ctx* ctx, const HashLaunch& qjob, const HashLaunch& kjob, const void* q, const void* K,
                      const void* V, const uint32_t* codes, int64_t n_tokens, int k, int n_sink, int n_local,
                      float scale, int32_t* out_idx, float* out);

// Host-only argument checks of the decode step (SPOTLIGHT_OK or the error spotlight_decode_step returns).
int check_step_args(const spotlight_ctx* ctx, const void* q, const void* K, const void* V, const spotlight_hash_weights* w,
                    const uint32_t* codes, int64_t n_tokens, int32_t k, int32_t n_sink, int32_t n_local,
                    const int32_t* out_idx, const float* out);
// spotlight_decode_step on any context, also one that lives on the caller's stack.
int decode_step(spotlight_ctx* ctx, const void* q, const void* K, const void* V, const spotlight_hash_weights* w,
                uint32_t* codes, int64_t n_tokens, int32_t k, int32_t n_sink, int32_t n_local, float scale,
                int32_t* out_idx, float* out);

inline int hip_rc(hipError_t e) { return e == hipSuccess ? SPOTLIGHT_OK : SPOTLIGHT_ERR_HIP; }

}  // namespace spotlight
