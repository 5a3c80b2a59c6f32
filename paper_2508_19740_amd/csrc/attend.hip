// Gather + sparse attention (paper Sec. 3.1: Eq. 2 gather, Eq. 1 restricted to the gathered rows).
//
// The work of one query head (k scattered rows of K and of V, 256 or 512 bytes each) is split over
// ceil(k / RB) workgroups so that a few dozen heads still fill 256 compute units.  A row is read
// by LPR adjacent lanes, 16 bytes per lane, so a wavefront fetches 64 / LPR whole rows per load
// instruction.  A wavefront first issues the loads of ALL its K rows and V rows (up to 16 KB in
// flight per wave: the kernel is bound by random-row HBM latency x bandwidth, not arithmetic),
// then forms the scores, a wave-local softmax in binary32, and the weighted sum of its V rows.
// Workgroup partials (max, sum, acc[128]) go to the workspace and a second small kernel merges the
// partials of each head with the usual max-rescaling.  (Merging in the last workgroup to arrive
// needs a device-wide fence per workgroup, which on this chip writes back the L2: measured 8x
// slower than the extra launch.)
#include "attend_rows.h"

namespace spotlight {
using namespace rows;
namespace {

// RB rows per workgroup, RB / 4 per wavefront.
template <typename T, int RB>
__global__ __launch_bounds__(kThreads) void attend_kernel(
    const T* __restrict__ q, const T* __restrict__ K, const T* __restrict__ V, const int32_t* __restrict__ idx,
    float2* __restrict__ part_ml, float* __restrict__ part_acc, int k, float scale, int64_t Nmax, int Hq, int Hkv,
    int nsplit, int max_splits)
{
    constexpr int LPR = RowTraits<T>::kLanesPerRow;   // lanes per row
    constexpr int E = RowTraits<T>::kElems;           // elements per lane
    constexpr int RPI = 64 / LPR;                     // rows per load instruction
    constexpr int RPW = RB / 4;                       // rows per wave
    constexpr int ITERS = RPW / RPI;
    static_assert(RPW % RPI == 0 && RPW <= 64, "row tiling");

    __shared__ float s_m[4], s_l[4];
    __shared__ float s_acc[4][kHeadDim];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int split = blockIdx.x;
    const int64_t bh = blockIdx.y;
    const int b = static_cast<int>(bh / Hq), hq = static_cast<int>(bh % Hq);
    const int hk = hq / (Hq / Hkv);
    const int sub = lane % LPR, grp = lane / LPR;

    const T* Kh = K + (static_cast<int64_t>(b) * Hkv + hk) * Nmax * kHeadDim;
    const T* Vh = V + (static_cast<int64_t>(b) * Hkv + hk) * Nmax * kHeadDim;

    // this lane's slice of q
    float qf[E];
    {
        const uint4 u = *reinterpret_cast<const uint4*>(q + bh * kHeadDim + sub * E);
        unpack<T>(u, qf);
    }

    // Row indices of this wave, straight from the index list (the lanes of a row read the same
    // word).  A missing row (past k, or an index outside the cache) loads row 0 and is masked below,
    // so that every load is unconditional and all of them are in flight together.
    const int row0 = split * RB + wave * RPW;
    int ridx[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int j = row0 + it * RPI + grp;
        ridx[it] = idx[bh * k + (j < k ? j : 0)];
        if (j >= k || static_cast<int64_t>(ridx[it]) >= Nmax) ridx[it] = -1;
    }
    uint4 kr[ITERS], vr[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int64_t off = static_cast<int64_t>(ridx[it] >= 0 ? ridx[it] : 0) * kHeadDim + sub * E;
        kr[it] = load_row16(Kh + off);
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int64_t off = static_cast<int64_t>(ridx[it] >= 0 ? ridx[it] : 0) * kHeadDim + sub * E;
        vr[it] = load_row16(Vh + off);
    }

    // scores
    float s[ITERS];
    float m = -INFINITY;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        float kf[E];
        unpack<T>(kr[it], kf);
        float dot = 0.0f;
#pragma unroll
        for (int e = 0; e < E; ++e) dot = __builtin_fmaf(qf[e], kf[e], dot);
        dot = add_across_row<LPR>(dot);
        s[it] = ridx[it] >= 0 ? dot * scale : -INFINITY;
        m = fmaxf(m, s[it]);
    }
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) m = fmaxf(m, __shfl_xor(m, off));

    // wave-local softmax numerators and weighted V sum
    float l = 0.0f;
    float acc[E];
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.0f;
    if (m > -INFINITY) {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            const float p = ridx[it] >= 0 ? __expf(s[it] - m) : 0.0f;
            l += p;
            float vf[E];
            unpack<T>(vr[it], vf);
#pragma unroll
            for (int e = 0; e < E; ++e) acc[e] = __builtin_fmaf(p, vf[e], acc[e]);
        }
    }
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
        l += __shfl_xor(l, off);
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] += __shfl_xor(acc[e], off);
    }
    if (grp == 0) {
#pragma unroll
        for (int e = 0; e < E; ++e) s_acc[wave][sub * E + e] = acc[e];
    }
    if (lane == 0) { s_m[wave] = m; s_l[wave] = l; }
    __syncthreads();

    // merge the four waves; thread c < 128 owns output column c
    if (tid < kHeadDim) {
        const float M = fmaxf(fmaxf(s_m[0], s_m[1]), fmaxf(s_m[2], s_m[3]));
        float a = 0.0f, lsum = 0.0f;
        if (M > -INFINITY) {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float f = s_m[w] > -INFINITY ? __expf(s_m[w] - M) : 0.0f;
                a = __builtin_fmaf(f, s_acc[w][tid], a);
                lsum = __builtin_fmaf(f, s_l[w], lsum);
            }
        }
        const int64_t pi = bh * max_splits + split;
        part_acc[pi * kHeadDim + tid] = a;
        if (tid == 0) part_ml[pi] = make_float2(M, lsum);
    }
}

// Merge of the partials of a head.  A workgroup owns 32 output columns of one head; thread
// (c, part) folds the splits part, part + 8, ... of column c in split order with a running maximum
// (loads issued twelve splits at a time, ahead of the arithmetic), then the eight parts are
// combined in part order through LDS.  Latency-bound: the point is one round trip to memory.
constexpr int kMergeCols = 32, kMergeParts = kThreads / kMergeCols;

__global__ __launch_bounds__(kThreads) void merge_kernel(const float2* __restrict__ part_ml,
                                                         const float* __restrict__ part_acc,
                                                         float* __restrict__ out, int nsplit, int max_splits)
{
    constexpr int NB = 12;
    __shared__ float s_m[kMergeParts][kMergeCols], s_a[kMergeParts][kMergeCols], s_l[kMergeParts][kMergeCols];
    const int tid = threadIdx.x;
    const int64_t bh = blockIdx.y;
    const int c = tid & (kMergeCols - 1), part = tid / kMergeCols;
    const int col = blockIdx.x * kMergeCols + c;
    const float2* ml = part_ml + bh * max_splits;
    const float* pa = part_acc + bh * max_splits * kHeadDim + col;
    float m = -INFINITY, a = 0.0f, l = 0.0f;
    for (int s0 = part; s0 < nsplit; s0 += kMergeParts * NB) {
        float2 v[NB];
        float av[NB];
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int sp = s0 + kMergeParts * i;
            const int spc = sp < nsplit ? sp : s0;         // in-bounds stand-in, masked below
            v[i] = ml[spc];
            av[i] = pa[static_cast<int64_t>(spc) * kHeadDim];
            if (sp >= nsplit) v[i].x = -INFINITY;
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            if (v[i].x > -INFINITY) {
                const float mn = fmaxf(m, v[i].x);
                const float fo = __expf(m - mn), fn = __expf(v[i].x - mn);  // exp(-inf) = 0 on the first split
                a = __builtin_fmaf(a, fo, fn * av[i]);
                l = __builtin_fmaf(l, fo, fn * v[i].y);
                m = mn;
            }
        }
    }
    s_m[part][c] = m; s_a[part][c] = a; s_l[part][c] = l;
    __syncthreads();
    if (part == 0) {
        float M = -INFINITY;
#pragma unroll
        for (int p = 0; p < kMergeParts; ++p) M = fmaxf(M, s_m[p][c]);
        float at = 0.0f, lt = 0.0f;
        if (M > -INFINITY) {
#pragma unroll
            for (int p = 0; p < kMergeParts; ++p) {
                const float f = s_m[p][c] > -INFINITY ? __expf(s_m[p][c] - M) : 0.0f;
                at = __builtin_fmaf(f, s_a[p][c], at);
                lt = __builtin_fmaf(f, s_l[p][c], lt);
            }
        }
        out[bh * kHeadDim + col] = lt > 0.0f ? at / lt : 0.0f;
    }
}

template <typename T, int RB>
void launch_rb(spotlight_ctx* ctx, StageTimer& timer, const void* q, const void* K, const void* V, const int32_t* idx,
               int k, float scale, int nsplit)
{
    const Plan& p = ctx->plan;
    dim3 grid(static_cast<unsigned>(nsplit), static_cast<unsigned>(p.B * p.Hq));
    timer.launch(attend_kernel<T, RB>, grid, dim3(kThreads), 0, static_cast<const T*>(q), static_cast<const T*>(K),
                 static_cast<const T*>(V), idx, reinterpret_cast<float2*>(ctx->workspace + p.off_part_ml),
                 reinterpret_cast<float*>(ctx->workspace + p.off_part_acc), k, scale, p.Nmax, p.Hq, p.Hkv, nsplit,
                 p.max_splits);
}

template <typename T>
int launch_t(spotlight_ctx* ctx, const void* q, const void* K, const void* V, const int32_t* idx, int k,
             float scale, float* out)
{
    const Plan& p = ctx->plan;
    const int64_t heads = static_cast<int64_t>(p.B) * p.Hq;
    // the largest row tile that still gives the chip about four workgroups per compute unit
    int RB = 128;
    while (RB > kAttendMinRows && heads * ((k + RB - 1) / RB) < 1024) RB >>= 1;
    const int nsplit = (k + RB - 1) / RB;
    {
        StageTimer timer(ctx, SPOTLIGHT_STAGE_ATTEND);
        if (RB == 128) launch_rb<T, 128>(ctx, timer, q, K, V, idx, k, scale, nsplit);
        else if (RB == 64) launch_rb<T, 64>(ctx, timer, q, K, V, idx, k, scale, nsplit);
        else launch_rb<T, 32>(ctx, timer, q, K, V, idx, k, scale, nsplit);
        if (hipGetLastError() != hipSuccess) return SPOTLIGHT_ERR_HIP;
    }
    StageTimer timer(ctx, SPOTLIGHT_STAGE_MERGE);
    timer.launch(merge_kernel, dim3(kHeadDim / kMergeCols, static_cast<unsigned>(heads)), dim3(kThreads), 0,
                 reinterpret_cast<const float2*>(ctx->workspace + p.off_part_ml),
                 reinterpret_cast<const float*>(ctx->workspace + p.off_part_acc), out, nsplit, p.max_splits);
    return hip_rc(hipGetLastError());
}

}  // namespace

int launch_attend(spotlight_ctx* ctx, const void* q, const void* K, const void* V, const int32_t* idx, int k,
                  float scale, float* out)
{
    if (ctx->plan.kv_dtype == SPOTLIGHT_BF16) return launch_t<bf16_raw>(ctx, q, K, V, idx, k, scale, out);
    return launch_t<float>(ctx, q, K, V, idx, k, scale, out);
}

}  // namespace spotlight
