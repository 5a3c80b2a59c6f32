// Hamming scoring and per-head top-k (paper Sec. 3.2, Eq. 3 and the top-k that follows it).
//
// Distances are integers in 0..L, so the k nearest tokens are found by counting, not sorting:
//
//   score   one workgroup per (batch, key-value head, block of tokens) streams the packed key
//           codes once, XORs them with the G query codes of the group, popcounts, stores one small
//           integer distance per (query head, token) and counts the distances of its block in an
//           LDS histogram (replicated over lanes to keep same-address atomics apart);
//   scan    one workgroup per query head adds the block histograms, finds the threshold T with
//           count(d < T) < k <= count(d <= T) and the number r = k - count(d < T) of tokens to take
//           from the tie bucket d == T, and turns the per-block counts into an output offset and a
//           tie quota per block (prefix sums over blocks, in token order);
//   select  one workgroup per (query head, block) re-reads its distances (one or two bytes per
//           token, not the codes), keeps d < T plus the first `quota` tokens with d == T, and writes
//           the kept token indices at offset + rank.
//
// The result is exactly the first k tokens in (distance, token index) order, listed by increasing
// token index, with no atomics on the output path: identical bits on every run.
#include "internal.h"

namespace spotlight {
namespace {

constexpr int kMaxBins = 513;  // L <= 512

__device__ __forceinline__ int popc(uint32_t x) { return __builtin_popcount(x); }

// ------------------------------------------------------------------------------------ score
// LPK lanes share one key (LPK * 4 words per key) when W is a multiple of 4; otherwise one lane
// reads the W words of its key one by one (WORDS_GENERIC).
template <int W, int G, typename DistT, int R>
__global__ __launch_bounds__(kThreads) void score_kernel(
    const uint32_t* __restrict__ codes, const uint32_t* __restrict__ qcode, DistT* __restrict__ dist,
    uint32_t* __restrict__ blockhist, int64_t n_tokens, int64_t Nmax, int64_t dist_stride, int Hkv,
    int tokens_per_block, int max_blocks)
{
    constexpr int L = W * 32;
    constexpr int BINS = L + 1;
    __shared__ uint32_t hist[G * BINS * R];

    const int tid = threadIdx.x;
    const int bk = blockIdx.y;               // b * Hkv + hk
    const int blk = blockIdx.x;
    const int Hq = Hkv * G;
    const int b = bk / Hkv, hk = bk % Hkv;
    const int64_t bh0 = static_cast<int64_t>(b) * Hq + hk * G;  // first query head of the group

    for (int i = tid; i < G * BINS * R; i += kThreads) hist[i] = 0;

    // query codes of the group: uniform over the workgroup
    uint32_t qc[G][W];
#pragma unroll
    for (int g = 0; g < G; ++g)
#pragma unroll
        for (int w = 0; w < W; ++w) qc[g][w] = qcode[(bh0 + g) * W + w];
    __syncthreads();

    const int64_t t_begin = static_cast<int64_t>(blk) * tokens_per_block;
    const int64_t t_end = min(n_tokens, t_begin + tokens_per_block);
    const uint32_t* cbase = codes + static_cast<int64_t>(bk) * Nmax * W;
    const int rep = tid & (R - 1);

    constexpr int U = 4;  // keys in flight per lane
    for (int64_t t0 = t_begin + tid; t0 < t_end; t0 += U * kThreads) {
        uint32_t kw[U][W];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t t = t0 + u * kThreads;
            if (t < t_end) {
                if constexpr (W % 4 == 0) {
#pragma unroll
                    for (int w4 = 0; w4 < W / 4; ++w4) {
                        const uint4 v = *reinterpret_cast<const uint4*>(cbase + t * W + w4 * 4);
                        kw[u][w4 * 4 + 0] = v.x; kw[u][w4 * 4 + 1] = v.y;
                        kw[u][w4 * 4 + 2] = v.z; kw[u][w4 * 4 + 3] = v.w;
                    }
                } else {
#pragma unroll
                    for (int w = 0; w < W; ++w) kw[u][w] = cbase[t * W + w];
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t t = t0 + u * kThreads;
            if (t < t_end) {
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    int d = 0;
#pragma unroll
                    for (int w = 0; w < W; ++w) d += popc(kw[u][w] ^ qc[g][w]);
                    dist[(bh0 + g) * dist_stride + t] = static_cast<DistT>(d);
                    atomicAdd(&hist[(g * BINS + d) * R + rep], 1u);
                }
            }
        }
    }
    __syncthreads();

    // fold the replicas and publish this block's histogram
    for (int i = tid; i < G * BINS; i += kThreads) {
        uint32_t s = 0;
#pragma unroll
        for (int r = 0; r < R; ++r) s += hist[i * R + r];
        const int g = i / BINS, bin = i % BINS;
        blockhist[((bh0 + g) * max_blocks + blk) * BINS + bin] = s;
    }
}

// ------------------------------------------------------------------------------------ scan
// blockinfo[bh][blk] = {output offset of the block, tie quota of the block}; headinfo[bh] = {T, r}.
__global__ __launch_bounds__(kThreads) void scan_kernel(
    const uint32_t* __restrict__ blockhist, uint2* __restrict__ blockinfo, uint2* __restrict__ headinfo,
    int bins, int nblk, int max_blocks, int k)
{
    __shared__ uint32_t ghist[kMaxBins];
    __shared__ uint32_t s_T, s_r;
    __shared__ uint32_t wave_lt[kThreads / 64], wave_eq[kThreads / 64];
    __shared__ uint32_t carry_lt, carry_eq;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bh = blockIdx.x;
    const uint32_t* bhist = blockhist + bh * max_blocks * bins;

    for (int bin = tid; bin < bins; bin += kThreads) {
        uint32_t s = 0;
        for (int blk = 0; blk < nblk; ++blk) s += bhist[static_cast<int64_t>(blk) * bins + bin];
        ghist[bin] = s;
    }
    if (tid == 0) { carry_lt = 0; carry_eq = 0; }
    __syncthreads();
    if (tid == 0) {
        uint32_t below = 0;
        int T = 0;
        for (; T < bins - 1; ++T) {
            if (below + ghist[T] >= static_cast<uint32_t>(k)) break;
            below += ghist[T];
        }
        s_T = T;
        s_r = static_cast<uint32_t>(k) - below;  // 1 <= r <= ghist[T]
        headinfo[bh] = make_uint2(static_cast<uint32_t>(T), s_r);
    }
    __syncthreads();
    const int T = s_T;
    const uint32_t r = s_r;

    // blocks in chunks of 256, running prefix over (lt, eq) in block order
    for (int base = 0; base < nblk; base += kThreads) {
        const int blk = base + tid;
        uint32_t lt = 0, eq = 0;
        if (blk < nblk) {
            const uint32_t* h = bhist + static_cast<int64_t>(blk) * bins;
            for (int bin = 0; bin < T; ++bin) lt += h[bin];
            eq = h[T];
        }
        // inclusive scan inside the wave
        uint32_t slt = lt, seq = eq;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const uint32_t a = __shfl_up(slt, off), c = __shfl_up(seq, off);
            if (lane >= off) { slt += a; seq += c; }
        }
        if (lane == 63) { wave_lt[wave] = slt; wave_eq[wave] = seq; }
        __syncthreads();
        uint32_t plt = carry_lt, peq = carry_eq;
        for (int w = 0; w < wave; ++w) { plt += wave_lt[w]; peq += wave_eq[w]; }
        const uint32_t lt_before = plt + slt - lt;   // exclusive prefixes in block order
        const uint32_t eq_before = peq + seq - eq;
        if (blk < nblk) {
            const uint32_t taken_before = eq_before < r ? eq_before : r;
            const uint32_t quota = r > eq_before ? min(r - eq_before, eq) : 0u;
            blockinfo[bh * max_blocks + blk] = make_uint2(lt_before + taken_before, quota);
        }
        __syncthreads();
        if (tid == kThreads - 1) { carry_lt = plt + slt; carry_eq = peq + seq; }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------ select
// One thread owns 16 consecutive tokens; the workgroup owns tokens_per_block (<= 4096) tokens.
template <typename DistT>
__global__ __launch_bounds__(kThreads) void select_kernel(
    const DistT* __restrict__ dist, const uint2* __restrict__ blockinfo, const uint2* __restrict__ headinfo,
    int32_t* __restrict__ out_idx, int64_t n_tokens, int64_t dist_stride, int tokens_per_block, int max_blocks, int k)
{
    __shared__ uint32_t wave_a[kThreads / 64], wave_b[kThreads / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bh = blockIdx.y;
    const int blk = blockIdx.x;
    const uint2 info = blockinfo[bh * max_blocks + blk];
    const uint32_t T = headinfo[bh].x;
    const uint32_t quota = info.y;

    const int64_t t_begin = static_cast<int64_t>(blk) * tokens_per_block;
    const int64_t t_end = min(n_tokens, t_begin + tokens_per_block);
    const int64_t t0 = t_begin + static_cast<int64_t>(tid) * 16;
    const DistT* dp = dist + bh * dist_stride;

    uint32_t d[16];
    if (t0 + 16 <= t_end && tid * 16 < tokens_per_block) {
        if constexpr (sizeof(DistT) == 1) {
            const uint4 v = *reinterpret_cast<const uint4*>(dp + t0);
            const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int i = 0; i < 16; ++i) d[i] = (w[i >> 2] >> ((i & 3) * 8)) & 0xffu;
        } else {
            const uint4 v0 = reinterpret_cast<const uint4*>(dp + t0)[0];
            const uint4 v1 = reinterpret_cast<const uint4*>(dp + t0)[1];
            const uint32_t w[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
            for (int i = 0; i < 16; ++i) d[i] = (w[i >> 1] >> ((i & 1) * 16)) & 0xffffu;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t t = t0 + i;
            d[i] = (t < t_end && tid * 16 < tokens_per_block) ? static_cast<uint32_t>(dp[t]) : 0xffffffffu;
        }
    }
    uint32_t lt = 0, eq = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) { lt += d[i] < T; eq += d[i] == T; }

    // exclusive prefix of eq over threads (token order)
    uint32_t seq = eq;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t a = __shfl_up(seq, off);
        if (lane >= off) seq += a;
    }
    if (lane == 63) wave_a[wave] = seq;
    __syncthreads();
    uint32_t eq_before = seq - eq;
    for (int w = 0; w < wave; ++w) eq_before += wave_a[w];
    const uint32_t take_eq = quota > eq_before ? min(quota - eq_before, eq) : 0u;
    const uint32_t cnt = lt + take_eq;

    uint32_t scnt = cnt;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t a = __shfl_up(scnt, off);
        if (lane >= off) scnt += a;
    }
    if (lane == 63) wave_b[wave] = scnt;
    __syncthreads();
    uint32_t pos = info.x + scnt - cnt;
    for (int w = 0; w < wave; ++w) pos += wave_b[w];

    if (cnt) {
        int32_t* op = out_idx + bh * k;
        uint32_t eq_left = take_eq;
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            bool keep = d[i] < T;
            if (d[i] == T && eq_left) { keep = true; --eq_left; }
            if (keep && pos < static_cast<uint32_t>(k)) { op[pos] = static_cast<int32_t>(t0 + i); ++pos; }
        }
    }
}

template <typename DistT>
__global__ __launch_bounds__(kThreads) void dump_dist_kernel(const DistT* __restrict__ dist, uint16_t* __restrict__ out,
                                                             int64_t n_tokens, int64_t dist_stride)
{
    const int64_t bh = blockIdx.y;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (t < n_tokens) out[bh * n_tokens + t] = static_cast<uint16_t>(dist[bh * dist_stride + t]);
}

// ------------------------------------------------------------------------------------ dispatch
template <int W, int G, typename DistT>
void launch_score_wg(spotlight_ctx* ctx, const uint32_t* codes, int64_t n_tokens, int nblk)
{
    const Plan& p = ctx->plan;
    constexpr int BINS = W * 32 + 1;
    // replicas: as many as fit in 40 KB of LDS, at most 32
    constexpr int kCap = 40960;
    constexpr int R = (G * BINS * 32 * 4 <= kCap) ? 32 : (G * BINS * 16 * 4 <= kCap) ? 16
                    : (G * BINS * 8 * 4 <= kCap) ? 8 : (G * BINS * 4 * 4 <= kCap) ? 4
                    : (G * BINS * 2 * 4 <= kCap) ? 2 : 1;
    dim3 grid(static_cast<unsigned>(nblk), static_cast<unsigned>(p.B * p.Hkv));
    hipLaunchKernelGGL((score_kernel<W, G, DistT, R>), grid, dim3(kThreads), 0, ctx->stream, codes,
                       reinterpret_cast<const uint32_t*>(ctx->workspace + p.off_qcode),
                       reinterpret_cast<DistT*>(ctx->workspace + p.off_dist),
                       reinterpret_cast<uint32_t*>(ctx->workspace + p.off_blockhist), n_tokens, p.Nmax,
                       p.dist_stride, p.Hkv, p.tokens_per_block, p.max_blocks);
}

template <int W, int G>
void launch_score_w(spotlight_ctx* ctx, const uint32_t* codes, int64_t n_tokens, int nblk)
{
    if constexpr (W * 32 < 256) launch_score_wg<W, G, uint8_t>(ctx, codes, n_tokens, nblk);
    else launch_score_wg<W, G, uint16_t>(ctx, codes, n_tokens, nblk);
}

template <int W>
int launch_score_g(spotlight_ctx* ctx, const uint32_t* codes, int64_t n_tokens, int nblk)
{
    switch (ctx->plan.G) {
    case 1: launch_score_w<W, 1>(ctx, codes, n_tokens, nblk); return SPOTLIGHT_OK;
    case 2: launch_score_w<W, 2>(ctx, codes, n_tokens, nblk); return SPOTLIGHT_OK;
    case 4: launch_score_w<W, 4>(ctx, codes, n_tokens, nblk); return SPOTLIGHT_OK;
    case 8: launch_score_w<W, 8>(ctx, codes, n_tokens, nblk); return SPOTLIGHT_OK;
    default: return SPOTLIGHT_ERR_UNSUPPORTED;
    }
}

int launch_score(spotlight_ctx* ctx, const uint32_t* codes, int64_t n_tokens, int nblk)
{
    switch (ctx->plan.W) {
    case 1: return launch_score_g<1>(ctx, codes, n_tokens, nblk);
    case 2: return launch_score_g<2>(ctx, codes, n_tokens, nblk);
    case 3: return launch_score_g<3>(ctx, codes, n_tokens, nblk);
    case 4: return launch_score_g<4>(ctx, codes, n_tokens, nblk);
    case 5: return launch_score_g<5>(ctx, codes, n_tokens, nblk);
    case 6: return launch_score_g<6>(ctx, codes, n_tokens, nblk);
    case 7: return launch_score_g<7>(ctx, codes, n_tokens, nblk);
    case 8: return launch_score_g<8>(ctx, codes, n_tokens, nblk);
    case 9: return launch_score_g<9>(ctx, codes, n_tokens, nblk);
    case 10: return launch_score_g<10>(ctx, codes, n_tokens, nblk);
    case 11: return launch_score_g<11>(ctx, codes, n_tokens, nblk);
    case 12: return launch_score_g<12>(ctx, codes, n_tokens, nblk);
    case 13: return launch_score_g<13>(ctx, codes, n_tokens, nblk);
    case 14: return launch_score_g<14>(ctx, codes, n_tokens, nblk);
    case 15: return launch_score_g<15>(ctx, codes, n_tokens, nblk);
    case 16: return launch_score_g<16>(ctx, codes, n_tokens, nblk);
    default: return SPOTLIGHT_ERR_UNSUPPORTED;
    }
}

}  // namespace

int launch_retrieve(spotlight_ctx* ctx, const uint32_t* codes, int64_t n_tokens, int k,
                    int32_t* out_idx, uint16_t* out_dist)
{
    const Plan& p = ctx->plan;
    const int nblk = static_cast<int>((n_tokens + p.tokens_per_block - 1) / p.tokens_per_block);
    const int BH = p.B * p.Hq;
    uint2* blockinfo = reinterpret_cast<uint2*>(ctx->workspace + p.off_blockinfo);
    uint2* headinfo = reinterpret_cast<uint2*>(ctx->workspace + p.off_headinfo);
    {
        StageTimer timer(ctx, SPOTLIGHT_STAGE_SCORE);
        const int rc = launch_score(ctx, codes, n_tokens, nblk);
        if (rc != SPOTLIGHT_OK) return rc;
        if (hipGetLastError() != hipSuccess) return SPOTLIGHT_ERR_HIP;
    }
    {
        StageTimer timer(ctx, SPOTLIGHT_STAGE_SCAN);
        hipLaunchKernelGGL(scan_kernel, dim3(BH), dim3(kThreads), 0, ctx->stream,
                           reinterpret_cast<const uint32_t*>(ctx->workspace + p.off_blockhist), blockinfo, headinfo,
                           p.L + 1, nblk, p.max_blocks, k);
        if (hipGetLastError() != hipSuccess) return SPOTLIGHT_ERR_HIP;
    }
    {
        StageTimer timer(ctx, SPOTLIGHT_STAGE_SELECT);
        dim3 grid(static_cast<unsigned>(nblk), static_cast<unsigned>(BH));
        if (p.dist_bytes == 1)
            hipLaunchKernelGGL(select_kernel<uint8_t>, grid, dim3(kThreads), 0, ctx->stream,
                               reinterpret_cast<const uint8_t*>(ctx->workspace + p.off_dist), blockinfo, headinfo,
                               out_idx, n_tokens, p.dist_stride, p.tokens_per_block, p.max_blocks, k);
        else
            hipLaunchKernelGGL(select_kernel<uint16_t>, grid, dim3(kThreads), 0, ctx->stream,
                               reinterpret_cast<const uint16_t*>(ctx->workspace + p.off_dist), blockinfo, headinfo,
                               out_idx, n_tokens, p.dist_stride, p.tokens_per_block, p.max_blocks, k);
        if (hipGetLastError() != hipSuccess) return SPOTLIGHT_ERR_HIP;
    }
    if (out_dist) {
        dim3 grid(static_cast<unsigned>((n_tokens + kThreads - 1) / kThreads), static_cast<unsigned>(BH));
        if (p.dist_bytes == 1)
            hipLaunchKernelGGL(dump_dist_kernel<uint8_t>, grid, dim3(kThreads), 0, ctx->stream,
                               reinterpret_cast<const uint8_t*>(ctx->workspace + p.off_dist), out_dist, n_tokens, p.dist_stride);
        else
            hipLaunchKernelGGL(dump_dist_kernel<uint16_t>, grid, dim3(kThreads), 0, ctx->stream,
                               reinterpret_cast<const uint16_t*>(ctx->workspace + p.off_dist), out_dist, n_tokens, p.dist_stride);
        if (hipGetLastError() != hipSuccess) return SPOTLIGHT_ERR_HIP;
    }
    return SPOTLIGHT_OK;
}

}  // namespace spotlight
