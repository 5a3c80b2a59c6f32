// The decode step of a SHORT context as one kernel launch (paper Sec. 3.1-3.2: Eq. 5-6 hash, Eq. 3
// Hamming score, top-k, Eq. 2 gather, Eq. 1 attention over the gathered rows).
//
// With a few tens of thousands of cached tokens per head, the five kernels of the general step
// (hash, score, select, attend, merge) take 4 - 7 us each and almost all of that is launch and
// drain.  The general path needs them because a head's tokens are spread over many workgroups and
// the top-k threshold depends on every one of them.  Here ONE workgroup of 512 threads owns a
// (batch, key-value head) outright, so every dependency is a workgroup barrier:
//
//   hash     the appended key and the G queries of the group, two vectors at a time (256 threads
//            each, the same code as the stand-alone kernel: hash_vec.h); codes to LDS and to memory
//   count    every cached code of the head is read once, XOR + popcount against the G query codes,
//            distances counted in an LDS histogram (bin 0: forced tokens, bin d + 1: distance d)
//   bound    per query head, the bin T with count(bin < T) < k <= count(bin <= T), r = k - count(bin < T)
//   select   per query head: every token's bin comes back from an LDS copy made while counting (or,
//            if that does not fit, the codes are read again: they are in the cache now), tokens with
//            bin < T and bin == T are marked in two LDS bitmaps by wave ballots, the ties trimmed to
//            the first r in token order, the indices written in increasing order
//   attend   the selected rows gathered by the eight wavefronts (online softmax per wavefront over
//            batches of rows, merged through LDS), output written
//
// Same results as the general path: codes and index arrays bit for bit (the selection is the first
// k tokens in (bin, token) order either way); the attention output differs in summation order only.
//
// Measured, it does NOT pay on this chip beyond a few thousand tokens per head, which is why the path
// is an option that is off by default: one compute unit streams about 85 GB/s, so a head of 32768
// tokens x 16 bytes costs 6 us per pass where the general path spreads it over eight compute units.
// Batch 1, 32 heads, top-k 2 %: 32768 tokens 46 us as one launch (dispatch 4, hash 8, count 14, bound
// + select 9, attend 10) against 27 us as five; 16384 tokens 31 against 25; 8192 tokens 25.0 against
// 24.1; 4096 tokens 22.3 against 23.7; 2048 tokens 21.0 against 23.8.
#pragma once
#include <type_traits>

#include "attend_rows.h"
#include "hash_vec.h"

namespace spotlight {
namespace small {

constexpr int kSmThreads = 512;       // eight wavefronts: the hash keeps whole weight rows in registers (up to 256 per lane)
constexpr int kSmWaves = kSmThreads / 64;
constexpr int kSmRep = 4;             // histogram replicas
constexpr int kSmMaxTokens = 65536;   // four bitmap words per thread at most
constexpr int kSmMaxChw = kSmMaxTokens / (32 * kSmThreads);
constexpr int kSmMaxHidden = 1024;
constexpr int64_t kSmMaxCodeBytes = 32ll << 20;   // beyond this the general path's many workgroups per head win

struct SmallArgs {
    hashdev::HashArgs job[2];   // [0] the queries, [1] the appended key
    const void* q;
    const void* K;
    const void* V;
    const uint32_t* codes;
    int32_t* out_idx;
    float* out;
    int64_t n_tokens, Nmax, n_sink, local_begin;   // token t is forced iff t < n_sink or t >= local_begin
    int k, Hq, Hkv, G;
    int act_dim;      // floats of hidden activations per hashing group
    int chw;          // bitmap words per thread (tokens / 16384, rounded up)
    int n_pad;        // tokens rounded up to a multiple of the workgroup size
    int cache_bins;   // the histogram bin of every (query head, token) is kept in LDS between the two passes
    int packed;
    float scale;
};

template <int W>
__device__ __forceinline__ void load_code(const uint32_t* __restrict__ p, uint32_t (&kw)[W])
{
    if constexpr (W % 4 == 0) {
#pragma unroll
        for (int w4 = 0; w4 < W / 4; ++w4) {
            const uint4 v = reinterpret_cast<const uint4*>(p)[w4];
            kw[w4 * 4 + 0] = v.x; kw[w4 * 4 + 1] = v.y; kw[w4 * 4 + 2] = v.z; kw[w4 * 4 + 3] = v.w;
        }
    } else if constexpr (W % 2 == 0) {
#pragma unroll
        for (int w2 = 0; w2 < W / 2; ++w2) {
            const uint2 v = reinterpret_cast<const uint2*>(p)[w2];
            kw[w2 * 2 + 0] = v.x; kw[w2 * 2 + 1] = v.y;
        }
    } else {
#pragma unroll
        for (int w = 0; w < W; ++w) kw[w] = p[w];
    }
}

// Exclusive prefix sum of x over the workgroup (thread order).  Two barriers; wsum has one word per wavefront.
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t x, uint32_t* wsum, int lane, int wave)
{
    const uint32_t incl = wave_inclusive_scan(x);
    if (lane == 63) wsum[wave] = incl;
    __syncthreads();
    uint32_t base = 0;
#pragma unroll
    for (int w = 0; w < kSmWaves; ++w) base += w < wave ? wsum[w] : 0u;
    __syncthreads();   // wsum may be reused
    return base + incl - x;
}

template <bool BF16, bool WBF16, int W>
__global__ __launch_bounds__(kSmThreads) void step_small_kernel(SmallArgs a)
{
    using XT = typename std::conditional<BF16, hashdev::bf16_raw, float>::type;   // element type for the hash
    using WT = typename std::conditional<WBF16, hashdev::bf16_raw, float>::type;  // element type of the hash weights
    using RT = typename std::conditional<BF16, rows::bf16_raw, float>::type;      // element type for the gather
    constexpr int L = W * 32;
    constexpr int BINS = L + 2;
    constexpr int CH = (BINS + 63) / 64;
    constexpr int R = kSmRep;
    constexpr int U = 8;   // keys a thread has in flight

    extern __shared__ __align__(16) uint32_t lds[];
    const int G = a.G;
    constexpr int NGRP = kSmThreads / 256;                             // vectors hashed side by side
    float* act = reinterpret_cast<float*>(lds);                        // [NGRP][act_dim]
    uint32_t* qcode = lds + NGRP * a.act_dim;                          // [G][W]
    uint32_t* newkey = qcode + G * W;                                  // [W]
    uint32_t* sT = newkey + W;                                         // [G]
    uint32_t* sR = sT + G;                                             // [G]
    uint32_t* wsum = sR + G;                                           // [waves]
    uint32_t* hist = wsum + kSmWaves;                                  // [G][BINS][R]
    uint32_t* lt_bits = hist + G * BINS * R;                           // [threads * chw]
    uint32_t* eq_bits = lt_bits + kSmThreads * a.chw;                  // [threads * chw]
    float* s_m = reinterpret_cast<float*>(eq_bits + kSmThreads * a.chw);   // [waves]
    float* s_l = s_m + kSmWaves;                                       // [waves]
    float* s_acc = s_l + kSmWaves;                                     // [waves][128]
    uint16_t* bin_cache = reinterpret_cast<uint16_t*>(s_acc + kSmWaves * kHeadDim);   // [G][n_pad], if cache_bins

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = tid >> 8, gtid = tid & 255;
    const int bk = blockIdx.x, b = bk / a.Hkv, hk = bk % a.Hkv;
    const int n = static_cast<int>(a.n_tokens);

    // ---------------------------------------------------------------- hash: G queries and the new key
    for (int v0 = 0; v0 <= G; v0 += NGRP) {
        // everything about the vector a group hashes is uniform over its wavefronts: kept in scalars
        const int v = v0 + __builtin_amdgcn_readfirstlane(grp);
        const bool live = v <= G;
        const int is_key = v == G ? 1 : 0;
        const hashdev::HashArgs& job = a.job[is_key];
        const int xhead = !live ? 0 : (is_key ? bk : b * a.Hq + hk * G + v);
        uint32_t* code_out = is_key ? newkey : qcode + (live ? v : 0) * W;
        float* my_act = act + __builtin_amdgcn_readfirstlane(grp) * a.act_dim;
        if (a.packed) hashdev::hash_one_vector<XT, WT, true>(job, xhead, live, gtid, my_act, code_out);
        else hashdev::hash_one_vector<XT, WT, false>(job, xhead, live, gtid, my_act, code_out);
        __syncthreads();   // the activations are free for the next vectors; the codes are in LDS
    }

    // ---------------------------------------------------------------- count
    for (int i = tid; i < G * BINS * R; i += kSmThreads) hist[i] = 0;
    __syncthreads();
    const uint32_t* hc = a.codes + static_cast<int64_t>(bk) * a.Nmax * W;
    const int rep = tid & (R - 1);
    // distance of one key to query head g
    auto distance = [&](const uint32_t (&kw)[W], int g) {
        uint32_t d = 0;
#pragma unroll
        for (int w = 0; w < W; ++w) d += static_cast<uint32_t>(__builtin_popcount(kw[w] ^ qcode[g * W + w]));
        return d;
    };
    // (The code of the key appended by this step was stored to memory by this workgroup before the
    // barrier above, so the loads below see it.)
    const int sink_end = static_cast<int>(min(a.n_sink, a.n_tokens));          // forced: t < sink_end or t >= local_begin
    const int local_begin = static_cast<int>(max(static_cast<int64_t>(0), a.local_begin));
    for (int t0 = tid; t0 < n; t0 += kSmThreads * U) {
        uint32_t kw[U][W];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * kSmThreads;
            if (t < n) load_code<W>(hc + static_cast<int64_t>(t) * W, kw[u]);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int t = t0 + u * kSmThreads;
            if (t < n) {
                const bool forced = t < sink_end || t >= local_begin;
                for (int g = 0; g < G; ++g) {
                    const uint32_t bin = forced ? 0u : 1u + distance(kw[u], g);
                    atomicAdd(&hist[(g * BINS + bin) * R + rep], 1u);
                    if (a.cache_bins) bin_cache[g * a.n_pad + t] = static_cast<uint16_t>(bin);
                }
            }
        }
    }
    __syncthreads();

    // ---------------------------------------------------------------- bound: one wavefront per query head
    for (int g = wave; g < G; g += kSmWaves) {
        uint32_t v[CH];
        uint32_t tot = 0;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int bin = lane * CH + c;
            uint32_t s = 0;
            if (bin < BINS) {
#pragma unroll
                for (int r = 0; r < R; ++r) s += hist[(g * BINS + bin) * R + r];
            }
            tot += s;
            v[c] = tot;
        }
        const uint32_t before = wave_inclusive_scan(tot) - tot;
        uint32_t prev = before;
#pragma unroll
        for (int c = 0; c < CH; ++c) {
            const int bin = lane * CH + c;
            const uint32_t cv = before + v[c];
            // exactly one bin qualifies (k <= n_tokens); the last bin also takes "never reaches k"
            if (bin < BINS && (cv >= static_cast<uint32_t>(a.k) || bin == BINS - 1) && prev < static_cast<uint32_t>(a.k)) {
                sT[g] = static_cast<uint32_t>(bin);
                sR[g] = static_cast<uint32_t>(a.k) - prev;
            }
            prev = cv;
        }
    }
    __syncthreads();

    // ---------------------------------------------------------------- per query head: select, then attend
    constexpr int LPR = rows::RowTraits<RT>::kLanesPerRow;   // lanes per row
    constexpr int E = rows::RowTraits<RT>::kElems;           // elements per lane
    constexpr int RPI = 64 / LPR;                            // rows per load instruction
    constexpr int ITERS = 8;                                 // load instructions in flight per wavefront (K, then V)
    constexpr int RPB = RPI * ITERS;                         // rows per wavefront and batch
    const int sub = lane % LPR, rgrp = lane / LPR;
    const RT* Kh = static_cast<const RT*>(a.K) + static_cast<int64_t>(bk) * a.Nmax * kHeadDim;
    const RT* Vh = static_cast<const RT*>(a.V) + static_cast<int64_t>(bk) * a.Nmax * kHeadDim;
    const int n_iter = a.chw * 32;   // passes of one token per thread that cover the bitmaps

    for (int g = 0; g < G; ++g) {
        const uint32_t T = sT[g], r = sR[g];
        const int64_t bh = static_cast<int64_t>(b) * a.Hq + hk * G + g;

        // bitmaps: wavefront w of pass `it` covers tokens it * threads + 64 w ...: two words of each bitmap
        for (int it0 = 0; it0 < n_iter; it0 += U) {
            uint32_t kw[U][W];
            if (!a.cache_bins) {
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int t = (it0 + u) * kSmThreads + tid;
                    if (it0 + u < n_iter && t < n) load_code<W>(hc + static_cast<int64_t>(t) * W, kw[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (it0 + u >= n_iter) break;   // uniform
                const int t = (it0 + u) * kSmThreads + tid;
                uint32_t bin = 0xffffffffu;
                if (t < n) {
                    if (a.cache_bins) {
                        bin = bin_cache[g * a.n_pad + t];
                    } else {
                        const bool forced = t < sink_end || t >= local_begin;
                        bin = forced ? 0u : 1u + distance(kw[u], g);
                    }
                }
                const unsigned long long mlt = __ballot(bin < T);
                const unsigned long long meq = __ballot(bin == T);
                if (lane == 0) {
                    const int word = (it0 + u) * (kSmThreads / 32) + 2 * wave;
                    lt_bits[word] = static_cast<uint32_t>(mlt);
                    lt_bits[word + 1] = static_cast<uint32_t>(mlt >> 32);
                    eq_bits[word] = static_cast<uint32_t>(meq);
                    eq_bits[word + 1] = static_cast<uint32_t>(meq >> 32);
                }
            }
        }
        __syncthreads();

        // thread j owns the chw bitmap words from chw j on, i.e. tokens 32 chw j ...; ties go to the lower token index
        uint32_t lw[kSmMaxChw], ew[kSmMaxChw];
        uint32_t ecount = 0;
#pragma unroll
        for (int i = 0; i < kSmMaxChw; ++i) {
            lw[i] = i < a.chw ? lt_bits[tid * a.chw + i] : 0u;
            ew[i] = i < a.chw ? eq_bits[tid * a.chw + i] : 0u;
            ecount += static_cast<uint32_t>(__builtin_popcount(ew[i]));
        }
        const uint32_t eq_before = block_exclusive_scan(ecount, wsum, lane, wave);
        const uint32_t gone = eq_before < r ? eq_before : r;                  // quota used by earlier threads
        uint32_t left = (r - gone) < ecount ? (r - gone) : ecount;            // ties this thread takes: its first ones
        uint32_t cnt = 0;
#pragma unroll
        for (int i = 0; i < kSmMaxChw; ++i) {
            while (static_cast<uint32_t>(__builtin_popcount(ew[i])) > left) ew[i] &= ~(0x80000000u >> __builtin_clz(ew[i]));
            left -= static_cast<uint32_t>(__builtin_popcount(ew[i]));
            lw[i] |= ew[i];
            cnt += static_cast<uint32_t>(__builtin_popcount(lw[i]));
        }
        uint32_t pos = block_exclusive_scan(cnt, wsum, lane, wave);
        int32_t* op = a.out_idx + bh * a.k;
#pragma unroll
        for (int i = 0; i < kSmMaxChw; ++i) {
            const int32_t tok0 = (tid * a.chw + i) * 32;
            uint32_t sel = lw[i];
            while (sel) {
                const int bit = __builtin_ctz(sel);
                sel &= sel - 1;
                if (pos < static_cast<uint32_t>(a.k)) op[pos] = tok0 + bit;
                ++pos;
            }
        }
        __syncthreads();   // the index list of this head is complete (and the bitmaps are free)

        // attention over the k listed rows: wavefront w takes rows [(waves i + w) RPB, +RPB) for i = 0, 1, ...
        float qf[E];
        {
            const uint4 u = *reinterpret_cast<const uint4*>(static_cast<const RT*>(a.q) + bh * kHeadDim + sub * E);
            rows::unpack<RT>(u, qf);
        }
        float m_run = -INFINITY, l_run = 0.0f;
        float acc[E];
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = 0.0f;
        for (int row0 = wave * RPB; row0 < a.k; row0 += kSmWaves * RPB) {
            int ridx[ITERS];
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                const int j = row0 + it * RPI + rgrp;
                ridx[it] = op[j < a.k ? j : 0];
                if (j >= a.k || static_cast<int64_t>(ridx[it]) >= a.Nmax) ridx[it] = -1;
            }
            uint4 kr[ITERS], vr[ITERS];
#pragma unroll
            for (int it = 0; it < ITERS; ++it)
                kr[it] = rows::load_row16(Kh + static_cast<int64_t>(ridx[it] >= 0 ? ridx[it] : 0) * kHeadDim + sub * E);
#pragma unroll
            for (int it = 0; it < ITERS; ++it)
                vr[it] = rows::load_row16(Vh + static_cast<int64_t>(ridx[it] >= 0 ? ridx[it] : 0) * kHeadDim + sub * E);
            float s[ITERS];
            float mb = -INFINITY;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                float kf[E];
                rows::unpack<RT>(kr[it], kf);
                float dot = 0.0f;
#pragma unroll
                for (int e = 0; e < E; ++e) dot = __builtin_fmaf(qf[e], kf[e], dot);
                dot = rows::add_across_row<LPR>(dot);
                s[it] = ridx[it] >= 0 ? dot * a.scale : -INFINITY;
                mb = fmaxf(mb, s[it]);
            }
#pragma unroll
            for (int off = LPR; off < 64; off <<= 1) mb = fmaxf(mb, __shfl_xor(mb, off));
            if (mb > -INFINITY) {   // uniform over the wavefront
                const float m_new = fmaxf(m_run, mb);
                const float keep = m_run > -INFINITY ? __expf(m_run - m_new) : 0.0f;
                l_run *= keep;
#pragma unroll
                for (int e = 0; e < E; ++e) acc[e] *= keep;
#pragma unroll
                for (int it = 0; it < ITERS; ++it) {
                    const float p = ridx[it] >= 0 ? __expf(s[it] - m_new) : 0.0f;
                    l_run += p;
                    float vf[E];
                    rows::unpack<RT>(vr[it], vf);
#pragma unroll
                    for (int e = 0; e < E; ++e) acc[e] = __builtin_fmaf(p, vf[e], acc[e]);
                }
                m_run = m_new;
            }
        }
#pragma unroll
        for (int off = LPR; off < 64; off <<= 1) {
            l_run += __shfl_xor(l_run, off);
#pragma unroll
            for (int e = 0; e < E; ++e) acc[e] += __shfl_xor(acc[e], off);
        }
        if (rgrp == 0) {
#pragma unroll
            for (int e = 0; e < E; ++e) s_acc[wave * kHeadDim + sub * E + e] = acc[e];
        }
        if (lane == 0) { s_m[wave] = m_run; s_l[wave] = l_run; }
        __syncthreads();
        if (tid < kHeadDim) {
            float M = -INFINITY;
#pragma unroll
            for (int w = 0; w < kSmWaves; ++w) M = fmaxf(M, s_m[w]);
            float at = 0.0f, lt = 0.0f;
            if (M > -INFINITY) {
#pragma unroll
                for (int w = 0; w < kSmWaves; ++w) {
                    const float f = s_m[w] > -INFINITY ? __expf(s_m[w] - M) : 0.0f;
                    at = __builtin_fmaf(f, s_acc[w * kHeadDim + tid], at);
                    lt = __builtin_fmaf(f, s_l[w], lt);
                }
            }
            a.out[bh * kHeadDim + tid] = lt > 0.0f ? at / lt : 0.0f;
        }
        __syncthreads();   // LDS is reused by the next head
    }
}

inline int small_chw(int64_t n_tokens) { return static_cast<int>((n_tokens + 32 * kSmThreads - 1) / (32 * kSmThreads)); }

inline int small_n_pad(int64_t n_tokens) { return static_cast<int>((n_tokens + kSmThreads - 1) / kSmThreads * kSmThreads); }

// LDS of one workgroup without / with the cache of every token's histogram bin.
inline size_t small_lds_bytes(const Plan& p, int64_t n_tokens, bool cache_bins)
{
    const int act_dim = p.hidden > 0 ? p.hidden : kHeadDim;
    const int chw = small_chw(n_tokens);
    const size_t words = (kSmThreads / 256) * static_cast<size_t>(act_dim) + static_cast<size_t>(p.G) * p.W + p.W + 2 * p.G + kSmWaves +
                         static_cast<size_t>(p.G) * (p.L + 2) * kSmRep + 2 * static_cast<size_t>(kSmThreads) * chw +
                         2 * kSmWaves + static_cast<size_t>(kSmWaves) * kHeadDim;
    return words * 4 + (cache_bins ? static_cast<size_t>(p.G) * small_n_pad(n_tokens) * 2 : 0);
}

// The launch for one (key / value type, weight type) pair; step_small_bf16w.hip and
// step_small_f32w.hip instantiate it for bfloat16 and binary32 hash weights.
template <bool BF16, bool WBF16>
int launch_small(spotlight_ctx* ctx, const SmallArgs& a, size_t lds)
{
    void (*kern)(SmallArgs) = nullptr;
    switch (ctx->plan.W) {
    case 1: kern = step_small_kernel<BF16, WBF16, 1>; break;
    case 2: kern = step_small_kernel<BF16, WBF16, 2>; break;
    case 3: kern = step_small_kernel<BF16, WBF16, 3>; break;
    case 4: kern = step_small_kernel<BF16, WBF16, 4>; break;
    case 5: kern = step_small_kernel<BF16, WBF16, 5>; break;
    case 6: kern = step_small_kernel<BF16, WBF16, 6>; break;
    case 7: kern = step_small_kernel<BF16, WBF16, 7>; break;
    case 8: kern = step_small_kernel<BF16, WBF16, 8>; break;
    default: return SPOTLIGHT_ERR_UNSUPPORTED;
    }
    if (allow_dynamic_lds(ctx, reinterpret_cast<const void*>(kern), lds) != SPOTLIGHT_OK) return SPOTLIGHT_ERR_HIP;
    StageTimer timer(ctx, SPOTLIGHT_STAGE_STEP_SMALL);
    timer.launch(kern, dim3(static_cast<unsigned>(ctx->plan.B * ctx->plan.Hkv)), dim3(kSmThreads), lds, a);
    return hip_rc(hipGetLastError());
}

}  // namespace small
}  // namespace spotlight
