// Device code shared by the kernels that hash ONE vector per group of 256 threads (the query of a
// head, or the key appended by a decode step): hash_vec_kernel in hash.hip and the single-launch
// decode step in step_small.hip.  Same arithmetic as every other hash kernel: one binary32
// accumulator per output, fused multiply-adds in increasing index order (paper Sec. 3.2 Eq. 4-6,
// appendix "Bit-Packing CUDA Kernel").
#pragma once
#include "internal.h"

namespace spotlight {
namespace hashdev {

struct bf16_raw { uint16_t v; };

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t hi16) { return __uint_as_float(hi16 << 16); }

// load 8 consecutive elements starting at p (16-byte aligned for bf16, 32-byte for f32) as floats
__device__ __forceinline__ void load8(const float* p, float (&o)[8])
{
    const float4 a = reinterpret_cast<const float4*>(p)[0];
    const float4 b = reinterpret_cast<const float4*>(p)[1];
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_raw* p, float (&o)[8])
{
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    o[0] = __uint_as_float(u.x << 16); o[1] = __uint_as_float(u.x & 0xffff0000u);
    o[2] = __uint_as_float(u.y << 16); o[3] = __uint_as_float(u.y & 0xffff0000u);
    o[4] = __uint_as_float(u.z << 16); o[5] = __uint_as_float(u.z & 0xffff0000u);
    o[6] = __uint_as_float(u.w << 16); o[7] = __uint_as_float(u.w & 0xffff0000u);
}
// 8 consecutive weights kept in their stored form (converted when used)
template <typename WT> struct Raw8;
template <> struct Raw8<float> { float4 a, b; };
template <> struct Raw8<bf16_raw> { uint4 u; };
__device__ __forceinline__ void load_raw(const float* p, Raw8<float>& r)
{
    r.a = reinterpret_cast<const float4*>(p)[0];
    r.b = reinterpret_cast<const float4*>(p)[1];
}
__device__ __forceinline__ void load_raw(const bf16_raw* p, Raw8<bf16_raw>& r) { r.u = *reinterpret_cast<const uint4*>(p); }
__device__ __forceinline__ void expand(const Raw8<float>& r, float (&o)[8])
{
    o[0] = r.a.x; o[1] = r.a.y; o[2] = r.a.z; o[3] = r.a.w; o[4] = r.b.x; o[5] = r.b.y; o[6] = r.b.z; o[7] = r.b.w;
}
__device__ __forceinline__ void expand(const Raw8<bf16_raw>& r, float (&o)[8])
{
    o[0] = __uint_as_float(r.u.x << 16); o[1] = __uint_as_float(r.u.x & 0xffff0000u);
    o[2] = __uint_as_float(r.u.y << 16); o[3] = __uint_as_float(r.u.y & 0xffff0000u);
    o[4] = __uint_as_float(r.u.z << 16); o[5] = __uint_as_float(r.u.z & 0xffff0000u);
    o[6] = __uint_as_float(r.u.w << 16); o[7] = __uint_as_float(r.u.w & 0xffff0000u);
}
__device__ __forceinline__ float load1(const float* p) { return *p; }
__device__ __forceinline__ float load1(const bf16_raw* p) { return bf16_bits_to_f32(p->v); }

__device__ __forceinline__ float silu_exp(float t)
{
    t = (t > -87.0f) ? t : -87.0f;  // NaN goes to -87 as well
    t = (t < 88.0f) ? t : 88.0f;
    const float n = __builtin_rintf(t * 0x1.715476p+0f);
    float r = __builtin_fmaf(n, -0x1.62e400p-1f, t);
    r = __builtin_fmaf(n, -0x1.7f7d1cp-20f, r);
    float p = 0x1.a01a02p-13f;
    p = __builtin_fmaf(p, r, 0x1.6c16c2p-10f);
    p = __builtin_fmaf(p, r, 0x1.111112p-7f);
    p = __builtin_fmaf(p, r, 0x1.555556p-5f);
    p = __builtin_fmaf(p, r, 0x1.555556p-3f);
    p = __builtin_fmaf(p, r, 0.5f);
    p = __builtin_fmaf(p, r, 1.0f);
    p = __builtin_fmaf(p, r, 1.0f);
    const float s = __uint_as_float(static_cast<uint32_t>(static_cast<int>(n) + 127) << 23);
    return p * s;
}

__device__ __forceinline__ float silu(float a)
{
    const float e = silu_exp(-a);
    const float den = 1.0f + e;
    return a / den;  // IEEE-correct binary32 division
}


struct HashArgs {
    const void* x;
    int64_t x_head_stride, x_row0, n_rows;
    int heads_per_batch, group, n_wheads;
    const void* w1;
    const void* b1;
    const void* w2;
    int hidden, L, W;
    uint32_t* codes;
    int64_t code_head_stride, code_row0;
    uint32_t* zero;
    int zero_words;
    float* wnorm;   // scratch for the output-row norms of the matrix-core path, or null
    AuditRec* audit;   // totals of the audited matrix-core path, or null
    const void* pack_w1;   // packed copies for the single-vector kernel, or null
    const void* pack_out;
};

__device__ __forceinline__ int whead_of(const HashArgs& a, int xhead) { return (xhead % a.heads_per_batch) / a.group; }


// Hashes the vector of x-head `xhead` of job `a` with the 256 threads tid = 0 .. 255 of one group.
// EVERY thread of the workgroup must call it (it contains one workgroup barrier); groups with
// live == false only take part in the barrier.  `act` is LDS for the hidden activations of this
// group (max(hidden, 128) floats).  The packed code words go to a.codes and, if lds_code is set,
// to lds_code[0 .. W).
//
// x is read through uniform addresses, and every thread fetches its whole W1 row and the first 128
// weights of its W2 row (kept in their stored form) before any arithmetic.  (Fetching more ahead,
// or staging the weights through LDS with coalesced loads, measured slower: rows are 256 B or more
// apart, so every 16-byte load of a wave touches 64 cache lines and issue time dominates.)  The
// only LDS traffic is the broadcast of the hidden activations.
//
// PACKED: the weights come from a copy laid out in the order this code reads them (made once by
// pack_weights_kernel), so that the 64 lanes of every 16-byte load read 1 KB of consecutive
// memory.  From the arrays as the caller stores them, a row per lane, every load of a wavefront
// touches 64 cache lines and the kernel is bound by the issue of those loads: 28 us against 15 us
// for 640 vectors of a 128 -> 512 -> 256 network.  Same values, same arithmetic, same codes.
//   first layer:   [weight head][i / 256][g][i % 256][8]       = W1[i][8g .. 8g+7], rows past hidden zero
//   output matrix: [weight head][pair][run][g][lane][8]        = Wout[o(pair, lane)][128 run + 8g ...]
// with o(pair, lane) = (31 - lane % 32) * W + 2 pair + lane / 32, the output that lands in bit
// lane % 32 of word 2 pair + lane / 32 (zeros where that word does not exist).
template <typename XT, typename WT, bool PACKED>
__device__ __forceinline__ void hash_one_vector(const HashArgs& a, int xhead, bool live, int tid, float* act,
                                                uint32_t* lds_code)
{
    constexpr int G16 = kHeadDim / 8;             // groups of 8 in a run of 128 weights
    constexpr int GT = 256;                       // threads of a group

    const int lane = tid & 63, wave = tid >> 6;
    const int whead = (xhead % a.heads_per_batch) / a.group;
    const XT* x = static_cast<const XT*>(a.x) + xhead * a.x_head_stride + a.x_row0 * kHeadDim;
    const int act_dim = a.hidden > 0 ? a.hidden : kHeadDim;   // multiple of 128
    const int n16 = act_dim / kHeadDim;                        // runs of 128 weights per output row
    const WT* wout = a.hidden > 0 ? static_cast<const WT*>(a.w2) + static_cast<int64_t>(whead) * a.L * a.hidden
                                  : static_cast<const WT*>(a.w1) + static_cast<int64_t>(whead) * a.L * kHeadDim;
    const int npairs = (a.W + 1) / 2;

    // fetch the first run of this thread's first output row
    const int word0 = 2 * wave + (lane >> 5);
    const bool live0 = wave < npairs && word0 < a.W;
    const int o0 = live0 ? (31 - (lane & 31)) * a.W + word0 : 0;
    Raw8<WT> ra[G16], rb[G16];
    // group g of run r of this lane's output row of pair `pair`
    const WT* pout = PACKED ? static_cast<const WT*>(a.pack_out) + static_cast<int64_t>(whead) * npairs * act_dim * 64 : nullptr;
    auto out_group = [&](int pair, int o, int r, int g) {
        if constexpr (PACKED) return pout + ((static_cast<int64_t>(pair) * n16 + r) * G16 + g) * (64 * 8) + lane * 8;
        else return wout + static_cast<int64_t>(o) * act_dim + r * kHeadDim + g * 8;
    };
    if (live) {
#pragma unroll
        for (int g = 0; g < G16; ++g) load_raw(out_group(wave < npairs ? wave : 0, o0, 0, g), ra[g]);

        if (a.hidden > 0) {
            const WT* w1 = static_cast<const WT*>(a.w1) + static_cast<int64_t>(whead) * a.hidden * kHeadDim;
            const WT* b1 = static_cast<const WT*>(a.b1) + static_cast<int64_t>(whead) * a.hidden;
            for (int i = tid; i < a.hidden; i += GT) {
                Raw8<WT> w1r[G16];
#pragma unroll
                for (int g = 0; g < G16; ++g) {
                    if constexpr (PACKED)
                        load_raw(static_cast<const WT*>(a.pack_w1) +
                                     (((static_cast<int64_t>(whead) * ((a.hidden + GT - 1) / GT) + i / GT) * G16 + g) * GT + tid) * 8,
                                 w1r[g]);
                    else
                        load_raw(w1 + static_cast<int64_t>(i) * kHeadDim + g * 8, w1r[g]);
                }
                float acc = load1(b1 + i);
#pragma unroll
                for (int g = 0; g < G16; ++g) {
                    float xv[8], wv[8];
                    load8(x + g * 8, xv);
                    expand(w1r[g], wv);
#pragma unroll
                    for (int j = 0; j < 8; ++j) acc = __builtin_fmaf(wv[j], xv[j], acc);
                }
                act[i] = silu(acc);
            }
        } else {
            for (int e = tid; e < G16; e += GT) {
                float xv[8];
                load8(x + e * 8, xv);
#pragma unroll
                for (int j = 0; j < 8; ++j) act[e * 8 + j] = xv[j];
            }
        }
    }
    __syncthreads();
    if (!live) return;

    auto run128 = [&](const Raw8<WT> (&r)[G16], const float* h, float y) {
#pragma unroll
        for (int g = 0; g < G16; ++g) {
            float wv[8];
            expand(r[g], wv);
            const float4 h0 = reinterpret_cast<const float4*>(h + g * 8)[0];
            const float4 h1 = reinterpret_cast<const float4*>(h + g * 8)[1];
            y = __builtin_fmaf(wv[0], h0.x, y); y = __builtin_fmaf(wv[1], h0.y, y);
            y = __builtin_fmaf(wv[2], h0.z, y); y = __builtin_fmaf(wv[3], h0.w, y);
            y = __builtin_fmaf(wv[4], h1.x, y); y = __builtin_fmaf(wv[5], h1.y, y);
            y = __builtin_fmaf(wv[6], h1.z, y); y = __builtin_fmaf(wv[7], h1.w, y);
        }
        return y;
    };

    uint32_t* cbase = a.codes + xhead * a.code_head_stride + a.code_row0 * a.W;
    for (int pair = wave; pair < npairs; pair += GT / 64) {
        const int word = 2 * pair + (lane >> 5);
        const bool lv = word < a.W;
        const int o = lv ? (31 - (lane & 31)) * a.W + word : 0;
        float y = 0.0f;
        for (int r0 = 0; r0 < n16; r0 += 2) {
            if (pair != wave || r0 != 0) {   // the first run of the first row is already here
#pragma unroll
                for (int g = 0; g < G16; ++g) load_raw(out_group(pair, o, r0, g), ra[g]);
            }
            if (r0 + 1 < n16) {
#pragma unroll
                for (int g = 0; g < G16; ++g) load_raw(out_group(pair, o, r0 + 1, g), rb[g]);
            }
            y = run128(ra, act + r0 * kHeadDim, y);
            if (r0 + 1 < n16) y = run128(rb, act + (r0 + 1) * kHeadDim, y);
        }
        const unsigned long long m = __ballot(lv && (y > 0.0f));
        if (lane == 0) {
            cbase[2 * pair] = static_cast<uint32_t>(m);
            if (2 * pair + 1 < a.W) cbase[2 * pair + 1] = static_cast<uint32_t>(m >> 32);
            if (lds_code) {
                lds_code[2 * pair] = static_cast<uint32_t>(m);
                if (2 * pair + 1 < a.W) lds_code[2 * pair + 1] = static_cast<uint32_t>(m >> 32);
            }
        }
    }
    if (a.zero)
        for (int i = tid; i < a.zero_words; i += GT) a.zero[static_cast<int64_t>(xhead) * a.zero_words + i] = 0u;
}

}  // namespace hashdev

// Kernel arguments of one hash job (host side: hash.hip).
hashdev::HashArgs make_hash_args(const HashLaunch& h);

}  // namespace spotlight
