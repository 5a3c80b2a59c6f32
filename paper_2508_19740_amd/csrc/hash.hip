// Hash MLP + sign + bit-packing (paper Sec. 3.2 Eq. 4-6, appendix "Bit-Packing CUDA Kernel").
//
// One workgroup hashes a tile of TK vectors of one head.  Every output keeps its own binary32
// accumulator and takes its fused multiply-adds in increasing index order, so the sign bits do not
// depend on the tile size or launch shape:
//   a_i = b1_i + sum_k W1[i][k] x[k];  h_i = a_i / (1 + exp(-a_i));  y_j = sum_i W2[j][i] h_i
// exp is the fixed routine silu_exp() (range clamp, round-to-nearest reduction by ln 2 in two fused
// steps, degree-7 Horner polynomial, exact power-of-two scaling).
//
// Phase 1: thread i owns hidden unit i (+256, ...), streams its W1 row from global memory 8 values
//          at a time and reads x from LDS (stored [k][t], so one 16-byte LDS read feeds 4 vectors).
// Phase 2: a wavefront owns two code words; lane l computes the hash output that belongs to bit
//          (l & 31) of word 2p + (l >> 5), i.e. output (31 - (l & 31)) * W + word, so a wave-wide
//          ballot of (y > 0) IS the pair of packed words.  No boolean tensor is ever stored.
#include "hash_vec.h"

namespace spotlight {
using namespace hashdev;
namespace {

// TK consecutive floats from LDS (16-byte reads when TK is a multiple of 4)
template <int TK>
__device__ __forceinline__ void lds_tile(const float* p, float (&o)[TK])
{
    if constexpr (TK % 4 == 0) {
#pragma unroll
        for (int t = 0; t < TK / 4; ++t) {
            const float4 v = reinterpret_cast<const float4*>(p)[t];
            o[4 * t] = v.x; o[4 * t + 1] = v.y; o[4 * t + 2] = v.z; o[4 * t + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int t = 0; t < TK; ++t) o[t] = p[t];
    }
}

// acc[t] += sum over n8*8 consecutive weights of `row` times act[(i)*stride + t], in increasing i,
// one fused multiply-add per term.  PF groups of 8 weights are fetched ahead of their use.
template <typename WT, int TK, int PF>
__device__ __forceinline__ void dot_rows(const WT* __restrict__ row, int n8, const float* act, int stride,
                                         float (&acc)[TK])
{
    int g = 0;
    for (; g + PF <= n8; g += PF) {
        float wv[PF][8];
#pragma unroll
        for (int p = 0; p < PF; ++p) load8(row + (g + p) * 8, wv[p]);
#pragma unroll
        for (int p = 0; p < PF; ++p)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                float xr[TK];
                lds_tile<TK>(act + ((g + p) * 8 + j) * stride, xr);
#pragma unroll
                for (int t = 0; t < TK; ++t) acc[t] = __builtin_fmaf(wv[p][j], xr[t], acc[t]);
            }
    }
    for (; g < n8; ++g) {
        float wv[8];
        load8(row + g * 8, wv);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            float xr[TK];
            lds_tile<TK>(act + (g * 8 + j) * stride, xr);
#pragma unroll
            for (int t = 0; t < TK; ++t) acc[t] = __builtin_fmaf(wv[j], xr[t], acc[t]);
        }
    }
}

// LDS: xs [128][TK] floats, then hs [hidden][TK] floats (hidden > 0 only).
template <typename XT, typename WT, int TK, int KSPLIT>
__global__ __launch_bounds__(kThreads) void hash_kernel(HashArgs a)
{
    constexpr int TK2 = TK / KSPLIT;
    constexpr int PF = TK == 1 ? 16 : (TK <= 8 ? 2 : 1);  // weight groups fetched ahead
    extern __shared__ __align__(16) float lds[];
    float* xs = lds;
    float* hs = lds + kHeadDim * TK;

    const int tid = threadIdx.x;
    const int xhead = blockIdx.y;
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * TK;
    const int rows = static_cast<int>(min(static_cast<int64_t>(TK), a.n_rows - r0));
    const int whead = (xhead % a.heads_per_batch) / a.group;
    if (a.zero && blockIdx.x == 0)
        for (int i = tid; i < a.zero_words; i += kThreads) a.zero[static_cast<int64_t>(xhead) * a.zero_words + i] = 0u;

    // ---- stage the x tile, transposed to [k][t], rows past the end as zeros
    const XT* xbase = static_cast<const XT*>(a.x) + xhead * a.x_head_stride + (a.x_row0 + r0) * kHeadDim;
    for (int e = tid; e < TK * (kHeadDim / 8); e += kThreads) {
        const int t = e / (kHeadDim / 8), k8 = e % (kHeadDim / 8);
        float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        if (t < rows) load8(xbase + static_cast<int64_t>(t) * kHeadDim + k8 * 8, v);
#pragma unroll
        for (int j = 0; j < 8; ++j) xs[(k8 * 8 + j) * TK + t] = v[j];
    }
    __syncthreads();

    // ---- phase 1: hidden activations
    const float* act = xs;   // what phase 2 contracts over
    int act_dim = kHeadDim;
    const WT* wout = static_cast<const WT*>(a.w1) + static_cast<int64_t>(whead) * a.L * kHeadDim;  // linear hash: R
    if (a.hidden > 0) {
        const WT* w1 = static_cast<const WT*>(a.w1) + static_cast<int64_t>(whead) * a.hidden * kHeadDim;
        const WT* b1 = static_cast<const WT*>(a.b1) + static_cast<int64_t>(whead) * a.hidden;
        for (int i = tid; i < a.hidden; i += kThreads) {
            float acc[TK];
            const float bias = load1(b1 + i);
#pragma unroll
            for (int t = 0; t < TK; ++t) acc[t] = bias;
            dot_rows<WT, TK, PF>(w1 + static_cast<int64_t>(i) * kHeadDim, kHeadDim / 8, xs, TK, acc);
#pragma unroll
            for (int t = 0; t < TK; ++t) hs[i * TK + t] = silu(acc[t]);
        }
        __syncthreads();
        act = hs;
        act_dim = a.hidden;
        wout = static_cast<const WT*>(a.w2) + static_cast<int64_t>(whead) * a.L * a.hidden;
    }

    // ---- phase 2: outputs, sign, ballot-pack
    const int lane = tid & 63, wave = tid >> 6;
    const int npairs = (a.W + 1) / 2;
    uint32_t* cbase = a.codes + xhead * a.code_head_stride + (a.code_row0 + r0) * a.W;
    for (int item = wave; item < npairs * KSPLIT; item += kThreads / 64) {
        const int pair = item / KSPLIT, ks = item % KSPLIT;
        const int word = 2 * pair + (lane >> 5);
        const bool live = word < a.W;
        const int o = live ? (31 - (lane & 31)) * a.W + word : 0;
        const WT* row = wout + static_cast<int64_t>(o) * act_dim;
        float y[TK2];
#pragma unroll
        for (int t = 0; t < TK2; ++t) y[t] = 0.0f;
        dot_rows<WT, TK2, PF>(row, act_dim / 8, act + ks * TK2, TK, y);
#pragma unroll
        for (int t = 0; t < TK2; ++t) {
            const unsigned long long m = __ballot(live && (y[t] > 0.0f));
            const int r = ks * TK2 + t;
            if (lane == 0 && r < rows) {
                cbase[static_cast<int64_t>(r) * a.W + 2 * pair] = static_cast<uint32_t>(m);
                if (2 * pair + 1 < a.W) cbase[static_cast<int64_t>(r) * a.W + 2 * pair + 1] = static_cast<uint32_t>(m >> 32);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Bulk hashing with the second layer on the matrix cores.
//
// Phase 1 is the canonical binary32 chain above (the hidden activations feed a non-linear function,
// so nothing but the defined arithmetic will do).  Phase 2, Y = H W2^T for a tile of 32 vectors, is
// a dense contraction and runs as v_mfma_f32_32x32x16_bf16: W2 is bfloat16 as stored, and each
// activation h is split on the fly into hi + lo (both bfloat16, |h - hi - lo| <= 2^-18 |h|), so
// the products are exact and two accumulating MFMA passes give y to within
//     |y_mfma - y_canonical| <= eps * sum_i |W2[j][i] h_i| <= eps * ||W2[j]|| * ||h||
// with eps = 1.01 * (hidden * (2^-24 + 1.01 * 2^-22) + 2^-17):  hidden roundings of 2^-24 in the
// canonical chain, at most 2 * hidden additions in the matrix core each assumed to err by at most
// one unit in the last place of binary32 whatever their order, and the split residue (2^-18, taken
// as 2^-17).  A fixed 1e-30 on top covers activations so small that a conversion flushes them.
// The sign of y_mfma is therefore the canonical sign wherever |y_mfma| exceeds that bound; the few
// outputs that do not (about 0.2 %) are recomputed with the canonical chain from the binary32
// activations still in LDS.  The codes are identical to the all-binary32 kernel's, bit for bit.
//
// The 32 columns of an MFMA tile are the 32 outputs of ONE code word in bit order (column c is
// output (31 - c) * W + word), so a wave ballot over an accumulator register is two packed words.
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));

constexpr int kMfmaTile = 32;       // vectors per tile (rows of the MFMA)
constexpr int kMfmaListCap = 1024;  // outputs of a tile that may go to the canonical recomputation

struct MfmaLds {   // lives in the x tile's LDS once phase 1 is done with it
    float part[8][kMfmaTile];
    float hn[kMfmaTile];              // ||h_t||
    uint32_t codes[kMfmaTile][16];
    uint16_t list[kMfmaListCap];
    uint32_t count;
};
static_assert(sizeof(MfmaLds) <= sizeof(float) * kHeadDim * kMfmaTile, "fits in the x tile");

// hi / lo split of 8 activations into two MFMA operands: hi = bf16(h) and lo = bf16(h - hi), both
// rounded to nearest by the packed conversion instruction; h - hi is exact.
__device__ __forceinline__ void split8(const float (&h)[8], bf16x8_t& hi, bf16x8_t& lo)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    union { bf16x8_t v; uint32_t u[4]; } a, b;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const f32x2_t hv = {h[2 * p], h[2 * p + 1]};
        const uint32_t hp = __builtin_bit_cast(uint32_t, __builtin_convertvector(hv, bf16x2_t));
        const f32x2_t rv = {h[2 * p] - __uint_as_float(hp << 16), h[2 * p + 1] - __uint_as_float(hp & 0xffff0000u)};
        a.u[p] = hp;
        b.u[p] = __builtin_bit_cast(uint32_t, __builtin_convertvector(rv, bf16x2_t));
    }
    hi = a.v;
    lo = b.v;
}

// ||W2[j]|| of every output row of every weight head, for the bound above.
__global__ __launch_bounds__(kThreads) void w2_norm_kernel(const bf16_raw* __restrict__ w2, float* __restrict__ wnorm,
                                                          int n_rows, int hidden)
{
    const int j = blockIdx.x * kThreads + threadIdx.x;
    if (j >= n_rows) return;
    float s = 0.0f;
    for (int g = 0; g < hidden / 8; ++g) {
        float wv[8];
        load8(w2 + static_cast<int64_t>(j) * hidden + g * 8, wv);
#pragma unroll
        for (int e = 0; e < 8; ++e) s = __builtin_fmaf(wv[e], wv[e], s);
    }
    wnorm[j] = __builtin_sqrtf(s);
}

// NBW: code words (MFMA column blocks) per wavefront = ceil(W / 4).
// AUDIT: every output is also evaluated with the canonical chain and compared with the matrix
// cores' value (distance in units of ||W2[j]|| ||h||, settled signs that disagree); the totals go to
// a.audit.  The codes written are the same either way.
template <typename XT, int NBW, bool AUDIT>
__global__ __launch_bounds__(kThreads) void hash_mfma_kernel(HashArgs a, const float* __restrict__ wnorm, float eps,
                                                            int tiles_per_group)
{
    using WT = bf16_raw;
    constexpr int TK = kMfmaTile;
    extern __shared__ __align__(16) float lds[];
    float* xs = lds;                                   // [128][TK], later MfmaLds
    float* hs = lds + kHeadDim * TK;                   // [hidden][TK]
    MfmaLds& m = *reinterpret_cast<MfmaLds*>(xs);
    float* hn = m.hn;
    const float* wn = wnorm + static_cast<int64_t>(whead_of(a, blockIdx.y)) * a.L;   // ||W2[j]|| of this head

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int xhead = blockIdx.y;
    const int whead = (xhead % a.heads_per_batch) / a.group;
    const WT* w1 = static_cast<const WT*>(a.w1) + static_cast<int64_t>(whead) * a.hidden * kHeadDim;
    const WT* b1 = static_cast<const WT*>(a.b1) + static_cast<int64_t>(whead) * a.hidden;
    const WT* w2 = static_cast<const WT*>(a.w2) + static_cast<int64_t>(whead) * a.L * a.hidden;
    const int n8 = a.hidden / 8;

    uint32_t au_outputs = 0, au_listed = 0, au_wrong = 0;   // this lane's audit totals
    float au_ratio = 0.0f;

    const int64_t n_tiles = (a.n_rows + TK - 1) / TK;
    const int64_t tile0 = static_cast<int64_t>(blockIdx.x) * tiles_per_group;
    const int64_t tile1 = min(n_tiles, tile0 + tiles_per_group);
    for (int64_t tile = tile0; tile < tile1; ++tile) {
        const int64_t r0 = tile * TK;
        const int rows = static_cast<int>(min(static_cast<int64_t>(TK), a.n_rows - r0));
        __syncthreads();   // the previous tile is done with LDS

        // ---- stage the x tile, transposed to [k][t], rows past the end as zeros
        const XT* xbase = static_cast<const XT*>(a.x) + xhead * a.x_head_stride + (a.x_row0 + r0) * kHeadDim;
        for (int e = tid; e < TK * (kHeadDim / 8); e += kThreads) {
            const int t = e / (kHeadDim / 8), k8 = e % (kHeadDim / 8);
            float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (t < rows) load8(xbase + static_cast<int64_t>(t) * kHeadDim + k8 * 8, v);
#pragma unroll
            for (int j = 0; j < 8; ++j) xs[(k8 * 8 + j) * TK + t] = v[j];
        }
        __syncthreads();

        // ---- phase 1 (canonical): hidden activations
        for (int i = tid; i < a.hidden; i += kThreads) {
            float acc[TK];
            const float bias = load1(b1 + i);
#pragma unroll
            for (int t = 0; t < TK; ++t) acc[t] = bias;
            dot_rows<WT, TK, 1>(w1 + static_cast<int64_t>(i) * kHeadDim, kHeadDim / 8, xs, TK, acc);
#pragma unroll
            for (int t = 0; t < TK; ++t) hs[i * TK + t] = silu(acc[t]);
        }
        __syncthreads();

        // ---- norms of the activation rows; the x tile's LDS becomes scratch
        {
            const int t = tid & (TK - 1), part = tid / TK;   // 8 partial sums per vector
            float s = 0.0f;
            for (int i = part; i < a.hidden; i += kThreads / TK) s = __builtin_fmaf(hs[i * TK + t], hs[i * TK + t], s);
            m.part[part][t] = s;
            if (tid == 0) m.count = 0;
        }
        __syncthreads();
        if (tid < TK) {
            float s = 0.0f;
#pragma unroll
            for (int p8 = 0; p8 < 8; ++p8) s += m.part[p8][tid];
            hn[tid] = __builtin_sqrtf(s);
        }
        __syncthreads();

        // ---- phase 2 on the matrix cores: wave w owns code words w, w + 4, ...
        const int c = lane & 31, half = lane >> 5;
        f32x16_t acc[NBW];
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][v] = 0.0f;
        const WT* brow[NBW];
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            const int word = wave + 4 * nb;
            const int j = word < a.W ? (31 - c) * a.W + word : 0;
            brow[nb] = w2 + static_cast<int64_t>(j) * a.hidden + 8 * half;
        }
        const int n_ks = a.hidden / 16;
        union BFrag { bf16x8_t v; uint4 u; };
        BFrag bnext[NBW];
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) bnext[nb].u = *reinterpret_cast<const uint4*>(brow[nb]);
        for (int ks = 0; ks < n_ks; ++ks) {
            BFrag b[NBW];
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) b[nb] = bnext[nb];
            if (ks + 1 < n_ks) {   // the next step's weights are requested before this step's arithmetic
#pragma unroll
                for (int nb = 0; nb < NBW; ++nb) bnext[nb].u = *reinterpret_cast<const uint4*>(brow[nb] + (ks + 1) * 16);
            }
            float h8[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) h8[e] = hs[(ks * 16 + 8 * half + e) * TK + c];
            bf16x8_t ahi, alo;
            split8(h8, ahi, alo);
#pragma unroll
            for (int nb = 0; nb < NBW; ++nb) {
                acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ahi, b[nb].v, acc[nb], 0, 0, 0);
                acc[nb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(alo, b[nb].v, acc[nb], 0, 0, 0);
            }
        }

        if constexpr (AUDIT) {
            // the canonical chain for each of this lane's outputs: its 16 vectors share the weight row
#pragma unroll 1
            for (int nb = 0; nb < NBW; ++nb) {
                const int word = wave + 4 * nb;
                if (word >= a.W) continue;
                const int j = (31 - c) * a.W + word;
                const WT* row = w2 + static_cast<int64_t>(j) * a.hidden;
                float yc[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) yc[v] = 0.0f;
                for (int g = 0; g < n8; ++g) {
                    float wv[8];
                    load8(row + g * 8, wv);
#pragma unroll
                    for (int q = 0; q < 8; ++q)
#pragma unroll
                        for (int v = 0; v < 16; ++v)
                            yc[v] = __builtin_fmaf(wv[q], hs[(g * 8 + q) * TK + (v / 4) * 8 + half * 4 + (v % 4)], yc[v]);
                }
                const float tcol = eps * wn[j];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int t = (v / 4) * 8 + half * 4 + (v % 4);
                    if (t >= rows) continue;
                    const float y = acc[nb][v];
                    const bool sure = __builtin_fabsf(y) > __builtin_fmaf(tcol, hn[t], 1e-30f);
                    const float den = wn[j] * hn[t];
                    const float diff = __builtin_fabsf(y - yc[v]);
                    // a NaN or an infinity on either side is never settled and is not a distance
                    const float ratio = (diff == 0.0f || !(diff < INFINITY)) ? 0.0f : (den > 0.0f ? diff / den : INFINITY);
                    au_ratio = fmaxf(au_ratio, ratio);
                    au_outputs += 1;
                    au_listed += sure ? 0 : 1;
                    au_wrong += (sure && ((y > 0.0f) != (yc[v] > 0.0f))) ? 1 : 0;
                }
            }
        }

        // ---- signs, ballot-pack, and the list of outputs too close to zero to trust
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            const int word = wave + 4 * nb;
            if (word >= a.W) continue;   // uniform over the wavefront
            const float tcol = eps * wn[(31 - c) * a.W + word];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int t = (v / 4) * 8 + half * 4 + (v % 4);
                const float y = acc[nb][v];
                const float thr = __builtin_fmaf(tcol, hn[t], 1e-30f);
                const bool sure = __builtin_fabsf(y) > thr;   // false for NaN
                const unsigned long long pos = __ballot(y > 0.0f);
                if (c == 0) m.codes[t][word] = half ? static_cast<uint32_t>(pos >> 32) : static_cast<uint32_t>(pos);
                if (!sure) {
                    const uint32_t at = atomicAdd(&m.count, 1u);
                    if (at < static_cast<uint32_t>(kMfmaListCap))
                        m.list[at] = static_cast<uint16_t>(t | (word << 5) | (c << 9));
                }
            }
        }
        __syncthreads();

        // ---- canonical recomputation of the listed outputs (of every output if the list overflowed)
        const uint32_t listed = m.count;
        if (listed <= static_cast<uint32_t>(kMfmaListCap)) {
            for (uint32_t e = tid; e < listed; e += kThreads) {
                const int t = m.list[e] & 31, word = (m.list[e] >> 5) & 15, col = m.list[e] >> 9;
                const WT* row = w2 + static_cast<int64_t>((31 - col) * a.W + word) * a.hidden;
                float y = 0.0f;
                for (int g = 0; g < n8; ++g) {
                    float wv[8];
                    load8(row + g * 8, wv);
#pragma unroll
                    for (int q = 0; q < 8; ++q) y = __builtin_fmaf(wv[q], hs[(g * 8 + q) * TK + t], y);
                }
                const uint32_t bit = 1u << col;
                if (((m.codes[t][word] & bit) != 0) != (y > 0.0f)) atomicXor(&m.codes[t][word], bit);
            }
        } else {
            for (int item = tid; item < TK * a.L; item += kThreads) {
                const int t = item % TK, j = item / TK;
                const WT* row = w2 + static_cast<int64_t>(j) * a.hidden;
                float y = 0.0f;
                for (int g = 0; g < n8; ++g) {
                    float wv[8];
                    load8(row + g * 8, wv);
#pragma unroll
                    for (int q = 0; q < 8; ++q) y = __builtin_fmaf(wv[q], hs[(g * 8 + q) * TK + t], y);
                }
                const int word = j % a.W, col = 31 - j / a.W;
                const uint32_t bit = 1u << col;
                if (((m.codes[t][word] & bit) != 0) != (y > 0.0f)) atomicXor(&m.codes[t][word], bit);
            }
        }
        __syncthreads();

        // ---- the tile's codes: rows * W consecutive words
        uint32_t* cbase = a.codes + xhead * a.code_head_stride + (a.code_row0 + r0) * a.W;
        for (int e = tid; e < rows * a.W; e += kThreads) cbase[e] = m.codes[e / a.W][e % a.W];
    }
    if constexpr (AUDIT) {
        const uint32_t outputs = wave_sum(au_outputs), listed = wave_sum(au_listed), wrong = wave_sum(au_wrong);
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) au_ratio = fmaxf(au_ratio, __shfl_xor(au_ratio, off));
        if (lane == 0) {
            atomicAdd(&a.audit->outputs, static_cast<unsigned long long>(outputs));
            if (listed) atomicAdd(&a.audit->listed, static_cast<unsigned long long>(listed));
            if (wrong) atomicAdd(&a.audit->wrong, static_cast<unsigned long long>(wrong));
            atomicMax(&a.audit->max_ratio_bits, __float_as_uint(au_ratio));   // non-negative floats order like their bits
        }
    }
}

// One vector per workgroup (the query of a head, or the key appended by a decode step), for hidden
// widths that are multiples of 128 (or the linear hash).  Latency matters here, not throughput; the
// work is hashdev::hash_one_vector (hash_vec.h).
// Two independent jobs in one launch (the decode step hashes the queries and the appended keys
// together): workgroups [0, n_first) run job[0], the rest job[1].
struct HashVecArgs {
    HashArgs job[2];
    int n_first;
};

template <typename XT, typename WT, bool PACKED>
__global__ __launch_bounds__(kThreads) void hash_vec_kernel(HashVecArgs jobs)
{
    extern __shared__ __align__(16) float act[];  // hidden activations, or x itself for the linear hash
    const bool second = static_cast<int>(blockIdx.x) >= jobs.n_first;   // uniform over the workgroup
    const HashArgs& a = jobs.job[second ? 1 : 0];
    const int xhead = static_cast<int>(blockIdx.x) - (second ? jobs.n_first : 0);
    hash_one_vector<XT, WT, PACKED>(a, xhead, true, threadIdx.x, act, nullptr);
}

// One thread per group of 8 weights of the packed copies (layout: see hash_vec_kernel).
template <typename WT>
__global__ __launch_bounds__(kThreads) void pack_weights_kernel(const WT* __restrict__ w1, const WT* __restrict__ wout,
                                                               WT* __restrict__ pack_w1, WT* __restrict__ pack_out,
                                                               int n_wheads, int hidden, int L)
{
    constexpr int G16 = kHeadDim / 8;
    const int W = L / 32, npairs = (W + 1) / 2;
    const int act_dim = hidden > 0 ? hidden : kHeadDim, n16 = act_dim / kHeadDim;
    const int nib = (hidden + kThreads - 1) / kThreads;   // 0 for the linear hash: no first layer
    const int64_t groups1 = static_cast<int64_t>(n_wheads) * nib * G16 * kThreads;
    const int64_t groups2 = static_cast<int64_t>(n_wheads) * npairs * n16 * G16 * 64;
    const int64_t x = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    const WT* src = nullptr;
    WT* dst;
    if (x < groups1) {
        const int t = static_cast<int>(x % kThreads), g = static_cast<int>((x / kThreads) % G16);
        const int ib = static_cast<int>((x / (kThreads * G16)) % nib), whead = static_cast<int>(x / (static_cast<int64_t>(kThreads) * G16 * nib));
        const int row = ib * kThreads + t;
        if (row < hidden) src = w1 + (static_cast<int64_t>(whead) * hidden + row) * kHeadDim + g * 8;
        dst = pack_w1 + x * 8;
    } else if (x < groups1 + groups2) {
        const int64_t y = x - groups1;
        const int lane = static_cast<int>(y % 64), g = static_cast<int>((y / 64) % G16);
        const int r = static_cast<int>((y / (64 * G16)) % n16), pair = static_cast<int>((y / (static_cast<int64_t>(64) * G16 * n16)) % npairs);
        const int whead = static_cast<int>(y / (static_cast<int64_t>(64) * G16 * n16 * npairs));
        const int word = 2 * pair + (lane >> 5);
        if (word < W) {
            const int o = (31 - (lane & 31)) * W + word;
            src = wout + (static_cast<int64_t>(whead) * L + o) * act_dim + r * kHeadDim + g * 8;
        }
        dst = pack_out + y * 8;
    } else {
        return;
    }
    if constexpr (sizeof(WT) == 2) {
        uint4 v = make_uint4(0u, 0u, 0u, 0u);
        if (src) v = *reinterpret_cast<const uint4*>(src);
        *reinterpret_cast<uint4*>(dst) = v;
    } else {
        float4 v0 = make_float4(0.f, 0.f, 0.f, 0.f), v1 = v0;
        if (src) { v0 = reinterpret_cast<const float4*>(src)[0]; v1 = reinterpret_cast<const float4*>(src)[1]; }
        reinterpret_cast<float4*>(dst)[0] = v0;
        reinterpret_cast<float4*>(dst)[1] = v1;
    }
}

template <typename XT, typename WT>
int run_vec(spotlight_ctx* ctx, const HashArgs& a, int n_xheads, const HashArgs* b, int n_xheads_b, int stage)
{
    const size_t lds = sizeof(float) * (a.hidden > 0 ? a.hidden : kHeadDim);
    HashVecArgs jobs;
    jobs.job[0] = a;
    jobs.job[1] = b ? *b : a;
    jobs.n_first = n_xheads;
    const int grid = n_xheads + (b ? n_xheads_b : 0);
    const bool packed = a.pack_out && (a.hidden == 0 || a.pack_w1) && (!b || (b->pack_out == a.pack_out && b->pack_w1 == a.pack_w1));
    auto kern = hash_vec_kernel<XT, WT, false>;
    if (packed) kern = hash_vec_kernel<XT, WT, true>;
    StageTimer timer(ctx, stage);
    timer.launch(kern, dim3(static_cast<unsigned>(grid)), dim3(kThreads), lds, jobs);
    return hip_rc(hipGetLastError());
}

inline size_t lds_bytes(int tk, int hidden) { return sizeof(float) * tk * (kHeadDim + hidden); }

template <typename XT, typename WT, int TK, int KSPLIT>
int run(spotlight_ctx* ctx, const HashArgs& a, int n_xheads, int stage)
{
    const size_t lds = lds_bytes(TK, a.hidden);
    if (lds > static_cast<size_t>(ctx->max_lds)) return SPOTLIGHT_ERR_UNSUPPORTED;
    auto kern = hash_kernel<XT, WT, TK, KSPLIT>;
    if (allow_dynamic_lds(ctx, reinterpret_cast<const void*>(kern), lds) != SPOTLIGHT_OK) return SPOTLIGHT_ERR_HIP;
    const int64_t tiles = (a.n_rows + TK - 1) / TK;
    dim3 grid(static_cast<unsigned>(tiles), static_cast<unsigned>(n_xheads));
    StageTimer timer(ctx, stage);
    timer.launch(kern, grid, dim3(kThreads), lds, a);
    return hip_rc(hipGetLastError());
}

template <typename XT, typename WT, int TK>
int run_ks(spotlight_ctx* ctx, const HashArgs& a, int n_xheads, int stage)
{
    const int npairs = (a.W + 1) / 2;
    if constexpr (TK >= 4) {
        if (npairs == 1) return run<XT, WT, TK, 4>(ctx, a, n_xheads, stage);
    }
    if constexpr (TK >= 2) {
        if (npairs <= 2) return run<XT, WT, TK, 2>(ctx, a, n_xheads, stage);
    }
    return run<XT, WT, TK, 1>(ctx, a, n_xheads, stage);
}

// Second layer on the matrix cores: bfloat16 weights, hidden a multiple of 16, at least one full tile.
template <typename XT, int NBW>
int run_mfma_nbw(spotlight_ctx* ctx, const HashArgs& a, int n_xheads, int stage, size_t lds, float* wnorm)
{
    auto kern = hash_mfma_kernel<XT, NBW, false>;
    if (a.audit) kern = hash_mfma_kernel<XT, NBW, true>;
    if (allow_dynamic_lds(ctx, reinterpret_cast<const void*>(kern), lds) != SPOTLIGHT_OK) return SPOTLIGHT_ERR_HIP;
    const int64_t tiles = (a.n_rows + kMfmaTile - 1) / kMfmaTile;
    // a workgroup takes a run of tiles of one head (the output-row norms are computed once per run),
    // short enough that the grid still has a few thousand workgroups
    int tpg = 8;
    while (tpg > 1 && ((tiles + tpg - 1) / tpg) * n_xheads < 4096) tpg /= 2;
    const double eps = bulk_hash_eps(a.hidden);   // error bound per unit of ||W2[j]|| * ||h||
    dim3 grid(static_cast<unsigned>((tiles + tpg - 1) / tpg), static_cast<unsigned>(n_xheads));
    const int n_out = a.n_wheads * a.L;
    hipLaunchKernelGGL(w2_norm_kernel, dim3(static_cast<unsigned>((n_out + kThreads - 1) / kThreads)), dim3(kThreads), 0,
                       ctx->stream, static_cast<const bf16_raw*>(a.w2), wnorm, n_out, a.hidden);   // microseconds: not timed
    StageTimer timer(ctx, stage);
    timer.launch(kern, grid, dim3(kThreads), lds, a, wnorm, static_cast<float>(eps), tpg);
    return hip_rc(hipGetLastError());
}

inline size_t mfma_lds_bytes(int hidden) { return sizeof(float) * kMfmaTile * (kHeadDim + hidden); }

template <typename XT>
int run_mfma(spotlight_ctx* ctx, const HashArgs& a, int n_xheads, int stage, float* wnorm)
{
    const size_t lds = mfma_lds_bytes(a.hidden);
    if (a.W <= 4) return run_mfma_nbw<XT, 1>(ctx, a, n_xheads, stage, lds, wnorm);
    if (a.W <= 8) return run_mfma_nbw<XT, 2>(ctx, a, n_xheads, stage, lds, wnorm);
    return run_mfma_nbw<XT, 4>(ctx, a, n_xheads, stage, lds, wnorm);
}

template <typename XT, typename WT>
int run_tk(spotlight_ctx* ctx, const HashArgs& a, int n_xheads, int stage)
{
    const size_t cap = static_cast<size_t>(ctx->max_lds);
    if constexpr (sizeof(WT) == 2) {
        if (a.n_rows >= kMfmaTile && a.hidden > 0 && a.hidden % 16 == 0 && a.W <= 16 &&
            mfma_lds_bytes(a.hidden) <= cap && a.wnorm)
            return run_mfma<XT>(ctx, a, n_xheads, stage, a.wnorm);
    }
    // a single vector per head, hidden width a multiple of 128: the latency-oriented kernel
    if (a.n_rows == 1 && a.hidden % kHeadDim == 0) return run_vec<XT, WT>(ctx, a, n_xheads, nullptr, 0, stage);
    if (a.n_rows >= 32 && lds_bytes(32, a.hidden) <= cap) return run_ks<XT, WT, 32>(ctx, a, n_xheads, stage);
    if (a.n_rows >= 4 && lds_bytes(8, a.hidden) <= cap) return run_ks<XT, WT, 8>(ctx, a, n_xheads, stage);
    return run_ks<XT, WT, 1>(ctx, a, n_xheads, stage);
}

}  // namespace

HashArgs make_hash_args(const HashLaunch& h)
{
    HashArgs a;
    a.x = h.x;
    a.x_head_stride = h.x_head_stride;
    a.x_row0 = h.x_row0;
    a.n_rows = h.n_rows;
    a.heads_per_batch = h.heads_per_batch;
    a.group = h.group;
    a.n_wheads = h.heads_per_batch / h.group;
    a.w1 = h.w1;
    a.b1 = h.b1;
    a.w2 = h.w2;
    a.hidden = h.hidden;
    a.L = h.L;
    a.W = h.L / 32;
    a.codes = h.codes;
    a.code_head_stride = h.code_head_stride;
    a.code_row0 = h.code_row0;
    a.zero = h.zero;
    a.zero_words = h.zero_words;
    a.wnorm = h.wnorm;
    a.audit = h.audit;
    a.pack_w1 = h.pack_w1;
    a.pack_out = h.pack_out;
    return a;
}

void pack_sizes(int hidden, int L, size_t* w1_elems, size_t* out_elems)
{
    *w1_elems = *out_elems = 0;
    if (hidden % kHeadDim != 0) return;   // the single-vector kernel takes hidden widths that are multiples of 128 (or 0)
    const int W = L / 32, npairs = (W + 1) / 2;
    const int act_dim = hidden > 0 ? hidden : kHeadDim;
    *w1_elems = static_cast<size_t>((hidden + kThreads - 1) / kThreads) * kThreads * kHeadDim;
    *out_elems = static_cast<size_t>(npairs) * 64 * act_dim;
}

int launch_pack_weights(spotlight_ctx* ctx, const void* w1, const void* w2, int w_dtype, void* pack_w1, void* pack_out)
{
    const Plan& p = ctx->plan;
    const int64_t groups = static_cast<int64_t>(p.Hkv) * (p.pack_w1_elems + p.pack_out_elems) / 8;
    if (groups <= 0) return SPOTLIGHT_OK;
    const void* wout = p.hidden > 0 ? w2 : w1;
    const dim3 grid(static_cast<unsigned>((groups + kThreads - 1) / kThreads));
    if (w_dtype == SPOTLIGHT_BF16)
        hipLaunchKernelGGL(pack_weights_kernel<bf16_raw>, grid, dim3(kThreads), 0, ctx->stream, static_cast<const bf16_raw*>(w1),
                           static_cast<const bf16_raw*>(wout), static_cast<bf16_raw*>(pack_w1), static_cast<bf16_raw*>(pack_out),
                           p.Hkv, p.hidden, p.L);
    else
        hipLaunchKernelGGL(pack_weights_kernel<float>, grid, dim3(kThreads), 0, ctx->stream, static_cast<const float*>(w1),
                           static_cast<const float*>(wout), static_cast<float*>(pack_w1), static_cast<float*>(pack_out), p.Hkv,
                           p.hidden, p.L);
    return hip_rc(hipGetLastError());
}

int launch_hash(spotlight_ctx* ctx, const HashLaunch& h, int stage)
{
    if (h.n_rows <= 0 || h.n_xheads <= 0) return SPOTLIGHT_OK;
    // the weight rows are read 8 elements at a time
    if (h.hidden % 8 != 0) return SPOTLIGHT_ERR_UNSUPPORTED;
    const HashArgs a = make_hash_args(h);
    const bool xb = h.x_dtype == SPOTLIGHT_BF16, wb = h.w_dtype == SPOTLIGHT_BF16;
    if (xb && wb) return run_tk<bf16_raw, bf16_raw>(ctx, a, h.n_xheads, stage);
    if (xb && !wb) return run_tk<bf16_raw, float>(ctx, a, h.n_xheads, stage);
    if (!xb && wb) return run_tk<float, bf16_raw>(ctx, a, h.n_xheads, stage);
    return run_tk<float, float>(ctx, a, h.n_xheads, stage);
}

int launch_hash_pair(spotlight_ctx* ctx, const HashLaunch& h0, const HashLaunch& h1, int stage)
{
    const bool one_launch = h0.n_rows == 1 && h1.n_rows == 1 && h0.n_xheads > 0 && h1.n_xheads > 0 &&
                            h0.hidden == h1.hidden && h0.hidden % kHeadDim == 0 && h0.L == h1.L &&
                            h0.x_dtype == h1.x_dtype && h0.w_dtype == h1.w_dtype;
    if (!one_launch) {
        const int rc = launch_hash(ctx, h0, stage);
        return rc != SPOTLIGHT_OK ? rc : launch_hash(ctx, h1, stage);
    }
    const HashArgs a = make_hash_args(h0), b = make_hash_args(h1);
    const bool xb = h0.x_dtype == SPOTLIGHT_BF16, wb = h0.w_dtype == SPOTLIGHT_BF16;
    if (xb && wb) return run_vec<bf16_raw, bf16_raw>(ctx, a, h0.n_xheads, &b, h1.n_xheads, stage);
    if (xb && !wb) return run_vec<bf16_raw, float>(ctx, a, h0.n_xheads, &b, h1.n_xheads, stage);
    if (!xb && wb) return run_vec<float, bf16_raw>(ctx, a, h0.n_xheads, &b, h1.n_xheads, stage);
    return run_vec<float, float>(ctx, a, h0.n_xheads, &b, h1.n_xheads, stage);
}

}  // namespace spotlight
