// Hamming scoring and per-head top-k (paper Sec. 3.2, Eq. 3 and the top-k that follows it).
//
// Distances are integers in 0..L, so the k nearest tokens are found by counting, not sorting, and
// the key codes are streamed from HBM exactly once:
//
//   score   one workgroup per (batch, key-value head, block of 4096 tokens) reads the packed key
//           codes of its block, XORs them with the G query codes of the group and popcounts; the
//           16 distances of each thread stay in registers.  The block counts them in an LDS
//           histogram (replicated over lanes so that same-address atomics stay apart), turns it
//           into a cumulative histogram and adds it to a running one that covers the blocks of
//           the head the workgroup has counted so far (its "run" of consecutive blocks).  The
//           running histogram is stored per block, and once per run added to the cumulative
//           histogram of the head (integer atomics).  It then keeps a short list of CANDIDATES:
//           the tokens up to a block-local distance bound chosen so that about twice the block's
//           fair share of k qualifies (one sub-list per wavefront).  Nothing else is written per
//           token.  Workgroups are persistent and fetch the next keys before finishing a block.
//   select  one workgroup per (query head, block).  The head's cumulative histogram gives the
//           exact threshold T with count(d < T) < k <= count(d <= T) and r = k - count(d < T),
//           the number of tokens to take from the tie bucket d == T.  The stored histograms of
//           the block in front (same run) and of the last block of every run before give this
//           block's own counts, its output offset and its share of the tie bucket (ties go to
//           the lower token index).  If T is within the block's candidate bound, the
//           block's tokens with d <= T are all in its list; otherwise (rare) the block recomputes
//           its distances from the codes.  Selected tokens are marked in an LDS bitmap and written
//           out in increasing token order.
//
// The result is exactly the first k tokens in (distance, token index) order, listed by increasing
// token index, with integer arithmetic only: identical bits on every run.
//
// Forced tokens (the first n_sink and the last n_local of the cache: the "Sink" and "Local"
// columns of the paper's comparison with MagicPIG; a local window of one is the current token that
// Eq. 1 concatenates) use the same machinery: every histogram has one bin below distance 0.  A
// token is counted in bin 0 if it is forced and in bin distance + 1 otherwise, so forced tokens
// sort in front of everything else and the selection is "forced tokens, then the nearest of the
// others", k in all.  The shift costs nothing (it is a constant in the LDS address), and only the
// few blocks that hold forced tokens do extra work: score re-reads their forced tokens and moves
// them from the bin of their distance to bin 0, select marks them by position.
#pragma once
// Kernel templates and launchers; included by retrieve.hip (dispatch) and by the retrieve_w*.hip
// translation units, each of which instantiates a few code lengths (so that they compile side by side).
#include "internal.h"

#include <type_traits>

namespace spotlight {
namespace retrieve_detail {

constexpr int kTPB = kTokensPerBlock;       // tokens per workgroup
constexpr int kKPT = kTPB / kThreads;       // keys per thread (16)

constexpr int kWaveCap = kCandCap / (kThreads / 64);  // entries of one wavefront's candidate sub-list (256)
constexpr int kWaveFull = 255;              // count value meaning "this sub-list overflowed"
constexpr int kLongRun = 16;                // blocks per resident workgroup from which runs are cut short
constexpr int kShortRun = 4;

// Per (query head, token block): the block's candidate bound (a bin, low kBoundBits bits), the
// first block of the run of blocks its workgroup counted together (the bits above), and the four
// sub-list lengths.
constexpr int kBoundBits = 11;   // bins go up to 32 * 32 + 1
struct BlockMeta {
    uint32_t bound_run;
    uint8_t count[kThreads / 64];
};
static_assert(sizeof(BlockMeta) == 8, "workspace layout");

__device__ __forceinline__ int popc(uint32_t x) { return __builtin_popcount(x); }

// One key (W words) at base + lane_off bytes; base is uniform over the wavefront, so the address is
// a scalar base plus a 32-bit lane offset.  Codes are read once: non-temporal loads.
template <int W>
__device__ __forceinline__ void load_key(const char* __restrict__ base, uint32_t lane_off, uint32_t (&kw)[W])
{
    if constexpr (W % 4 == 0) {
#pragma unroll
        for (int w4 = 0; w4 < W / 4; ++w4) {
            const uint4* src = reinterpret_cast<const uint4*>(base + lane_off + w4 * 16);
            kw[w4 * 4 + 0] = __builtin_nontemporal_load(&src->x);
            kw[w4 * 4 + 1] = __builtin_nontemporal_load(&src->y);
            kw[w4 * 4 + 2] = __builtin_nontemporal_load(&src->z);
            kw[w4 * 4 + 3] = __builtin_nontemporal_load(&src->w);
        }
    } else {
        const uint32_t* src = reinterpret_cast<const uint32_t*>(base + lane_off);
#pragma unroll
        for (int w = 0; w < W; ++w) kw[w] = __builtin_nontemporal_load(src + w);
    }
}

// Sum of x over the LPK (1, 2, 4 or 8) adjacent lanes that share a key: data-parallel-primitive
// moves within a group of four lanes, then between the two fours of a group of eight; no LDS traffic.
template <int LPK>
__device__ __forceinline__ uint32_t add_across_key(uint32_t x)
{
    if constexpr (LPK >= 2)   // lanes 1 0 3 2
        x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0xB1, 0xf, 0xf, true));
    if constexpr (LPK >= 4)   // lanes 2 3 0 1
        x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x4E, 0xf, 0xf, true));
    if constexpr (LPK >= 8)   // lanes 7 6 5 4 3 2 1 0 (every lane of a four holds that four's sum by now)
        x += static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(x), 0x141, 0xf, 0xf, true));
    static_assert(LPK == 1 || LPK == 2 || LPK == 4 || LPK == 8, "a key spans at most eight lanes");
    return x;
}

// ------------------------------------------------------------------------------------ score
struct ScoreArgs {
    const uint32_t* codes;
    const uint32_t* qcode;
    uint32_t* gcum;
    uint32_t* blockcum;
    BlockMeta* blockmeta;
    uint32_t* cand;
    int64_t n_tokens, Nmax;
    int64_t n_sink, local_begin;   // token t is forced iff t < n_sink or t >= local_begin
    int Hkv, nblk, max_blocks, k, total_tasks, tasks_per_group;
};

// Wavefronts per SIMD the register allocation must leave room for.  Without the hint the allocator
// lands on either side of an occupancy step depending on unrelated code (256-bit codes with four
// heads per group: 4 waves measured 4 % faster than 3; 512-bit codes: 167 or 256 registers).
constexpr int score_min_waves(int W, int G) { return (W == 8 && G == 4) ? 4 : (W == 16 && G <= 4) ? 3 : 1; }

// Persistent workgroups.  A task is one (batch * kv head, token block); a workgroup takes
// tasks_per_group CONSECUTIVE tasks, which mostly belong to one head, and keeps that head's
// cumulative histogram in LDS across them, so the (slow, device-wide) atomics into the head's
// global histogram happen once per run of tasks instead of once per block.
template <int W, int G, int R>
__global__ __launch_bounds__(kThreads, score_min_waves(W, G)) void score_kernel(ScoreArgs a)
{
    constexpr int L = W * 32;
    constexpr int BINS = L + 2;            // bin 0: forced tokens; bin d + 1: distance d
    constexpr int CH = (BINS + 63) / 64;   // bins per lane in the scan
    // lanes per key: 16 bytes per lane when the code is 16, 32, 64 or 128 bytes, else one lane per key
    constexpr int LPK = (W == 4 || W == 8 || W == 16 || W == 32) ? W / 4 : 1;
    constexpr int CWL = W / LPK;           // code words per lane
    constexpr int SLOTS = kKPT * LPK;      // load instructions per thread and task
    constexpr int KPS = kThreads / LPK;    // keys per slot
    constexpr int KB = CWL <= 4 ? 4 : (CWL <= 8 ? 2 : 1);  // slots per batch of loads
    __shared__ uint32_t hist[G * BINS * R];
    __shared__ uint32_t cum[G * BINS];     // this block's histogram, then its cumulative form
    __shared__ uint32_t gacc[G * BINS];    // cumulative histogram summed over this run of tasks
    __shared__ uint32_t s_thi[G];
    __shared__ uint32_t escr[kThreads / 64][kKPT / 2][64];   // per-lane copy of one head's packed distances

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int rep = (tid / LPK) & (R - 1);   // the lanes of one key never record the same slot
    const int Hq = a.Hkv * G;
    const uint32_t lane_off = static_cast<uint32_t>(tid) * (CWL * 4);
    const int sub = tid % LPK, kq = tid / LPK;   // part of the key this lane reads, key within a slot

    for (int i = tid; i < G * BINS * R; i += kThreads) hist[i] = 0;
    for (int i = tid; i < G * BINS; i += kThreads) gacc[i] = 0;
    __syncthreads();

    const int task0 = blockIdx.x * a.tasks_per_group;
    const int task1 = min(a.total_tasks, task0 + a.tasks_per_group);

    // Loads run one batch (KB slots) ahead of the arithmetic, in two register buffers that swap
    // roles; the first batch of a task is fetched during the epilogue of the task in front of it
    // and is always in buf[0] (the number of batches is even).  Full blocks load unpredicated.
    // Groups of four or eight heads keep too many distances in registers for a second buffer (it
    // measured slower): they load each batch right before using it.
    constexpr int NB = SLOTS / KB;
    constexpr bool AHEAD = G <= 2;
    static_assert(NB % 2 == 0, "the first batch of every task lands in buf[0]");
    uint32_t buf[AHEAD ? 2 : 1][KB][CWL];
    auto fetch = [&](auto full, int t, int bt, uint32_t (&dst)[KB][CWL]) {
        const int bk = t / a.nblk, blk = t % a.nblk;
        const int64_t t_begin = static_cast<int64_t>(blk) * kTPB;
        const int n_blk = static_cast<int>(min(static_cast<int64_t>(kTPB), a.n_tokens - t_begin));
        const char* base = reinterpret_cast<const char*>(a.codes + (static_cast<int64_t>(bk) * a.Nmax + t_begin) * W);
#pragma unroll
        for (int u = 0; u < KB; ++u) {
            const int sl = bt * KB + u;
            if (decltype(full)::value || sl * KPS + kq < n_blk)
                load_key<CWL>(base + static_cast<size_t>(sl) * (kThreads * CWL * 4), lane_off, dst[u]);
        }
    };
    if (AHEAD && task0 < task1) fetch(std::false_type{}, task0, 0, buf[0]);

    int run_begin = 0;   // first block of the current run: consecutive blocks of one head counted by this workgroup
    for (int task = task0; task < task1; ++task) {
        const int bk = task / a.nblk, blk = task % a.nblk;
        const int b = bk / a.Hkv, hk = bk % a.Hkv;
        const int64_t bh0 = static_cast<int64_t>(b) * Hq + hk * G;  // first query head of the group
        const int64_t t_begin = static_cast<int64_t>(blk) * kTPB;
        const int n_blk = static_cast<int>(min(static_cast<int64_t>(kTPB), a.n_tokens - t_begin));
        if (task == task0 || blk == 0) run_begin = blk;   // gacc starts from zero here
        // this lane's part of the G query codes (the whole code when a lane owns whole keys)
        uint32_t qc[G][CWL];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int w = 0; w < CWL; ++w) qc[g][w] = a.qcode[(bh0 + g) * W + sub * CWL + w];

        // Forced tokens of this block, as offsets into it: [0, sink_end) and [local_off, n_blk).
        // Only the first and the last blocks of a head have any; such a block takes the predicated
        // path of the main loop, which counts a slot (KPS consecutive tokens) that is forced as a
        // whole in bin 0 directly.  The forced tokens of the one or two slots that are only partly
        // forced are counted at the bin of their distance like every other token and moved to bin
        // 0 here (the subtraction comes first: the counters wrap and come back).  The candidate
        // lists never hold forced tokens on purpose; select knows them by position.
        const int sink_end = static_cast<int>(max(static_cast<int64_t>(0), min(static_cast<int64_t>(n_blk), a.n_sink - t_begin)));
        const int local_off = max(sink_end,   // windows that meet: every token once
            static_cast<int>(max(static_cast<int64_t>(0), min(static_cast<int64_t>(n_blk), a.local_begin - t_begin))));
        const bool has_forced = sink_end > 0 || local_off < n_blk;
        // whole slots inside the windows: slots [0, sink_slots) and [local_slot, SLOTS)
        const int sink_slots = sink_end / KPS, local_slot = (local_off + KPS - 1) / KPS;
        if (has_forced) {
            const char* blk_base = reinterpret_cast<const char*>(a.codes + (static_cast<int64_t>(bk) * a.Nmax + t_begin) * W);
            auto move_to_bin0 = [&](int lo, int hi) {   // fewer than KPS tokens: at most one per thread
                for (int off = lo + tid; off < hi; off += kThreads) {
                    constexpr int CHUNK = W % 4 == 0 ? 4 : 1;   // words per load
                    uint32_t d[G];
#pragma unroll
                    for (int g = 0; g < G; ++g) d[g] = 0;
#pragma unroll 1
                    for (int w0 = 0; w0 < W; w0 += CHUNK) {
                        uint32_t key[CHUNK];
                        load_key<CHUNK>(blk_base, static_cast<uint32_t>(off) * (W * 4) + w0 * 4, key);
#pragma unroll
                        for (int g = 0; g < G; ++g)
#pragma unroll
                            for (int w = 0; w < CHUNK; ++w) d[g] += popc(key[w] ^ a.qcode[(bh0 + g) * W + w0 + w]);
                    }
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        atomicSub(&hist[(g * BINS + 1 + d[g]) * R + rep], 1u);
                        atomicAdd(&hist[(g * BINS + 0) * R + rep], 1u);
                    }
                }
            };
            move_to_bin0(sink_slots * KPS, sink_end);
            move_to_bin0(local_off, min(n_blk, local_slot * KPS));
        }

        // distances of the 16 keys this lane owns, two per register
        uint32_t dv[G][kKPT / 2];
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int i = 0; i < kKPT / 2; ++i) dv[g][i] = 0x7fff7fffu;   // absent keys: farther than any bound

        // A "slot" is one load instruction of the workgroup: KPS = 256 / LPK keys, LPK adjacent lanes
        // per key, 16 bytes per lane (fully coalesced).  The partial distances of a key are added
        // across its LPK lanes; lane `sub` of the key keeps the slots with s % LPK == sub, so every
        // lane ends up owning 16 keys: key j of a lane is slot j * LPK + sub, token offset
        // (j * LPK + sub) * KPS + kq.
        auto score_block = [&](auto full) {
#pragma unroll
        for (int bt = 0; bt < NB; ++bt) {
            uint32_t (&kw)[KB][CWL] = buf[AHEAD ? bt & 1 : 0];
            if constexpr (!AHEAD) fetch(full, task, bt, buf[0]);
            else if (bt + 1 < NB) fetch(full, task, bt + 1, buf[(bt + 1) & 1]);
            else if (task + 1 < task1) fetch(std::false_type{}, task + 1, 0, buf[0]);   // in flight during the epilogue
#pragma unroll
            for (int u = 0; u < KB; ++u) {
                const int sl = bt * KB + u;
                const bool valid = decltype(full)::value || sl * KPS + kq < n_blk;
                uint32_t d[G];   // distances; the histogram bin is d + 1
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    d[g] = 0;
#pragma unroll
                    for (int w = 0; w < CWL; ++w) d[g] += popc(kw[u][w] ^ qc[g][w]);
                    d[g] = add_across_key<LPK>(d[g]);
                }
                if constexpr (!decltype(full)::value) {
                    if (sl < sink_slots || sl >= local_slot) {   // a slot of forced tokens (uniform): bin 0
#pragma unroll
                        for (int g = 0; g < G; ++g) d[g] = 0xffffffffu;
                    }
                }
                if (valid && (LPK == 1 || sub == sl % LPK)) {
                    const int j = sl / LPK;   // index among the keys this lane owns
#pragma unroll
                    for (int g = 0; g < G; ++g) {
                        atomicAdd(&hist[(g * BINS + 1 + d[g]) * R + rep], 1u);
                        if constexpr (decltype(full)::value) {   // both halves get written: no mask needed
                            dv[g][j >> 1] = (j & 1) ? (d[g] << 16) | dv[g][j >> 1] : d[g];
                        } else {
                            const uint32_t d16 = d[g] & 0x7fffu;   // a forced slot's 0xffffffff: never a candidate
                            if (j & 1) dv[g][j >> 1] = (dv[g][j >> 1] & 0x0000ffffu) | (d16 << 16);
                            else dv[g][j >> 1] = (dv[g][j >> 1] & 0xffff0000u) | d16;
                        }
                    }
                }
            }
        }
        };
        if (n_blk == kTPB && !has_forced) score_block(std::true_type{});
        else score_block(std::false_type{});

        __syncthreads();

        // fold the replicas (rotated so that neighbouring threads hit different banks)
        for (int i = tid; i < G * BINS; i += kThreads) {
            uint32_t s = 0;
#pragma unroll
            for (int r = 0; r < R; ++r) s += hist[i * R + ((r + i) & (R - 1))];
            cum[i] = s;
        }
        __syncthreads();
        for (int i = tid; i < G * BINS * R; i += kThreads) hist[i] = 0;  // ready for the next task

        // cumulative histogram per head (one wave per head), and the block-local candidate bound:
        // the first bin at which about twice the block's fair share of k (plus a little) is reached,
        // counting only tokens outside the forced windows (bin 0 is not a distance; select places
        // forced tokens by position and needs no candidates for them)
        const uint32_t want = static_cast<uint32_t>(min(static_cast<int64_t>(n_blk),
            (static_cast<int64_t>(n_blk) * a.k * 2 + a.n_tokens - 1) / a.n_tokens + 32));
        for (int g = wave; g < G; g += kThreads / 64) {
            uint32_t v[CH];
            uint32_t tot = 0;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int bin = lane * CH + c;
                tot += bin < BINS ? cum[g * BINS + bin] : 0u;
                v[c] = tot;
            }
            const uint32_t before = wave_inclusive_scan(tot) - tot;
            const uint32_t c0 = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(v[0])));   // bin 0
            const uint32_t wantn = min(want, static_cast<uint32_t>(n_blk) - c0);
            if (lane == 0 && wantn == 0) s_thi[g] = BINS - 1;   // nothing but forced tokens: no candidate either way
            uint32_t prev = before;
#pragma unroll
            for (int c = 0; c < CH; ++c) {
                const int bin = lane * CH + c;
                if (bin < BINS) {
                    const uint32_t cv = before + v[c];
                    cum[g * BINS + bin] = cv;
                    gacc[g * BINS + bin] += cv;
                    if (bin > 0 && wantn > 0 && cv - c0 >= wantn && prev - c0 < wantn) s_thi[g] = static_cast<uint32_t>(bin);  // exactly one bin
                    prev = cv;
                }
            }
        }
        __syncthreads();

        // publish: the cumulative histogram of the run up to and including this block (contiguous
        // store; select takes differences of neighbouring blocks and sums over the runs in front,
        // instead of summing over every block in front), and, at the end of a run, the same
        // numbers into the head's global histogram
        const bool flush = task + 1 == task1 || (task + 1) / a.nblk != bk;
        for (int i = tid; i < G * BINS; i += kThreads) {
            const int g = i / BINS, bin = i % BINS;
            const uint32_t v = gacc[i];
            a.blockcum[((bh0 + g) * a.max_blocks + blk) * BINS + bin] = v;
            if (flush) {
                if (v) atomicAdd(&a.gcum[(bh0 + g) * BINS + bin], v);
                gacc[i] = 0;
            }
        }

        // Candidate lists, one sub-list per wavefront, in any fixed order.  Few keys qualify (a few
        // per cent), so the work is arranged per qualifying key, not per key: a packed 16-bit
        // subtraction per register marks the keys below the bound in a per-lane bit mask, a wave scan
        // of the mask populations gives every lane its place in the sub-list, and the lanes then
        // write their keys one per round (the longest mask of the wave sets the number of rounds).
        // The distance of the key a round picks comes back from a per-lane copy of the registers in
        // LDS, since registers cannot be indexed per lane.
        typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
        typedef uint16_t __attribute__((may_alias)) u16_view;   // halves of the 32-bit words written below
        static_assert(kKPT == 16, "the bit layout of the mask assumes eight registers of two keys");
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const uint32_t thi = __builtin_amdgcn_readfirstlane(s_thi[g]);   // a bin: bound on distance + 1
            const int64_t slot = (bh0 + g) * a.max_blocks + blk;
            uint32_t* cl = a.cand + (slot * (kThreads / 64) + wave) * kWaveCap;
            const u16x2 thi2 = __builtin_bit_cast(u16x2, thi | (thi << 16));
            uint32_t q = 0;   // bit 7 - r: low key of register r qualifies; bit 23 - r: high key
#pragma unroll
            for (int r = 0; r < kKPT / 2; ++r) {
                // d - thi in 16 bits: bit 15 set exactly when d < thi (d <= 0x7fff, thi <= L + 1)
                const uint32_t t = __builtin_bit_cast(uint32_t, __builtin_bit_cast(u16x2, dv[g][r]) - thi2);
                q = (q << 1) | ((t >> 15) & 0x00010001u);
                escr[wave][r][lane] = dv[g][r];
            }
            const uint32_t mine = popc(q);
            const uint32_t incl = wave_inclusive_scan(mine);
            const uint32_t total = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(incl), 63));
            uint32_t at = incl - mine;
            while (__ballot(q != 0)) {
                if (q) {
                    const int bit = __builtin_ctz(q);
                    q &= q - 1;
                    const int r = 7 - (bit & 15), half = bit >> 4;
                    const uint32_t d = reinterpret_cast<const u16_view*>(&escr[wave][r][lane])[half];
                    const int j = 2 * r + half;   // index among the keys this lane owns
                    if (at < static_cast<uint32_t>(kWaveCap))
                        cl[at] = (d << 16) + (0x10000u | static_cast<uint32_t>((j * LPK + sub) * KPS + kq));   // bin << 16 | offset
                    ++at;
                }
            }
            if (lane == 0) {
                BlockMeta* bm = a.blockmeta + slot;
                bm->count[wave] = total < static_cast<uint32_t>(kWaveFull) ? static_cast<uint8_t>(total) : static_cast<uint8_t>(kWaveFull);
                if (wave == 0) bm->bound_run = thi | (static_cast<uint32_t>(run_begin) << kBoundBits);
            }
        }
        // the next task's first barrier orders these reads of cum / s_thi / gacc before their reuse
    }
}

// ------------------------------------------------------------------------------------ select
// Workgroup sizes of the select kernel.  Two wavefronts per block (one thread per 32 tokens) have the
// shorter dependent chain; one wavefront (one thread per 64 tokens) lets twice as many blocks be
// resident per compute unit, which wins once the grid needs several rounds to pass through the chip.
constexpr int kSelThreads = 128;
constexpr int kSelThreadsNarrow = 64;
constexpr int kSelWideGrid = 256 * 16;   // workgroups of kSelThreads resident on the chip at once

template <int TOK> struct TokenMask { using type = uint32_t; };
template <> struct TokenMask<64> { using type = uint64_t; };
__device__ __forceinline__ uint32_t popc_m(uint32_t x) { return static_cast<uint32_t>(__builtin_popcount(x)); }
__device__ __forceinline__ uint32_t popc_m(uint64_t x) { return static_cast<uint32_t>(__builtin_popcountll(x)); }
__device__ __forceinline__ int ctz_m(uint32_t x) { return __builtin_ctz(x); }
__device__ __forceinline__ int ctz_m(uint64_t x) { return __builtin_ctzll(x); }
__device__ __forceinline__ uint32_t drop_highest(uint32_t x) { return x & ~(0x80000000u >> __builtin_clz(x)); }
__device__ __forceinline__ uint64_t drop_highest(uint64_t x) { return x & ~(0x8000000000000000ull >> __builtin_clzll(x)); }
// bits i of a 32-token bitmap word starting at token `first` with first + i < bound
__device__ __forceinline__ uint32_t bits_below(uint32_t first, uint32_t bound)
{
    if (bound <= first) return 0u;
    const uint32_t n = bound - first;
    return n >= 32 ? 0xffffffffu : (1u << n) - 1u;
}

// FORCED: the call has sink / local tokens (otherwise that code is compiled out).
template <int W, bool FORCED, int THREADS>
__global__ __launch_bounds__(THREADS) void select_kernel(
    const uint32_t* __restrict__ codes, const uint32_t* __restrict__ qcode, const uint32_t* __restrict__ gcum,
    const uint32_t* __restrict__ blockcum, const BlockMeta* __restrict__ blockmeta, const uint32_t* __restrict__ cand,
    int32_t* __restrict__ out_idx, int64_t n_tokens, int64_t Nmax, int Hq, int Hkv, int max_blocks, int k,
    int64_t n_sink, int64_t local_begin, int tasks_per_group)
{
    constexpr int BINS = W * 32 + 2;   // bin 0: forced tokens; bin d + 1: distance d
    constexpr int NW = THREADS / 64;
    constexpr int SUB = kThreads / 64;          // candidate sub-lists per block
    constexpr int PER = kWaveCap / THREADS;     // sub-list entries per thread
    constexpr int WORDS = kTPB / 32;            // bitmap words of a block
    constexpr int TOK = kTPB / THREADS;         // tokens owned by a thread
    constexpr int WPT = TOK / 32;               // bitmap words owned by a thread
    static_assert(NW == 1 || NW == 2, "one or two wavefronts");
    static_assert(TOK == 32 || TOK == 64, "a thread's tokens fit one mask");
    using mask_t = typename TokenMask<TOK>::type;
    constexpr uint32_t kDenseOutput = 512;
    constexpr uint32_t kDenseChunk = 1024;
    __shared__ uint32_t s_T, s_r;
    __shared__ uint32_t red[3][2];
    __shared__ uint32_t lt_bits[WORDS], eq_bits[WORDS];
    __shared__ uint32_t wsum[NW];
    __shared__ uint16_t dense[kDenseChunk];   // offsets of selected tokens, for blocks selected almost whole

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t bh = blockIdx.y;
    const int blk = blockIdx.x;
    const uint32_t* gc = gcum + bh * BINS;
    const uint32_t* bc = blockcum + bh * max_blocks * BINS;
    const int64_t slot = bh * max_blocks + blk;
    // The candidate entries are fetched before the threshold is known, so that their latency
    // overlaps the threshold search; the first THREADS of every sub-list (which is all of it unless
    // the block is unusually dense) even before the sub-list lengths are known.  Entries past a
    // sub-list's length hold whatever the workspace held: they are never looked at.
    uint32_t ce[SUB][PER];
#pragma unroll
    for (int s = 0; s < SUB; ++s) ce[s][0] = cand[(slot * SUB + s) * kWaveCap + tid];
    const BlockMeta meta = blockmeta[slot];
#pragma unroll
    for (int s = 0; s < SUB; ++s)
#pragma unroll
        for (int h = 1; h < PER; ++h) {
            ce[s][h] = 0;
            if (meta.count[s] != kWaveFull && h * THREADS + tid < static_cast<int>(meta.count[s]))
                ce[s][h] = cand[(slot * SUB + s) * kWaveCap + h * THREADS + tid];
        }

#pragma unroll
    for (int i = 0; i < WPT; ++i) {
        lt_bits[i * THREADS + tid] = 0;
        eq_bits[i * THREADS + tid] = 0;
    }
#pragma unroll 4
    for (int bin = tid; bin < BINS; bin += THREADS) {
        const uint32_t c = gc[bin];
        const uint32_t p = bin ? gc[bin - 1] : 0u;
        // exactly one bin qualifies for a consistent histogram; the last bin also takes the case "never
        // reaches k", so T is a valid bin whatever the workspace holds
        if ((c >= static_cast<uint32_t>(k) || bin == BINS - 1) && p < static_cast<uint32_t>(k)) {
            s_T = bin;
            s_r = static_cast<uint32_t>(k) - p;
        }
    }
    __syncthreads();
    const uint32_t T = s_T, r = s_r;

    // The rows of `bc` are cumulative over the blocks of a run (the consecutive blocks of the head
    // that one score workgroup counted).  This block's own counts are its row minus the row in
    // front (within the run); the tokens below T and in the tie bucket in all blocks before this
    // one are that row in front plus the last rows of the runs before this one.  Every run between
    // the head's first and this one is tasks_per_group blocks long, so those last rows are
    // tasks_per_group apart.  All requested together.
    const int rb = min(static_cast<int>(meta.bound_run >> kBoundBits), blk);   // first block of this block's run
    const uint32_t cur_le = bc[static_cast<int64_t>(blk) * BINS + T];
    const uint32_t cur_lt = T ? bc[static_cast<int64_t>(blk) * BINS + T - 1] : 0u;
    // thread 0 takes the row in front, thread m >= 1 the last row of the m-th run before this one
    uint32_t lt = 0, eq = 0;
    const int step = min(tasks_per_group, blk + 1);   // a longer step leaves the head at once anyway
    int j = tid == 0 ? (blk > rb ? blk - 1 : -1) : rb - 1 - (tid - 1) * step;
    uint32_t first_le = 0, first_lt = 0;   // what thread 0 read
    if (j >= 0) {
        first_le = bc[static_cast<int64_t>(j) * BINS + T];
        first_lt = T ? bc[static_cast<int64_t>(j) * BINS + T - 1] : 0u;
        lt = first_lt;
        eq = first_le - first_lt;
    }
    // more than THREADS - 1 runs in front: the THREADS - 1 threads that walk them go round again
    for (j = tid == 0 ? -1 : j - (THREADS - 1) * step; j >= 0; j -= (THREADS - 1) * step) {
        const uint32_t le = bc[static_cast<int64_t>(j) * BINS + T];
        const uint32_t l = T ? bc[static_cast<int64_t>(j) * BINS + T - 1] : 0u;
        lt += l;
        eq += le - l;
    }
    uint32_t prev_le = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(first_le)));
    uint32_t prev_lt = static_cast<uint32_t>(__builtin_amdgcn_readfirstlane(static_cast<int>(first_lt)));
    lt = wave_sum(lt);
    eq = wave_sum(eq);
    if constexpr (NW > 1) {
        if (lane == 0) { red[0][wave] = lt; red[1][wave] = eq; }
        if (tid == 0) { red[2][0] = first_le; red[2][1] = first_lt; }
        __syncthreads();
        lt = red[0][0] + red[0][1];
        eq = red[1][0] + red[1][1];
        prev_le = red[2][0];
        prev_lt = red[2][1];
    }
    const uint32_t own_le = cur_le - prev_le;
    const uint32_t own_lt = cur_lt - prev_lt;
    const uint32_t own_eq = own_le - own_lt;
    // Ties go to earlier blocks first.  Written without any subtraction that could wrap.
    const uint32_t taken_before = eq < r ? eq : r;              // ties taken by the blocks before
    const uint32_t left = r - taken_before;                     // ties still to hand out
    const uint32_t quota = left < own_eq ? left : own_eq;       // ties this block may take
    uint32_t pos = lt + taken_before;                           // output offset of this block
    if (own_lt + quota == 0) return;                            // uniform over the workgroup

    const int64_t t_begin = static_cast<int64_t>(blk) * kTPB;
    const int n_blk = static_cast<int>(min(static_cast<int64_t>(kTPB), n_tokens - t_begin));
    // forced tokens of this block, as offsets into it: [0, sink_end) and [local_off, n_blk)
    const uint32_t sink_end = !FORCED ? 0u :
        static_cast<uint32_t>(max(static_cast<int64_t>(0), min(static_cast<int64_t>(n_blk), n_sink - t_begin)));
    const uint32_t local_off = !FORCED ? static_cast<uint32_t>(n_blk) :
        static_cast<uint32_t>(max(static_cast<int64_t>(0), min(static_cast<int64_t>(n_blk), local_begin - t_begin)));
    bool listed = T <= (meta.bound_run & ((1u << kBoundBits) - 1));
#pragma unroll
    for (int s = 0; s < SUB; ++s) listed = listed && meta.count[s] != kWaveFull;
    if (listed) {
#pragma unroll
        for (int s = 0; s < SUB; ++s)
#pragma unroll
            for (int h = 0; h < PER; ++h) {
                if (h * THREADS + tid < static_cast<int>(meta.count[s])) {
                    const uint32_t off = ce[s][h] & (kTPB - 1);
                    const uint32_t d = (FORCED && (off < sink_end || off >= local_off)) ? 0u : ce[s][h] >> 16;   // forced: bin 0
                    if (d < T) atomicOr(&lt_bits[off >> 5], 1u << (off & 31));
                    else if (d == T) atomicOr(&eq_bits[off >> 5], 1u << (off & 31));
                }
            }
    } else {
        // recompute this block's distances from the codes
        const int G = Hq / Hkv;
        const int b = static_cast<int>(bh / Hq), hq = static_cast<int>(bh % Hq);
        const char* cbase = reinterpret_cast<const char*>(codes + ((static_cast<int64_t>(b) * Hkv + hq / G) * Nmax + t_begin) * W);
        uint32_t qc[W];
#pragma unroll
        for (int w = 0; w < W; ++w) qc[w] = qcode[bh * W + w];
        constexpr int U = W <= 4 ? 8 : (W <= 8 ? 4 : (W <= 16 ? 2 : 1));   // keys in flight per thread (within 64 registers)
        for (int off0 = tid; off0 < n_blk; off0 += THREADS * U) {
            uint32_t kw[U][W];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int off = off0 + u * THREADS;
                if (off < n_blk) load_key<W>(cbase, static_cast<uint32_t>(off) * (W * 4), kw[u]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int off = off0 + u * THREADS;   // a wavefront holds 64 consecutive offsets
                uint32_t d = 1;
#pragma unroll
                for (int w = 0; w < W; ++w) d += popc(kw[u][w] ^ qc[w]);
                if (FORCED && (static_cast<uint32_t>(off) < sink_end || static_cast<uint32_t>(off) >= local_off)) d = 0;
                // one bitmap word per 32 lanes, written by one of them (32 lanes OR-ing single bits
                // into the same LDS word serialise: 85 us for a block that is all below T)
                const unsigned long long mlt = __ballot(off < n_blk && d < T);
                const unsigned long long meq = __ballot(off < n_blk && d == T);
                if ((lane & 31) == 0 && off < n_blk) {
                    const uint32_t wlt = static_cast<uint32_t>(lane ? mlt >> 32 : mlt);
                    const uint32_t weq = static_cast<uint32_t>(lane ? meq >> 32 : meq);
                    if (wlt) atomicOr(&lt_bits[off >> 5], wlt);
                    if (weq) atomicOr(&eq_bits[off >> 5], weq);
                }
            }
        }
    }
    // forced tokens are in bin 0 whether or not a list names them: marked by position
    if (FORCED && (sink_end > 0 || local_off < static_cast<uint32_t>(n_blk))) {
#pragma unroll
        for (int i = 0; i < WPT; ++i) {
            const int word = i * THREADS + tid;
            const uint32_t first = static_cast<uint32_t>(word) * 32;
            const uint32_t m = (bits_below(first, sink_end) | ~bits_below(first, local_off)) &
                               bits_below(first, static_cast<uint32_t>(n_blk));
            if (m) atomicOr(T > 0 ? &lt_bits[word] : &eq_bits[word], m);
        }
    }
    __syncthreads();

    // thread j owns tokens TOK*j .. TOK*j + TOK-1 of the block
    mask_t lw = lt_bits[tid * WPT];
    mask_t ew = eq_bits[tid * WPT];
    if constexpr (WPT == 2) {
        lw |= static_cast<mask_t>(lt_bits[tid * WPT + 1]) << 32;
        ew |= static_cast<mask_t>(eq_bits[tid * WPT + 1]) << 32;
    }
    const uint32_t ecount = popc_m(ew);
    const uint32_t sc = wave_inclusive_scan(ecount);  // tie counts over threads (token order)
    uint32_t eq_before = sc - ecount;
    if constexpr (NW > 1) {
        if (lane == 63) wsum[wave] = sc;
        __syncthreads();
        if (wave == 1) eq_before += wsum[0];
        __syncthreads();  // wsum is reused
    }
    const uint32_t gone = eq_before < quota ? eq_before : quota;  // quota used by earlier threads
    const uint32_t take = (quota - gone) < ecount ? (quota - gone) : ecount;
    while (popc_m(ew) > take) ew = drop_highest(ew);  // drop the highest ties
    mask_t sel = lw | ew;
    const uint32_t cnt = popc_m(sel);
    const uint32_t sn = wave_inclusive_scan(cnt);
    uint32_t local = sn - cnt;                      // place of this thread's first token among the block's
    uint32_t n_sel;                                 // tokens this block contributes (own_lt + quota)
    if constexpr (NW > 1) {
        if (lane == 63) wsum[wave] = sn;
        __syncthreads();
        if (wave == 1) local += wsum[0];
        n_sel = wsum[0] + wsum[1];
    } else {
        n_sel = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(sn), 63));
    }
    int32_t* op = out_idx + bh * k;
    if (n_sel <= kDenseOutput) {
        // the usual case, a few dozen tokens per block: every thread writes its own
        pos += local;
        const int32_t tok0 = static_cast<int32_t>(t_begin) + tid * TOK;
        while (sel) {
            const int bit = ctz_m(sel);
            sel &= sel - 1;
            if (pos < static_cast<uint32_t>(k)) op[pos] = tok0 + bit;
            ++pos;
        }
    } else {
        // a block that is selected almost whole (wide forced windows, k close to N): written thread by
        // thread, every store instruction touches 64 cache lines; through LDS, a chunk of the block's
        // output at a time, the stores are contiguous
        for (uint32_t base = 0; base < n_sel; base += kDenseChunk) {
            while (sel && local < base + kDenseChunk) {
                const int bit = ctz_m(sel);
                sel &= sel - 1;
                dense[local - base] = static_cast<uint16_t>(tid * TOK + bit);
                ++local;
            }
            __syncthreads();
            const uint32_t n_chunk = min(kDenseChunk, n_sel - base);
            for (uint32_t i = tid; i < n_chunk; i += THREADS)
                if (pos + base + i < static_cast<uint32_t>(k)) op[pos + base + i] = static_cast<int32_t>(t_begin) + dense[i];
            __syncthreads();
        }
    }
}

// All distances of every query head, for tests and debugging only.
template <int W>
__global__ __launch_bounds__(kThreads) void dist_kernel(const uint32_t* __restrict__ codes,
                                                        const uint32_t* __restrict__ qcode,
                                                        uint16_t* __restrict__ out, int64_t n_tokens,
                                                        int64_t Nmax, int Hq, int Hkv)
{
    const int64_t bh = blockIdx.y;
    const int64_t t = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
    if (t >= n_tokens) return;
    const int b = static_cast<int>(bh / Hq), hq = static_cast<int>(bh % Hq);
    const uint32_t* p = codes + ((static_cast<int64_t>(b) * Hkv + hq / (Hq / Hkv)) * Nmax + t) * W;
    int d = 0;
#pragma unroll
    for (int w = 0; w < W; ++w) d += popc(p[w] ^ qcode[bh * W + w]);
    out[bh * n_tokens + t] = static_cast<uint16_t>(d);
}

// ------------------------------------------------------------------------------------ dispatch
struct RetrieveArgs {
    const uint32_t* codes;
    int64_t n_tokens;
    int64_t n_sink, local_begin;
    int k, nblk;
    int32_t* out_idx;
    uint16_t* out_dist;
};

template <int W, int G>
int launch_score_wg(spotlight_ctx* ctx, StageTimer& timer, const RetrieveArgs& a, int* tasks_per_group)
{
    const Plan& p = ctx->plan;
    constexpr int BINS = W * 32 + 2;
    // histogram replicas: 8 if they fit in 32 KB of LDS (more did not make the LDS atomics faster
    // and make the per-block fold and re-zero slower), fewer for wide codes and big groups
    // and so that everything (replicas, two more histograms, 8 KB of emission scratch) stays under 64 KB
    constexpr int kCap = 32768;
    constexpr int kRest = G * BINS * 2 * 4 + 8192 + 256;
    constexpr int R = (G * BINS * 8 * 4 <= kCap && G * BINS * 8 * 4 + kRest <= 65536) ? 8
                    : (G * BINS * 4 * 4 <= kCap && G * BINS * 4 * 4 + kRest <= 65536) ? 4
                    : (G * BINS * 2 * 4 <= kCap && G * BINS * 2 * 4 + kRest <= 65536) ? 2 : 1;
    static_assert(G * BINS * R * 4 + kRest <= 65536, "LDS of the score kernel");
    auto kern = score_kernel<W, G, R>;
    // persistent grid: as many workgroups as the chip holds at once (a context has one code length
    // and one group size, hence one score kernel: asked once per context)
    if (ctx->score_resident == 0) {
        int per_cu = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kern, kThreads, 0) != hipSuccess || per_cu < 1)
            return SPOTLIGHT_ERR_HIP;
        ctx->score_resident = per_cu * ctx->n_cus;
    }
    const int resident = ctx->score_resident;
    ScoreArgs s;
    s.codes = a.codes;
    s.qcode = reinterpret_cast<const uint32_t*>(ctx->workspace + p.off_qcode);
    s.gcum = reinterpret_cast<uint32_t*>(ctx->workspace + p.off_gcum);
    s.blockcum = reinterpret_cast<uint32_t*>(ctx->workspace + p.off_blockcum);
    s.blockmeta = reinterpret_cast<BlockMeta*>(ctx->workspace + p.off_blockmeta);
    s.cand = reinterpret_cast<uint32_t*>(ctx->workspace + p.off_cand);
    s.n_tokens = a.n_tokens;
    s.n_sink = a.n_sink;
    s.local_begin = a.local_begin;
    s.Nmax = p.Nmax;
    s.Hkv = p.Hkv;
    s.nblk = a.nblk;
    s.max_blocks = p.max_blocks;
    s.k = a.k;
    s.total_tasks = a.nblk * p.B * p.Hkv;
    s.tasks_per_group = (s.total_tasks + resident - 1) / resident;
    // Long streams (gigabytes of codes): short runs, handed out by the hardware as workgroups
    // retire, instead of one long run per resident workgroup.  The workgroups in flight then read
    // one window of memory that moves through the cache in order, and uneven progress evens out
    // (1M tokens x 128 heads, 512-bit codes: 1474 us with runs of 32 blocks, 1438 us with runs of
    // 4, 1413 us with single blocks, which cost the shorter streams their look-ahead: 49 against
    // 46.5 us for 512K tokens x 32 heads).  Two generations of workgroups are the worst case.
    if (s.tasks_per_group >= kLongRun) s.tasks_per_group = kShortRun;
    *tasks_per_group = s.tasks_per_group;
    const int grid = (s.total_tasks + s.tasks_per_group - 1) / s.tasks_per_group;
    timer.launch(kern, dim3(static_cast<unsigned>(grid)), dim3(kThreads), 0, s);
    return SPOTLIGHT_OK;
}

template <int W>
int launch_w(spotlight_ctx* ctx, const RetrieveArgs& a)
{
    const Plan& p = ctx->plan;
    const int BH = p.B * p.Hq;
    const uint32_t* qcode = reinterpret_cast<const uint32_t*>(ctx->workspace + p.off_qcode);
    int tasks_per_group = 1;
    {
        StageTimer timer(ctx, SPOTLIGHT_STAGE_SCORE);
        int rc;
        switch (p.G) {
        case 1: rc = launch_score_wg<W, 1>(ctx, timer, a, &tasks_per_group); break;
        case 2: rc = launch_score_wg<W, 2>(ctx, timer, a, &tasks_per_group); break;
        // groups of three to eight heads; with 1024-bit codes their histograms do not fit in LDS
#define SPOTLIGHT_SCORE_GROUP(GG)                                                                          \
        case GG:                                                                                           \
            if constexpr (W <= 16) { rc = launch_score_wg<W, GG>(ctx, timer, a, &tasks_per_group); break; } \
            return SPOTLIGHT_ERR_UNSUPPORTED;
        SPOTLIGHT_SCORE_GROUP(3) SPOTLIGHT_SCORE_GROUP(4) SPOTLIGHT_SCORE_GROUP(5) SPOTLIGHT_SCORE_GROUP(6)
        SPOTLIGHT_SCORE_GROUP(7) SPOTLIGHT_SCORE_GROUP(8)
#undef SPOTLIGHT_SCORE_GROUP
        default: return SPOTLIGHT_ERR_UNSUPPORTED;
        }
        if (rc != SPOTLIGHT_OK) return rc;
        if (hipGetLastError() != hipSuccess) return SPOTLIGHT_ERR_HIP;
    }
    {
        StageTimer timer(ctx, SPOTLIGHT_STAGE_SELECT);
        dim3 grid(static_cast<unsigned>(a.nblk), static_cast<unsigned>(BH));
        const bool forced = a.n_sink > 0 || a.local_begin < a.n_tokens;
        // small grids: two wavefronts per block; grids of several rounds: one, twice as many resident
        const bool narrow = static_cast<int64_t>(a.nblk) * BH > kSelWideGrid;
        auto kern = select_kernel<W, false, kSelThreads>;
        if (forced && !narrow) kern = select_kernel<W, true, kSelThreads>;
        if (!forced && narrow) kern = select_kernel<W, false, kSelThreadsNarrow>;
        if (forced && narrow) kern = select_kernel<W, true, kSelThreadsNarrow>;
        timer.launch(kern, grid, dim3(narrow ? kSelThreadsNarrow : kSelThreads), 0, a.codes, qcode,
                     reinterpret_cast<const uint32_t*>(ctx->workspace + p.off_gcum),
                     reinterpret_cast<const uint32_t*>(ctx->workspace + p.off_blockcum),
                     reinterpret_cast<const BlockMeta*>(ctx->workspace + p.off_blockmeta),
                     reinterpret_cast<const uint32_t*>(ctx->workspace + p.off_cand), a.out_idx, a.n_tokens, p.Nmax,
                     p.Hq, p.Hkv, p.max_blocks, a.k, a.n_sink, a.local_begin, tasks_per_group);
        if (hipGetLastError() != hipSuccess) return SPOTLIGHT_ERR_HIP;
    }
    if (a.out_dist) {
        dim3 grid(static_cast<unsigned>((a.n_tokens + kThreads - 1) / kThreads), static_cast<unsigned>(BH));
        hipLaunchKernelGGL(dist_kernel<W>, grid, dim3(kThreads), 0, ctx->stream, a.codes, qcode, a.out_dist,
                           a.n_tokens, p.Nmax, p.Hq, p.Hkv);
        if (hipGetLastError() != hipSuccess) return SPOTLIGHT_ERR_HIP;
    }
    return SPOTLIGHT_OK;
}

}  // namespace retrieve_detail
}  // namespace spotlight
