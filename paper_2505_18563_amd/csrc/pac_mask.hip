// pac_build_mask: magnitude threshold at a target sparsity -> bitmask + exclusive prefix index.
//
// Per prune scope the kept set is "the k largest composites" (see pac_internal.h); C* is the k-th.
//
//   hist0    histogram of digit 0 (key bits 30..17) per scope: LDS histograms flushed to a global one.
//            Scopes from 4M elements on are only sampled: one 16384-element tile of every aligned group
//            of `stride`, at a hashed position.  The work is a list of slots shared evenly by the workgroups
//   select0  per scope: bracket [lo, hi) that holds the k-th key - exactly one digit-0 bin when every
//            element was counted; when the scope was sampled, the keys inside a confidence band around
//            the estimated rank, its two ends interpolated inside their bins.  Also the scope's tie key
//            (a key that very many in-bracket samples share, e.g. the zeros of a pruned model) and the
//            layout of digit 1 over the bracket
//   emit     one pass over the weights, one workgroup per 4096-element tile: mask bit = key >= hi,
//            a compare's lane mask being the mask word; elements with lo <= key < hi are undecided:
//            their composites go to the tile's record - except those with the tie key, which are
//            counted per tile - and the tile's counts to its header.  No atomics
//   count1   from the headers and records: digit-1 histogram of the undecided elements, kept and tie
//            counts per scope
//   select1  per scope: checks that the bracket did hold the k-th key (always true for exact
//            counts), then the digit-1 bin b1 of the k-th undecided element and its rank inside
//   (retry)  if a sampled bracket missed, hist0/select0/emit/count1/select1 run again with full
//            counts and whole bins; otherwise those five launches return at once
//   small    scopes of at most 32768 elements take no part in the above: one workgroup each selects
//            from LDS and writes the scope's mask bits
//   compact2 undecided elements whose digit 1 is their scope's b1 -> match lists (a few hundred per scope)
//   final    one workgroup per scope gathers its matches into LDS and resolves the remaining
//            bits there -> C*; if C* carries the tie key, its index part comes from the tiles' tie counts
//   fixup    undecided elements with composite >= C* get their mask bit set (atomic OR); tiles that
//            hold kept tie-key elements are read again for them
//   scan     exclusive prefix sum of the mask-word popcounts (single pass, decoupled look-back)
//
// A tile that holds more undecided elements than its record takes is not listed: count1, compact2 and
// fixup read that tile's weights instead.  A scope with more than 4096 matches is resolved by `final`
// from its weights.  Same results, slower; the status word tells (kDevSlowPath).
#include <cstdlib>
#include <type_traits>

#include "pac_internal.h"

namespace pac {
namespace {

typedef unsigned long long u64;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t key_of_bits(uint32_t bits) { return bits & 0x7FFFFFFFu; }
__device__ __forceinline__ u64 composite_of(uint32_t key, uint32_t i) {
    return ((u64)key << 32) | (u64)(0xFFFFFFFFu - i);
}
__device__ __forceinline__ uint32_t index_of(u64 composite) { return 0xFFFFFFFFu - (uint32_t)composite; }
__device__ __forceinline__ uint32_t digit0_of(uint32_t key) { return key >> kDigit0Shift; }
__device__ __forceinline__ uint32_t hash32(uint32_t x) {
    x ^= x >> 16; x *= 0x7FEB352Du; x ^= x >> 15; x *= 0x846CA68Bu; x ^= x >> 16;
    return x;
}
__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }
__device__ __forceinline__ uint32_t lanes_below(u64 m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// Sum of v over the 64 lanes, the same in every lane's return value; all lanes must be active.  Four
// cross-lane adds inside each row of 16 lanes, then the four row sums through scalar registers.  (An LDS
// atomic add of 64 different values to one address is turned by the compiler into a scalar loop over the
// lanes, seven scalar instructions each.)
__device__ __forceinline__ uint32_t wave_sum_rows(uint32_t v) {
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x141, 0xF, 0xF, true);   // row_half_mirror
    v += (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, 0x140, 0xF, 0xF, true);   // row_mirror
    return (uint32_t)__builtin_amdgcn_readlane((int)v, 0) + (uint32_t)__builtin_amdgcn_readlane((int)v, 16) +
           (uint32_t)__builtin_amdgcn_readlane((int)v, 32) + (uint32_t)__builtin_amdgcn_readlane((int)v, 48);
}

// atomicAdd(base + idx, 1) for every lane with `active`.  Equal magnitudes (all-zero biases, unit
// norm scales) put whole waves on one counter, and atomics on one address are serialised: when all
// active lanes agree on idx the wave issues a single atomic with their number; otherwise the lanes
// mostly differ and each issues its own.  Must be called by all lanes of the wave.
__device__ __forceinline__ void wave_aggregated_inc(uint32_t* __restrict__ base, uint32_t idx, bool active) {
    const u64 todo = __ballot(active);
    if (todo == 0) return;
    const uint32_t leader = (uint32_t)__ffsll((long long)todo) - 1u;
    const uint32_t lead_idx = (uint32_t)__shfl((int)idx, (int)leader, 64);
    if (__ballot(active && idx == lead_idx) == todo) {
        if (lane_id() == leader) atomicAdd(base + lead_idx, (uint32_t)__popcll(todo));
    } else if (active) {
        atomicAdd(base + idx, 1u);
    }
}

// First scope whose end exceeds flat index i (scopes ascending; empty scopes are never returned).
// Requires i < seg[nseg-1].end.
__device__ __forceinline__ uint32_t find_seg(const SegDesc* __restrict__ seg, uint32_t nseg, uint32_t i) {
    uint32_t lo = 0, hi = nseg - 1;
    while (lo < hi) {
        const uint32_t mid = (lo + hi) >> 1;
        if (seg[mid].end > i) hi = mid; else lo = mid + 1;
    }
    return lo;
}

// Exclusive prefix sum of v over the THREADS threads of the workgroup; `total` gets the sum.
template <int THREADS>
__device__ __forceinline__ uint32_t block_exclusive_scan(uint32_t v, uint32_t* wave_sums, uint32_t& total) {
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(inc, d, 64);
        if (lane >= (uint32_t)d) inc += t;
    }
    if (lane == 63) wave_sums[wave] = inc;
    __syncthreads();
    uint32_t off = 0, tot = 0;
#pragma unroll
    for (int i = 0; i < THREADS / 64; ++i) {
        const uint32_t x = wave_sums[i];
        if ((uint32_t)i < wave) off += x;
        tot += x;
    }
    total = tot;
    __syncthreads();
    return off + inc - v;
}

// ------------------------------------------------------------------------------------- hist0
constexpr int kHistBlock = 1024;
constexpr uint32_t kHistLoads = 4;                                 // 16-byte loads per thread per tile
constexpr uint32_t kHistTile = kHistBlock * 4 * kHistLoads;        // 16384 elements
static_assert(kHistTile == kHistTileElems, "the host counts histogram work in tiles of this size");

// ++lds[d] for every lane with `active`.  LDS atomics on one address are serialised lane by lane, and a
// tensor with very many equal magnitudes (the zeros of a pruned model) sends most lanes of every wave to
// one bin: the lanes that share the first active lane's bin go in as one add of their number.
__device__ __forceinline__ void count_digit0(uint32_t* lds, uint32_t d, bool active) {
    const u64 todo = __ballot(active);
    if (todo == 0) return;
    const uint32_t leader = (uint32_t)__ffsll((long long)todo) - 1u;
    const uint32_t d_lead = (uint32_t)__builtin_amdgcn_readlane((int)d, (int)leader);
    const u64 same = __ballot(active && d == d_lead);
    if (active && d != d_lead) atomicAdd(&lds[d], 1u);
    else if (lane_id() == leader) atomicAdd(&lds[d_lead], (uint32_t)__popcll(same));
}

__device__ __forceinline__ void flush_hist0(uint32_t* lds, uint32_t* __restrict__ global_hist) {
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < kDigit0Bins; b += kHistBlock) {
        const uint32_t v = lds[b];
        if (v) {
            atomicAdd(&global_hist[b], v);
            lds[b] = 0;
        }
    }
    __syncthreads();
}

// Counts the elements [from, to) of w, from < to, into the LDS histogram, the workgroup's threads
// striding over them with eight loads in flight each (indices clamped, not branched, so that the
// loads are issued together: one load per trip would wait for memory once per 1024 elements).
__device__ __forceinline__ void hist0_range(const float* __restrict__ w, u64 from, u64 to, uint32_t* lds) {
    constexpr uint32_t kFlight = 8;
    for (u64 i0 = from + threadIdx.x; i0 < to; i0 += (u64)kHistBlock * kFlight) {
        uint32_t v[kFlight];
#pragma unroll
        for (uint32_t q = 0; q < kFlight; ++q) v[q] = __float_as_uint(w[min(i0 + q * kHistBlock, to - 1)]);
#pragma unroll
        for (uint32_t q = 0; q < kFlight; ++q)
            count_digit0(lds, digit0_of(key_of_bits(v[q])), i0 + q * kHistBlock < to);
    }
}

// First slot of scope s in the given pass; nseg stands for "one past the last scope".
__device__ __forceinline__ uint32_t first_slot(const SegDesc* __restrict__ seg, uint32_t nseg, uint32_t s,
                                               uint32_t pass, uint32_t total_slots) {
    if (s >= nseg) return total_slots;
    return pass == 0 ? seg[s].slot0 : seg[s].slot1;
}

// The work of a histogram pass is a list of slots: per scope (in order) one slot for every aligned group
// of `stride` tiles that the scope touches - in the full pass, and for a scope counted in full, for every
// tile.  A slot stands for the group's sampled tile, clipped to the scope, or for nothing when that tile
// lies outside the scope (first and last group only).  The workgroups share the slots evenly, each taking
// a run of consecutive ones, so that the work is balanced whatever mix of strides the table holds, a
// workgroup meets few scope boundaries, and flushes its histogram rarely.
template <bool VEC>
__global__ __launch_bounds__(kHistBlock) void hist0_kernel(const float* __restrict__ w, uint32_t n,
                                                           const SegDesc* __restrict__ seg, uint32_t nseg,
                                                           uint32_t* __restrict__ hist0, Globals* glob,
                                                           uint32_t pass, uint32_t total_slots) {
    __shared__ uint32_t lds[kDigit0Bins];
    if (pass != 0 && !glob->retry) return;             // the retry pass has nothing to do
    for (uint32_t b = threadIdx.x; b < kDigit0Bins; b += kHistBlock) lds[b] = 0;
    if (blockIdx.x == 0) {
        // Counters of this call start from zero (the retry pass keeps `retry` itself).
        static_assert(sizeof(Globals) / 4 <= 2 * kHistBlock, "Globals cleared by one workgroup");
        uint32_t* g = reinterpret_cast<uint32_t*>(glob);
        const uint32_t keep = pass != 0 ? (uint32_t)(offsetof(Globals, retry) / 4) : 0xFFFFFFFFu;
        for (uint32_t j = threadIdx.x; j < sizeof(Globals) / 4; j += kHistBlock)
            if (j != keep) g[j] = 0;
    }
    __syncthreads();

    const uint32_t per_block = (total_slots + gridDim.x - 1) / gridDim.x;
    const uint32_t j_begin = blockIdx.x * per_block;
    const uint32_t j_end = min(total_slots, j_begin + per_block);
    if (j_begin >= j_end) return;

    // The scope that owns slot j_begin: the last one whose first slot is <= j_begin (scopes without slots
    // share their first slot with the scope after them).
    uint32_t s;
    {
        uint32_t lo = 0, hi = nseg - 1;
        while (lo < hi) {
            const uint32_t mid = (lo + hi + 1) >> 1;
            if (first_slot(seg, nseg, mid, pass, total_slots) <= j_begin) lo = mid; else hi = mid - 1;
        }
        s = lo;
    }
    const uint32_t kNone = 0xFFFFFFFFu;
    uint32_t counted = kNone;   // scope whose counts sit in the LDS histogram
    uint32_t s_first = first_slot(seg, nseg, s, pass, total_slots);
    uint32_t s_next = first_slot(seg, nseg, s + 1, pass, total_slots);
    uint32_t sb = seg[s].begin, se = seg[s].end, m = pass == 0 ? seg[s].stride : 1u;
    for (uint32_t j = j_begin; j < j_end; ++j) {
        while (j >= s_next) {                           // s_next <= total_slots > j for the last scope: ends
            ++s;
            s_first = s_next;
            s_next = first_slot(seg, nseg, s + 1, pass, total_slots);
            sb = seg[s].begin; se = seg[s].end; m = pass == 0 ? seg[s].stride : 1u;
        }
        const uint32_t sh = 31 - __clz((int)m);         // m is a power of two >= 1 for a scope with slots
        const uint32_t first_tile = sb / kHistTile, last_tile = (se - 1) / kHistTile;
        const uint32_t group = (first_tile >> sh) + (j - s_first);
        // one tile of every aligned group of m, at a hashed position so that no period of the tensor
        // layout can line up with the sample
        const uint32_t t = (group << sh) + (hash32(group) & (m - 1));
        if (t < first_tile || t > last_tile) continue;
        if (s != counted) {
            if (counted != kNone) flush_hist0(lds, hist0 + (size_t)counted * kDigit0Bins);
            counted = s;
        }
        const u64 a = max((u64)t * kHistTile, (u64)sb);
        const u64 b = min(((u64)t + 1) * kHistTile, (u64)se);
        if (VEC && b - a == kHistTile) {
            const u32x4* p = reinterpret_cast<const u32x4*>(w + a) + threadIdx.x;
            u32x4 v[kHistLoads];
#pragma unroll
            for (uint32_t u = 0; u < kHistLoads; ++u) v[u] = __builtin_nontemporal_load(p + u * kHistBlock);
#pragma unroll
            for (uint32_t u = 0; u < kHistLoads; ++u) {
                count_digit0(lds, digit0_of(key_of_bits(v[u].x)), true);
                count_digit0(lds, digit0_of(key_of_bits(v[u].y)), true);
                count_digit0(lds, digit0_of(key_of_bits(v[u].z)), true);
                count_digit0(lds, digit0_of(key_of_bits(v[u].w)), true);
            }
        } else {
            hist0_range(w, a, b, lds);
        }
    }
    if (counted != kNone) flush_hist0(lds, hist0 + (size_t)counted * kDigit0Bins);
}

// ---------------------------------------------------------------------------- select0 / select1
// Finds, in a histogram of BINS bins owned 16 per thread, the bin that holds the k-th element when
// bins are walked from the highest digit down.  `extra_cnt` further elements count in bin `extra_bin`
// (they are not in the histogram).  Zeroes the histogram.  Exactly one thread returns true (if
// 1 <= k <= total count) with bin / rank-inside-bin / bin count.
template <int BINS>
__device__ __forceinline__ bool select_bin(uint32_t* __restrict__ h, uint32_t k, uint32_t extra_bin, uint32_t extra_cnt,
                                           uint32_t* wave_sums, uint32_t& bin, uint32_t& krem, uint32_t& cnt) {
    constexpr int THREADS = BINS / 16;
    uint32_t loc[16];
    uint4* hv = reinterpret_cast<uint4*>(h) + threadIdx.x * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint4 x = hv[j];
        loc[4 * j] = x.x; loc[4 * j + 1] = x.y; loc[4 * j + 2] = x.z; loc[4 * j + 3] = x.w;
        hv[j] = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 16; ++j)
        if (threadIdx.x * 16 + j == extra_bin) loc[j] += extra_cnt;
    uint32_t sum = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) sum += loc[j];
    uint32_t total;
    const uint32_t below = block_exclusive_scan<THREADS>(sum, wave_sums, total);
    const uint32_t above = total - below - sum;     // elements in bins owned by higher threads
    bool mine = false;
    if (k >= 1 && above < k && k <= above + sum) {
        uint32_t acc = above;
#pragma unroll
        for (int j = 15; j >= 0; --j) {
            if (!mine) {
                if (acc + loc[j] >= k) {
                    mine = true;
                    bin = threadIdx.x * 16 + j;
                    krem = k - acc;
                    cnt = loc[j];
                } else {
                    acc += loc[j];
                }
            }
        }
    }
    return mine;
}

constexpr uint32_t kFinalList = 4096;   // matches of one scope that `final` can hold in LDS

// Width of the confidence band around the estimated sample rank, in standard deviations of a
// simple random sample.  Tiles are clusters, which can inflate the variance; a bracket that misses
// is detected after emit and the call falls back to full counts.
constexpr double kBandSigmas = 8.0;

// Digit 1 of an undecided key (see SegState).
__device__ __forceinline__ uint32_t digit1_of(uint32_t key, uint32_t lo1, uint32_t sh1, uint32_t off1) {
    return key < lo1 ? 0u : ((key - lo1) >> sh1) + off1;
}

// Samples of a scope that select0 looks at to find a tie key: one per thread, at hashed positions.
constexpr uint32_t kTieVoters = 256;    // in-bracket samples that take part in the vote
constexpr uint32_t kTieMinVotes = 8;    // a key with at least this many of them becomes the tie key

__global__ __launch_bounds__(kDigit0Bins / 16) void select0_kernel(const float* __restrict__ w,
                                                                   const SegDesc* __restrict__ seg,
                                                                   SegState* __restrict__ state,
                                                                   uint32_t* __restrict__ hist0,
                                                                   uint32_t* __restrict__ kept_above,
                                                                   uint32_t* __restrict__ tie_count, Globals* glob,
                                                                   uint32_t pass) {
    constexpr int THREADS = kDigit0Bins / 16;
    __shared__ uint32_t wave_sums[THREADS / 64];
    __shared__ uint32_t sh_hi, sh_lo, sh_above_hi, sh_lo_key, sh_hi_cut;
    __shared__ uint32_t voters[kTieVoters];
    __shared__ uint32_t n_in, n_in_tie_bin, sh_next;
    __shared__ u64 best;
    if (pass != 0 && !glob->retry) return;
    const uint32_t s = blockIdx.x;
    const uint32_t k = seg[s].k;
    const uint32_t begin = seg[s].begin;
    const uint32_t n_s = seg[s].end - begin;
    SegState* st = state + s;
    auto settle = [&](u64 cstar, uint32_t edge) {   // nothing undecided: every key is below (or at least) `edge`
        st->cstar = cstar;
        st->active = 0;
        st->lo = st->hi = st->lo1 = edge;
        st->sh1 = 0; st->off1 = 0; st->tie_key = kNoTieKey; st->tie_in = 0;
        st->exact = 1; st->krem0 = 0; st->bin1 = 0; st->cnt1 = 0; st->krem1 = 0; st->heavy = 0;
    };
    if (seg[s].stride == 0) {
        // A small scope takes no part in the streaming passes: emit leaves it all-zero (no key reaches
        // hi) and its own workgroup writes its bits afterwards.  Its histogram rows stay zero.
        if (threadIdx.x == 0) settle(~0ull, kKeyEnd);
        return;
    }

    // One sample of the scope per thread, for the tie-key vote further down (issued early: the histogram
    // work below hides its latency).
    const uint32_t sample_pos = begin + (uint32_t)(((u64)hash32(threadIdx.x * 0x9E3779B1u + s) * n_s) >> 32);
    const uint32_t sample_key = key_of_bits(__float_as_uint(w[sample_pos]));

    // this scope's counters start from zero
    if (threadIdx.x == 0) { kept_above[s] = 0; tie_count[s] = 0; }

    // thread t owns bins [16t, 16t+16); read them (and the two bins next to them), then clear them
    uint32_t loc[16];
    uint32_t* row = hist0 + (size_t)s * kDigit0Bins;
    uint4* hv = reinterpret_cast<uint4*>(row) + threadIdx.x * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint4 x = hv[j];
        loc[4 * j] = x.x; loc[4 * j + 1] = x.y; loc[4 * j + 2] = x.z; loc[4 * j + 3] = x.w;
    }
    const uint32_t bin_before = threadIdx.x > 0 ? row[threadIdx.x * 16 - 1] : 0u;
    const uint32_t bin_after = threadIdx.x + 1 < THREADS ? row[threadIdx.x * 16 + 16] : 0u;
    uint32_t sum = 0;
#pragma unroll
    for (int j = 0; j < 16; ++j) sum += loc[j];
    uint32_t counted;   // elements the histogram pass visited
    const uint32_t below = block_exclusive_scan<THREADS>(sum, wave_sums, counted);   // (barriers: every read above is done)
#pragma unroll
    for (int j = 0; j < 4; ++j) hv[j] = make_uint4(0, 0, 0, 0);
    const uint32_t above = counted - below - sum;   // elements in bins owned by higher threads

    if (k == 0 || k == n_s) {
        // Nothing to resolve: keep nothing (hi above every key) or everything (hi = 0).
        if (threadIdx.x == 0) settle(k == 0 ? ~0ull : 0ull, k == 0 ? kKeyEnd : 0u);
        return;
    }

    // Rank band [lo_rank, hi_rank] (in counted elements, from the top) that holds the k-th element.
    const bool exact = counted == n_s;
    double lo_rank, hi_rank;
    if (exact) {
        lo_rank = (double)k - 1.0;   // bins with at most k-1 elements above them ...
        hi_rank = (double)k;         // ... and at least k elements at or above them: one bin
    } else {
        const double frac = (double)k / (double)n_s;
        const double ks = frac * (double)counted;
        const double sd = sqrt(fmax(ks * (1.0 - frac), 1.0));
        lo_rank = ks - kBandSigmas * sd - 2.0;
        hi_rank = ks + kBandSigmas * sd + 2.0;
    }
    if (threadIdx.x == 0) {
        sh_hi = kDigit0Bins - 1; sh_lo = 0; sh_above_hi = 0;
        n_in = 0; n_in_tie_bin = 0; sh_next = kDigit0Bins; best = 0;
    }
    __syncthreads();
    {
        // b_hi = smallest bin with (#counted above it) <= lo_rank; b_lo = largest bin with
        // (#counted at or above it) >= hi_rank.  Both conditions are monotone in the bin index.
        uint32_t cgt = above, my_hi = 0xFFFFFFFFu, my_lo = 0;
        bool any_lo = false;
#pragma unroll
        for (int j = 15; j >= 0; --j) {
            const uint32_t bin = threadIdx.x * 16 + j;
            if ((double)cgt <= lo_rank) my_hi = bin;                         // descending j: ends at the smallest
            if (!any_lo && (double)(cgt + loc[j]) >= hi_rank) { my_lo = bin; any_lo = true; }   // first hit is the largest
            cgt += loc[j];
        }
        if (my_hi != 0xFFFFFFFFu) atomicMin(&sh_hi, my_hi);
        if (any_lo) atomicMax(&sh_lo, my_lo);
    }
    __syncthreads();
    const uint32_t b_hi = sh_hi;
    const uint32_t b_lo = min(sh_lo, b_hi);
    {
        // A sampled bracket need not end on bin boundaries (emit counts what lies above it, select1 checks
        // that it held the k-th key): inside its two end bins the ends move to where the rank band ends,
        // taking the keys of a bin as evenly spread - if the bin is well filled and both bins next to it
        // hold comparable numbers (a bin that stands alone is a lump of equal values, like the zeros of a
        // pruned model, and is taken whole).  Where the guess is wrong the check fails and the call falls
        // back to full counts and whole bins.
        constexpr uint32_t kBinKeys = 1u << kDigit0Shift;
        constexpr uint32_t kMinForCut = 64;      // sampled elements in a bin before its inside is trusted
        uint32_t cgt = above;
#pragma unroll
        for (int j = 15; j >= 0; --j) {
            const uint32_t bin = threadIdx.x * 16 + j, c = loc[j];
            const uint32_t left = j > 0 ? loc[j > 0 ? j - 1 : 0] : bin_before;
            const uint32_t right = j < 15 ? loc[j < 15 ? j + 1 : 15] : bin_after;
            const bool smooth = c >= kMinForCut && left >= c / 4 && right >= c / 4;
            if (bin == b_hi) {
                sh_above_hi = cgt;
                uint32_t cut = 0;                // keys taken off the top of bin b_hi (they count as kept)
                if (!exact && smooth) {
                    const double f = (lo_rank - (double)cgt) / (double)c;
                    if (f > 0.0) cut = (uint32_t)fmin(f * (double)kBinKeys, (double)(kBinKeys - 1u));
                }
                sh_hi_cut = cut;
            }
            if (bin == b_lo) {
                uint32_t lo_key = bin << kDigit0Shift;
                if (!exact && smooth) {
                    const double f = ((hi_rank - (double)cgt) / (double)c) * (double)kBinKeys;
                    if (f < (double)kBinKeys) lo_key += kBinKeys - (uint32_t)ceil(fmax(f, 1.0));
                }
                sh_lo_key = lo_key;
            }
            cgt += c;
        }
    }
    __syncthreads();
    // (two ends in one bin: the band is at least a few elements wide, so lo stays below hi; an empty
    // bracket would simply fail select1's check)
    const u64 hi_key = ((u64)(b_hi + 1u) << kDigit0Shift) - sh_hi_cut;       // up to 2^31
    const uint32_t lo = (u64)sh_lo_key < hi_key ? sh_lo_key : (uint32_t)hi_key;
    const uint32_t width = (uint32_t)(hi_key - lo);

    // Tie key: the samples that fall into the bracket vote; a key that very many of them share (the zeros
    // of a pruned model, a constant tensor) would overflow every tile's list, so its elements are only
    // counted.  Any choice is correct - the key only decides which elements are listed and which counted.
    const bool in_bracket = sample_key - lo < width;
    uint32_t my_slot = kTieVoters;
    if (in_bracket) my_slot = atomicAdd(&n_in, 1u);
    if (my_slot < kTieVoters) voters[my_slot] = sample_key;
    __syncthreads();
    const uint32_t n_voters = min(n_in, kTieVoters);
    if (my_slot < kTieVoters && n_voters >= kTieMinVotes) {
        uint32_t votes = 0;
        for (uint32_t i = 0; i < n_voters; ++i) votes += voters[i] == sample_key ? 1u : 0u;
        if (votes >= kTieMinVotes) atomicMax(&best, ((u64)votes << 32) | sample_key);
    }
    __syncthreads();
    const bool has_tie = best != 0;
    const uint32_t tie_key = has_tie ? (uint32_t)best : kNoTieKey;
    // Where digit 1 starts.  If the tie key fills the lowest bin of a bracket of several bins (every sample
    // of that bin is the tie key: the zeros below all other magnitudes), digit 1 starts at the next bin
    // that holds anything, so that it resolves the listed elements and not the empty range above the zeros.
    uint32_t b1_lo = b_lo;
    if (has_tie && digit0_of(tie_key) == b_lo && b_lo < b_hi) {
        if (digit0_of(sample_key) == b_lo && sample_key != tie_key) atomicAdd(&n_in_tie_bin, 1u);   // impure
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            const uint32_t bin = threadIdx.x * 16 + j;
            if (bin > b_lo && bin <= b_hi && loc[j] != 0) atomicMin(&sh_next, bin);
        }
        __syncthreads();
        if (n_in_tie_bin == 0) b1_lo = min(sh_next, b_hi);
    } else {
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        // the finest digit 1 whose values stay below kDigit1Bins, with lo1 aligned to its width
        const uint32_t off1 = b1_lo > b_lo ? 1u : 0u;
        const uint32_t first_key = off1 ? b1_lo << kDigit0Shift : lo;
        const u64 last_key = hi_key - 1u;
        uint32_t sh1 = 0, lo1 = 0;
        for (;; ++sh1) {
            lo1 = first_key & ~((1u << sh1) - 1u);
            if (last_key < lo1 || ((last_key - lo1) >> sh1) + off1 <= kDigit1Bins - 1u) break;
        }
        st->cstar = 0;
        st->active = 1;
        st->lo = lo;
        st->hi = lo + width;                             // up to 2^31
        st->lo1 = lo1; st->sh1 = sh1; st->off1 = off1;
        st->tie_key = tie_key; st->tie_in = 0;
        st->exact = exact ? 1u : 0u;
        st->krem0 = exact ? k - sh_above_hi : 0u;
        st->bin1 = 0; st->cnt1 = 0; st->krem1 = 0;
        st->heavy = 0;
    }
}

__global__ __launch_bounds__(kDigit1Bins / 16) void select1_kernel(const SegDesc* __restrict__ seg,
                                                                   SegState* __restrict__ state,
                                                                   uint32_t* __restrict__ hist1,
                                                                   const uint32_t* __restrict__ kept_above,
                                                                   const uint32_t* __restrict__ tie_count,
                                                                   Globals* glob, uint32_t* __restrict__ status,
                                                                   uint32_t pass) {
    __shared__ uint32_t wave_sums[kDigit1Bins / 16 / 64];
    __shared__ uint32_t sh_rank;
    if (pass != 0 && !glob->retry) return;
    const uint32_t s = blockIdx.x;
    SegState* st = state + s;
    const uint32_t active = st->active;
    // Rank of the k-th element among the undecided ones.  Exact counts gave it before emit; a sampled
    // bracket gets it from the number of elements emit found above the bracket, and is checked here.
    if (threadIdx.x == 0) {
        uint32_t rank = 0;
        if (active) {
            if (st->exact) {
                rank = st->krem0;
            } else {
                const uint32_t kept = kept_above[s];
                const uint32_t k = seg[s].k;
                rank = k > kept ? k - kept : 0u;   // 0: more than k elements above the bracket
            }
        }
        sh_rank = rank;
    }
    __syncthreads();
    const uint32_t rank = sh_rank;
    // the tie key's elements were counted, not listed: they join the histogram as one lump
    const uint32_t tie_key = active ? st->tie_key : kNoTieKey;
    const uint32_t ties = tie_key != kNoTieKey ? tie_count[s] : 0u;
    const uint32_t tie_bin = tie_key != kNoTieKey ? digit1_of(tie_key, st->lo1, st->sh1, st->off1) : 0xFFFFFFFFu;
    uint32_t bin = 0, krem = 0, cnt = 0;
    // (select_bin clears the histogram and finds nothing when rank is 0 or beyond the undecided count)
    const bool mine = select_bin<(int)kDigit1Bins>(hist1 + (size_t)s * kDigit1Bins, rank, tie_bin, ties, wave_sums, bin, krem, cnt);
    if (threadIdx.x == 0) sh_rank = 0;
    __syncthreads();
    if (mine) {
        const bool tie_in = ties != 0 && bin == tie_bin;
        const uint32_t listed = tie_in ? cnt - ties : cnt;
        st->krem0 = rank; st->bin1 = bin; st->cnt1 = cnt; st->krem1 = krem;
        st->tie_in = tie_in ? 1u : 0u;
        st->heavy = listed > kFinalList ? 1u : 0u;
        if (listed > kFinalList) atomicOr(status, kDevSlowPath);
        sh_rank = 1;
    }
    __syncthreads();
    if (threadIdx.x == 0 && active && sh_rank == 0) {   // the bracket missed the k-th element
        glob->retry = 1;
        atomicOr(status, kDevRetryTaken);
    }
}

// -------------------------------------------------------------------------------------- emit
// The pass over the weights that writes the mask.  With [lo, hi) the scope's bracket:
// key >= hi -> kept;   lo <= key < hi -> undecided (candidate).
//
// One workgroup of 4 waves per 4096-element tile, one 1024-element quarter per wave.  A lane loads
// one element per step (16 dword loads at a stride of 64 elements, all issued before the first is
// used), so the lane mask of the compare `key >= hi` IS the mask word of those 64 elements: no
// cross-lane assembly.  Lane u keeps word u; 16 lanes store the wave's 128 bytes of mask.
// The workgroup ends with stores and takes part in no atomics: a workgroup's wave slots stay taken
// until its last memory operation is acknowledged, and a returning atomic is the slowest of them.
//
// Undecided elements are rare for continuous weight distributions (~0.5 %).  Their composites go,
// through a small per-wave LDS stage, into the tile's record: 128 u64 slots per tile.  The tile's header
// (listed entries, kept elements, tie-key elements of its first and of its last scope: 16 bits each) goes
// into a dense array of its own, so that the passes which need only headers read 8 bytes per tile.
// Elements whose key is the scope's tie key are counted, not listed.  A tile that still holds more
// undecided elements than its record takes is marked kRecWalk: the kernels that consume the records then
// walk that tile's 4096 weights instead - the overflow is local, every other tile keeps its list.
constexpr int kEmitBlock = 256;
constexpr int kEmitWaves = kEmitBlock / 64;
constexpr uint32_t kEmitLoads = 16;                                 // dword loads per lane per tile
constexpr uint32_t kEmitWaveTile = 64 * kEmitLoads;                 // 1024 elements = 16 mask words
constexpr uint32_t kEmitTile = kEmitWaves * kEmitWaveTile;          // 4096 elements
constexpr uint32_t kWaveStage = 64;                                 // staged composites per wave
static_assert(kEmitTile == kEmitTileElems, "records are per emit tile");

__device__ __forceinline__ void wave_lds_sync() {
    // Orders this wave's LDS writes before its later LDS accesses of other lanes.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

struct EmitShared {
    u64 stage[kEmitWaves][kWaveStage];
    uint32_t wcount[kEmitWaves];     // undecided elements each wave met (more than kWaveStage: its stage overflowed)
    uint32_t wkept[kEmitWaves];
    uint32_t wtie[kEmitWaves];       // tie-key elements: head scope in the low half, tail scope in the high half
};

__device__ __forceinline__ u64 pack_header(uint32_t listed, uint32_t kept, uint32_t tie_head, uint32_t tie_tail) {
    return (u64)listed | ((u64)kept << 16) | ((u64)tie_head << 32) | ((u64)tie_tail << 48);
}
__device__ __forceinline__ uint32_t header_listed(u64 h) { return (uint32_t)h & 0xFFFFu; }
__device__ __forceinline__ uint32_t header_kept(u64 h) { return (uint32_t)(h >> 16) & 0xFFFFu; }
__device__ __forceinline__ uint32_t header_tie_head(u64 h) { return (uint32_t)(h >> 32) & 0xFFFFu; }
__device__ __forceinline__ uint32_t header_tie_tail(u64 h) { return (uint32_t)(h >> 48); }

// Scope of element i for a lane whose elements come in ascending order: moves (sc, sc_end) forward.
// Returns true when the scope changed.  Requires i < n (the last scope ends at n).
__device__ __forceinline__ bool advance_scope(const SegDesc* __restrict__ seg, uint32_t i, uint32_t& sc,
                                              uint32_t& sc_end) {
    bool moved = false;
    while (i >= sc_end) {
        ++sc;
        sc_end = seg[sc].end;
        moved = true;
    }
    return moved;
}

// Lane U of the pair (lo, hi) replaced by the two halves of the wave-uniform 64-bit value m: two
// v_writelane_b32 with the lane as an immediate.  (The compiler's own lowering of `lane == U ? x : old`
// keeps sixteen lane masks in scalar registers, which it then spills.)  m is the result of the vector
// compare just before: the s_nop covers the "a vector instruction writes a scalar register, the next one
// reads it: two wait states" rule of this chip, which the compiler cannot apply inside an asm statement.
template <uint32_t U>
__device__ __forceinline__ void set_lane_pair(u64 m, uint32_t& lo, uint32_t& hi) {
    asm volatile("s_nop 1\n\tv_writelane_b32 %0, %2, %4\n\tv_writelane_b32 %1, %3, %4"
                 : "+v"(lo), "+v"(hi) : "s"((uint32_t)m), "s"((uint32_t)(m >> 32)), "n"(U));
}

// f(std::integral_constant<uint32_t, U>) for U = 0 .. N-1, so that U is a constant where an asm operand needs one.
template <uint32_t U, uint32_t N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (U < N) {
        f(std::integral_constant<uint32_t, U>{});
        static_for<U + 1, N>(f);
    }
}

__global__ __launch_bounds__(kEmitBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) void emit_kernel(const float* __restrict__ w, uint32_t n,
                                                          const SegDesc* __restrict__ seg, uint32_t nseg,
                                                          const SegState* __restrict__ state, const Globals* glob,
                                                          const uint32_t* __restrict__ tile_scope,
                                                          uint32_t* __restrict__ kept_above, u64* __restrict__ hdrs,
                                                          u64* __restrict__ rec, uint32_t rec_cap,
                                                          u64* __restrict__ mask, uint32_t pass) {
    __shared__ EmitShared sh;
    if (pass != 0 && !glob->retry) return;             // the retry pass has nothing to do
    const uint32_t lane = lane_id();
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t num_tiles = (uint32_t)(((u64)n + kEmitTile - 1) / kEmitTile);
    const uint32_t words = (uint32_t)(((u64)n + 63) >> 6);

    for (uint32_t t = blockIdx.x; t < num_tiles;) {                  // one trip when the grid covers the tiles
        const u64 a = (u64)t * kEmitTile;                            // < n
        const bool whole = a + kEmitTile <= n;
        const u64 wave_first = a + wave * kEmitWaveTile;
        // A whole tile's loads go out before anything is known about its scopes (a tile that turns out to
        // cross a scope boundary reads its elements again, a few at a time, on the general path below).
        uint32_t v[kEmitLoads];
        if (whole) {
            const uint32_t* p = reinterpret_cast<const uint32_t*>(w) + wave_first + lane;
#pragma unroll
            for (uint32_t u = 0; u < kEmitLoads; ++u) v[u] = __builtin_nontemporal_load(p + u * 64);
        }
        const uint32_t s0 = nseg > 1 ? tile_scope[t] : 0u;
        const uint32_t s0_end = seg[s0].end;

        // The wave's counters live in LDS: the per-element work below is vector instructions only (a
        // compute unit issues one scalar instruction per clock for all of its waves together, and ballots
        // that are counted step by step cost several each).  Undecided elements are rare: the few lanes
        // that hold one append it with an LDS atomic; their order in the record does not matter.
        if (lane == 0) sh.wcount[wave] = 0;
        wave_lds_sync();
        uint32_t mine_lo = 0, mine_hi = 0;   // lane u: mask word u of this wave
        uint32_t my_tie = 0;                 // this lane's tie-key elements: head scope | tail scope << 16
        u64* my = sh.stage[wave];
        if (whole && (u64)s0_end >= a + kEmitTile) {
            // the whole tile inside one scope: nothing per element but the compares
            const uint32_t lo = state[s0].lo, hi = state[s0].hi, width = hi - lo, tie = state[s0].tie_key;
            const uint32_t i0 = (uint32_t)wave_first + lane;
            static_for<0, kEmitLoads>([&](auto uc) {
                constexpr uint32_t u = decltype(uc)::value;
                const uint32_t key = key_of_bits(v[u]);
                const u64 km = __ballot(key >= hi);
                set_lane_pair<u>(km, mine_lo, mine_hi);
                const bool is_tie = key == tie;                      // never true without a tie key
                my_tie += is_tie ? 1u : 0u;
                const uint32_t listed_key = is_tie ? 0xFFFFFFFFu : key;   // outside every bracket
                // The accumulators take their new values here and now.  (Left to itself the compiler sinks
                // these updates to the end of the tile and keeps sixteen steps' lane masks alive in scalar
                // registers it does not have: they spill, and the loaded values after them.)
                asm volatile("" : "+v"(mine_lo), "+v"(mine_hi), "+v"(my_tie));
                if (listed_key - lo < width) {
                    const uint32_t pos = atomicAdd(&sh.wcount[wave], 1u);
                    if (pos < kWaveStage) my[pos] = composite_of(key, i0 + u * 64);
                }
            });
        } else {
            // The ragged last tile, or a tile that crosses scope boundaries: every lane follows the
            // scopes of its own (ascending) elements.  Kept counts of sampled scopes go straight to
            // their counters (the record's count is only used for tiles inside one scope).  At most one
            // other large scope begins inside a tile: its tie-key elements are the header's tail count.
            const bool single = (u64)s0_end >= min(a + kEmitTile, (u64)n);
            uint32_t sc = s0, sc_end = s0_end;
            uint32_t lo = state[s0].lo, hi = state[s0].hi, exact = state[s0].exact, tie = state[s0].tie_key;
            constexpr uint32_t kGroup = 4;      // loads in flight: such tiles are few, their code is kept small
#pragma unroll 1
            for (uint32_t u0 = 0; u0 < kEmitLoads; u0 += kGroup) {
                uint32_t x[kGroup];
#pragma unroll
                for (uint32_t q = 0; q < kGroup; ++q) {
                    const u64 i = wave_first + (u0 + q) * 64 + lane;
                    x[q] = i < n ? __float_as_uint(w[i]) : 0u;
                }
#pragma unroll
                for (uint32_t q = 0; q < kGroup; ++q) {
                    const uint32_t u = u0 + q;
                    const u64 i = wave_first + u * 64 + lane;
                    const bool valid = i < n;
                    if (valid && advance_scope(seg, (uint32_t)i, sc, sc_end)) {
                        lo = state[sc].lo; hi = state[sc].hi; exact = state[sc].exact; tie = state[sc].tie_key;
                    }
                    const uint32_t key = key_of_bits(x[q]);
                    const bool kept = valid && key >= hi;
                    const u64 km = __ballot(kept);
                    mine_lo = lane == u ? (uint32_t)km : mine_lo;
                    mine_hi = lane == u ? (uint32_t)(km >> 32) : mine_hi;
                    if (!single) wave_aggregated_inc(kept_above, sc, kept && !exact);
                    const bool is_tie = valid && key == tie;
                    my_tie += is_tie ? (sc == s0 ? 1u : 0x10000u) : 0u;
                    if (valid && !is_tie && key - lo < hi - lo) {
                        const uint32_t pos = atomicAdd(&sh.wcount[wave], 1u);
                        if (pos < kWaveStage) my[pos] = composite_of(key, (uint32_t)i);
                    }
                }
            }
        }
        const u64 mine = ((u64)mine_hi << 32) | mine_lo;     // lanes 0..15; zero in the others
        if (lane < kEmitLoads) {
            const u64 wi = (wave_first >> 6) + lane;
            if (wi < words) __builtin_nontemporal_store(mine, mask + wi);
        }
        const uint32_t kept_n = wave_sum_rows((uint32_t)__popcll(mine));
        const uint32_t tie_n = wave_sum_rows(my_tie);         // two 16-bit sums side by side, each at most 1024
        if (lane == 0) { sh.wkept[wave] = kept_n; sh.wtie[wave] = tie_n; }

        // the tile's record: header, then the waves' entries back to back
        __syncthreads();
        const uint32_t staged = sh.wcount[wave];
        uint32_t off = 0, total = 0, kept_total = 0, tie_total = 0;
        bool walk = false;
#pragma unroll
        for (int j = 0; j < kEmitWaves; ++j) {
            const uint32_t c = sh.wcount[j];
            if (c > kWaveStage) walk = true;      // that wave's stage overflowed
            if ((uint32_t)j < wave) off += c;
            total += c;
            kept_total += sh.wkept[j];
            tie_total += sh.wtie[j];              // still two 16-bit sums, each at most 4096
        }
        if (total > rec_cap) walk = true;
        u64* r = rec + (size_t)t * kRecSlots;
        if (threadIdx.x == 0) hdrs[t] = pack_header(walk ? kRecWalk : total, kept_total, tie_total & 0xFFFFu, tie_total >> 16);
        if (!walk) {
            for (uint32_t j = lane; j < staged; j += 64) r[off + j] = my[j];
        }
        t += gridDim.x;
        if (t >= num_tiles) break;
        __syncthreads();   // the stage and the counts are reused by the next tile
    }
}

// First scope of every emit tile, so that a workgroup finds its scope with one load.
__global__ void tile_scope_kernel(const SegDesc* __restrict__ seg, uint32_t nseg, uint32_t num_tiles,
                                  uint32_t* __restrict__ tile_scope) {
    const uint32_t t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < num_tiles) tile_scope[t] = find_seg(seg, nseg, t * kEmitTile);
}

// ---------------------------------------------------------------------- walking the tile records
// count1, compact2 and fixup all visit "every undecided element": the entries of the tiles'
// records, or, for a tile marked kRecWalk, the tile's weights.  A wave takes 64 tiles at a time, one
// header per lane, then runs over the entries of all 64 records as one flat sequence (an entry
// finds its tile by a search over the running counts), so that the loads of a step are independent
// of each other.  `header(t, hdr, s0, single)` is called once per tile by its lane,
// `visit(composite, scope)` by the lanes that hold an undecided element, under divergence.
struct WalkShared {
    uint32_t excl[64];     // entries in the records of the lanes below
    uint32_t meta[64];     // tile's first scope | bit 31: the tile lies inside that scope
};

__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
    const uint32_t lane = lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t t = __shfl_up(v, d, 64);
        if (lane >= (uint32_t)d) v += t;
    }
    return v;
}

template <typename Header, typename Visit>
__device__ __forceinline__ void visit_tiles(const float* __restrict__ w, uint32_t n,
                                            const SegDesc* __restrict__ seg, uint32_t nseg,
                                            const SegState* __restrict__ state,
                                            const uint32_t* __restrict__ tile_scope, const u64* __restrict__ hdrs,
                                            const u64* __restrict__ rec,
                                            uint32_t t0, uint32_t t_end, WalkShared& ws, Header header,
                                            Visit visit) {
    const uint32_t lane = lane_id();
    const uint32_t t = t0 + lane;
    const bool valid = t < t_end;
    const u64 hdr = valid ? hdrs[t] : 0ull;
    const uint32_t s0 = valid && nseg > 1 ? tile_scope[t] : 0u;
    const bool single = valid && (u64)seg[s0].end >= min((u64)(t + 1) * kEmitTile, (u64)n);
    if (valid) header(t, hdr, s0, single);
    const uint32_t cnt = header_listed(hdr);
    const bool walk = valid && cnt == kRecWalk;
    const uint32_t c = valid && !walk ? cnt : 0u;
    const uint32_t incl = wave_inclusive_scan(c);
    const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
    wave_lds_sync();                       // the previous step's readers are done
    ws.excl[lane] = incl - c;
    ws.meta[lane] = s0 | (single ? 0x80000000u : 0u);
    wave_lds_sync();
    constexpr uint32_t kAhead = 4;         // entry loads in flight per lane
    for (uint32_t e0 = 0; e0 < total; e0 += 64 * kAhead) {
        u64 cmp[kAhead];
        uint32_t m[kAhead];
#pragma unroll
        for (uint32_t q = 0; q < kAhead; ++q) {
            const uint32_t e = e0 + q * 64 + lane;
            cmp[q] = 0;
            m[q] = 0;
            if (e < total) {
                uint32_t j = 0;            // the last lane whose running count does not exceed e owns entry e
#pragma unroll
                for (uint32_t step = 32; step >= 1; step >>= 1)
                    if (ws.excl[j + step] <= e) j += step;   // j + step <= 63
                cmp[q] = rec[(size_t)(t0 + j) * kRecSlots + (e - ws.excl[j])];
                m[q] = ws.meta[j];
            }
        }
#pragma unroll
        for (uint32_t q = 0; q < kAhead; ++q) {
            if (e0 + q * 64 + lane < total)
                visit(cmp[q], (m[q] & 0x80000000u) ? (m[q] & 0x7FFFFFFFu) : find_seg(seg, nseg, index_of(cmp[q])));
        }
    }
    // tiles whose undecided elements are not listed: the wave reads their weights
    u64 todo = __ballot(walk);
    while (todo != 0) {
        const uint32_t j = (uint32_t)__ffsll((long long)todo) - 1u;
        todo &= todo - 1;
        const uint32_t tw = t0 + j;
        const u64 a = (u64)tw * kEmitTile;
        const u64 b = min(a + kEmitTile, (u64)n);
        uint32_t sc = nseg > 1 ? tile_scope[tw] : 0u;
        uint32_t sc_end = seg[sc].end;
        uint32_t lo = state[sc].lo, hi = state[sc].hi, tie = state[sc].tie_key;
        for (u64 i = a + lane; i < b; i += 64) {
            if (advance_scope(seg, (uint32_t)i, sc, sc_end)) { lo = state[sc].lo; hi = state[sc].hi; tie = state[sc].tie_key; }
            const uint32_t key = key_of_bits(__float_as_uint(w[i]));
            if (key - lo < hi - lo && key != tie) visit(composite_of(key, (uint32_t)i), sc);   // tie-key elements are counted, never visited
        }
    }
}

// -------------------------------------------------------------------------------------- count1
// Digit-1 histogram of the undecided elements and, for sampled scopes, the number of elements above
// the bracket, per scope.  Few large workgroups, each over a contiguous range of tiles, so that
// the counts of a range meet in one LDS histogram before they go to the global one.  A workgroup
// works in rounds of up to 1024 tiles that start in the same scope; what a round meets of another
// scope (in a tile that crosses a boundary) is counted in global memory.
constexpr int kCountBlock = 1024;
constexpr uint32_t kCountBlocks = 256;

__global__ __launch_bounds__(kCountBlock) void count1_kernel(const float* __restrict__ w, uint32_t n,
                                                             const SegDesc* __restrict__ seg, uint32_t nseg,
                                                             const SegState* __restrict__ state, const Globals* glob,
                                                             const uint32_t* __restrict__ tile_scope,
                                                             const u64* __restrict__ hdrs, const u64* __restrict__ rec,
                                                             uint32_t* __restrict__ hist1,
                                                             uint32_t* __restrict__ kept_above,
                                                             uint32_t* __restrict__ tie_count, uint32_t pass) {
    constexpr uint32_t kWaves = kCountBlock / 64;
    __shared__ uint32_t lds[kDigit1Bins];
    __shared__ WalkShared ws[kWaves];
    __shared__ uint32_t sh_kept, sh_tie;
    if (pass != 0 && !glob->retry) return;
    for (uint32_t b = threadIdx.x; b < kDigit1Bins; b += kCountBlock) lds[b] = 0;
    if (threadIdx.x == 0) { sh_kept = 0; sh_tie = 0; }
    __syncthreads();
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t num_tiles = (uint32_t)(((u64)n + kEmitTile - 1) / kEmitTile);
    const uint32_t per_block = (num_tiles + gridDim.x - 1) / gridDim.x;
    const uint32_t t_begin = min(num_tiles, blockIdx.x * per_block);
    const uint32_t t_end = min(num_tiles, t_begin + per_block);
    const uint32_t kNone = 0xFFFFFFFFu;
    uint32_t cur = kNone;    // scope whose counts sit in LDS (same in every thread)

    auto flush = [&]() {
        __syncthreads();
        for (uint32_t b = threadIdx.x; b < kDigit1Bins; b += kCountBlock) {
            const uint32_t v = lds[b];
            if (v) {
                atomicAdd(&hist1[(size_t)cur * kDigit1Bins + b], v);
                lds[b] = 0;
            }
        }
        if (threadIdx.x == 0) {
            if (sh_kept) atomicAdd(&kept_above[cur], sh_kept);
            if (sh_tie) atomicAdd(&tie_count[cur], sh_tie);
            sh_kept = 0;
            sh_tie = 0;
        }
        __syncthreads();
    };

    uint32_t t = t_begin;
    while (t < t_end) {                                         // same trips in every thread
        const uint32_t s_round = nseg > 1 ? tile_scope[t] : 0u;
        uint32_t r_end = min(t_end, t + kWaves * 64);
        if (nseg > 1 && tile_scope[r_end - 1] != s_round) {
            // the round stops before the first tile that starts in another scope (tile_scope ascends)
            uint32_t lo_t = t, hi_t = r_end - 1;                // tile_scope[lo_t] == s_round < tile_scope[hi_t]
            while (hi_t - lo_t > 1) {
                const uint32_t mid = (lo_t + hi_t) >> 1;
                if (tile_scope[mid] == s_round) lo_t = mid; else hi_t = mid;
            }
            r_end = hi_t;
        }
        if (s_round != cur) {
            if (cur != kNone) flush();
            cur = s_round;
        }
        // the round's tiles in equal shares (of at most 64) over the waves, so that a short round
        // still occupies all of them
        const uint32_t share = (r_end - t + kWaves - 1) / kWaves;
        const uint32_t t0 = t + wave * share;
        if (t0 < r_end) {
            visit_tiles(w, n, seg, nseg, state, tile_scope, hdrs, rec, t0, min(r_end, t0 + share), ws[wave],
                [&](uint32_t tile, u64 hdr, uint32_t s0, bool single) {
                    // kept elements of a tile inside one scope (emit counted the others itself)
                    const uint32_t kept = header_kept(hdr);
                    if (single && kept != 0 && !state[s0].exact) {
                        if (s0 == cur) atomicAdd(&sh_kept, kept);
                        else atomicAdd(&kept_above[s0], kept);
                    }
                    // tie-key elements: of the tile's first scope, and of the large scope that begins inside it
                    const uint32_t th = header_tie_head(hdr), tt = header_tie_tail(hdr);
                    if (th != 0) {
                        if (s0 == cur) atomicAdd(&sh_tie, th);
                        else atomicAdd(&tie_count[s0], th);
                    }
                    if (tt != 0) {
                        const uint32_t last = (uint32_t)(min((u64)(tile + 1) * kEmitTile, (u64)n) - 1);
                        atomicAdd(&tie_count[find_seg(seg, nseg, last)], tt);
                    }
                },
                [&](u64 c, uint32_t s) {
                    const uint32_t d1 = digit1_of((uint32_t)(c >> 32), state[s].lo1, state[s].sh1, state[s].off1);
                    if (s == cur) atomicAdd(&lds[d1], 1u);
                    else atomicAdd(&hist1[(size_t)s * kDigit1Bins + d1], 1u);
                });
        }
        t = r_end;
    }
    if (cur != kNone) flush();
}

// ----------------------------------------------------------------------------------- compact2
// An undecided element whose digit 1 equals its scope's bin is a match.  There are only a few
// hundred matches per scope, and an append counter shared by all workgroups would cost one
// serialised global atomic per match; instead every workgroup collects the matches of its tiles in
// LDS and writes them to slots of its own, with their number, for `final` to pick up.
constexpr int kListBlock = 256;
constexpr uint32_t kListWaves = kMatchBlocks * (kListBlock / 64);   // waves of a compact2 / fixup launch

// Tiles [begin, end) of wave `gw` out of kListWaves: contiguous, equal shares.
__device__ __forceinline__ void wave_tile_range(uint32_t num_tiles, uint32_t gw, uint32_t& begin, uint32_t& end) {
    const uint32_t per_wave = (num_tiles + kListWaves - 1) / kListWaves;
    begin = min(num_tiles, gw * per_wave);
    end = min(num_tiles, begin + per_wave);
}

__global__ __launch_bounds__(kListBlock) void compact2_kernel(const float* __restrict__ w, uint32_t n,
                                                              const SegDesc* __restrict__ seg, uint32_t nseg,
                                                              const SegState* __restrict__ state, Globals* glob,
                                                              const uint32_t* __restrict__ tile_scope,
                                                              const u64* __restrict__ hdrs, const u64* __restrict__ rec,
                                                              u64* __restrict__ match,
                                                              uint32_t* __restrict__ match_count,
                                                              uint32_t* __restrict__ status) {
    __shared__ u64 found[kMatchSlotsPerBlock];
    __shared__ WalkShared ws[kListBlock / 64];
    __shared__ uint32_t nfound;
    if (threadIdx.x == 0) nfound = 0;
    __syncthreads();
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t num_tiles = (uint32_t)(((u64)n + kEmitTile - 1) / kEmitTile);
    uint32_t t_begin, t_end;
    wave_tile_range(num_tiles, blockIdx.x * (kListBlock / 64) + wave, t_begin, t_end);
    for (uint32_t t0 = t_begin; t0 < t_end; t0 += 64) {
        visit_tiles(w, n, seg, nseg, state, tile_scope, hdrs, rec, t0, t_end, ws[wave],
            [](uint32_t, u64, uint32_t, bool) {},
            [&](u64 c, uint32_t s) {
                if (!state[s].heavy &&
                    digit1_of((uint32_t)(c >> 32), state[s].lo1, state[s].sh1, state[s].off1) == state[s].bin1) {
                    const uint32_t pos = atomicAdd(&nfound, 1u);
                    if (pos < kMatchSlotsPerBlock) found[pos] = c;
                }
            });
    }
    __syncthreads();
    const uint32_t total = nfound;
    if (total > kMatchSlotsPerBlock && threadIdx.x == 0) {   // `final` uses the weights
        glob->match_overflow = 1;
        atomicOr(status, kDevSlowPath);
    }
    const uint32_t kept = min(total, kMatchSlotsPerBlock);
    if (threadIdx.x < kept) match[(size_t)blockIdx.x * kMatchSlotsPerBlock + threadIdx.x] = found[threadIdx.x];
    if (threadIdx.x == 0) match_count[blockIdx.x] = kept;
}

// -------------------------------------------------------------------------------------- final
// Resolves what digits 0 and 1 left open of C* for one scope: first the remaining bits of the key, then
// the 32 index bits.  The source is the scope's matches, gathered from the match slots into LDS (every
// one agrees with C* on digits 0 and 1), or, when the lists are not usable, the scope's weights filtered
// on the fly.  The tie key's elements are in no list: while key bits are resolved they count as one lump
// at their key; if the k-th key turns out to BE the tie key, the index of the k-th element follows from
// the tiles' tie counts in flat order (ties are kept in ascending index order) and one tile's weights.
constexpr int kFinalBlock = 1024;

// Digits of at most 8 bits, most significant first, from bit `from` of the composite down to bit `to`
// (both multiples of... any values with from > to >= 0; a digit never straddles bit 32, where the key ends).
// `lump` elements with composite bits `lump_c` (only its bits >= 32 matter) count besides the listed ones.
// Read from the weights, only keys in [key_lo, key_hi) take part.
template <bool FROM_LIST>
__device__ __forceinline__ void final_levels(const u64* list, uint32_t list_cnt,
                                             const float* __restrict__ w, uint32_t begin, uint32_t end,
                                             uint32_t key_lo, uint32_t key_hi,
                                             uint32_t from, uint32_t to, u64 lump_c, uint32_t lump,
                                             u64& prefix, uint32_t& krem, uint32_t* hist,
                                             uint32_t* wave_sums, uint32_t* found) {
    uint32_t resolved_above = from;   // bits >= this position are already fixed in `prefix`
    while (resolved_above > to) {
        const uint32_t room = resolved_above > 32 && to < 32 ? resolved_above - 32 : resolved_above - to;
        const uint32_t width = room >= 8 ? 8u : room;
        const uint32_t shift = resolved_above - width;
        if (threadIdx.x < 256) hist[threadIdx.x] = 0;
        __syncthreads();
        const uint32_t count = FROM_LIST ? list_cnt : end - begin;
        for (u64 j = threadIdx.x; j < count; j += kFinalBlock) {
            u64 c;
            if (FROM_LIST) {
                c = list[j];
            } else {
                const uint32_t i = begin + (uint32_t)j;
                const uint32_t key = key_of_bits(__float_as_uint(w[i]));
                if (key - key_lo >= key_hi - key_lo) continue;
                c = composite_of(key, i);
            }
            if (((c ^ prefix) >> resolved_above) == 0)
                atomicAdd(&hist[(uint32_t)(c >> shift) & ((1u << width) - 1u)], 1u);
        }
        if (threadIdx.x == 0 && lump != 0 && ((lump_c ^ prefix) >> resolved_above) == 0)
            atomicAdd(&hist[(uint32_t)(lump_c >> shift) & ((1u << width) - 1u)], lump);
        __syncthreads();
        // thread t < 256 owns bin t; walk from the highest bin down
        const uint32_t v = threadIdx.x < 256 ? hist[threadIdx.x] : 0u;
        uint32_t total;
        const uint32_t below = block_exclusive_scan<kFinalBlock>(v, wave_sums, total);
        const uint32_t above = total - below - v;
        if (v != 0 && above < krem && krem <= above + v) {
            found[0] = threadIdx.x;
            found[1] = krem - above;
        }
        __syncthreads();
        prefix |= (u64)found[0] << shift;
        krem = found[1];
        resolved_above = shift;
        __syncthreads();
    }
}

__global__ __launch_bounds__(kFinalBlock) void final_kernel(const float* __restrict__ w, uint32_t n,
                                                            const SegDesc* __restrict__ seg, uint32_t nseg,
                                                            SegState* __restrict__ state, const Globals* glob,
                                                            const uint32_t* __restrict__ tile_scope,
                                                            const u64* __restrict__ hdrs,
                                                            const uint32_t* __restrict__ tie_count,
                                                            const u64* __restrict__ match,
                                                            const uint32_t* __restrict__ match_count) {
    __shared__ u64 list[kFinalList];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t wave_sums[kFinalBlock / 64];
    __shared__ uint32_t found[2];
    __shared__ uint32_t gathered;
    __shared__ uint32_t sh_tile, sh_rank, sh_index;
    const uint32_t s = blockIdx.x;
    SegState* st = state + s;
    if (!st->active) return;
    // The keys of digit-1 bin b1 share all bits from sh1 up (lo1 is a multiple of 2^sh1) - except for
    // digit 0 of a digit 1 that starts above the bracket's lower end, which is just "every key below lo1".
    const uint32_t bin1 = st->bin1, off1 = st->off1;
    const bool below_lo1 = off1 != 0 && bin1 == 0;
    const uint32_t key_bits = below_lo1 ? 31u : st->sh1;
    u64 prefix = below_lo1 ? 0ull : (u64)(st->lo1 + ((bin1 - off1) << st->sh1)) << 32;
    uint32_t krem = st->krem1;
    const uint32_t begin = seg[s].begin, end = seg[s].end;
    if (threadIdx.x == 0) {
        found[0] = 0; found[1] = 0; gathered = 0;
        sh_tile = begin / kEmitTile; sh_rank = 0; sh_index = begin;   // in range whatever the counts say
    }
    __syncthreads();
    const bool from_list = !glob->match_overflow && !st->heavy;
    const uint32_t tie_key = st->tie_key;
    if (!from_list) {
        // every element of the scope is read from the weights, the tie key's among them: no lump
        // (only undecided keys take part: a digit-1 bin may reach beyond the bracket's upper end)
        final_levels<false>(nullptr, 0, w, begin, end, st->lo, below_lo1 ? st->lo1 : st->hi,
                            32u + key_bits, 0u, 0ull, 0u, prefix, krem, hist, wave_sums, found);
        if (threadIdx.x == 0) st->cstar = prefix;
        return;
    }
    // Matches of this scope: thread t looks through the slots of compact2's workgroup t.
    static_assert(kFinalBlock == (int)kMatchBlocks, "one thread per compact2 workgroup");
    const uint32_t mine = min(match_count[threadIdx.x], kMatchSlotsPerBlock);
    for (uint32_t e = 0; e < mine; ++e) {
        const u64 c = match[(size_t)threadIdx.x * kMatchSlotsPerBlock + e];
        const uint32_t i = index_of(c);
        if (i >= begin && i < end) {
            const uint32_t pos = atomicAdd(&gathered, 1u);
            if (pos < kFinalList) list[pos] = c;
        }
    }
    __syncthreads();
    const uint32_t count = min(gathered, kFinalList);
    const uint32_t lump = st->tie_in ? tie_count[s] : 0u;
    const u64 lump_c = (u64)tie_key << 32;
    final_levels<true>(list, count, nullptr, 0, 0, 0u, 0u, 32u + key_bits, 32u, lump_c, lump, prefix, krem, hist, wave_sums, found);
    if (lump == 0 || (uint32_t)(prefix >> 32) != tie_key) {
        // an ordinary key: the listed elements that carry it, by index
        final_levels<true>(list, count, nullptr, 0, 0, 0u, 0u, 32u, 0u, 0ull, 0u, prefix, krem, hist, wave_sums, found);
        if (threadIdx.x == 0) st->cstar = prefix;
        return;
    }

    // The k-th key is the tie key: the krem-th of its elements in flat order is the last one kept.
    // Tile counts in order: the scope's first tile may hold it as the tile's tail scope; every later tile
    // of the scope starts inside it.
    const uint32_t t_first = begin / kEmitTile, t_end = (end - 1u) / kEmitTile + 1u;
    const uint32_t first_is_head = (nseg > 1 ? tile_scope[t_first] : 0u) == s ? 1u : 0u;
    auto ties_of = [&](uint32_t t) {
        const u64 hdr = hdrs[t];
        return t == t_first && !first_is_head ? header_tie_tail(hdr) : header_tie_head(hdr);
    };
    const uint32_t per = (t_end - t_first + kFinalBlock - 1) / kFinalBlock;
    const uint32_t my_first = min(t_end, t_first + threadIdx.x * per), my_end = min(t_end, my_first + per);
    uint32_t my_sum = 0;
    for (uint32_t t = my_first; t < my_end; t += 8) {        // eight header loads in flight
        uint32_t c[8];
#pragma unroll
        for (uint32_t q = 0; q < 8; ++q) c[q] = ties_of(min(t + q, my_end - 1));
#pragma unroll
        for (uint32_t q = 0; q < 8; ++q) my_sum += t + q < my_end ? c[q] : 0u;
    }
    uint32_t total;
    const uint32_t before = block_exclusive_scan<kFinalBlock>(my_sum, wave_sums, total);
    if (before < krem && krem <= before + my_sum) {
        uint32_t acc = before;
        for (uint32_t t = my_first; t < my_end; ++t) {
            const uint32_t c = ties_of(t);
            if (krem <= acc + c) { sh_tile = t; sh_rank = krem - acc; break; }
            acc += c;
        }
    }
    __syncthreads();
    // that tile's part of the scope, four consecutive elements per thread: the sh_rank-th tie-key element
    const uint32_t tile = sh_tile, want = sh_rank;
    const u64 ta = max((u64)tile * kEmitTile, (u64)begin), tb = min((u64)(tile + 1) * kEmitTile, (u64)end);
    uint32_t hits[4], mine_n = 0;
#pragma unroll
    for (uint32_t q = 0; q < 4; ++q) {
        const u64 i = (u64)tile * kEmitTile + threadIdx.x * 4u + q;
        hits[q] = i >= ta && i < tb && key_of_bits(__float_as_uint(w[i])) == tie_key ? 1u : 0u;
        mine_n += hits[q];
    }
    const uint32_t ahead = block_exclusive_scan<kFinalBlock>(mine_n, wave_sums, total);
    if (ahead < want && want <= ahead + mine_n) {
        uint32_t acc = ahead;
#pragma unroll
        for (uint32_t q = 0; q < 4; ++q) {
            acc += hits[q];
            if (hits[q] && acc == want) sh_index = tile * kEmitTile + threadIdx.x * 4u + q;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) st->cstar = composite_of(tie_key, sh_index);
}

// -------------------------------------------------------------------------------- small scopes
// One workgroup resolves one small scope completely: keys into LDS, a radix select over the 31 key
// bits, then the tie rule by position - among the elements equal
// to the threshold key the first r in flat order are kept - with one ballot per mask word, a wave
// owning the 64 elements of one word.  Words that lie inside the scope are stored (emit left them
// zero), the two words shared with neighbouring scopes are OR-ed.
// Two size classes, so that the many very short vectors of a model run with small workgroups and
// little LDS, many to a compute unit: scopes of up to kTinyScope elements with 256 threads, the rest
// with 1024.
template <int kSmallBlock, uint32_t kMaxLen>
__global__ __launch_bounds__(kSmallBlock) void small_scope_kernel(const float* __restrict__ w,
                                                                  const SegDesc* __restrict__ seg,
                                                                  u64* __restrict__ mask, uint32_t min_len) {
    constexpr uint32_t kSmallWords = kMaxLen / 64 + 2;     // mask words one scope of this class can touch
    static_assert(kSmallWords <= (uint32_t)kSmallBlock, "one thread per word in the scan over words");
    extern __shared__ uint32_t keys[];                     // [scope length]
    __shared__ uint32_t hist[2048];
    __shared__ uint32_t wave_sums[kSmallBlock / 64];
    __shared__ uint32_t found[2];
    __shared__ uint32_t eq_before[kSmallWords];
    const SegDesc d = seg[blockIdx.x];
    if (d.stride != 0) return;                             // not a small scope
    const uint32_t begin = d.begin, end = d.end, len = end - begin, k = d.k;
    if (len < min_len || len > kMaxLen) return;            // the other size class
    if (len == 0 || k == 0) return;                        // nothing kept: emit wrote the zeros
    // eight loads in flight per thread: one load per trip would make a long scope wait for memory
    // thirty-two times in a row
    for (uint32_t j0 = threadIdx.x; j0 < len; j0 += kSmallBlock * 8) {
        uint32_t v[8];
#pragma unroll
        for (uint32_t q = 0; q < 8; ++q) {
            const uint32_t j = min(j0 + q * kSmallBlock, len - 1u);   // clamped, not branched: the loads stay together
            v[q] = __float_as_uint(w[begin + j]);
        }
#pragma unroll
        for (uint32_t q = 0; q < 8; ++q) {
            const uint32_t j = j0 + q * kSmallBlock;
            if (j < len) keys[j] = key_of_bits(v[q]);
        }
    }
    if (threadIdx.x == 0) { found[0] = 0; found[1] = 0; }
    __syncthreads();

    // key of the k-th largest element, and its rank r among the elements with that key: digits of
    // 11, 10 and 10 bits, most significant first.  (The leading byte of a float key is its exponent,
    // which takes only a handful of values in a weight tensor and would serialise the LDS atomics
    // on a few bins; three more bits spread the counts.)  A thread adds a run of equal digits at once.
    constexpr uint32_t kBins = 2048, kPer = kBins / kSmallBlock;
    uint32_t prefix = 0, krem = k, resolved_above = 31;
    while (resolved_above > 0) {
        const uint32_t width = resolved_above == 31 ? 11u : 10u;
        const uint32_t shift = resolved_above - width;
        for (uint32_t b = threadIdx.x; b < kBins; b += kSmallBlock) hist[b] = 0;
        __syncthreads();
        uint32_t run_digit = 0, run = 0;
        for (uint32_t j = threadIdx.x; j < len; j += kSmallBlock) {
            const uint32_t key = keys[j];
            if (((key ^ prefix) >> resolved_above) == 0) {
                const uint32_t digit = (key >> shift) & ((1u << width) - 1u);
                if (run != 0 && digit != run_digit) {
                    atomicAdd(&hist[run_digit], run);
                    run = 0;
                }
                run_digit = digit;
                ++run;
            }
        }
        if (run != 0) atomicAdd(&hist[run_digit], run);
        __syncthreads();
        // thread t owns bins [t * kPer, (t + 1) * kPer); walk from the highest bin down
        uint32_t loc[kPer], v = 0;
#pragma unroll
        for (uint32_t q = 0; q < kPer; ++q) { loc[q] = hist[threadIdx.x * kPer + q]; v += loc[q]; }
        uint32_t total;
        const uint32_t below = block_exclusive_scan<kSmallBlock>(v, wave_sums, total);
        uint32_t above = total - below - v;
        if (v != 0 && above < krem && krem <= above + v) {
#pragma unroll
            for (int q = (int)kPer - 1; q >= 0; --q) {
                if (above < krem && krem <= above + loc[q]) {
                    found[0] = threadIdx.x * kPer + (uint32_t)q;
                    found[1] = krem - above;
                }
                above += loc[q];
            }
        }
        __syncthreads();
        prefix |= found[0] << shift;
        krem = found[1];
        resolved_above = shift;
        __syncthreads();
    }
    const uint32_t thr = prefix, r = krem;

    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6;
    const uint32_t base0 = begin & ~63u;                   // first element of the first word touched
    const uint32_t words = (uint32_t)(((u64)end - base0 + 63) >> 6);
    for (uint32_t wd = wave; wd < words; wd += kSmallBlock / 64) {
        const u64 g = (u64)base0 + wd * 64u + lane;
        const bool eq = g >= begin && g < end && keys[g - begin] == thr;
        const u64 m = __ballot(eq);
        if (lane == 0) eq_before[wd] = (uint32_t)__popcll(m);
    }
    __syncthreads();
    {
        // exclusive scan over the words' counts of threshold-equal elements
        uint32_t total;
        const uint32_t v = threadIdx.x < words ? eq_before[threadIdx.x] : 0u;
        const uint32_t ex = block_exclusive_scan<kSmallBlock>(v, wave_sums, total);
        if (threadIdx.x < words) eq_before[threadIdx.x] = ex;
        __syncthreads();
    }
    for (uint32_t wd = wave; wd < words; wd += kSmallBlock / 64) {
        const u64 g0 = (u64)base0 + wd * 64u;
        const u64 g = g0 + lane;
        const bool valid = g >= begin && g < end;
        const uint32_t key = valid ? keys[g - begin] : 0u;
        const bool eq = valid && key == thr;
        const u64 eqm = __ballot(eq);
        const bool keep = valid && (key > thr || (eq && eq_before[wd] + lanes_below(eqm) < r));
        const u64 bits = __ballot(keep);
        if (lane == 0 && bits != 0) {
            if (g0 >= begin && g0 + 64 <= end) mask[g0 >> 6] = bits;
            else atomicOr(&mask[g0 >> 6], bits);
        }
    }
}

// -------------------------------------------------------------------------------------- fixup
// Undecided elements at or above their scope's C* are kept: set their mask bits.  Listed elements (and
// those of walked tiles) one by one; the tie key's elements, which no list holds, by reading again the
// tiles in which some of them are kept - none if the k-th key lies above the tie key (the zeros of a
// pruned model), the tiles up to the one that holds the k-th element if it is the tie key itself.
__global__ __launch_bounds__(kListBlock) void fixup_kernel(const float* __restrict__ w, uint32_t n,
                                                           const SegDesc* __restrict__ seg, uint32_t nseg,
                                                           const SegState* __restrict__ state,
                                                           const uint32_t* __restrict__ tile_scope,
                                                           const u64* __restrict__ hdrs, const u64* __restrict__ rec,
                                                           u64* __restrict__ mask, u64* __restrict__ tile_state,
                                                           uint32_t scan_tiles) {
    __shared__ WalkShared ws[kListBlock / 64];
    // The scan that follows starts from cleared tile states.
    for (u64 j = (u64)blockIdx.x * kListBlock + threadIdx.x; j < scan_tiles; j += (u64)gridDim.x * kListBlock)
        tile_state[j] = 0;
    const uint32_t lane = lane_id();
    const uint32_t wave = threadIdx.x >> 6;
    const uint32_t num_tiles = (uint32_t)(((u64)n + kEmitTile - 1) / kEmitTile);
    uint32_t t_begin, t_end;
    wave_tile_range(num_tiles, blockIdx.x * (kListBlock / 64) + wave, t_begin, t_end);
    for (uint32_t t0 = t_begin; t0 < t_end; t0 += 64) {
        visit_tiles(w, n, seg, nseg, state, tile_scope, hdrs, rec, t0, t_end, ws[wave],
            [](uint32_t, u64, uint32_t, bool) {},
            [&](u64 c, uint32_t s) {
                if (c >= state[s].cstar) {
                    const uint32_t i = index_of(c);
                    atomicOr(&mask[i >> 6], 1ull << (i & 63u));
                }
            });
    }

    // Tie-key elements that are kept.  The tiles concerned form runs (all tiles of a constant tensor up to
    // the one that holds the k-th element), so the waves take tiles at a stride of the whole launch: a
    // run is shared by all of them.  Lane l looks at the header of the wave's l-th tile.
    const uint32_t gw = blockIdx.x * (kListBlock / 64) + wave;
    for (uint32_t base = gw; base < num_tiles; base += 64u * kListWaves) {
        const u64 tl = (u64)base + (u64)lane * kListWaves;
        bool reread = false;
        if (tl < num_tiles) {
            const uint32_t tile = (uint32_t)tl;
            const u64 hdr = hdrs[tile];
            const uint32_t s0 = nseg > 1 ? tile_scope[tile] : 0u;
            // The first element of a part has the largest composite its tie-key elements can have.
            if (header_tie_head(hdr) != 0 && state[s0].tie_key != kNoTieKey &&
                composite_of(state[s0].tie_key, tile * kEmitTile) >= state[s0].cstar)
                reread = true;
            if (header_tie_tail(hdr) != 0) {
                const uint32_t last = (uint32_t)(min((u64)(tile + 1) * kEmitTile, (u64)n) - 1);
                const uint32_t s1 = find_seg(seg, nseg, last);
                if (state[s1].tie_key != kNoTieKey && composite_of(state[s1].tie_key, seg[s1].begin) >= state[s1].cstar)
                    reread = true;
            }
        }
        u64 todo = __ballot(reread);
        while (todo != 0) {
            const uint32_t j = (uint32_t)__ffsll((long long)todo) - 1u;
            todo &= todo - 1;
            const uint32_t tw = base + j * kListWaves;
            const u64 a = (u64)tw * kEmitTile;
            uint32_t sc = nseg > 1 ? tile_scope[tw] : 0u;
            uint32_t sc_end = seg[sc].end;
            uint32_t tie = state[sc].tie_key;
            u64 cstar = state[sc].cstar;
            // 64 rows of 64 elements, one mask word per row; 16 rows' loads in flight
            for (uint32_t r0 = 0; r0 < kEmitTile / 64; r0 += 16) {
                uint32_t v[16];
#pragma unroll
                for (uint32_t q = 0; q < 16; ++q) {
                    const u64 i = a + (u64)(r0 + q) * 64 + lane;
                    v[q] = i < n ? __float_as_uint(w[i]) : 0u;
                }
#pragma unroll
                for (uint32_t q = 0; q < 16; ++q) {
                    const u64 i = a + (u64)(r0 + q) * 64 + lane;
                    const bool valid = i < n;
                    if (valid && advance_scope(seg, (uint32_t)i, sc, sc_end)) { tie = state[sc].tie_key; cstar = state[sc].cstar; }
                    const uint32_t key = key_of_bits(v[q]);
                    const u64 bits = __ballot(valid && key == tie && composite_of(key, (uint32_t)i) >= cstar);
                    if (bits != 0 && lane == 0) atomicOr(&mask[(a >> 6) + r0 + q], bits);
                }
            }
        }
    }
}

// --------------------------------------------------------------------------------------- scan
// prefix[j] = number of set bits in mask words 0..j-1: a single-pass scan with decoupled
// look-back.  A workgroup takes the next tile from a ticket counter (so every tile before it is
// owned by a workgroup that is already running), publishes the tile's bit count, then walks back
// over its predecessors' published values until it meets one that already holds an inclusive
// prefix.  Status and value share one 64-bit word, read and written with device-scope atomics, so
// no other data needs ordering across the XCDs' L2 caches.  The wait for a predecessor is bounded:
// a workgroup that gives up raises kDevScanStalled in the context's status word and finishes (with
// wrong offsets) rather than spin; the caller reads the word with pac_device_status.  The last tile
// compares the total with the count the host expects (kDevCountMismatch).
// The tile size follows the size of the mask (scan_iters_for): a tile per workgroup must be small
// enough for the tiles to fill the chip, and large enough that the look-back chain stays short.
constexpr int kScanBlock = 1024;
constexpr int kScanWaves = kScanBlock / 64;
constexpr uint32_t scan_tile_words(uint32_t iters) { return kScanWaves * 64u * 2u * iters; }   // iters 16-byte loads per lane
constexpr u64 kTileAggregate = 1ull << 32;   // value = bits in this tile
constexpr u64 kTileInclusive = 2ull << 32;   // value = bits in this tile and all before it

__device__ __forceinline__ u64 tile_load(const u64* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void tile_store(u64* p, u64 v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

template <uint32_t kScanIters>
__global__ __launch_bounds__(kScanBlock) void scan_lookback_kernel(const u64* __restrict__ mask, uint32_t words,
                                                                   u64* __restrict__ tile_state, Globals* glob,
                                                                   uint32_t* __restrict__ prefix,
                                                                   u64* __restrict__ total_out, u64 expect_total,
                                                                   uint32_t* __restrict__ status, uint32_t spin_limit) {
    __shared__ uint32_t ex_lds[kScanIters][kScanBlock];
    __shared__ uint32_t wave_totals[kScanWaves];
    __shared__ uint32_t sh_tile, sh_base;
    if (threadIdx.x == 0) sh_tile = atomicAdd(&glob->scan_ticket, 1u);
    __syncthreads();
    const uint32_t tile = sh_tile;
    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6;
    constexpr uint32_t kScanWaveWords = 64 * 2 * kScanIters, kScanTile = kScanWaves * kScanWaveWords;

    // A lane owns two consecutive words per iteration (one 16-byte load); a wave kScanWaveWords consecutive words.
    const u64 wave_first = (u64)tile * kScanTile + wave * kScanWaveWords;
    uint32_t pp[kScanIters];   // popcounts of the lane's two words, packed: low byte first word, next byte second
#pragma unroll
    for (uint32_t it = 0; it < kScanIters; ++it) {
        const u64 w0 = wave_first + it * 128u + lane * 2u;
        if (w0 + 1 < words) {
            const ulonglong2 v = *reinterpret_cast<const ulonglong2*>(mask + w0);
            pp[it] = (uint32_t)__popcll(v.x) | ((uint32_t)__popcll(v.y) << 8);
        } else {
            pp[it] = w0 < words ? (uint32_t)__popcll(mask[w0]) : 0u;
        }
    }
    // ex_lds[it][thread]: bits before the lane's first word, within the wave's chunk (parked in LDS
    // to keep the register count of a 16-wave workgroup down)
    uint32_t running = 0;
#pragma unroll
    for (uint32_t it = 0; it < kScanIters; ++it) {
        const uint32_t s = (pp[it] & 0xFFu) + (pp[it] >> 8);
        const uint32_t inc = wave_inclusive_scan(s);
        ex_lds[it][threadIdx.x] = running + inc - s;
        running += (uint32_t)__shfl((int)inc, 63, 64);
    }
    if (lane == 0) wave_totals[wave] = running;
    __syncthreads();
    uint32_t wave_off = 0, tile_total = 0;
#pragma unroll
    for (int i = 0; i < kScanWaves; ++i) {
        const uint32_t x = wave_totals[i];
        if ((uint32_t)i < wave) wave_off += x;
        tile_total += x;
    }

    if (threadIdx.x < 64) {   // wave 0 publishes and looks back
        if (tile == 0) {
            if (lane == 0) {
                tile_store(&tile_state[0], kTileInclusive | tile_total);
                sh_base = 0;
            }
        } else {
            if (lane == 0) tile_store(&tile_state[tile], kTileAggregate | tile_total);
            uint32_t before = 0;          // bits in the tiles walked so far
            uint32_t window = tile;       // lanes look at tiles window-1, window-2, ...
            bool stalled = false;
            while (true) {
                const bool real = lane < window;
                const u64* slot = &tile_state[real ? window - 1 - lane : 0];
                u64 st = real ? tile_load(slot) : kTileInclusive;   // "before tile 0": inclusive 0
                uint32_t spins = 0;
                while (__any((st >> 32) == 0)) {
                    if ((st >> 32) == 0) st = tile_load(slot);
                    if (++spins > spin_limit) { stalled = true; break; }
                    __builtin_amdgcn_s_sleep(1);
                }
                if (stalled) break;
                const u64 incl = __ballot((st >> 32) == 2);
                if (incl != 0) {
                    const uint32_t stop = (uint32_t)__ffsll((long long)incl) - 1u;   // nearest inclusive tile
                    before += wave_sum(lane <= stop ? (uint32_t)st : 0u);
                    break;
                }
                before += wave_sum((uint32_t)st);
                window -= 64;
            }
            if (lane == 0) {
                if (stalled) atomicOr(status, kDevScanStalled);
                tile_store(&tile_state[tile], kTileInclusive | (u64)(before + tile_total));
                sh_base = before;
            }
        }
    }
    __syncthreads();
    const uint32_t base = sh_base + wave_off;
    // the last tile knows the number of set bits of the whole mask
    if (tile == gridDim.x - 1 && threadIdx.x == 0) {
        const u64 total = (u64)sh_base + tile_total;
        if (total_out != nullptr) *total_out = total;
        if (expect_total != kNoExpectedTotal && total != expect_total) atomicOr(status, kDevCountMismatch);
    }
#pragma unroll
    for (uint32_t it = 0; it < kScanIters; ++it) {
        const u64 w0 = wave_first + it * 128u + lane * 2u;
        const uint32_t a = base + ex_lds[it][threadIdx.x];
        if (w0 + 1 < words) {
            *reinterpret_cast<uint2*>(prefix + w0) = make_uint2(a, a + (pp[it] & 0xFFu));
        } else if (w0 < words) {
            prefix[w0] = a;
        }
    }
}

// Clears the scan's tile states and ticket for a scan that does not follow a mask build.
__global__ void scan_reset_kernel(u64* __restrict__ tile_state, uint32_t tiles, Globals* glob, uint32_t* clear_status) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i <= tiles) tile_state[i] = 0;
    if (i == 0) {
        glob->scan_ticket = 0;
        if (clear_status != nullptr) *clear_status = 0;
    }
}

inline uint32_t div_up_u64(u64 a, u64 b) { return (uint32_t)((a + b - 1) / b); }

// 16-byte loads per lane of the scan for a mask of `words` words (measured: 4096-word tiles up to
// 32M elements, 8192-word tiles up to 256M, 32768-word tiles above).
inline uint32_t scan_iters_for(uint32_t words) { return words <= (1u << 19) ? 2u : words <= (1u << 22) ? 4u : 16u; }
inline uint32_t scan_tiles_for(uint32_t words) { return div_up_u64(words, scan_tile_words(scan_iters_for(words))); }

inline void launch_scan(const MaskScratch& s, const u64* d_mask, uint32_t words, uint32_t* d_prefix,
                        u64* d_total_out, u64 expect_total, hipStream_t stream) {
    const uint32_t tiles = scan_tiles_for(words);
    switch (scan_iters_for(words)) {
        case 2:
            hipLaunchKernelGGL((scan_lookback_kernel<2>), dim3(tiles), dim3(kScanBlock), 0, stream, d_mask, words,
                               s.tile_state, s.glob, d_prefix, d_total_out, expect_total, s.status, s.scan_spin_limit);
            break;
        case 4:
            hipLaunchKernelGGL((scan_lookback_kernel<4>), dim3(tiles), dim3(kScanBlock), 0, stream, d_mask, words,
                               s.tile_state, s.glob, d_prefix, d_total_out, expect_total, s.status, s.scan_spin_limit);
            break;
        default:
            hipLaunchKernelGGL((scan_lookback_kernel<16>), dim3(tiles), dim3(kScanBlock), 0, stream, d_mask, words,
                               s.tile_state, s.glob, d_prefix, d_total_out, expect_total, s.status, s.scan_spin_limit);
    }
}

__global__ void status_read_kernel(uint32_t* status, uint32_t* out, uint32_t clear) {
    const uint32_t v = clear ? atomicExch(status, 0u) : __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (out != nullptr) *out = v;
}

// Workgroups of a persistent kernel that fit on the device at once.
template <typename K>
uint32_t resident_blocks(K kernel, int block, int num_cu, uint32_t fallback_per_cu) {
    int per_cu = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, block, 0) != hipSuccess || per_cu <= 0)
        per_cu = (int)fallback_per_cu;
    return (uint32_t)per_cu * (uint32_t)num_cu;
}

}  // namespace

hipError_t prepare_mask_kernels() {
    return hipFuncSetAttribute(reinterpret_cast<const void*>(small_scope_kernel<1024, kSmallScope>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kSmallScope * sizeof(uint32_t)));
}

uint32_t mask_hist_blocks(int num_cu) { return resident_blocks(hist0_kernel<true>, kHistBlock, num_cu, 2); }

hipError_t launch_status_read(uint32_t* d_status, uint32_t* d_out, bool clear, hipStream_t stream) {
    hipLaunchKernelGGL(status_read_kernel, dim3(1), dim3(1), 0, stream, d_status, d_out, clear ? 1u : 0u);
    return hipGetLastError();
}

hipError_t launch_build_mask(const MaskScratch& s, const float* d_weights, uint32_t n, uint32_t nseg,
                             uint32_t slots0, uint32_t slots1, bool any_sampled, uint32_t max_tiny, uint32_t max_small,
                             bool fresh_table, unsigned long long* d_mask, uint32_t* d_prefix,
                             unsigned long long expect_total, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const uint32_t words = div_up_u64(n, 64);
    const bool aligned = (reinterpret_cast<uintptr_t>(d_weights) & 15u) == 0;
    const uint32_t emit_tiles = div_up_u64(n, kEmitTile);

    if (fresh_table && nseg > 1)
        hipLaunchKernelGGL(tile_scope_kernel, dim3(div_up_u64(emit_tiles, 256)), dim3(256), 0, stream, s.seg, nseg,
                           emit_tiles, s.tile_scope);

    // a record takes what the candidate capacity allows per tile (all of its slots unless a test lowered it)
    const uint32_t per_tile = (uint32_t)(s.cand_cap / emit_tiles);
    const uint32_t rec_cap = per_tile < kRecSlots ? per_tile : kRecSlots;
    // Pass 0 works from (possibly sampled) histograms; pass 1 repeats the five kernels with full
    // counts if a sampled bracket missed, and returns at once otherwise.
    // (A table with no sampled scope cannot miss: the second round is not even launched.)
    const uint32_t passes = any_sampled ? 2u : 1u;
    for (uint32_t pass = 0; pass < passes; ++pass) {
        // No more workgroups than fit on the device at once, nor than there are slots (the sampled pass
        // has few).  A table of small scopes only has no slot: one workgroup still clears the counters.
        const uint32_t slots = pass == 0 ? slots0 : slots1;
        uint32_t grid = slots < s.hist_blocks ? slots : s.hist_blocks;
        if (grid == 0) grid = 1;
        if (aligned)
            hipLaunchKernelGGL((hist0_kernel<true>), dim3(grid), dim3(kHistBlock), 0, stream, d_weights, n,
                               s.seg, nseg, s.hist0, s.glob, pass, slots);
        else
            hipLaunchKernelGGL((hist0_kernel<false>), dim3(grid), dim3(kHistBlock), 0, stream, d_weights, n,
                               s.seg, nseg, s.hist0, s.glob, pass, slots);
        hipLaunchKernelGGL(select0_kernel, dim3(nseg), dim3(kDigit0Bins / 16), 0, stream, d_weights, s.seg, s.state,
                           s.hist0, s.kept_above, s.tie_count, s.glob, pass);
        // One workgroup per tile; the retry pass, which almost never runs, strides over the tiles
        // with a small grid so that its launch costs little.
        const uint32_t emit_grid = pass == 0 || emit_tiles < 2048 ? emit_tiles : 2048u;
        hipLaunchKernelGGL(emit_kernel, dim3(emit_grid), dim3(kEmitBlock), 0, stream, d_weights, n, s.seg, nseg,
                           s.state, s.glob, s.tile_scope, s.kept_above, s.hdrs, s.rec, rec_cap, d_mask, pass);
        if (pass + 1 == passes && max_small != 0) {
            // after the last emit (it writes the small scopes' words as zero): fork
            hipError_t r = hipEventRecord(s.fork_event, stream);
            if (r == hipSuccess) r = hipStreamWaitEvent(s.side_stream, s.fork_event, 0);
            if (r != hipSuccess) return r;
            if (max_tiny != 0)
                hipLaunchKernelGGL((small_scope_kernel<256, kTinyScope>), dim3(nseg), dim3(256),
                                   (size_t)max_tiny * sizeof(uint32_t), s.side_stream, d_weights, s.seg, d_mask, 0u);
            if (max_small > kTinyScope)
                hipLaunchKernelGGL((small_scope_kernel<1024, kSmallScope>), dim3(nseg), dim3(1024),
                                   (size_t)max_small * sizeof(uint32_t), s.side_stream, d_weights, s.seg, d_mask,
                                   kTinyScope + 1u);
            r = hipEventRecord(s.join_event, s.side_stream);
            if (r != hipSuccess) return r;
        }
        const uint32_t count_grid = emit_tiles < kCountBlocks ? emit_tiles : kCountBlocks;
        hipLaunchKernelGGL(count1_kernel, dim3(count_grid), dim3(kCountBlock), 0, stream, d_weights, n, s.seg, nseg,
                           s.state, s.glob, s.tile_scope, s.hdrs, s.rec, s.hist1, s.kept_above, s.tie_count, pass);
        hipLaunchKernelGGL(select1_kernel, dim3(nseg), dim3(kDigit1Bins / 16), 0, stream, s.seg, s.state, s.hist1,
                           s.kept_above, s.tie_count, s.glob, s.status, pass);
    }

    hipLaunchKernelGGL(compact2_kernel, dim3(kMatchBlocks), dim3(kListBlock), 0, stream, d_weights, n, s.seg, nseg,
                       s.state, s.glob, s.tile_scope, s.hdrs, s.rec, s.match, s.match_count, s.status);
    hipLaunchKernelGGL(final_kernel, dim3(nseg), dim3(kFinalBlock), 0, stream, d_weights, n, s.seg, nseg, s.state,
                       s.glob, s.tile_scope, s.hdrs, s.tie_count, s.match, s.match_count);
    const uint32_t scan_tiles = scan_tiles_for(words);
    hipLaunchKernelGGL(fixup_kernel, dim3(kMatchBlocks), dim3(kListBlock), 0, stream, d_weights, n, s.seg, nseg,
                       s.state, s.tile_scope, s.hdrs, s.rec, d_mask, s.tile_state, scan_tiles);
    if (max_small != 0) {   // join: the scan reads the small scopes' words
        hipError_t r = hipStreamWaitEvent(stream, s.join_event, 0);
        if (r != hipSuccess) return r;
    }
    launch_scan(s, d_mask, words, d_prefix, static_cast<u64*>(nullptr), expect_total, stream);
    return hipGetLastError();
}

static_assert(scan_tile_words(2) * 128 >= (1u << 19) && scan_tile_words(4) * 512 >= (1u << 22) &&
              (u64)scan_tile_words(16) * kScanMaxTiles >= (1ull << 26), "no mask below 2^32 bits needs more than kScanMaxTiles tiles");

hipError_t launch_prefix_scan(const MaskScratch& s, const unsigned long long* d_mask, uint32_t words,
                              uint32_t* d_prefix, unsigned long long* d_total_out, bool reset_status,
                              hipStream_t stream) {
    if (words == 0) return hipSuccess;
    const uint32_t scan_tiles = scan_tiles_for(words);
    hipLaunchKernelGGL(scan_reset_kernel, dim3(div_up_u64(scan_tiles + 1, 256)), dim3(256), 0, stream, s.tile_state,
                       scan_tiles, s.glob, reset_status ? s.status : static_cast<uint32_t*>(nullptr));
    launch_scan(s, d_mask, words, d_prefix, d_total_out, kNoExpectedTotal, stream);
    return hipGetLastError();
}

}  // namespace pac
