// pac_build_mask: magnitude threshold at a target sparsity -> bitmask + exclusive prefix index.
//
// Per prune scope the kept set is "the k largest composites" (see pac_internal.h).  The k-th
// composite C* is found by a most-significant-digit radix select:
//
//   hist0    one pass over the weights: per-scope histogram of digit 0 (LDS histograms,
//            flushed to a global histogram per scope)
//   select0  per scope: the digit-0 bin b0 that holds the k-th element, its rank inside the bin
//   emit     second pass over the weights: mask bit = digit0 > b0 (wave ballot -> 64-bit word);
//            elements with digit0 == b0 are undecided: their composites go to the scope's
//            candidate list and are counted by digit 1
//   select1  per scope: digit-1 bin b1, rank inside it
//   compact2 candidates whose digit 1 is b1 -> second-level list (a few hundred elements)
//   final    one workgroup per scope resolves the remaining 37 bits on that list -> C*
//   fixup    candidates with composite >= C* get their mask bit set (atomic OR)
//   scan     exclusive prefix sum of the mask-word popcounts
//
// A scope whose candidates do not fit the candidate list (very many equal magnitudes) skips the
// lists: `final` and `fixup` then walk the scope's weights instead.  Same result, slower.
#include "pac_internal.h"

namespace pac {
namespace {

typedef unsigned long long u64;

__device__ __forceinline__ uint32_t key_of_bits(uint32_t bits) { return bits & 0x7FFFFFFFu; }
__device__ __forceinline__ u64 composite_of(uint32_t key, uint32_t i) {
    return ((u64)key << 32) | (u64)(0xFFFFFFFFu - i);
}
__device__ __forceinline__ uint32_t digit0_of(uint32_t key) { return key >> kDigit0Shift; }
__device__ __forceinline__ uint32_t digit1_of(uint32_t key) { return (key >> kDigit1Shift) & (kDigit1Bins - 1u); }

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }
__device__ __forceinline__ uint32_t lanes_below(u64 m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
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

__device__ __forceinline__ void flush_hist(uint32_t* lds, uint32_t* __restrict__ global_hist) {
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

template <bool VEC>
__global__ __launch_bounds__(kHistBlock) void hist0_kernel(const float* __restrict__ w, uint32_t n,
                                                           const SegDesc* __restrict__ seg, uint32_t nseg,
                                                           uint32_t* __restrict__ hist0, Globals* glob,
                                                           uint32_t tiles_per_block) {
    __shared__ uint32_t lds[kDigit0Bins];
    for (uint32_t b = threadIdx.x; b < kDigit0Bins; b += kHistBlock) lds[b] = 0;
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        glob->cand_total = 0;
        glob->list2_total = 0;
        glob->any_full = 0;
    }
    __syncthreads();

    const uint32_t num_tiles = (uint32_t)(((u64)n + kHistTile - 1) / kHistTile);
    const uint32_t t0 = blockIdx.x * tiles_per_block;
    const uint32_t t1 = min(t0 + tiles_per_block, num_tiles);
    const uint32_t kNone = 0xFFFFFFFFu;
    uint32_t cur = kNone;   // scope whose counts sit in the LDS histogram

    for (uint32_t t = t0; t < t1; ++t) {
        const uint32_t a = t * kHistTile;
        const uint32_t b = (uint32_t)min((u64)a + kHistTile, (u64)n);
        const uint32_t s = find_seg(seg, nseg, a);
        if (seg[s].end >= b) {
            if (s != cur) {
                if (cur != kNone) flush_hist(lds, hist0 + (size_t)cur * kDigit0Bins);
                cur = s;
            }
            if (VEC && b - a == kHistTile) {
                const uint4* p = reinterpret_cast<const uint4*>(w + a) + threadIdx.x;
                uint4 v[kHistLoads];
#pragma unroll
                for (uint32_t u = 0; u < kHistLoads; ++u) v[u] = p[u * kHistBlock];
#pragma unroll
                for (uint32_t u = 0; u < kHistLoads; ++u) {
                    atomicAdd(&lds[digit0_of(key_of_bits(v[u].x))], 1u);
                    atomicAdd(&lds[digit0_of(key_of_bits(v[u].y))], 1u);
                    atomicAdd(&lds[digit0_of(key_of_bits(v[u].z))], 1u);
                    atomicAdd(&lds[digit0_of(key_of_bits(v[u].w))], 1u);
                }
            } else {
                for (u64 i = (u64)a + threadIdx.x; i < b; i += kHistBlock)
                    atomicAdd(&lds[digit0_of(key_of_bits(__float_as_uint(w[i])))], 1u);
            }
        } else {
            // The tile crosses scope boundaries: count element by element into the global histograms.
            for (u64 i = (u64)a + threadIdx.x; i < b; i += kHistBlock) {
                const uint32_t si = find_seg(seg, nseg, (uint32_t)i);
                atomicAdd(&hist0[(size_t)si * kDigit0Bins + digit0_of(key_of_bits(__float_as_uint(w[i])))], 1u);
            }
        }
    }
    if (cur != kNone) flush_hist(lds, hist0 + (size_t)cur * kDigit0Bins);
}

// ---------------------------------------------------------------------------- select0 / select1
// Finds, in a histogram of BINS bins owned 16 per thread, the bin that holds the k-th element when
// bins are walked from the highest digit down.  Zeroes the histogram.  Exactly one thread returns
// true (if 1 <= k <= total count) with bin / rank-inside-bin / bin count.
template <int BINS>
__device__ __forceinline__ bool select_bin(uint32_t* __restrict__ h, uint32_t k, uint32_t* wave_sums,
                                           uint32_t& bin, uint32_t& krem, uint32_t& cnt) {
    constexpr int THREADS = BINS / 16;
    uint32_t loc[16];
    uint4* hv = reinterpret_cast<uint4*>(h) + threadIdx.x * 4;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const uint4 x = hv[j];
        loc[4 * j] = x.x; loc[4 * j + 1] = x.y; loc[4 * j + 2] = x.z; loc[4 * j + 3] = x.w;
        hv[j] = make_uint4(0, 0, 0, 0);
    }
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

__global__ __launch_bounds__(kDigit0Bins / 16) void select0_kernel(const SegDesc* __restrict__ seg,
                                                                   SegState* __restrict__ state,
                                                                   uint32_t* __restrict__ hist0, Globals* glob,
                                                                   uint32_t cand_cap) {
    __shared__ uint32_t wave_sums[kDigit0Bins / 16 / 64];
    const uint32_t s = blockIdx.x;
    const uint32_t k = seg[s].k;
    uint32_t bin = 0, krem = 0, cnt = 0;
    const bool mine = select_bin<(int)kDigit0Bins>(hist0 + (size_t)s * kDigit0Bins, k, wave_sums, bin, krem, cnt);
    SegState* st = state + s;
    if (k == 0) {
        if (threadIdx.x == 0) {
            st->cstar = ~0ull;
            st->bin0 = kNoBin; st->cnt0 = 0; st->krem0 = 0; st->mode = kModeNone;
            st->cand_off = 0; st->cand_fill = 0;
            st->bin1 = 0; st->cnt1 = 0; st->krem1 = 0; st->list2_off = 0; st->list2_fill = 0;
        }
        return;
    }
    if (mine) {
        const uint32_t off = atomicAdd(&glob->cand_total, cnt);
        const bool fits = (u64)off + cnt <= (u64)cand_cap;
        if (!fits) glob->any_full = 1;
        st->cstar = 0;
        st->bin0 = bin; st->cnt0 = cnt; st->krem0 = krem; st->mode = fits ? kModeCand : kModeFull;
        st->cand_off = fits ? off : 0; st->cand_fill = 0;
        st->bin1 = 0; st->cnt1 = 0; st->krem1 = 0; st->list2_off = 0; st->list2_fill = 0;
    }
}

__global__ __launch_bounds__(kDigit1Bins / 16) void select1_kernel(SegState* __restrict__ state,
                                                                   uint32_t* __restrict__ hist1, Globals* glob) {
    __shared__ uint32_t wave_sums[kDigit1Bins / 16 / 64];
    const uint32_t s = blockIdx.x;
    SegState* st = state + s;
    const uint32_t mode = st->mode;
    const uint32_t k = mode == kModeNone ? 0u : st->krem0;
    uint32_t bin = 0, krem = 0, cnt = 0;
    const bool mine = select_bin<(int)kDigit1Bins>(hist1 + (size_t)s * kDigit1Bins, k, wave_sums, bin, krem, cnt);
    if (mine) {
        st->bin1 = bin; st->cnt1 = cnt; st->krem1 = krem;
        st->list2_off = mode == kModeCand ? atomicAdd(&glob->list2_total, cnt) : 0u;
        st->list2_fill = 0;
    }
}

// -------------------------------------------------------------------------------------- emit
// Persistent workgroups of 16 waves; a wave owns 16 consecutive mask words of a tile and loads one
// element per lane per word, so the wave ballot of the keep predicate IS the mask word.
// Undecided elements (digit 0 equal to the scope's bin) are rare for continuous weight
// distributions; they are staged in LDS (composites) and counted by digit 1 in an LDS histogram,
// and reach global memory once per workgroup and scope, so global atomics on the scope's fill
// counter stay few.  The all-zero composite cannot occur (flat indices are below 2^32 - 1), it
// marks an empty staging slot.
constexpr int kEmitBlock = 1024;
constexpr uint32_t kEmitWordsPerWave = 16;
constexpr uint32_t kEmitTile = (kEmitBlock / 64) * kEmitWordsPerWave * 64;   // 16384 elements
constexpr uint32_t kStageCap = 2048;

struct EmitShared {
    u64 stage[kStageCap];
    uint32_t hist1[kDigit1Bins];
    uint32_t wave_sums[kEmitBlock / 64];
    uint32_t stage_count;
    uint32_t flush_base;
};

// Moves the staged composites of scope `s` to its candidate list.  Called by all threads.
__device__ __forceinline__ void flush_stage(EmitShared& sh, SegState* __restrict__ st, u64* __restrict__ cand,
                                            uint32_t cand_off) {
    __syncthreads();
    if (sh.stage_count != 0) {   // uniform: read after the barrier
        constexpr uint32_t kPer = kStageCap / kEmitBlock;
        u64 e[kPer];
        uint32_t have = 0;
#pragma unroll
        for (uint32_t j = 0; j < kPer; ++j) {
            e[j] = sh.stage[threadIdx.x * kPer + j];
            have += e[j] != 0 ? 1u : 0u;
        }
        uint32_t total;
        uint32_t pos = block_exclusive_scan<kEmitBlock>(have, sh.wave_sums, total);
        if (threadIdx.x == 0) sh.flush_base = total ? atomicAdd(&st->cand_fill, total) : 0u;
        __syncthreads();
        pos += sh.flush_base;
#pragma unroll
        for (uint32_t j = 0; j < kPer; ++j) {
            if (e[j] != 0) {
                cand[(size_t)cand_off + pos] = e[j];
                ++pos;
                sh.stage[threadIdx.x * kPer + j] = 0;
            }
        }
        if (threadIdx.x == 0) sh.stage_count = 0;
    }
    __syncthreads();
}

__device__ __forceinline__ void flush_hist1(EmitShared& sh, uint32_t* __restrict__ global_hist1) {
    __syncthreads();
    for (uint32_t b = threadIdx.x; b < kDigit1Bins; b += kEmitBlock) {
        const uint32_t v = sh.hist1[b];
        if (v) {
            atomicAdd(&global_hist1[b], v);
            sh.hist1[b] = 0;
        }
    }
    __syncthreads();
}

__global__ __launch_bounds__(kEmitBlock) void emit_kernel(const float* __restrict__ w, uint32_t n,
                                                          const SegDesc* __restrict__ seg, uint32_t nseg,
                                                          SegState* __restrict__ state,
                                                          uint32_t* __restrict__ hist1, u64* __restrict__ cand,
                                                          u64* __restrict__ mask, uint32_t tiles_per_block) {
    __shared__ EmitShared sh;
    for (uint32_t j = threadIdx.x; j < kStageCap; j += kEmitBlock) sh.stage[j] = 0;
    for (uint32_t j = threadIdx.x; j < kDigit1Bins; j += kEmitBlock) sh.hist1[j] = 0;
    if (threadIdx.x == 0) { sh.stage_count = 0; sh.flush_base = 0; }
    __syncthreads();

    const uint32_t lane = lane_id(), wave = threadIdx.x >> 6;
    const uint32_t num_tiles = (uint32_t)(((u64)n + kEmitTile - 1) / kEmitTile);
    const uint32_t t0 = blockIdx.x * tiles_per_block;
    const uint32_t t1 = min(t0 + tiles_per_block, num_tiles);
    const uint32_t kNone = 0xFFFFFFFFu;
    uint32_t cur = kNone;                       // scope whose undecided elements sit in LDS
    uint32_t s_bin0 = 0, s_mode = 0, s_off = 0; // of scope `cur`

    for (uint32_t t = t0; t < t1; ++t) {
        const uint32_t a = t * kEmitTile;                               // < n
        const uint32_t b = (uint32_t)min((u64)a + kEmitTile, (u64)n);
        const uint32_t s0 = find_seg(seg, nseg, a);
        const bool single = seg[s0].end >= b;                           // whole tile inside one scope
        const u64 wave_first = (u64)a + wave * (kEmitWordsPerWave * 64);

        uint32_t bits[kEmitWordsPerWave];
#pragma unroll
        for (uint32_t j = 0; j < kEmitWordsPerWave; ++j) {
            const u64 i = wave_first + j * 64 + lane;
            bits[j] = i < n ? __float_as_uint(w[i]) : 0u;
        }

        if (single) {
            if (s0 != cur) {
                if (cur != kNone) {
                    if (s_mode == kModeCand) flush_stage(sh, state + cur, cand, s_off);
                    flush_hist1(sh, hist1 + (size_t)cur * kDigit1Bins);
                }
                cur = s0;
                s_bin0 = state[s0].bin0;
                s_mode = state[s0].mode;
                s_off = state[s0].cand_off;
            } else if (s_mode == kModeCand) {
                // Read the fill level between two barriers so that every thread sees the same value.
                __syncthreads();
                const uint32_t staged = sh.stage_count;
                __syncthreads();
                if (staged >= kStageCap / 2) flush_stage(sh, state + cur, cand, s_off);
            }
        }

        u64 my_word = 0;
#pragma unroll
        for (uint32_t j = 0; j < kEmitWordsPerWave; ++j) {
            const u64 i64 = wave_first + j * 64 + lane;
            const bool valid = i64 < n;
            const uint32_t i = (uint32_t)i64;
            const uint32_t key = key_of_bits(bits[j]);
            const uint32_t d0 = digit0_of(key);
            if (single) {
                const bool keep = valid && d0 > s_bin0;
                const bool undecided = valid && d0 == s_bin0;
                const u64 word = __ballot(keep);
                if (lane == j) my_word = word;
                const u64 cm = __ballot(undecided);
                if (cm != 0) {
                    if (undecided) atomicAdd(&sh.hist1[digit1_of(key)], 1u);
                    if (s_mode == kModeCand) {
                        const uint32_t cnt = (uint32_t)__popcll(cm);
                        const uint32_t leader = (uint32_t)__ffsll((long long)cm) - 1u;
                        uint32_t base = 0;
                        if (lane == leader) base = atomicAdd(&sh.stage_count, cnt);
                        base = __shfl(base, (int)leader, 64);
                        if (base + cnt <= kStageCap) {
                            if (undecided) sh.stage[base + lanes_below(cm)] = composite_of(key, i);
                        } else {
                            // staging area full: straight to the candidate list
                            uint32_t g = 0;
                            if (lane == leader) g = atomicAdd(&state[cur].cand_fill, cnt);
                            g = __shfl(g, (int)leader, 64);
                            if (undecided) cand[(size_t)s_off + g + lanes_below(cm)] = composite_of(key, i);
                        }
                    }
                }
            } else {
                // The tile crosses scope boundaries: every lane looks its scope up.
                bool keep = false;
                if (valid) {
                    const uint32_t si = find_seg(seg, nseg, i);
                    const uint32_t bin0 = state[si].bin0;
                    keep = d0 > bin0;
                    if (d0 == bin0) {
                        atomicAdd(&hist1[(size_t)si * kDigit1Bins + digit1_of(key)], 1u);
                        if (state[si].mode == kModeCand) {
                            const uint32_t pos = atomicAdd(&state[si].cand_fill, 1u);
                            cand[(size_t)state[si].cand_off + pos] = composite_of(key, i);
                        }
                    }
                }
                const u64 word = __ballot(keep);
                if (lane == j) my_word = word;
            }
        }
        if (lane < kEmitWordsPerWave) {
            const u64 word_idx = (wave_first >> 6) + lane;
            if (word_idx * 64 < n) mask[word_idx] = my_word;
        }
    }
    if (cur != kNone) {
        if (s_mode == kModeCand) flush_stage(sh, state + cur, cand, s_off);
        flush_hist1(sh, hist1 + (size_t)cur * kDigit1Bins);
    }
}

// ----------------------------------------------------------------------------------- compact2
constexpr int kListBlock = 256;

__global__ __launch_bounds__(kListBlock) void compact2_kernel(SegState* __restrict__ state,
                                                              const u64* __restrict__ cand,
                                                              u64* __restrict__ list2) {
    const uint32_t s = blockIdx.y;
    SegState* st = state + s;
    if (st->mode != kModeCand) return;
    const uint32_t cnt0 = st->cnt0, off = st->cand_off, bin1 = st->bin1, off2 = st->list2_off;
    const uint32_t lane = lane_id();
    for (u64 base = (u64)blockIdx.x * kListBlock; base < cnt0; base += (u64)gridDim.x * kListBlock) {
        const u64 j = base + threadIdx.x;
        const bool valid = j < cnt0;
        const u64 c = valid ? cand[(size_t)off + j] : 0ull;
        const bool match = valid && digit1_of((uint32_t)(c >> 32)) == bin1;
        const u64 mm = __ballot(match);
        if (mm != 0) {
            const uint32_t leader = (uint32_t)__ffsll((long long)mm) - 1u;
            uint32_t pos = 0;
            if (lane == leader) pos = atomicAdd(&st->list2_fill, (uint32_t)__popcll(mm));
            pos = __shfl(pos, (int)leader, 64);
            if (match) list2[(size_t)off2 + pos + lanes_below(mm)] = c;
        }
    }
}

// -------------------------------------------------------------------------------------- final
// Resolves the low kTailBits bits of C* for one scope.  The source is either the scope's
// second-level list (every entry already agrees with C* on digits 0 and 1) or, for a scope without
// lists, the scope's weights filtered on the fly.
constexpr int kFinalBlock = 256;

template <bool FROM_LIST>
__device__ __forceinline__ void final_levels(const u64* __restrict__ list, uint32_t list_cnt,
                                             const float* __restrict__ w, uint32_t begin, uint32_t end,
                                             u64& prefix, uint32_t& krem, uint32_t* hist, uint32_t* wave_sums,
                                             uint32_t* found) {
    // digit widths over the 37 tail bits, most significant first
    const uint32_t shifts[5] = {29, 21, 13, 5, 0};
    const uint32_t widths[5] = {8, 8, 8, 8, 5};
    uint32_t resolved_above = kTailBits;   // bits >= this position are already fixed in `prefix`
    for (int level = 0; level < 5; ++level) {
        const uint32_t shift = shifts[level], width = widths[level];
        hist[threadIdx.x] = 0;
        __syncthreads();
        const uint32_t count = FROM_LIST ? list_cnt : end - begin;
        for (u64 j = threadIdx.x; j < count; j += kFinalBlock) {
            u64 c;
            if (FROM_LIST) {
                c = list[j];
            } else {
                const uint32_t i = begin + (uint32_t)j;
                c = composite_of(key_of_bits(__float_as_uint(w[i])), i);
            }
            if (((c ^ prefix) >> resolved_above) == 0)
                atomicAdd(&hist[(uint32_t)(c >> shift) & ((1u << width) - 1u)], 1u);
        }
        __syncthreads();
        // thread t owns bin t; walk from the highest bin down
        const uint32_t v = hist[threadIdx.x];
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

__global__ __launch_bounds__(kFinalBlock) void final_kernel(const float* __restrict__ w,
                                                            const SegDesc* __restrict__ seg,
                                                            SegState* __restrict__ state,
                                                            const u64* __restrict__ list2) {
    __shared__ uint32_t hist[kFinalBlock];
    __shared__ uint32_t wave_sums[kFinalBlock / 64];
    __shared__ uint32_t found[2];
    const uint32_t s = blockIdx.x;
    SegState* st = state + s;
    const uint32_t mode = st->mode;
    if (mode == kModeNone) return;
    u64 prefix = ((u64)st->bin0 << (32 + kDigit0Shift)) | ((u64)st->bin1 << (32 + kDigit1Shift));
    uint32_t krem = st->krem1;
    if (threadIdx.x == 0) { found[0] = 0; found[1] = 0; }
    __syncthreads();
    if (mode == kModeCand)
        final_levels<true>(list2 + st->list2_off, st->cnt1, nullptr, 0, 0, prefix, krem, hist, wave_sums, found);
    else
        final_levels<false>(nullptr, 0, w, seg[s].begin, seg[s].end, prefix, krem, hist, wave_sums, found);
    if (threadIdx.x == 0) st->cstar = prefix;
}

// -------------------------------------------------------------------------------------- fixup
__global__ __launch_bounds__(kListBlock) void fixup_kernel(const float* __restrict__ w,
                                                           const SegDesc* __restrict__ seg,
                                                           const SegState* __restrict__ state,
                                                           const u64* __restrict__ cand, u64* __restrict__ mask) {
    const uint32_t s = blockIdx.y;
    const SegState* st = state + s;
    const uint32_t mode = st->mode;
    if (mode == kModeNone) return;
    const u64 cstar = st->cstar;
    if (mode == kModeCand) {
        const uint32_t cnt0 = st->cnt0, off = st->cand_off;
        for (u64 j = (u64)blockIdx.x * kListBlock + threadIdx.x; j < cnt0; j += (u64)gridDim.x * kListBlock) {
            const u64 c = cand[(size_t)off + j];
            if (c >= cstar) {
                const uint32_t i = 0xFFFFFFFFu - (uint32_t)c;
                atomicOr(&mask[i >> 6], 1ull << (i & 63u));
            }
        }
    } else {
        const uint32_t begin = seg[s].begin, end = seg[s].end, bin0 = st->bin0;
        for (u64 i = (u64)begin + (u64)blockIdx.x * kListBlock + threadIdx.x; i < end; i += (u64)gridDim.x * kListBlock) {
            const uint32_t key = key_of_bits(__float_as_uint(w[i]));
            if (digit0_of(key) == bin0 && composite_of(key, (uint32_t)i) >= cstar)
                atomicOr(&mask[i >> 6], 1ull << (i & 63u));
        }
    }
}

// --------------------------------------------------------------------------------------- scan
// prefix[j] = number of set bits in mask words 0..j-1.  Three small kernels over the mask words:
// per-tile popcount sums, one workgroup scanning the tile sums, per-tile rescan with the offset.
constexpr int kScanBlock = 256;
constexpr uint32_t kScanWordsPerThread = 8;
constexpr uint32_t kScanTile = kScanBlock * kScanWordsPerThread;   // 2048 words

__device__ __forceinline__ void load_words(const u64* __restrict__ mask, uint32_t words, uint32_t first,
                                           uint32_t pc[kScanWordsPerThread]) {
#pragma unroll
    for (uint32_t j = 0; j < kScanWordsPerThread; ++j) {
        const u64 idx = (u64)first + j;
        pc[j] = idx < words ? (uint32_t)__popcll(mask[idx]) : 0u;
    }
}

__global__ __launch_bounds__(kScanBlock) void scan_tile_sums_kernel(const u64* __restrict__ mask, uint32_t words,
                                                                    uint32_t* __restrict__ tile_sums) {
    __shared__ uint32_t wave_sums[kScanBlock / 64];
    uint32_t pc[kScanWordsPerThread];
    load_words(mask, words, blockIdx.x * kScanTile + threadIdx.x * kScanWordsPerThread, pc);
    uint32_t sum = 0;
#pragma unroll
    for (uint32_t j = 0; j < kScanWordsPerThread; ++j) sum += pc[j];
    uint32_t total;
    block_exclusive_scan<kScanBlock>(sum, wave_sums, total);
    if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

constexpr int kScanTopBlock = 1024;
__global__ __launch_bounds__(kScanTopBlock) void scan_tile_offsets_kernel(uint32_t* __restrict__ tile_sums,
                                                                          uint32_t num_tiles) {
    __shared__ uint32_t wave_sums[kScanTopBlock / 64];
    const uint32_t per = (num_tiles + kScanTopBlock - 1) / kScanTopBlock;
    const uint32_t first = threadIdx.x * per;
    uint32_t sum = 0;
    for (uint32_t j = 0; j < per; ++j)
        if (first + j < num_tiles) sum += tile_sums[first + j];
    uint32_t total;
    uint32_t run = block_exclusive_scan<kScanTopBlock>(sum, wave_sums, total);
    for (uint32_t j = 0; j < per; ++j) {
        if (first + j < num_tiles) {
            const uint32_t v = tile_sums[first + j];
            tile_sums[first + j] = run;
            run += v;
        }
    }
}

__global__ __launch_bounds__(kScanBlock) void scan_write_prefix_kernel(const u64* __restrict__ mask, uint32_t words,
                                                                       const uint32_t* __restrict__ tile_offsets,
                                                                       uint32_t* __restrict__ prefix) {
    __shared__ uint32_t wave_sums[kScanBlock / 64];
    uint32_t pc[kScanWordsPerThread];
    const uint32_t first = blockIdx.x * kScanTile + threadIdx.x * kScanWordsPerThread;
    load_words(mask, words, first, pc);
    uint32_t sum = 0;
#pragma unroll
    for (uint32_t j = 0; j < kScanWordsPerThread; ++j) sum += pc[j];
    uint32_t total;
    uint32_t run = tile_offsets[blockIdx.x] + block_exclusive_scan<kScanBlock>(sum, wave_sums, total);
#pragma unroll
    for (uint32_t j = 0; j < kScanWordsPerThread; ++j) {
        const u64 idx = (u64)first + j;
        if (idx < words) prefix[idx] = run;
        run += pc[j];
    }
}

inline uint32_t div_up_u64(u64 a, u64 b) { return (uint32_t)((a + b - 1) / b); }

}  // namespace

hipError_t launch_build_mask(const MaskScratch& s, const float* d_weights, uint32_t n, uint32_t nseg,
                             unsigned long long* d_mask, uint32_t* d_prefix, int num_cu, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    const uint32_t words = div_up_u64(n, 64);

    // hist0: persistent workgroups, each walks a contiguous run of tiles
    {
        const uint32_t num_tiles = div_up_u64(n, kHistTile);
        const uint32_t want = (uint32_t)num_cu * 2u;
        const uint32_t blocks = num_tiles < want ? num_tiles : want;
        const uint32_t per = div_up_u64(num_tiles, blocks);
        const uint32_t grid = div_up_u64(num_tiles, per);
        if ((reinterpret_cast<uintptr_t>(d_weights) & 15u) == 0)
            hipLaunchKernelGGL((hist0_kernel<true>), dim3(grid), dim3(kHistBlock), 0, stream, d_weights, n, s.seg,
                               nseg, s.hist0, s.glob, per);
        else
            hipLaunchKernelGGL((hist0_kernel<false>), dim3(grid), dim3(kHistBlock), 0, stream, d_weights, n, s.seg,
                               nseg, s.hist0, s.glob, per);
    }
    hipLaunchKernelGGL(select0_kernel, dim3(nseg), dim3(kDigit0Bins / 16), 0, stream, s.seg, s.state, s.hist0,
                       s.glob, s.cand_cap);
    {
        const uint32_t num_tiles = div_up_u64(n, kEmitTile);
        const uint32_t want = (uint32_t)num_cu * 2u;
        const uint32_t blocks = num_tiles < want ? num_tiles : want;
        const uint32_t per = div_up_u64(num_tiles, blocks);
        const uint32_t grid = div_up_u64(num_tiles, per);
        hipLaunchKernelGGL(emit_kernel, dim3(grid), dim3(kEmitBlock), 0, stream, d_weights, n, s.seg, nseg, s.state,
                           s.hist1, s.cand, d_mask, per);
    }
    hipLaunchKernelGGL(select1_kernel, dim3(nseg), dim3(kDigit1Bins / 16), 0, stream, s.state, s.hist1, s.glob);

    uint32_t per_seg_blocks = 16384u / nseg;
    if (per_seg_blocks < 1) per_seg_blocks = 1;
    if (per_seg_blocks > 256) per_seg_blocks = 256;
    hipLaunchKernelGGL(compact2_kernel, dim3(per_seg_blocks, nseg), dim3(kListBlock), 0, stream, s.state, s.cand,
                       s.list2);
    hipLaunchKernelGGL(final_kernel, dim3(nseg), dim3(kFinalBlock), 0, stream, d_weights, s.seg, s.state, s.list2);
    hipLaunchKernelGGL(fixup_kernel, dim3(per_seg_blocks, nseg), dim3(kListBlock), 0, stream, d_weights, s.seg,
                       s.state, s.cand, d_mask);

    const uint32_t scan_tiles = div_up_u64(words, kScanTile);
    hipLaunchKernelGGL(scan_tile_sums_kernel, dim3(scan_tiles), dim3(kScanBlock), 0, stream, d_mask, words,
                       s.tile_sums);
    hipLaunchKernelGGL(scan_tile_offsets_kernel, dim3(1), dim3(kScanTopBlock), 0, stream, s.tile_sums, scan_tiles);
    hipLaunchKernelGGL(scan_write_prefix_kernel, dim3(scan_tiles), dim3(kScanBlock), 0, stream, d_mask, words,
                       s.tile_sums, d_prefix);
    return hipGetLastError();
}

}  // namespace pac
