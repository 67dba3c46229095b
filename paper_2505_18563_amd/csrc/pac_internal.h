// Internal declarations shared by the translation units of libpactrain (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pac {

// ---- magnitude order ------------------------------------------------------------------------
// key(w) = bit pattern with the sign cleared (31 bits).  Elements of a prune scope are ordered by
// the 63-bit composite (key << 32) | (0xFFFFFFFF - flat_index): larger composite = kept first,
// i.e. |w| descending, flat index ascending.  The selection finds the composite C* of the k-th
// element in three steps:
//   bracket: a key range [lo, hi) that holds the k-th key, from a histogram of digit 0 (key bits 30..17)
//            over all of the scope's elements (one whole bin) or over a sample of them (a rank band)
//   tie key: if one key holds a visible share of the bracket's elements (the zeros of an already pruned
//            model, a constant tensor), its elements are not listed one by one: every tile only counts
//            them, and their flat order decides among them at the end
//   digit 1: the other undecided elements (lo <= key < hi) are counted by a second digit (see
//            SegState) while they are collected; the bin of the k-th among them narrows the range
//   tail   : the remaining key bits and the 32 index bits, resolved inside one workgroup
constexpr uint32_t kDigit0Bits = 14;
constexpr uint32_t kDigit0Bins = 1u << kDigit0Bits;   // 16384
constexpr uint32_t kDigit0Shift = 17;                 // within the 31-bit key
constexpr uint32_t kDigit1Bits = 11;
constexpr uint32_t kDigit1Bins = 1u << kDigit1Bits;   // 2048
constexpr uint32_t kKeyEnd = 0x80000000u;             // one past the largest key

// One prune scope, written by the host.
struct SegDesc {
    uint32_t begin;    // first flat element
    uint32_t end;      // one past the last flat element
    uint32_t k;        // keep count
    uint32_t stride;   // the first histogram pass visits one tile in `stride` (power of two; 1 = every tile);
                       // 0 marks a small scope (at most kSmallScope elements), which takes no part in the
                       // histogram passes: one workgroup selects and writes its mask bits from LDS
    uint32_t slot0;    // work items ("slots") of the histogram passes before this scope: in the first pass one slot
    uint32_t slot1;    // per aligned group of `stride` tiles that the scope touches (slot0), in the full pass one
                       // per tile that it touches (slot1).  See hist_slots().
};

// Tiles of the histogram passes: kHistTileElems consecutive flat elements, counted from element 0 of the flat
// tensor (not from the scope's begin).  A scope at stride m takes part in the first pass with one tile of every
// aligned group of m tiles; the number of such groups (m = 1: of tiles) that [begin, end) touches:
constexpr uint32_t kHistTileElems = 16384;
inline uint32_t hist_slots(uint32_t begin, uint32_t end, uint32_t m) {
    if (m == 0 || begin >= end) return 0;
    uint32_t sh = 0;
    while ((1u << sh) < m) ++sh;
    return (((end - 1) / kHistTileElems) >> sh) - ((begin / kHistTileElems) >> sh) + 1;
}

// Selection state of one prune scope, device only.
constexpr uint32_t kNoTieKey = 0xFFFFFFFFu;   // no key is 0xFFFFFFFF (keys have 31 bits)
struct SegState {
    unsigned long long cstar;  // composite of the k-th element: kept iff composite >= cstar
    uint32_t active;           // 0 if nothing is undecided (k == 0 or k == n): cstar is already final
    uint32_t lo;               // bracket: key >= hi is kept, lo <= key < hi is undecided
    uint32_t hi;
    uint32_t lo1;              // digit 1 of an undecided key: 0 below lo1, ((key - lo1) >> sh1) + off1 from lo1 on,
    uint32_t sh1;              // always below kDigit1Bins; lo1 is a multiple of 2^sh1, so the keys of one digit
    uint32_t off1;             // (other than a digit 0 below lo1) share all bits from sh1 up.  off1 = 1 iff lo1 > lo
    uint32_t tie_key;          // kNoTieKey, or the key inside the bracket whose elements are counted per tile, not listed
    uint32_t tie_in;           // the tie key's elements fall into digit-1 bin bin1 (cnt1 includes them)
    uint32_t exact;            // the histogram counted every element, so krem0 was known before emit
    uint32_t krem0;            // rank of the k-th element among the undecided ones (1-based, descending)
    uint32_t bin1;             // digit 1 of the k-th element
    uint32_t cnt1;             // undecided elements with that digit
    uint32_t krem1;            // rank of the k-th element among those
    uint32_t heavy;            // too many listed elements share digit 1 for `final`'s LDS list:
                               // `final` walks this scope's weights
};
static_assert(sizeof(SegState) == 64, "one cache line half per scope");

constexpr uint32_t kMaxSampleStride = 64;  // largest SegDesc::stride (power of two)

// Scopes of up to this many elements (norm and bias vectors, small kernels) are resolved by one
// workgroup each with the keys held in LDS: exact whatever the ties, and no per-scope traffic in
// the streaming passes.
constexpr uint32_t kSmallScope = 32768;

// emit leaves one record per tile of kEmitTileElems elements: a 64-bit header (in an array of its own, so
// that the passes that only need headers read them densely) and up to kRecSlots composites of listed
// undecided elements (room for 3 % of the tile; a sampled bracket holds a few tenths of a percent).
// Header fields, 16 bits each from the low end:
//   listed   undecided elements listed in the record; kRecWalk = not listed, consumers walk the tile's weights
//   kept     elements above their bracket (used for tiles that lie inside one scope)
//   tie_head elements equal to the tie key of the scope that holds the tile's first element
//   tie_tail the same for the other large scope that begins inside the tile, if there is one
// Tie-key elements are never listed and never visited by a walk: they exist as these counts only.
constexpr uint32_t kEmitTileElems = 4096;
constexpr uint32_t kRecSlots = 128;
constexpr uint32_t kRecWalk = 0xFFFFu;

// compact2 runs with a fixed number of workgroups, each owning a short list of matches.
constexpr uint32_t kMatchBlocks = 1024;
constexpr uint32_t kMatchSlotsPerBlock = 64;
constexpr uint32_t kMatchSlots = kMatchBlocks * kMatchSlotsPerBlock;         // 65536

// Counters shared by all scopes of one pac_build_mask call.
struct Globals {
    uint32_t retry;                      // a sampled bracket missed the k-th element: redo with full counts
    uint32_t match_overflow;             // a workgroup of compact2 ran out of match slots
    uint32_t scan_ticket;                // next tile of the prefix scan
    uint32_t pad[5];
};

// Bits of the context's device status word; the values are those of the PAC_DEV_* enumerators of the
// public header (checked where both are visible).
constexpr uint32_t kDevScanStalled = 0x01u;
constexpr uint32_t kDevCountMismatch = 0x02u;
constexpr uint32_t kDevMetaMismatch = 0x04u;
constexpr uint32_t kDevRetryTaken = 0x100u;
constexpr uint32_t kDevSlowPath = 0x200u;
constexpr unsigned long long kNoExpectedTotal = ~0ull;   // "do not check the scan's total"

struct MaskScratch {
    uint32_t* status;              // the context's device status word (sticky PAC_DEV_* bits)
    uint32_t scan_spin_limit;      // polls after which a scan workgroup gives up waiting (a test hook lowers it)
    uint32_t hist_blocks;          // workgroups of the first histogram pass that fit on the device at once
    SegDesc* seg;                  // [max_segments] scope table of the current call (one of the context's resident tables)
    SegState* state;               // [max_segments]
    uint32_t* hist0;               // [max_segments * kDigit0Bins], all zero between calls
    uint32_t* hist1;               // [max_segments * kDigit1Bins], all zero between calls
    uint32_t* kept_above;          // [max_segments] elements with key >= hi (counted for sampled scopes)
    uint32_t* tie_count;           // [max_segments] elements equal to the scope's tie key
    Globals* glob;
    unsigned long long* hdrs;      // [tiles] tile record headers
    unsigned long long* rec;       // [tiles * kRecSlots] tile records: the listed composites
    uint32_t* tile_scope;          // [tiles] scope of each tile's first element (belongs to the table in `seg`)
    unsigned long long* match;     // [kMatchSlots] undecided elements whose digit 1 is their scope's bin1 as
                                   // well, kMatchSlotsPerBlock slots per workgroup of compact2
    uint32_t* match_count;         // [kMatchBlocks] slots used by each workgroup
    unsigned long long cand_cap;   // undecided elements the records may list in total (a test hook lowers it)
    unsigned long long* tile_state; // per scan tile: status and running count of the look-back scan
    // The small scopes' workgroups only need the weights and emit's zeroed words: they run on a side
    // stream, next to the kernels that resolve the large scopes, and join before the scan.
    hipStream_t side_stream;
    hipEvent_t fork_event;
    hipEvent_t join_event;
};

// Launchers (defined in pac_mask.hip / pac_pack.hip).  All enqueue on `stream` and return the
// first launch error.
// `slots0` / `slots1`: work items of the sampled and of the full histogram pass (sums of hist_slots() over
// the table).  `any_sampled`: some scope has a stride above 1.  `max_tiny` / `max_small`: length of the
// longest small scope of at most kTinyScope elements / of any length in the table (0 = none).
// `fresh_table`: s.tile_scope has not been filled for the table in s.seg yet.  `expect_total`: the sum of
// the scopes' keep counts (the scan raises kDevCountMismatch if the mask holds another number of bits).
constexpr uint32_t kTinyScope = 4096;
hipError_t launch_build_mask(const MaskScratch& s, const float* d_weights, uint32_t n, uint32_t nseg,
                             uint32_t slots0, uint32_t slots1, bool any_sampled, uint32_t max_tiny, uint32_t max_small,
                             bool fresh_table, unsigned long long* d_mask, uint32_t* d_prefix,
                             unsigned long long expect_total, hipStream_t stream);
// Raises the small-scope kernel's LDS limit; once per device, before the first launch.
hipError_t prepare_mask_kernels();
// Workgroups of the first histogram pass that fit on a device with `num_cu` compute units at once.
uint32_t mask_hist_blocks(int num_cu);

// prefix[j] = set bits in words < j of any mask of at most 2^32 - 1 bits; *d_total_out (device, may be
// null) receives the number of set bits.  Uses s.tile_state (at least kScanMaxTiles + 1 words),
// s.glob, s.status and s.scan_spin_limit only.
constexpr uint32_t kScanMaxTiles = 2048;
// `reset_status`: the kernel that clears the scan state also zeroes *s.status (for scratch that is
// shared by unrelated calls; a context's status word is sticky and is left alone).
hipError_t launch_prefix_scan(const MaskScratch& s, const unsigned long long* d_mask, uint32_t words,
                              uint32_t* d_prefix, unsigned long long* d_total_out, bool reset_status,
                              hipStream_t stream);

// Records a formatted error text where pac_last_error(NULL) finds it (calls without a context) and
// returns `code`.
int32_t thread_fail(int32_t code, const char* fmt, ...);

// d_status: the device status word that receives kDevMetaMismatch / kDevCountMismatch.
hipError_t launch_compress(const void* d_grad, int dtype, uint32_t n, const unsigned long long* d_mask,
                           const uint32_t* d_prefix, void* d_compact, uint32_t nnz, uint32_t* d_status,
                           hipStream_t stream);

hipError_t launch_decompress(const void* d_compact, int dtype, uint32_t nnz, const unsigned long long* d_mask,
                             const uint32_t* d_prefix, void* d_dense, uint32_t n, uint32_t* d_status,
                             hipStream_t stream);

// x <- x - alpha * g on kept weights (g = the next value of the summed compact buffer), +0 on pruned ones.
hipError_t launch_decompress_update(const void* d_compact, int dtype, uint32_t nnz, const unsigned long long* d_mask,
                                    const uint32_t* d_prefix, float alpha, float* d_weights, uint32_t n,
                                    uint32_t* d_status, hipStream_t stream);

// Copies the status word to d_out (may be null) and, with clear, resets it; one thread.
hipError_t launch_status_read(uint32_t* d_status, uint32_t* d_out, bool clear, hipStream_t stream);

// Mask Tracker kernels (pac_track.hip).
hipError_t launch_nonzero_mask(const void* d_values, int dtype, uint32_t n, unsigned long long* d_mask,
                               hipStream_t stream);
// *d_diff_out = number of positions below n where the masks differ; if d_copy_to is not null, mask b is
// copied there in the same pass (d_copy_to may be mask a).
hipError_t launch_mask_diff(const unsigned long long* d_a, const unsigned long long* d_b, uint32_t n,
                            unsigned long long* d_diff_out, unsigned long long* d_copy_to, hipStream_t stream);
hipError_t launch_mask_copy(const unsigned long long* d_src, unsigned long long* d_dst, uint32_t words,
                            hipStream_t stream);
struct TrackerState {
    unsigned long long diff;   // scratch of the comparison
    uint32_t unchanged;        // consecutive comparisons that found no difference
    uint32_t stable;           // unchanged >= patience
};
// After a comparison (fresh = 0) or a first / resized observation (fresh = 1): updates the counters and
// writes {unchanged, stable} to d_state_out (device uint32[2], may be null).
hipError_t launch_tracker_finalize(TrackerState* d_state, uint32_t patience, uint32_t fresh, uint32_t* d_state_out,
                                   hipStream_t stream);

struct WorkerPtrs {
    const void* p[64];
};

// Ternary payload (pac_ternary.hip).  *d_scale is a device float.
hipError_t launch_absmax(const void* d_values, int dtype, uint32_t count, bool accumulate, float* d_scale,
                         hipStream_t stream);
hipError_t launch_ternarize(const void* d_values, int dtype, uint32_t count, const float* d_scale,
                            unsigned long long seed, unsigned long long stream_id, uint8_t* d_packed,
                            hipStream_t stream);
hipError_t launch_ternary_reduce(const WorkerPtrs& bufs, uint32_t W, uint32_t count, const float* d_scale,
                                 int out_dtype, void* d_out, hipStream_t stream);

hipError_t launch_reduce(const WorkerPtrs& bufs, uint32_t W, int dtype, uint32_t nnz, void* d_out,
                         hipStream_t stream);

// reduced[slot(i)] = ((g_0[i] + g_1[i]) + ...) + g_{W-1}[i] for kept i: gather and sum in one pass over the W
// dense gradients.
hipError_t launch_step_fused(const WorkerPtrs& grads, uint32_t W, int dtype, uint32_t n,
                             const unsigned long long* d_mask, const uint32_t* d_prefix, void* d_reduced, uint32_t nnz,
                             uint32_t* d_status, hipStream_t stream);

}  // namespace pac
