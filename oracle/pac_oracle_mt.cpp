// PacTrain compression path: the CPU oracle's all-core leg.
//
// TEST INFRASTRUCTURE ONLY, like pac_oracle.cpp.  The definition-level oracle there is single threaded
// on purpose.  The benchmark also reports what the host's cores do together, so this file holds the same
// four operations spread over OpenMP threads, with the work split by 64-element mask words:
//   mask      per prune scope, the threshold key by two counting passes over the scope (top 16 key
//             bits, then the low 15), the tie rule by position (equal-magnitude counts per thread
//             range, prefix over the ranges), bits written by the thread that owns the word
//   gather    each thread walks its own words; a word's first slot is its prefix entry
//   sum       each thread folds its own range of slots, workers in order
//   scatter   each thread writes the 64 outputs of its own words
// Results are defined by pac_oracle.cpp: tests/test_oracle_pins.py checks every function here against
// the function there, element for element.  Nothing here is shared with the GPU library.
// (Magnitude criterion Sec. II-B / III-B; Prune step Sec. III-C and Alg. 1; shared mask and dense
// reformatting Sec. I, III-B; Eq. 2; the sum of Eq. 1.)
#include <omp.h>
#include <sched.h>

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>

extern "C" uint64_t orc_keep_count(uint64_t n, double sparsity);

namespace {

inline uint32_t key_of(float x) {
    uint32_t u;
    std::memcpy(&u, &x, sizeof u);
    return u & 0x7FFFFFFFu;
}

inline float widen_bf16(uint16_t h) {
    const uint32_t u = uint32_t(h) << 16;
    float x;
    std::memcpy(&x, &u, sizeof x);
    return x;
}

inline uint16_t narrow_bf16(float x) {
    uint32_t u;
    std::memcpy(&u, &x, sizeof u);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return uint16_t((u >> 16) | 0x0040u);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return uint16_t(u >> 16);
}

// Walks a histogram from its highest bin down to the bin that holds the `rank`-th element
// (1-based); returns the bin and leaves the rank inside it in `rank`.
uint32_t descend(const std::vector<uint64_t>& hist, uint64_t& rank) {
    for (size_t b = hist.size(); b-- > 0;) {
        if (hist[b] >= rank) return uint32_t(b);
        rank -= hist[b];
    }
    return 0;
}

}  // namespace

extern "C" {

// Threads the functions below use: the cores this process may run on (sched_getaffinity), capped by
// OMP_NUM_THREADS when the environment sets it.
int orc_mt_threads() {
    cpu_set_t set;
    CPU_ZERO(&set);
    int cores = 1;
    if (sched_getaffinity(0, sizeof set, &set) == 0) cores = CPU_COUNT(&set);
    const int cap = omp_get_max_threads();
    return cores < cap ? cores : cap;
}

int orc_build_mask_mt(const float* w, uint64_t n, const uint64_t* seg_off, uint32_t nseg, const double* sparsity,
                      uint64_t* mask, uint32_t* prefix, uint64_t* nnz_out) {
    if (n >= (uint64_t(1) << 32) || nseg == 0 || seg_off[0] != 0 || seg_off[nseg] != n) return -1;
    for (uint32_t s = 0; s < nseg; ++s) {
        if (seg_off[s] > seg_off[s + 1]) return -1;
        if (!(sparsity[s] >= 0.0 && sparsity[s] <= 1.0)) return -1;
    }
    const int T = orc_mt_threads();
    const uint64_t words = (n + 63) / 64;
#pragma omp parallel for num_threads(T) schedule(static)
    for (uint64_t j = 0; j < words; ++j) mask[j] = 0;

    uint64_t total = 0;
    std::vector<uint64_t> hist_hi(1u << 16), hist_lo(1u << 15);
    std::vector<std::vector<uint64_t>> local(T);
    std::vector<uint64_t> eq_in_range(T + 1);
    for (uint32_t s = 0; s < nseg; ++s) {
        const uint64_t b = seg_off[s], e = seg_off[s + 1], len = e - b;
        const uint64_t k = orc_keep_count(len, sparsity[s]);
        total += k;
        if (k == 0) continue;
        // Thread t owns the elements of the scope inside words [wb + t*per, wb + (t+1)*per): whole
        // words, so no two threads write one mask word.
        const uint64_t wb = b / 64, we = (e + 63) / 64;
        const uint64_t per = (we - wb + T - 1) / T;
        auto range = [&](int t, uint64_t& lo, uint64_t& hi) {
            lo = (wb + uint64_t(t) * per) * 64;
            hi = lo + per * 64;
            if (lo < b) lo = b;
            if (hi > e) hi = e;
            if (lo > hi) lo = hi;
        };
        uint32_t thr = 0;     // key of the k-th element
        uint64_t ties = 0;    // elements with that key that are kept (the first `ties` in flat order)
        if (k < len) {
            // top 16 bits of the 31-bit key
#pragma omp parallel num_threads(T)
            {
                const int t = omp_get_thread_num();
                std::vector<uint64_t>& h = local[t];
                h.assign(1u << 16, 0);
                uint64_t lo, hi;
                range(t, lo, hi);
                for (uint64_t i = lo; i < hi; ++i) ++h[key_of(w[i]) >> 15];
            }
            for (size_t bin = 0; bin < hist_hi.size(); ++bin) {
                uint64_t c = 0;
                for (int t = 0; t < T; ++t) c += local[t][bin];
                hist_hi[bin] = c;
            }
            uint64_t rank = k;
            const uint32_t top = descend(hist_hi, rank);
            // low 15 bits among the elements that share those top bits
#pragma omp parallel num_threads(T)
            {
                const int t = omp_get_thread_num();
                std::vector<uint64_t>& h = local[t];
                h.assign(1u << 15, 0);
                uint64_t lo, hi;
                range(t, lo, hi);
                for (uint64_t i = lo; i < hi; ++i) {
                    const uint32_t key = key_of(w[i]);
                    if ((key >> 15) == top) ++h[key & 0x7FFFu];
                }
            }
            for (size_t bin = 0; bin < hist_lo.size(); ++bin) {
                uint64_t c = 0;
                for (int t = 0; t < T; ++t) c += local[t][bin];
                hist_lo[bin] = c;
            }
            const uint32_t low = descend(hist_lo, rank);
            thr = (top << 15) | low;
            ties = rank;
        } else {
            thr = 0;          // everything is kept: every key is >= 0 ...
            ties = len;       // ... and all ties at key 0 are kept too
        }
        // tie rule by position: equal-magnitude elements per thread range, then the ranges in order
#pragma omp parallel num_threads(T)
        {
            const int t = omp_get_thread_num();
            uint64_t lo, hi, c = 0;
            range(t, lo, hi);
            for (uint64_t i = lo; i < hi; ++i) c += key_of(w[i]) == thr;
            eq_in_range[t + 1] = c;
        }
        eq_in_range[0] = 0;
        for (int t = 0; t < T; ++t) eq_in_range[t + 1] += eq_in_range[t];
#pragma omp parallel num_threads(T)
        {
            const int t = omp_get_thread_num();
            uint64_t lo, hi;
            range(t, lo, hi);
            uint64_t seen = eq_in_range[t];
            for (uint64_t i = lo; i < hi; ++i) {
                const uint32_t key = key_of(w[i]);
                bool keep = key > thr;
                if (key == thr) keep = seen++ < ties;
                if (keep) mask[i >> 6] |= uint64_t(1) << (i & 63);
            }
        }
    }
    // prefix: bits per thread range of words, the ranges in order, then each range again
    std::vector<uint64_t> bits(T + 1, 0);
    const uint64_t wper = (words + T - 1) / T;
#pragma omp parallel num_threads(T)
    {
        const int t = omp_get_thread_num();
        const uint64_t lo = uint64_t(t) * wper < words ? uint64_t(t) * wper : words;
        const uint64_t hi = lo + wper < words ? lo + wper : words;
        uint64_t c = 0;
        for (uint64_t j = lo; j < hi; ++j) c += uint64_t(__builtin_popcountll(mask[j]));
        bits[t + 1] = c;
    }
    for (int t = 0; t < T; ++t) bits[t + 1] += bits[t];
#pragma omp parallel num_threads(T)
    {
        const int t = omp_get_thread_num();
        const uint64_t lo = uint64_t(t) * wper < words ? uint64_t(t) * wper : words;
        const uint64_t hi = lo + wper < words ? lo + wper : words;
        uint64_t run = bits[t];
        for (uint64_t j = lo; j < hi; ++j) {
            prefix[j] = uint32_t(run);
            run += uint64_t(__builtin_popcountll(mask[j]));
        }
    }
    if (nnz_out) *nnz_out = total;
    return 0;
}

// compact[prefix[j] + rank of bit b in word j] = grad[64 j + b] for every set bit, words in parallel.
void orc_compress_mt(const void* grad, int dtype, uint64_t n, const uint64_t* mask, const uint32_t* prefix, void* compact) {
    const int T = orc_mt_threads();
    const int64_t words = int64_t((n + 63) / 64);
#pragma omp parallel for num_threads(T) schedule(static)
    for (int64_t j = 0; j < words; ++j) {
        uint64_t m = mask[j];
        uint64_t slot = prefix[j];
        while (m) {
            const uint64_t i = uint64_t(j) * 64 + uint64_t(__builtin_ctzll(m));
            m &= m - 1;
            if (dtype == 0) static_cast<uint32_t*>(compact)[slot] = static_cast<const uint32_t*>(grad)[i];
            else static_cast<uint16_t*>(compact)[slot] = static_cast<const uint16_t*>(grad)[i];
            ++slot;
        }
    }
}

// out[j] = ((c_0[j] + c_1[j]) + ...) + c_{W-1}[j], slots in parallel, workers in order.
void orc_reduce_mt(const void* const* bufs, uint32_t W, int dtype, uint64_t nnz, void* out) {
    const int T = orc_mt_threads();
#pragma omp parallel for num_threads(T) schedule(static)
    for (int64_t j = 0; j < int64_t(nnz); ++j) {
        if (dtype == 0) {
            float acc = static_cast<const float*>(bufs[0])[j];
            for (uint32_t w = 1; w < W; ++w) acc = acc + static_cast<const float*>(bufs[w])[j];
            static_cast<float*>(out)[j] = acc;
        } else {
            float acc = widen_bf16(static_cast<const uint16_t*>(bufs[0])[j]);
            for (uint32_t w = 1; w < W; ++w) acc = acc + widen_bf16(static_cast<const uint16_t*>(bufs[w])[j]);
            static_cast<uint16_t*>(out)[j] = narrow_bf16(acc);
        }
    }
}

// out[i] = compact[slot(i)] where the bit is set, the all-zero pattern elsewhere; words in parallel.
void orc_decompress_mt(const void* compact, int dtype, const uint64_t* mask, const uint32_t* prefix, void* out, uint64_t n) {
    const int T = orc_mt_threads();
    const int64_t words = int64_t((n + 63) / 64);
#pragma omp parallel for num_threads(T) schedule(static)
    for (int64_t j = 0; j < words; ++j) {
        const uint64_t m = mask[j];
        uint64_t slot = prefix[j];
        const uint64_t first = uint64_t(j) * 64;
        const uint64_t last = first + 64 < n ? first + 64 : n;
        for (uint64_t i = first; i < last; ++i) {
            const bool kept = (m >> (i & 63)) & 1u;
            if (dtype == 0) static_cast<uint32_t*>(out)[i] = kept ? static_cast<const uint32_t*>(compact)[slot] : 0u;
            else static_cast<uint16_t*>(out)[i] = kept ? static_cast<const uint16_t*>(compact)[slot] : uint16_t(0);
            slot += kept;
        }
    }
}

}  // extern "C"
