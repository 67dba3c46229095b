// PacTrain compression path: CPU oracle.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
// mask -> compress -> sum -> decompress path computes.  It is used by the tests,
// by the smoke check and by the benchmark's CPU-baseline leg; the product never
// calls it and it shares no code with the GPU library.
//
// Every function is single threaded and written as the definition reads: no
// blocking, no vector intrinsics, no reordering.  Built with the host compiler
// without fast-math, so float adds are IEEE single adds in the written order and
// denormals are kept.
//
// What the paper fixes and what it leaves open:
//  * Importance of a weight is its absolute value (Sec. II-B, first criterion named;
//    Sec. III-B: gradient elements are selected by local weight magnitude, identical on
//    every worker).  Prune(model, pruning_ratio) is step 1 of the algorithm in Sec. III-C
//    and line 2 of Alg. 1.
//  * The mask is shared by all workers and is used to reformat a sparse flat gradient
//    into a shorter dense tensor that a floating-point all-reduce can sum
//    (Sec. I contribution 2, Sec. III-B, Alg. 1 compress step, Mask Tracker paragraph).
//  * Gradient sparsity enforcement, Eq. 2: gradient entries of pruned weights are zero.
//  * Aggregation is the sum over workers inside Eq. 1 (the 1/n and the learning rate
//    belong to the weight update, which is outside this path).
// Readings where the paper is silent (count rounding, tie order, special floats, slot
// order, fill value, summation order, bf16 rounding) are stated at each function.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <vector>

namespace {

inline uint32_t float_bits(float x) {
    uint32_t u;
    std::memcpy(&u, &x, sizeof u);
    return u;
}

inline float bits_float(uint32_t u) {
    float x;
    std::memcpy(&x, &u, sizeof x);
    return x;
}

// Magnitude key: the IEEE-754 single bit pattern with the sign cleared, compared as an
// unsigned integer.  For every non-NaN float this order equals the order of |x|
// (denormals included, -0 ties +0); NaN patterns sort above infinity.
inline uint32_t magnitude_key(float x) { return float_bits(x) & 0x7FFFFFFFu; }

// bf16 <-> float.  Widening is exact (append 16 zero bits).  Narrowing rounds to nearest,
// ties to even, on the 32-bit pattern; a NaN stays a NaN (quiet bit forced) instead of
// being rounded into infinity.
inline float bf16_to_float(uint16_t h) { return bits_float(uint32_t(h) << 16); }

inline uint16_t float_to_bf16_rne(float x) {
    uint32_t u = float_bits(x);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return uint16_t((u >> 16) | 0x0040u);
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    return uint16_t(u >> 16);
}

inline bool mask_bit(const uint64_t* mask, uint64_t i) { return (mask[i >> 6] >> (i & 63)) & 1u; }

}  // namespace

extern "C" {

enum { ORC_F32 = 0, ORC_BF16 = 1 };

// Keep count of one prune scope: k = ceil((1 - s) * n), evaluated in integers with the
// sparsity taken to the nearest millionth so that the result does not depend on how a
// double happens to round (1 - s) * n.   (Pruning ratio: Alg. 1 input, Sec. III-C step 1.)
uint64_t orc_keep_count(uint64_t n, double sparsity) {
    const uint64_t M = 1000000u;
    long long ppm = std::llround(sparsity * 1e6);
    if (ppm < 0) ppm = 0;
    if (ppm > (long long)M) ppm = (long long)M;
    return (n * (M - (uint64_t)ppm) + M - 1) / M;
}

// Mask of the kept weights, one prune scope per segment [seg_off[s], seg_off[s+1]).
//
// Kept set of a scope with n elements and keep count k: the k elements that come first
// when the scope is ordered by |w| descending, flat index ascending.  Written out: give
// element i the composite (key_i << 32) | (0xFFFFFFFF - i); composites are distinct, and
// element i is kept iff its composite is among the k largest.
//
// mask:   ceil(n/64) words, bit b of word j stands for flat element 64*j + b, bits at or
//         beyond n are zero.
// prefix: prefix[j] = number of set bits in words 0 .. j-1 (over the whole flat set,
//         regardless of segments).
// Returns 0, or -1 on bad arguments (n >= 2^32, offsets not ascending / not ending at n,
// sparsity outside [0,1] or NaN).
int orc_build_mask(const float* weights, uint64_t n, const uint64_t* seg_off, uint32_t nseg,
                   const double* sparsity, uint64_t* mask, uint32_t* prefix, uint64_t* nnz_out) {
    if (n >= (uint64_t(1) << 32) || nseg == 0 || seg_off[0] != 0 || seg_off[nseg] != n) return -1;
    for (uint32_t s = 0; s < nseg; ++s) {
        if (seg_off[s] > seg_off[s + 1]) return -1;
        if (!(sparsity[s] >= 0.0 && sparsity[s] <= 1.0)) return -1;
    }
    const uint64_t words = (n + 63) / 64;
    for (uint64_t j = 0; j < words; ++j) mask[j] = 0;

    uint64_t total = 0;
    std::vector<uint64_t> comp;
    for (uint32_t s = 0; s < nseg; ++s) {
        const uint64_t b = seg_off[s], e = seg_off[s + 1];
        const uint64_t len = e - b;
        const uint64_t k = orc_keep_count(len, sparsity[s]);
        total += k;
        if (k == 0) continue;
        comp.resize(len);
        for (uint64_t i = b; i < e; ++i)
            comp[i - b] = (uint64_t(magnitude_key(weights[i])) << 32) | uint64_t(0xFFFFFFFFu - uint32_t(i));
        // k-th largest composite lands at position k-1 of a descending order.
        std::nth_element(comp.begin(), comp.begin() + (k - 1), comp.end(), std::greater<uint64_t>());
        const uint64_t kth = comp[k - 1];
        for (uint64_t i = b; i < e; ++i) {
            const uint64_t c = (uint64_t(magnitude_key(weights[i])) << 32) | uint64_t(0xFFFFFFFFu - uint32_t(i));
            if (c >= kth) mask[i >> 6] |= uint64_t(1) << (i & 63);
        }
    }

    uint64_t running = 0;
    for (uint64_t j = 0; j < words; ++j) {
        prefix[j] = uint32_t(running);
        running += (uint64_t)__builtin_popcountll(mask[j]);
    }
    if (nnz_out) *nnz_out = total;
    return 0;
}

// Compress one worker's flat gradient: walk flat positions in ascending order and append
// the element wherever the mask bit is set.  Elements are copied as bit patterns.  The
// slot order (ascending flat index) is the one boolean-mask indexing gives; any order
// shared by all workers would serve the method, this one is fixed here.
// Returns the number of set bits met; elements beyond `capacity` are counted, not written.
uint64_t orc_compress(const void* grad, int dtype, uint64_t n, const uint64_t* mask, void* compact,
                      uint64_t capacity) {
    uint64_t out = 0;
    if (dtype == ORC_F32) {
        const uint32_t* g = static_cast<const uint32_t*>(grad);
        uint32_t* c = static_cast<uint32_t*>(compact);
        for (uint64_t i = 0; i < n; ++i)
            if (mask_bit(mask, i)) {
                if (out < capacity) c[out] = g[i];
                ++out;
            }
    } else {
        const uint16_t* g = static_cast<const uint16_t*>(grad);
        uint16_t* c = static_cast<uint16_t*>(compact);
        for (uint64_t i = 0; i < n; ++i)
            if (mask_bit(mask, i)) {
                if (out < capacity) c[out] = g[i];
                ++out;
            }
    }
    return out;
}

// Sum of W compact buffers, slot by slot: the Sigma of Eq. 1 over the workers, as a native
// floating-point all-reduce would produce it, with the order fixed here to
// (((c_0 + c_1) + c_2) + ... + c_{W-1}) starting from worker 0's value.
// fp32: single-precision adds.  bf16 payload: every input is widened to single, the same
// ordered single-precision adds, one round-to-nearest-even back to bf16.
void orc_reduce(const void* const* bufs, uint32_t W, int dtype, uint64_t nnz, void* out) {
    if (dtype == ORC_F32) {
        float* o = static_cast<float*>(out);
        for (uint64_t j = 0; j < nnz; ++j) {
            float acc = static_cast<const float*>(bufs[0])[j];
            for (uint32_t w = 1; w < W; ++w) acc = acc + static_cast<const float*>(bufs[w])[j];
            o[j] = acc;
        }
    } else {
        uint16_t* o = static_cast<uint16_t*>(out);
        for (uint64_t j = 0; j < nnz; ++j) {
            float acc = bf16_to_float(static_cast<const uint16_t*>(bufs[0])[j]);
            for (uint32_t w = 1; w < W; ++w)
                acc = acc + bf16_to_float(static_cast<const uint16_t*>(bufs[w])[j]);
            o[j] = float_to_bf16_rne(acc);
        }
    }
}

// Decompress: the dense output is first filled with the all-zero bit pattern (+0.0), then
// flat positions are walked in ascending order and each set bit takes the next compact
// value.  Pruned positions are selected to zero, not multiplied by zero, so they are +0
// whatever the gradient held (Eq. 2 read as a selection).
// Returns the number of set bits met; bits beyond `nnz` compact values leave the zero fill.
uint64_t orc_decompress(const void* compact, int dtype, uint64_t nnz, const uint64_t* mask, void* dense,
                        uint64_t n) {
    uint64_t next = 0;
    if (dtype == ORC_F32) {
        const uint32_t* c = static_cast<const uint32_t*>(compact);
        uint32_t* d = static_cast<uint32_t*>(dense);
        for (uint64_t i = 0; i < n; ++i) d[i] = 0u;
        for (uint64_t i = 0; i < n; ++i)
            if (mask_bit(mask, i)) {
                if (next < nnz) d[i] = c[next];
                ++next;
            }
    } else {
        const uint16_t* c = static_cast<const uint16_t*>(compact);
        uint16_t* d = static_cast<uint16_t*>(dense);
        for (uint64_t i = 0; i < n; ++i) d[i] = 0u;
        for (uint64_t i = 0; i < n; ++i)
            if (mask_bit(mask, i)) {
                if (next < nnz) d[i] = c[next];
                ++next;
            }
    }
    return next;
}

// Round a float array to bf16 patterns with the rule above (exposed so that tests can pin
// the rounding against an independent bf16 implementation).
void orc_f32_to_bf16(const float* in, uint16_t* out, uint64_t n) {
    for (uint64_t i = 0; i < n; ++i) out[i] = float_to_bf16_rne(in[i]);
}

// ---- around the hot path: Mask Tracker and the weight update -------------------------------

// Mask of the non-zero elements of a flat tensor: the (Weight != 0) of Eq. 2, which is also how
// the Mask Tracker (Sec. III-B, Mask Tracker paragraph) reads the sparsity pattern off a
// flattened bucket without names or shapes.  "!= 0" is the IEEE comparison: -0 is zero, NaN
// and denormals are non-zero.  bf16 values are compared after exact widening.
// Writes the bitmask (bits >= n zero) and the exclusive prefix; returns the number of set bits.
uint64_t orc_mask_from_nonzero(const void* values, int dtype, uint64_t n, uint64_t* mask, uint32_t* prefix) {
    const uint64_t words = (n + 63) / 64;
    for (uint64_t w = 0; w < words; ++w) mask[w] = 0;
    for (uint64_t i = 0; i < n; ++i) {
        const float x = dtype == ORC_F32 ? static_cast<const float*>(values)[i]
                                         : bf16_to_float(static_cast<const uint16_t*>(values)[i]);
        if (x != 0.0f) mask[i >> 6] |= 1ull << (i & 63);
    }
    uint64_t running = 0;
    for (uint64_t w = 0; w < words; ++w) {
        prefix[w] = static_cast<uint32_t>(running);
        running += static_cast<uint64_t>(__builtin_popcountll(mask[w]));
    }
    return running;
}

// Number of positions below n at which two masks differ: the Mask Tracker's comparison of this
// iteration's mask with the previous one (zero = unchanged).
uint64_t orc_mask_diff(const uint64_t* a, const uint64_t* b, uint64_t n) {
    uint64_t diff = 0;
    for (uint64_t i = 0; i < n; ++i)
        if (mask_bit(a, i) != mask_bit(b, i)) ++diff;
    return diff;
}

// Weight update of Eq. 1 on the sparse model, fused with the decompression of the summed
// compact buffer: a kept weight becomes x - alpha * g with g the next compact value (widened
// exactly if bf16) and alpha = eta / n supplied by the caller as one single-precision number;
// a pruned weight becomes +0 (Prune made it zero and Eq. 2 keeps it there).  Two IEEE single
// operations per kept element, a multiply and a subtract, each rounded to nearest (no fused
// multiply-add).  Bits beyond `nnz` compact values take g = +0.
// Returns the number of set bits met.
uint64_t orc_decompress_update(const void* compact, int dtype, uint64_t nnz, const uint64_t* mask, float alpha,
                               float* weights, uint64_t n) {
    uint64_t next = 0;
    for (uint64_t i = 0; i < n; ++i) {
        if (!mask_bit(mask, i)) {
            weights[i] = 0.0f;
            continue;
        }
        float g = 0.0f;
        if (next < nnz)
            g = dtype == ORC_F32 ? static_cast<const float*>(compact)[next]
                                 : bf16_to_float(static_cast<const uint16_t*>(compact)[next]);
        ++next;
        const float step = alpha * g;
        weights[i] = weights[i] - step;
    }
    return next;
}

// ---- ternary payload (Sec. III-D) ---------------------
// ternarize(.) of Sec. III-D is the TernGrad quantiser the section names: with a scale s >= max|g|,
// every element becomes s * sign(g) * b with b ~ Bernoulli(|g| / s), so that E[s * t] = g (Eq. 3 is
// that expectation).  The paper fixes neither the random source nor the layout; here:
//  * random bits: the Philox4x32-10 counter-based generator (Salmon et al., SC'11), key = the two
//    halves of `seed`, counter = (block, block >> 32, stream, stream >> 32) with block = j / 4; the
//    four output words serve elements 4*block .. 4*block+3.  A worker passes its own `stream`.
//  * u = (word >> 8) * 2^-24, a uniform in [0,1) that is exact in single precision;
//    p = |g| / s as one IEEE single division; the element is kept iff u < p.
//  * code 0 = 0, 1 = +1, 2 = -1; element j sits in bits 2*(j%4).. of byte j/4; unused bits zero.
//  * a scale that is zero, negative, infinite or NaN, and NaN elements, give code 0.
//  * the scale is shared by the workers (TernGrad's scaler sharing), so that the ternaries can be
//    summed as integers by an all-reduce: sum = s * (float)(t_0 + ... + t_{W-1}).

static inline void philox_round(uint32_t c[4], uint32_t k0, uint32_t k1) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c[0];
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c[2];
    const uint32_t n0 = (uint32_t)(p1 >> 32) ^ c[1] ^ k0;
    const uint32_t n1 = (uint32_t)p1;
    const uint32_t n2 = (uint32_t)(p0 >> 32) ^ c[3] ^ k1;
    const uint32_t n3 = (uint32_t)p0;
    c[0] = n0; c[1] = n1; c[2] = n2; c[3] = n3;
}

// Philox4x32 with 10 rounds; the key is bumped by the Weyl constants between rounds.
void orc_philox4x32_10(const uint32_t counter[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c[4] = {counter[0], counter[1], counter[2], counter[3]};
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        philox_round(c, k0, k1);
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    for (int i = 0; i < 4; ++i) out[i] = c[i];
}

// max |x| over the buffer, NaN elements ignored; 0 for an empty buffer.  If `start` is given the
// result is max(*start, max|x|): calls over the W workers' buffers build the shared scale.
float orc_absmax(const void* values, int dtype, uint64_t count, const float* start) {
    float m = start ? *start : 0.0f;
    for (uint64_t j = 0; j < count; ++j) {
        const float x = dtype == ORC_F32 ? static_cast<const float*>(values)[j]
                                         : bf16_to_float(static_cast<const uint16_t*>(values)[j]);
        const float a = std::fabs(x);
        if (a > m) m = a;          // false for NaN
    }
    return m;
}

void orc_ternarize(const void* values, int dtype, uint64_t count, float scale, uint64_t seed, uint64_t stream,
                   uint8_t* packed) {
    const uint64_t bytes = (count + 3) / 4;
    for (uint64_t b = 0; b < bytes; ++b) packed[b] = 0;
    const bool usable = scale > 0.0f && !std::isinf(scale);     // false for NaN too
    if (!usable) return;
    const uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (uint64_t block = 0; block * 4 < count; ++block) {
        const uint32_t counter[4] = {(uint32_t)block, (uint32_t)(block >> 32), (uint32_t)stream, (uint32_t)(stream >> 32)};
        uint32_t r[4];
        orc_philox4x32_10(counter, key, r);
        for (uint64_t e = 0; e < 4 && block * 4 + e < count; ++e) {
            const uint64_t j = block * 4 + e;
            const float x = dtype == ORC_F32 ? static_cast<const float*>(values)[j]
                                             : bf16_to_float(static_cast<const uint16_t*>(values)[j]);
            const float u = (float)(r[e] >> 8) * 5.9604644775390625e-08f;     // 2^-24, exact
            const float p = std::fabs(x) / scale;
            if (u < p) packed[j >> 2] |= (uint8_t)((std::signbit(x) ? 2u : 1u) << (2 * (j & 3)));
        }
    }
}

// out[j] = scale * (float)(t_0[j] + ... + t_{W-1}[j]): an exact integer sum, one multiply, and for a
// bf16 output one rounding to nearest even.
void orc_ternary_reduce(const uint8_t* const* packed, uint32_t W, uint64_t count, float scale, int out_dtype,
                        void* out) {
    for (uint64_t j = 0; j < count; ++j) {
        int32_t sum = 0;
        for (uint32_t w = 0; w < W; ++w) {
            const uint32_t code = (packed[w][j >> 2] >> (2 * (j & 3))) & 3u;
            sum += code == 1 ? 1 : code == 2 ? -1 : 0;
        }
        const float v = scale * (float)sum;
        if (out_dtype == ORC_F32) static_cast<float*>(out)[j] = v;
        else static_cast<uint16_t*>(out)[j] = float_to_bf16_rne(v);
    }
}

}  // extern "C"
