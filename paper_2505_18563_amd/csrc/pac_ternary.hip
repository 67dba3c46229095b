// Ternary payload (Sec. III-D): the TernGrad quantiser on the
// compact buffer.  Shared scale s = max |g| over the workers' buffers; element -> s * sign(g) * b,
// b ~ Bernoulli(|g| / s); 2-bit codes, four per byte; the workers' ternaries are summed as integers.
// Random bits come from the Philox4x32-10 counter-based generator (Salmon et al., SC'11):
// key = seed, counter = (element / 4, stream), so any element's draw can be recomputed anywhere.
// The kernels stream e*k (or k/4) bytes once.  The quantiser is bound by arithmetic, not by HBM:
// ten Philox rounds per four elements plus one correctly rounded division per element come to
// about 35 vector operations per element.
#include "pac_internal.h"

namespace pac {
namespace {

typedef unsigned long long u64;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;

struct Philox {
    uint32_t c0, c1, c2, c3;
};

// Ten rounds of Philox4x32; the key is bumped by the Weyl constants between rounds.
__device__ __forceinline__ Philox philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                                uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        const uint32_t n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Philox{c0, c1, c2, c3};
}

// 2-bit code of one element: kept iff u < |x| / s with u = (word >> 8) * 2^-24.
__device__ __forceinline__ uint32_t tern_code(float x, float s, uint32_t word) {
    const float u = __uint2float_rn(word >> 8) * 5.9604644775390625e-08f;   // exact: 24 bits
    const float p = __fdiv_rn(fabsf(x), s);
    if (!(u < p)) return 0u;                                                  // also when p is NaN
    return (__float_as_uint(x) >> 31) ? 2u : 1u;
}

__device__ __forceinline__ bool scale_usable(float s) { return s > 0.0f && s < __uint_as_float(0x7F800000u); }

__device__ __forceinline__ float widen16(uint32_t h) { return __uint_as_float(h << 16); }

// codes of the four elements of Philox block `block`, packed into one byte
__device__ __forceinline__ uint32_t tern_byte(float x0, float x1, float x2, float x3, float s, u64 block, u64 stream,
                                              uint32_t k0, uint32_t k1) {
    const Philox r = philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), (uint32_t)stream,
                                   (uint32_t)(stream >> 32), k0, k1);
    return tern_code(x0, s, r.c0) | (tern_code(x1, s, r.c1) << 2) | (tern_code(x2, s, r.c2) << 4) |
           (tern_code(x3, s, r.c3) << 6);
}

// -------------------------------------------------------------------------------------- absmax
__global__ void set_float_kernel(float* p, float v) { *p = v; }

// max over the non-NaN |x| as a bit pattern (non-negative floats order like their patterns)
template <int DT>
__device__ __forceinline__ uint32_t absmax_chunk(const u32x4 v) {
    uint32_t m = 0;
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (DT == 0) {
            const uint32_t k = d[i] & 0x7FFFFFFFu;
            if (k <= 0x7F800000u && k > m) m = k;
        } else {
            const uint32_t a = (d[i] & 0x7FFFu) << 16, b = d[i] & 0x7FFF0000u;
            if (a <= 0x7F800000u && a > m) m = a;
            if (b <= 0x7F800000u && b > m) m = b;
        }
    }
    return m;
}

template <int DT>
__global__ __launch_bounds__(kBlock) void absmax_kernel(const void* __restrict__ values, uint32_t count,
                                                        uint32_t vec_ok, uint32_t* __restrict__ scale_bits) {
    __shared__ uint32_t wave_max[kBlock / 64];
    constexpr uint32_t E = DT == 0 ? 4u : 8u;
    uint32_t m = 0;
    const uint32_t n_chunks = vec_ok ? count / E : 0u;
    for (u64 q = (u64)blockIdx.x * kBlock + threadIdx.x; q < n_chunks; q += (u64)gridDim.x * kBlock) {
        const uint32_t c = absmax_chunk<DT>(__builtin_nontemporal_load(static_cast<const u32x4*>(values) + q));
        if (c > m) m = c;
    }
    // what the 16-byte loads did not cover, element by element
    for (u64 j = (u64)n_chunks * E + (u64)blockIdx.x * kBlock + threadIdx.x; j < count; j += (u64)gridDim.x * kBlock) {
        const uint32_t k = DT == 0 ? (static_cast<const uint32_t*>(values)[j] & 0x7FFFFFFFu)
                                   : ((uint32_t)(static_cast<const uint16_t*>(values)[j] & 0x7FFFu) << 16);
        if (k <= 0x7F800000u && k > m) m = k;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, d, 64));
    if ((threadIdx.x & 63u) == 0) wave_max[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int i = 1; i < kBlock / 64; ++i) m = max(m, wave_max[i]);
        if (m != 0) atomicMax(scale_bits, m);
    }
}

// ----------------------------------------------------------------------------------- ternarize
// A thread owns one 16-byte chunk: one Philox block and one output byte for fp32, two blocks and two
// bytes for bf16.  The (at most 3 or 7) elements after the last whole chunk go to one more thread.
template <int DT>
__global__ __launch_bounds__(kBlock) void ternarize_kernel(const void* __restrict__ values, uint32_t count,
                                                           uint32_t vec_ok, const float* __restrict__ scale,
                                                           u64 seed, u64 stream, uint8_t* __restrict__ packed) {
    constexpr uint32_t E = DT == 0 ? 4u : 8u;
    const float s = *scale;
    const bool usable = scale_usable(s);
    const uint32_t k0 = (uint32_t)seed, k1 = (uint32_t)(seed >> 32);
    const uint32_t n_chunks = count / E;
    const uint32_t q = blockIdx.x * kBlock + threadIdx.x;
    if (q < n_chunks) {
        float x[8];
        if (vec_ok) {
            const u32x4 v = __builtin_nontemporal_load(static_cast<const u32x4*>(values) + q);
            if (DT == 0) {
                x[0] = __uint_as_float(v.x); x[1] = __uint_as_float(v.y); x[2] = __uint_as_float(v.z); x[3] = __uint_as_float(v.w);
            } else {
                x[0] = widen16(v.x & 0xFFFFu); x[1] = widen16(v.x >> 16); x[2] = widen16(v.y & 0xFFFFu); x[3] = widen16(v.y >> 16);
                x[4] = widen16(v.z & 0xFFFFu); x[5] = widen16(v.z >> 16); x[6] = widen16(v.w & 0xFFFFu); x[7] = widen16(v.w >> 16);
            }
        } else {
#pragma unroll
            for (uint32_t e = 0; e < E; ++e)
                x[e] = DT == 0 ? static_cast<const float*>(values)[(u64)q * E + e]
                               : widen16(static_cast<const uint16_t*>(values)[(u64)q * E + e]);
        }
        if (DT == 0) {
            packed[q] = usable ? (uint8_t)tern_byte(x[0], x[1], x[2], x[3], s, q, stream, k0, k1) : (uint8_t)0;
        } else {
            uint32_t lo = 0, hi = 0;
            if (usable) {
                lo = tern_byte(x[0], x[1], x[2], x[3], s, 2ull * q, stream, k0, k1);
                hi = tern_byte(x[4], x[5], x[6], x[7], s, 2ull * q + 1, stream, k0, k1);
            }
            reinterpret_cast<uint16_t*>(packed)[q] = (uint16_t)(lo | (hi << 8));   // packed is 4-byte aligned
        }
    } else if (q == n_chunks && count % E != 0) {
        // the tail: up to E-1 elements, one output byte per started group of four
        const u64 first = (u64)n_chunks * E;
        for (u64 g = first / 4; g * 4 < count; ++g) {
            float x[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            for (uint32_t e = 0; e < 4 && g * 4 + e < count; ++e)
                x[e] = DT == 0 ? static_cast<const float*>(values)[g * 4 + e]
                               : widen16(static_cast<const uint16_t*>(values)[g * 4 + e]);
            // elements beyond count are +0 and take code 0
            packed[g] = usable ? (uint8_t)tern_byte(x[0], x[1], x[2], x[3], s, g, stream, k0, k1) : (uint8_t)0;
        }
    }
}

// ------------------------------------------------------------------------------ ternary reduce
__device__ __forceinline__ int32_t tern_value(uint32_t code) { return (int32_t)(code & 1u) - (int32_t)(code >> 1); }

__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

// A thread owns one 16-byte output chunk: 4 fp32 elements (one packed byte per worker) or 8 bf16
// elements (two bytes per worker).  Integer sums, one multiply by the scale.
template <int DT>
__global__ __launch_bounds__(kBlock) void ternary_reduce_kernel(WorkerPtrs bufs, uint32_t W, uint32_t count,
                                                                uint32_t vec_ok, const float* __restrict__ scale,
                                                                void* __restrict__ out) {
    constexpr uint32_t E = DT == 0 ? 4u : 8u;
    const float s = *scale;
    const uint32_t n_chunks = count / E;
    const uint32_t q = blockIdx.x * kBlock + threadIdx.x;
    if (q < n_chunks) {
        int32_t sum[E];
#pragma unroll
        for (uint32_t e = 0; e < E; ++e) sum[e] = 0;
        auto load_bits = [&](uint32_t w) -> uint32_t {
            if (DT == 0) return static_cast<const uint8_t*>(bufs.p[w])[q];
            return static_cast<const uint16_t*>(bufs.p[w])[q];         // packed buffers are 4-byte aligned
        };
        auto add_bits = [&](uint32_t bits) {
#pragma unroll
            for (uint32_t e = 0; e < E; ++e) sum[e] += tern_value((bits >> (2 * e)) & 3u);
        };
        uint32_t w = 0;
        for (; w + 4 <= W; w += 4) {   // four loads in flight
            const uint32_t b0 = load_bits(w), b1 = load_bits(w + 1), b2 = load_bits(w + 2), b3 = load_bits(w + 3);
            add_bits(b0); add_bits(b1); add_bits(b2); add_bits(b3);
        }
        for (; w < W; ++w) add_bits(load_bits(w));
        float v[E];
#pragma unroll
        for (uint32_t e = 0; e < E; ++e) v[e] = __fmul_rn(s, (float)sum[e]);
        u32x4 o;
        if (DT == 0) {
            o = (u32x4){__float_as_uint(v[0]), __float_as_uint(v[1]), __float_as_uint(v[2]), __float_as_uint(v[3])};
        } else {
            o = (u32x4){f32_to_bf16_bits(v[0]) | (f32_to_bf16_bits(v[1]) << 16),
                        f32_to_bf16_bits(v[2]) | (f32_to_bf16_bits(v[3]) << 16),
                        f32_to_bf16_bits(v[4 % E]) | (f32_to_bf16_bits(v[5 % E]) << 16),
                        f32_to_bf16_bits(v[6 % E]) | (f32_to_bf16_bits(v[7 % E]) << 16)};
        }
        if (vec_ok) {
            static_cast<u32x4*>(out)[q] = o;   // plain store: the sum is read next by decompress
        } else {
            if (DT == 0) {
                uint32_t* d = static_cast<uint32_t*>(out) + (u64)q * 4;
                d[0] = o.x; d[1] = o.y; d[2] = o.z; d[3] = o.w;
            } else {
                uint16_t* d = static_cast<uint16_t*>(out) + (u64)q * 8;
                d[0] = (uint16_t)o.x; d[1] = (uint16_t)(o.x >> 16); d[2] = (uint16_t)o.y; d[3] = (uint16_t)(o.y >> 16);
                d[4] = (uint16_t)o.z; d[5] = (uint16_t)(o.z >> 16); d[6] = (uint16_t)o.w; d[7] = (uint16_t)(o.w >> 16);
            }
        }
    } else if (q == n_chunks) {
        for (u64 j = (u64)n_chunks * E; j < count; ++j) {
            int32_t sum = 0;
            for (uint32_t w = 0; w < W; ++w)
                sum += tern_value((static_cast<const uint8_t*>(bufs.p[w])[j >> 2] >> (2 * (j & 3))) & 3u);
            const float v = __fmul_rn(s, (float)sum);
            if (DT == 0) static_cast<float*>(out)[j] = v;
            else static_cast<uint16_t*>(out)[j] = (uint16_t)f32_to_bf16_bits(v);
        }
    }
}

inline uint32_t div_up(u64 a, u64 b) { return (uint32_t)((a + b - 1) / b); }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

hipError_t launch_absmax(const void* d_values, int dtype, uint32_t count, bool accumulate, float* d_scale,
                         hipStream_t stream) {
    if (!accumulate) hipLaunchKernelGGL(set_float_kernel, dim3(1), dim3(1), 0, stream, d_scale, 0.0f);
    if (count == 0) return hipGetLastError();
    const uint32_t E = dtype == 0 ? 4u : 8u;
    uint32_t blocks = div_up(div_up(count, E), kBlock * 4);
    if (blocks > 2048) blocks = 2048;
    const uint32_t vec_ok = aligned16(d_values) ? 1u : 0u;
    if (dtype == 0)
        hipLaunchKernelGGL((absmax_kernel<0>), dim3(blocks), dim3(kBlock), 0, stream, d_values, count, vec_ok,
                           reinterpret_cast<uint32_t*>(d_scale));
    else
        hipLaunchKernelGGL((absmax_kernel<1>), dim3(blocks), dim3(kBlock), 0, stream, d_values, count, vec_ok,
                           reinterpret_cast<uint32_t*>(d_scale));
    return hipGetLastError();
}

hipError_t launch_ternarize(const void* d_values, int dtype, uint32_t count, const float* d_scale,
                            unsigned long long seed, unsigned long long stream_id, uint8_t* d_packed,
                            hipStream_t stream) {
    if (count == 0) return hipSuccess;
    const uint32_t E = dtype == 0 ? 4u : 8u;
    const uint32_t threads = count / E + 1;        // one more for the tail
    const uint32_t vec_ok = aligned16(d_values) ? 1u : 0u;
    if (dtype == 0)
        hipLaunchKernelGGL((ternarize_kernel<0>), dim3(div_up(threads, kBlock)), dim3(kBlock), 0, stream, d_values,
                           count, vec_ok, d_scale, seed, stream_id, d_packed);
    else
        hipLaunchKernelGGL((ternarize_kernel<1>), dim3(div_up(threads, kBlock)), dim3(kBlock), 0, stream, d_values,
                           count, vec_ok, d_scale, seed, stream_id, d_packed);
    return hipGetLastError();
}

hipError_t launch_ternary_reduce(const WorkerPtrs& bufs, uint32_t W, uint32_t count, const float* d_scale,
                                 int out_dtype, void* d_out, hipStream_t stream) {
    if (count == 0) return hipSuccess;
    const uint32_t E = out_dtype == 0 ? 4u : 8u;
    const uint32_t threads = count / E + 1;
    const uint32_t vec_ok = aligned16(d_out) ? 1u : 0u;
    if (out_dtype == 0)
        hipLaunchKernelGGL((ternary_reduce_kernel<0>), dim3(div_up(threads, kBlock)), dim3(kBlock), 0, stream, bufs,
                           W, count, vec_ok, d_scale, d_out);
    else
        hipLaunchKernelGGL((ternary_reduce_kernel<1>), dim3(div_up(threads, kBlock)), dim3(kBlock), 0, stream, bufs,
                           W, count, vec_ok, d_scale, d_out);
    return hipGetLastError();
}

}  // namespace pac
