// Mask Tracker kernels (Sec. III-B, Mask Tracker paragraph; Alg. 1, mask-update step): the mask of
// the non-zero elements of a flat tensor (the Weight != 0 of Eq. 2), the comparison of two masks, and
// the stability counter.  All are streaming passes over n*e or n/8 bytes, bound by HBM bandwidth.
#include "pac_internal.h"

namespace pac {
namespace {

typedef unsigned long long u64;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kBlock = 256;

__device__ __forceinline__ uint32_t or_over_8_lanes(uint32_t x) {
    // After the three steps every lane of an aligned group of 8 holds the OR of the group.
    x |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0xB1, 0xF, 0xF, true);    // quad_perm [1,0,3,2]
    x |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x4E, 0xF, 0xF, true);    // quad_perm [2,3,0,1]
    x |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, 0x141, 0xF, 0xF, true);   // row_half_mirror
    return x;
}

// "!= 0" as the IEEE comparison on bit patterns: both zeros are zero, NaN and denormals are not.
__device__ __forceinline__ uint32_t nz32(uint32_t bits) { return (bits & 0x7FFFFFFFu) != 0 ? 1u : 0u; }
__device__ __forceinline__ uint32_t nz16(uint32_t bits) { return (bits & 0x7FFFu) != 0 ? 1u : 0u; }

// ---------------------------------------------------------------------------- mask of non-zeros
// A lane owns 16-byte chunks (4 fp32 or 8 bf16 elements); the 8 lanes that share a 32-bit half word
// (fp32) or a whole 64-bit word (bf16) OR their shifted bits together with DPP steps and one of
// them stores.  Chunk q >= n / E holds the at most E-1 elements after the last whole chunk.
constexpr uint32_t kNzLoads = 4;   // chunks per lane

template <int DT>   // 0 = fp32, 1 = bf16
__global__ __launch_bounds__(kBlock) void nonzero_mask_kernel(const u32x4* __restrict__ values, uint32_t n,
                                                              u64* __restrict__ mask) {
    constexpr uint32_t E = DT == 0 ? 4u : 8u;
    const uint32_t n_chunks = n / E;
    const uint32_t words = (uint32_t)(((u64)n + 63) >> 6);
    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t first = blockIdx.x * (kBlock * kNzLoads) + (threadIdx.x >> 6) * (64 * kNzLoads);   // wave's first chunk
    u32x4 v[kNzLoads];
#pragma unroll
    for (uint32_t u = 0; u < kNzLoads; ++u) {
        const uint32_t q = first + u * 64 + lane;
        v[u] = (u32x4){0, 0, 0, 0};
        if (q < n_chunks) {
            v[u] = __builtin_nontemporal_load(values + q);
        } else if (q == n_chunks) {   // the elements after the last whole chunk, one by one
            uint32_t d[4] = {0, 0, 0, 0};
            for (uint32_t e = 0; e < n - n_chunks * E; ++e) {
                if (DT == 0) d[e] = reinterpret_cast<const uint32_t*>(values)[n_chunks * E + e];
                else d[e >> 1] |= (uint32_t)reinterpret_cast<const uint16_t*>(values)[n_chunks * E + e] << ((e & 1u) * 16u);
            }
            v[u] = (u32x4){d[0], d[1], d[2], d[3]};
        }
    }
#pragma unroll
    for (uint32_t u = 0; u < kNzLoads; ++u) {
        const uint32_t q0 = first + u * 64;   // first chunk of this wave step
        if (DT == 0) {
            const uint32_t nib = nz32(v[u].x) | (nz32(v[u].y) << 1) | (nz32(v[u].z) << 2) | (nz32(v[u].w) << 3);
            const uint32_t half = or_over_8_lanes(nib << ((lane & 7u) * 4u));
            const u64 half_idx = (u64)(q0 >> 3) + (lane >> 3);   // 8 chunks of 4 elements per half word
            if ((lane & 7u) == 0 && half_idx < 2ull * words) reinterpret_cast<uint32_t*>(mask)[half_idx] = half;
        } else {
            const uint32_t byte = nz16(v[u].x) | (nz16(v[u].x >> 16) << 1) | (nz16(v[u].y) << 2) |
                                  (nz16(v[u].y >> 16) << 3) | (nz16(v[u].z) << 4) | (nz16(v[u].z >> 16) << 5) |
                                  (nz16(v[u].w) << 6) | (nz16(v[u].w >> 16) << 7);
            const uint32_t sh = (lane & 3u) * 8u;
            const uint32_t lo = or_over_8_lanes((lane & 4u) ? 0u : byte << sh);
            const uint32_t hi = or_over_8_lanes((lane & 4u) ? byte << sh : 0u);
            const u64 word_idx = (u64)(q0 >> 3) + (lane >> 3);   // 8 chunks of 8 elements per word
            if ((lane & 7u) == 0 && word_idx < words) mask[word_idx] = ((u64)hi << 32) | lo;
        }
    }
}

// Any element alignment: one element per lane, the wave's ballot is the mask word.
template <int DT>
__global__ __launch_bounds__(kBlock) void nonzero_mask_scalar_kernel(const void* __restrict__ values, uint32_t n,
                                                                     u64* __restrict__ mask) {
    const u64 i = (u64)blockIdx.x * kBlock + threadIdx.x;
    bool nz = false;
    if (i < n) nz = DT == 0 ? nz32(static_cast<const uint32_t*>(values)[i]) != 0
                            : nz16(static_cast<const uint16_t*>(values)[i]) != 0;
    const u64 word = __ballot(nz);
    if ((threadIdx.x & 63u) == 0 && i < n) mask[i >> 6] = word;
}

// --------------------------------------------------------------------------- mask comparison
__global__ void zero_u64_kernel(u64* p) { *p = 0; }

template <bool COPY>
__global__ __launch_bounds__(kBlock) void mask_diff_kernel(const u64* a, const u64* __restrict__ b,
                                                           uint32_t words, uint32_t n, u64* __restrict__ diff_out,
                                                           u64* copy_to) {   // copy_to may be a
    __shared__ uint32_t wave_sums[kBlock / 64];
    const u64 last_keep = (n & 63u) ? ((1ull << (n & 63u)) - 1ull) : ~0ull;   // bits of the last word below n
    uint32_t acc = 0;
    for (u64 w = (u64)blockIdx.x * kBlock + threadIdx.x; w < words; w += (u64)gridDim.x * kBlock) {
        const u64 x = a[w], y = b[w];
        u64 d = x ^ y;
        if (w == words - 1) d &= last_keep;
        acc += (uint32_t)__popcll(d);
        if (COPY) copy_to[w] = y;
    }
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) acc += __shfl_xor(acc, d, 64);
    if ((threadIdx.x & 63u) == 0) wave_sums[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        u64 t = 0;
        for (int i = 0; i < kBlock / 64; ++i) t += wave_sums[i];
        if (t) atomicAdd(diff_out, t);
    }
}

__global__ void copy_words_kernel(const u64* __restrict__ src, u64* __restrict__ dst, uint32_t words) {
    for (u64 w = (u64)blockIdx.x * blockDim.x + threadIdx.x; w < words; w += (u64)gridDim.x * blockDim.x) dst[w] = src[w];
}

__global__ void tracker_finalize_kernel(TrackerState* st, uint32_t patience, uint32_t fresh, uint32_t* out) {
    const uint32_t unchanged = (!fresh && st->diff == 0) ? st->unchanged + 1u : 0u;
    st->unchanged = unchanged;
    st->stable = unchanged >= patience ? 1u : 0u;
    st->diff = 0;
    if (out) { out[0] = unchanged; out[1] = st->stable; }
}

inline uint32_t div_up(u64 a, u64 b) { return (uint32_t)((a + b - 1) / b); }

}  // namespace

hipError_t launch_nonzero_mask(const void* d_values, int dtype, uint32_t n, unsigned long long* d_mask,
                               hipStream_t stream) {
    if (n == 0) return hipSuccess;
    if ((reinterpret_cast<uintptr_t>(d_values) & 15u) == 0) {
        const uint32_t E = dtype == 0 ? 4u : 8u;
        // chunks 0 .. n/E (the last one partial or empty), rounded up to whole mask words
        const uint32_t chunks = div_up((u64)div_up(n, 64) * 64, E);
        const uint32_t blocks = div_up(chunks, kBlock * kNzLoads);
        if (dtype == 0)
            hipLaunchKernelGGL((nonzero_mask_kernel<0>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const u32x4*>(d_values), n, d_mask);
        else
            hipLaunchKernelGGL((nonzero_mask_kernel<1>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const u32x4*>(d_values), n, d_mask);
    } else {
        const uint32_t blocks = div_up(n, kBlock);
        if (dtype == 0)
            hipLaunchKernelGGL((nonzero_mask_scalar_kernel<0>), dim3(blocks), dim3(kBlock), 0, stream, d_values, n, d_mask);
        else
            hipLaunchKernelGGL((nonzero_mask_scalar_kernel<1>), dim3(blocks), dim3(kBlock), 0, stream, d_values, n, d_mask);
    }
    return hipGetLastError();
}

hipError_t launch_mask_diff(const unsigned long long* d_a, const unsigned long long* d_b, uint32_t n,
                            unsigned long long* d_diff_out, unsigned long long* d_copy_to, hipStream_t stream) {
    hipLaunchKernelGGL(zero_u64_kernel, dim3(1), dim3(1), 0, stream, d_diff_out);
    if (n == 0) return hipGetLastError();
    const uint32_t words = div_up(n, 64);
    uint32_t blocks = div_up(words, kBlock * 4);
    if (blocks > 4096) blocks = 4096;
    if (d_copy_to)
        hipLaunchKernelGGL((mask_diff_kernel<true>), dim3(blocks), dim3(kBlock), 0, stream, d_a, d_b, words, n,
                           d_diff_out, d_copy_to);
    else
        hipLaunchKernelGGL((mask_diff_kernel<false>), dim3(blocks), dim3(kBlock), 0, stream, d_a, d_b, words, n,
                           d_diff_out, static_cast<u64*>(nullptr));
    return hipGetLastError();
}

hipError_t launch_mask_copy(const unsigned long long* d_src, unsigned long long* d_dst, uint32_t words,
                            hipStream_t stream) {
    if (words == 0) return hipSuccess;
    uint32_t blocks = div_up(words, kBlock * 4);
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(copy_words_kernel, dim3(blocks), dim3(kBlock), 0, stream, d_src, d_dst, words);
    return hipGetLastError();
}

hipError_t launch_tracker_finalize(TrackerState* d_state, uint32_t patience, uint32_t fresh, uint32_t* d_state_out,
                                   hipStream_t stream) {
    hipLaunchKernelGGL(tracker_finalize_kernel, dim3(1), dim3(1), 0, stream, d_state, patience, fresh, d_state_out);
    return hipGetLastError();
}

}  // namespace pac
