// Gather (compress), scatter (decompress) and the W-way sum of compact buffers.
//
// All three are streaming kernels bound by HBM bandwidth.  A lane owns one 16-byte chunk of the
// dense tensor (8 bf16 or 4 fp32 elements); consecutive lanes own consecutive chunks, so dense
// loads and stores are full 128-bit coalesced accesses.  The mask word and its prefix entry of the
// chunk are fetched by every lane that shares them (one cache line per wave).  Compact accesses of
// a wave fall into one short contiguous range.
#include "pac_internal.h"

namespace pac {
namespace {

constexpr int kBlock = 256;

template <typename T>
struct Chunk {
    static constexpr uint32_t kElems = 16 / sizeof(T);   // elements per 16-byte chunk
};

__device__ __forceinline__ uint32_t popc64(unsigned long long x) { return (uint32_t)__popcll(x); }

// Sub-mask and first compact slot of chunk q (kElems elements starting at q * kElems).
template <typename T>
__device__ __forceinline__ void chunk_meta(uint32_t q, unsigned long long word, uint32_t pre,
                                           uint32_t& sub, uint32_t& slot) {
    constexpr uint32_t E = Chunk<T>::kElems;
    const uint32_t bitoff = (q * E) & 63u;
    sub = (uint32_t)(word >> bitoff) & ((1u << E) - 1u);
    slot = pre + popc64(word & ((1ull << bitoff) - 1ull));
}

__device__ __forceinline__ uint32_t dword_of(const uint4& v, int i) {
    return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w;
}

template <typename T>
__device__ __forceinline__ T elem_of(const uint4& v, int e);
template <>
__device__ __forceinline__ uint32_t elem_of<uint32_t>(const uint4& v, int e) { return dword_of(v, e); }
template <>
__device__ __forceinline__ uint16_t elem_of<uint16_t>(const uint4& v, int e) {
    const uint32_t d = dword_of(v, e >> 1);
    return (uint16_t)((e & 1) ? (d >> 16) : d);
}

// ------------------------------------------------------------------------------------ compress
template <typename T, int UNROLL>
__global__ __launch_bounds__(kBlock) void compress_vec_kernel(const uint4* __restrict__ grad, uint32_t n,
                                                              const unsigned long long* __restrict__ mask,
                                                              const uint32_t* __restrict__ prefix,
                                                              T* __restrict__ compact, uint32_t nnz) {
    constexpr uint32_t E = Chunk<T>::kElems;
    const uint32_t n_chunks = n / E;
    const uint32_t first = blockIdx.x * (uint32_t)(kBlock * UNROLL) + threadIdx.x;

    uint4 v[UNROLL];
    unsigned long long word[UNROLL];
    uint32_t pre[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const uint32_t q = first + (uint32_t)u * kBlock;
        word[u] = 0;
        pre[u] = 0;
        v[u] = make_uint4(0, 0, 0, 0);
        if (q < n_chunks) {
            v[u] = grad[q];
            const uint32_t w = (q * E) >> 6;
            word[u] = mask[w];
            pre[u] = prefix[w];
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const uint32_t q = first + (uint32_t)u * kBlock;
        uint32_t sub, slot;
        chunk_meta<T>(q, word[u], pre[u], sub, slot);
        // A mask/prefix pair that disagrees with nnz must not make the kernel write out of bounds.
        if (slot > nnz || (uint32_t)__popc(sub) > nnz - slot) sub = 0;
        T* out = compact + slot;
#pragma unroll
        for (int e = 0; e < (int)E; ++e) {
            if (sub & (1u << e)) {
                *out = elem_of<T>(v[u], e);
                ++out;
            }
        }
    }

    // Elements after the last whole chunk (n not a multiple of the chunk size).
    if (blockIdx.x == gridDim.x - 1) {
        const uint32_t i = n_chunks * E + threadIdx.x;
        if (threadIdx.x < E && i < n) {
            const unsigned long long wd = mask[i >> 6];
            if ((wd >> (i & 63u)) & 1ull) {
                const uint32_t slot = prefix[i >> 6] + popc64(wd & ((1ull << (i & 63u)) - 1ull));
                if (slot < nnz) compact[slot] = reinterpret_cast<const T*>(grad)[i];
            }
        }
    }
}

// Any element alignment: one element per lane, lane b of a wave owns bit b of one mask word.
template <typename T>
__global__ __launch_bounds__(kBlock) void compress_scalar_kernel(const T* __restrict__ grad, uint32_t n,
                                                                 const unsigned long long* __restrict__ mask,
                                                                 const uint32_t* __restrict__ prefix,
                                                                 T* __restrict__ compact, uint32_t nnz) {
    const unsigned long long i = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const unsigned long long wd = mask[i >> 6];
    const uint32_t b = (uint32_t)i & 63u;
    if ((wd >> b) & 1ull) {
        const uint32_t slot = prefix[i >> 6] + popc64(wd & ((1ull << b) - 1ull));
        if (slot < nnz) compact[slot] = grad[i];
    }
}

// ---------------------------------------------------------------------------------- decompress
template <typename T>
__device__ __forceinline__ uint4 gather_chunk(const T* __restrict__ src, uint32_t sub);
template <>
__device__ __forceinline__ uint4 gather_chunk<uint32_t>(const uint32_t* __restrict__ src, uint32_t sub) {
    uint4 o = make_uint4(0, 0, 0, 0);
    if (sub & 1u) { o.x = *src; ++src; }
    if (sub & 2u) { o.y = *src; ++src; }
    if (sub & 4u) { o.z = *src; ++src; }
    if (sub & 8u) { o.w = *src; }
    return o;
}
template <>
__device__ __forceinline__ uint4 gather_chunk<uint16_t>(const uint16_t* __restrict__ src, uint32_t sub) {
    uint32_t d[4] = {0, 0, 0, 0};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (sub & (1u << e)) {
            d[e >> 1] |= (uint32_t)(*src) << ((e & 1) * 16);
            ++src;
        }
    }
    return make_uint4(d[0], d[1], d[2], d[3]);
}

template <typename T, int UNROLL>
__global__ __launch_bounds__(kBlock) void decompress_vec_kernel(const T* __restrict__ compact, uint32_t nnz,
                                                                const unsigned long long* __restrict__ mask,
                                                                const uint32_t* __restrict__ prefix,
                                                                uint4* __restrict__ dense, uint32_t n) {
    constexpr uint32_t E = Chunk<T>::kElems;
    const uint32_t n_chunks = n / E;
    const uint32_t first = blockIdx.x * (uint32_t)(kBlock * UNROLL) + threadIdx.x;

    unsigned long long word[UNROLL];
    uint32_t pre[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const uint32_t q = first + (uint32_t)u * kBlock;
        word[u] = 0;
        pre[u] = 0;
        if (q < n_chunks) {
            const uint32_t w = (q * E) >> 6;
            word[u] = mask[w];
            pre[u] = prefix[w];
        }
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
        const uint32_t q = first + (uint32_t)u * kBlock;
        if (q < n_chunks) {
            uint32_t sub, slot;
            chunk_meta<T>(q, word[u], pre[u], sub, slot);
            if (slot > nnz || (uint32_t)__popc(sub) > nnz - slot) sub = 0;   // never read beyond the compact buffer
            dense[q] = gather_chunk<T>(compact + slot, sub);
        }
    }

    if (blockIdx.x == gridDim.x - 1) {
        const uint32_t i = n_chunks * E + threadIdx.x;
        if (threadIdx.x < E && i < n) {
            const unsigned long long wd = mask[i >> 6];
            T val = 0;
            if ((wd >> (i & 63u)) & 1ull) {
                const uint32_t slot = prefix[i >> 6] + popc64(wd & ((1ull << (i & 63u)) - 1ull));
                if (slot < nnz) val = compact[slot];
            }
            reinterpret_cast<T*>(dense)[i] = val;
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void decompress_scalar_kernel(const T* __restrict__ compact, uint32_t nnz,
                                                                   const unsigned long long* __restrict__ mask,
                                                                   const uint32_t* __restrict__ prefix,
                                                                   T* __restrict__ dense, uint32_t n) {
    const unsigned long long i = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    const unsigned long long wd = mask[i >> 6];
    const uint32_t b = (uint32_t)i & 63u;
    T val = 0;
    if ((wd >> b) & 1ull) {
        const uint32_t slot = prefix[i >> 6] + popc64(wd & ((1ull << b) - 1ull));
        if (slot < nnz) val = compact[slot];
    }
    dense[i] = val;
}

// ---------------------------------------------------------------------------------------- sum
// bf16 <-> fp32 on bit patterns.  Narrowing is round-to-nearest-even; a NaN keeps its sign and
// top payload bits and gets the quiet bit, so it cannot round into infinity.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (u >> 16) | 0x0040u;
    return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

template <int DT>
struct Acc;
template <>
struct Acc<0> {   // fp32 payload: 4 values per chunk
    float a[4];
    __device__ __forceinline__ void set(const uint4& v) {
        a[0] = __uint_as_float(v.x); a[1] = __uint_as_float(v.y);
        a[2] = __uint_as_float(v.z); a[3] = __uint_as_float(v.w);
    }
    __device__ __forceinline__ void add(const uint4& v) {
        a[0] = __fadd_rn(a[0], __uint_as_float(v.x)); a[1] = __fadd_rn(a[1], __uint_as_float(v.y));
        a[2] = __fadd_rn(a[2], __uint_as_float(v.z)); a[3] = __fadd_rn(a[3], __uint_as_float(v.w));
    }
    __device__ __forceinline__ uint4 get() const {
        return make_uint4(__float_as_uint(a[0]), __float_as_uint(a[1]), __float_as_uint(a[2]), __float_as_uint(a[3]));
    }
};
template <>
struct Acc<1> {   // bf16 payload: 8 values per chunk, accumulated in fp32
    float a[8];
    __device__ __forceinline__ void set(const uint4& v) {
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[2 * i] = __uint_as_float(d[i] << 16);
            a[2 * i + 1] = __uint_as_float(d[i] & 0xFFFF0000u);
        }
    }
    __device__ __forceinline__ void add(const uint4& v) {
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[2 * i] = __fadd_rn(a[2 * i], __uint_as_float(d[i] << 16));
            a[2 * i + 1] = __fadd_rn(a[2 * i + 1], __uint_as_float(d[i] & 0xFFFF0000u));
        }
    }
    __device__ __forceinline__ uint4 get() const {
        uint32_t d[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) d[i] = f32_to_bf16_bits(a[2 * i]) | (f32_to_bf16_bits(a[2 * i + 1]) << 16);
        return make_uint4(d[0], d[1], d[2], d[3]);
    }
};

template <int DT>
__device__ __forceinline__ float load_scalar(const void* p, uint32_t j) {
    if (DT == 0) return static_cast<const float*>(p)[j];
    return __uint_as_float((uint32_t)static_cast<const uint16_t*>(p)[j] << 16);
}

template <int DT>
__device__ __forceinline__ void store_scalar(void* p, uint32_t j, float f) {
    if (DT == 0) static_cast<float*>(p)[j] = f;
    else static_cast<uint16_t*>(p)[j] = (uint16_t)f32_to_bf16_bits(f);
}

template <int DT>
__global__ __launch_bounds__(kBlock) void reduce_vec_kernel(WorkerPtrs bufs, uint32_t W, uint32_t nnz, void* out) {
    constexpr uint32_t E = DT == 0 ? 4 : 8;
    const uint32_t n_chunks = nnz / E;
    const uint32_t q = blockIdx.x * (uint32_t)kBlock + threadIdx.x;
    if (q < n_chunks) {
        Acc<DT> acc;
        acc.set(static_cast<const uint4*>(bufs.p[0])[q]);
        uint32_t w = 1;
        for (; w + 4 <= W; w += 4) {   // four loads in flight, adds in worker order
            const uint4 v0 = static_cast<const uint4*>(bufs.p[w])[q];
            const uint4 v1 = static_cast<const uint4*>(bufs.p[w + 1])[q];
            const uint4 v2 = static_cast<const uint4*>(bufs.p[w + 2])[q];
            const uint4 v3 = static_cast<const uint4*>(bufs.p[w + 3])[q];
            acc.add(v0); acc.add(v1); acc.add(v2); acc.add(v3);
        }
        for (; w < W; ++w) acc.add(static_cast<const uint4*>(bufs.p[w])[q]);
        static_cast<uint4*>(out)[q] = acc.get();
    }
    if (blockIdx.x == gridDim.x - 1) {
        const uint32_t j = n_chunks * E + threadIdx.x;
        if (threadIdx.x < E && j < nnz) {
            float a = load_scalar<DT>(bufs.p[0], j);
            for (uint32_t w = 1; w < W; ++w) a = __fadd_rn(a, load_scalar<DT>(bufs.p[w], j));
            store_scalar<DT>(out, j, a);
        }
    }
}

template <int DT>
__global__ __launch_bounds__(kBlock) void reduce_scalar_kernel(WorkerPtrs bufs, uint32_t W, uint32_t nnz, void* out) {
    const unsigned long long j = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    if (j >= nnz) return;
    float a = load_scalar<DT>(bufs.p[0], (uint32_t)j);
    for (uint32_t w = 1; w < W; ++w) a = __fadd_rn(a, load_scalar<DT>(bufs.p[w], (uint32_t)j));
    store_scalar<DT>(out, (uint32_t)j, a);
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline uint32_t div_up(unsigned long long a, unsigned long long b) { return (uint32_t)((a + b - 1) / b); }

}  // namespace

hipError_t launch_compress(const void* d_grad, int dtype, uint32_t n, const unsigned long long* d_mask,
                           const uint32_t* d_prefix, void* d_compact, uint32_t nnz, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    constexpr int U = 4;
    if (aligned16(d_grad)) {
        if (dtype == 0) {
            const uint32_t blocks = div_up((unsigned long long)n / 4 + 1, kBlock * U);
            hipLaunchKernelGGL((compress_vec_kernel<uint32_t, U>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint4*>(d_grad), n, d_mask, d_prefix,
                               static_cast<uint32_t*>(d_compact), nnz);
        } else {
            const uint32_t blocks = div_up((unsigned long long)n / 8 + 1, kBlock * U);
            hipLaunchKernelGGL((compress_vec_kernel<uint16_t, U>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint4*>(d_grad), n, d_mask, d_prefix,
                               static_cast<uint16_t*>(d_compact), nnz);
        }
    } else {
        const uint32_t blocks = div_up(n, kBlock);
        if (dtype == 0)
            hipLaunchKernelGGL((compress_scalar_kernel<uint32_t>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint32_t*>(d_grad), n, d_mask, d_prefix,
                               static_cast<uint32_t*>(d_compact), nnz);
        else
            hipLaunchKernelGGL((compress_scalar_kernel<uint16_t>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint16_t*>(d_grad), n, d_mask, d_prefix,
                               static_cast<uint16_t*>(d_compact), nnz);
    }
    return hipGetLastError();
}

hipError_t launch_decompress(const void* d_compact, int dtype, uint32_t nnz, const unsigned long long* d_mask,
                             const uint32_t* d_prefix, void* d_dense, uint32_t n, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    constexpr int U = 4;
    if (aligned16(d_dense)) {
        if (dtype == 0) {
            const uint32_t blocks = div_up((unsigned long long)n / 4 + 1, kBlock * U);
            hipLaunchKernelGGL((decompress_vec_kernel<uint32_t, U>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint32_t*>(d_compact), nnz, d_mask, d_prefix,
                               static_cast<uint4*>(d_dense), n);
        } else {
            const uint32_t blocks = div_up((unsigned long long)n / 8 + 1, kBlock * U);
            hipLaunchKernelGGL((decompress_vec_kernel<uint16_t, U>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint16_t*>(d_compact), nnz, d_mask, d_prefix,
                               static_cast<uint4*>(d_dense), n);
        }
    } else {
        const uint32_t blocks = div_up(n, kBlock);
        if (dtype == 0)
            hipLaunchKernelGGL((decompress_scalar_kernel<uint32_t>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint32_t*>(d_compact), nnz, d_mask, d_prefix,
                               static_cast<uint32_t*>(d_dense), n);
        else
            hipLaunchKernelGGL((decompress_scalar_kernel<uint16_t>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint16_t*>(d_compact), nnz, d_mask, d_prefix,
                               static_cast<uint16_t*>(d_dense), n);
    }
    return hipGetLastError();
}

hipError_t launch_reduce(const WorkerPtrs& bufs, uint32_t W, int dtype, uint32_t nnz, void* d_out,
                         hipStream_t stream) {
    if (nnz == 0) return hipSuccess;
    bool vec = aligned16(d_out);
    for (uint32_t w = 0; w < W; ++w) vec = vec && aligned16(bufs.p[w]);
    if (vec) {
        const uint32_t E = dtype == 0 ? 4 : 8;
        const uint32_t blocks = div_up((unsigned long long)nnz / E + 1, kBlock);
        if (dtype == 0)
            hipLaunchKernelGGL((reduce_vec_kernel<0>), dim3(blocks), dim3(kBlock), 0, stream, bufs, W, nnz, d_out);
        else
            hipLaunchKernelGGL((reduce_vec_kernel<1>), dim3(blocks), dim3(kBlock), 0, stream, bufs, W, nnz, d_out);
    } else {
        const uint32_t blocks = div_up(nnz, kBlock);
        if (dtype == 0)
            hipLaunchKernelGGL((reduce_scalar_kernel<0>), dim3(blocks), dim3(kBlock), 0, stream, bufs, W, nnz, d_out);
        else
            hipLaunchKernelGGL((reduce_scalar_kernel<1>), dim3(blocks), dim3(kBlock), 0, stream, bufs, W, nnz, d_out);
    }
    return hipGetLastError();
}

}  // namespace pac
