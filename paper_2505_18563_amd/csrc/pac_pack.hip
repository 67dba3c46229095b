// Gather (compress), scatter (decompress) and the W-way sum of compact buffers.
//
// All three are streaming kernels bound by HBM bandwidth.  A lane owns one 16-byte chunk of the
// dense tensor (8 bf16 or 4 fp32 elements); consecutive lanes own consecutive chunks, so dense
// loads and stores are full 128-bit coalesced accesses.  The mask word and its prefix entry of the
// chunk are fetched by every lane that shares them (one cache line per wave).  The compact side of
// a wave is one short contiguous range; it goes through the wave's LDS staging area so that it,
// too, moves in 128-bit accesses instead of one narrow access per surviving element.
#include "pac_internal.h"

namespace pac {
namespace {

constexpr int kBlock = 256;

template <typename T>
struct Chunk {
    static constexpr uint32_t kElems = 16 / sizeof(T);   // elements per 16-byte chunk
};

__device__ __forceinline__ uint32_t popc64(unsigned long long x) { return (uint32_t)__popcll(x); }

// Called by one thread of the workgroup that holds the end of the tensor: the mask's own bit count
// (last prefix entry + bits of the last word) against the nnz the caller passed.
__device__ __forceinline__ void check_total(const unsigned long long* __restrict__ mask,
                                            const uint32_t* __restrict__ prefix, uint32_t words, uint32_t nnz,
                                            uint32_t* __restrict__ status) {
    if (prefix[words - 1] + popc64(mask[words - 1]) != nnz) atomicOr(status, kDevCountMismatch);
}

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

// ------------------------------------------------------------------------- tile geometry
// A tile is a run of chunks that starts on a mask-word boundary, so its first compact slot S0 and
// the slot after its last survivor S1 are two entries of the prefix array (S1 = nnz for the tile that
// holds the end of the tensor): uniform values, read with scalar loads, no cross-lane reduction.
// Survivors are staged in LDS at (slot - S0 + phase), where phase makes LDS 16-byte chunks line up
// with 16-byte chunks of the compact buffer; the compact range is then moved with at most one head,
// one tail (element-wise) and full 16-byte accesses in between.
// Scatter (decompress) uses one wave per tile (kPackU * 64 chunks) and no workgroup barrier;
// gather (compress) uses one workgroup per tile, see below.
constexpr int kPackBlock = 128;
constexpr int kPackWaves = kPackBlock / 64;
constexpr int kPackU = 4;   // measured: 2 -> 4 takes 17 % off the bf16 scatter, 12 % off the fp32 one; 8 is slower again

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <typename T, int U>
struct Tile {
    static constexpr uint32_t E = 16 / sizeof(T);
    static constexpr uint32_t kChunks = 64 * U;
    static constexpr uint32_t kElems = kChunks * E;
    static constexpr uint32_t kWords = kElems / 64;       // = U * E
    static constexpr uint32_t kStage = kElems + 2 * E;    // + phase + tail elements
};

__device__ __forceinline__ void wave_lds_sync() {
    // Orders this wave's LDS writes before its later LDS reads of other lanes' data.
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
}

template <typename T>
__device__ __forceinline__ uint32_t phase_of(const T* p) {
    return (uint32_t)((reinterpret_cast<uintptr_t>(p) / sizeof(T)) & (16 / sizeof(T) - 1));
}

// ------------------------------------------------------------------------------------ compress
// One workgroup (4 waves) per tile of kCompressU * 256 chunks; the tile's survivors form one
// contiguous compact range, staged in LDS and written out cooperatively after one barrier, so that
// only the two ends of a ~0.8 KB range are partial cache lines.
constexpr int kCompressBlock = 256;
// 7 chunks per lane (tiles of 1792 chunks, 28 KB of staging) with the register count held to 64 so
// that the waves per SIMD are bounded by LDS, not registers: measured 5 % faster than 2 chunks per
// lane; 3 and 4 are slower than either, 8 and more slower again.
constexpr int kCompressU = 7;

template <typename T, int U>
struct BlockTile {
    static constexpr uint32_t E = 16 / sizeof(T);
    static constexpr uint32_t kChunks = kCompressBlock * U;
    static constexpr uint32_t kElems = kChunks * E;
    static constexpr uint32_t kWords = kElems / 64;
    static constexpr uint32_t kStage = kElems + 2 * E;    // + phase + tail elements
};

template <typename T, int U>
__global__ __launch_bounds__(kCompressBlock, 8) void compress_tile_kernel(const u32x4* __restrict__ grad, uint32_t n,
                                                                       const unsigned long long* __restrict__ mask,
                                                                       const uint32_t* __restrict__ prefix,
                                                                       T* __restrict__ compact, uint32_t nnz,
                                                                       uint32_t* __restrict__ status) {
    typedef BlockTile<T, U> G;
    constexpr uint32_t E = G::E;
    __shared__ __attribute__((aligned(16))) T stage[G::kStage];

    const uint32_t tile = blockIdx.x;
    const uint32_t n_chunks = n / E;
    const uint32_t words = (uint32_t)(((unsigned long long)n + 63) >> 6);
    const uint32_t chunk0 = tile * G::kChunks;

    u32x4 v[U];
    unsigned long long word[U];
    uint32_t pre[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t q = chunk0 + (uint32_t)u * kCompressBlock + threadIdx.x;
        word[u] = 0;
        pre[u] = 0;
        v[u] = (u32x4){0, 0, 0, 0};
        if (q < n_chunks) {
            v[u] = __builtin_nontemporal_load(grad + q);
            const uint32_t w = (q * E) >> 6;
            word[u] = mask[w];
            pre[u] = prefix[w];
        }
    }

    const uint32_t w0 = tile * G::kWords;   // < words by the launch shape
    const uint32_t w1 = w0 + G::kWords;
    const uint32_t s0 = prefix[w0];
    const uint32_t s1 = w1 < words ? prefix[w1] : nnz;
    if (tile == gridDim.x - 1 && threadIdx.x == 0) check_total(mask, prefix, words, nnz, status);
    // A mask/prefix/nnz triple that does not fit together must not make the kernel write out of
    // bounds: the tile is skipped and the status word says so.  (Same decision in every thread, so
    // the barrier below is safe.)
    if (s0 > s1 || s1 > nnz || s1 - s0 > G::kElems) {
        if (threadIdx.x == 0) atomicOr(status, kDevMetaMismatch);
        return;
    }
    const uint32_t count = s1 - s0;
    const uint32_t ph = phase_of(compact + s0);

#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t q = chunk0 + (uint32_t)u * kCompressBlock + threadIdx.x;
        const uint32_t bitoff = (q * E) & 63u;
        uint32_t sub = (uint32_t)(word[u] >> bitoff) & ((1u << E) - 1u);
        const uint32_t pos = pre[u] + popc64(word[u] & ((1ull << bitoff) - 1ull)) - s0 + ph;
        if (pos > G::kStage - E) sub = 0;
        T* p = stage + pos;
        const uint4 vv = make_uint4(v[u].x, v[u].y, v[u].z, v[u].w);
#pragma unroll
        for (int e = 0; e < (int)E; ++e) {
            if (sub & (1u << e)) {
                *p = elem_of<T>(vv, e);
                ++p;
            }
        }
    }
    // Elements after the last whole chunk (n not a multiple of E) belong to the tile they follow.
    if (tile == n_chunks / G::kChunks) {
        const uint32_t i = n_chunks * E + threadIdx.x;
        if (threadIdx.x < E && i < n) {
            const unsigned long long wd = mask[i >> 6];
            if ((wd >> (i & 63u)) & 1ull) {
                const uint32_t pos = prefix[i >> 6] + popc64(wd & ((1ull << (i & 63u)) - 1ull)) - s0 + ph;
                if (pos < G::kStage) stage[pos] = reinterpret_cast<const T*>(grad)[i];
            }
        }
    }
    __syncthreads();

    // LDS [ph, ph + count) -> compact [s0, s1); (compact + s0 - ph) is 16-byte aligned.
    T* gbase = compact + s0 - ph;
    const uint32_t a = ph, b = ph + count;
    uint32_t h_end = (a + E - 1u) & ~(E - 1u);
    if (h_end > b) h_end = b;
    if (threadIdx.x < h_end - a) gbase[a + threadIdx.x] = stage[a + threadIdx.x];
    // The 16-byte body goes out with nontemporal stores: a workgroup's wave slots stay taken until its
    // last store is acknowledged, and streaming stores come back sooner than write-back ones (measured:
    // 10 % of the kernel's time).  The few 2- or 4-byte head and tail stores are faster as plain stores.
    for (uint32_t c = h_end / E + threadIdx.x; c < b / E; c += kCompressBlock)
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4*>(stage + c * E),
                                    reinterpret_cast<u32x4*>(gbase + c * E));
    uint32_t t0 = b & ~(E - 1u);
    if (t0 < h_end) t0 = h_end;
    if (threadIdx.x < b - t0) gbase[t0 + threadIdx.x] = stage[t0 + threadIdx.x];
}

// Any element alignment: one element per lane, lane b of a wave owns bit b of one mask word.
template <typename T>
__global__ __launch_bounds__(kBlock) void compress_scalar_kernel(const T* __restrict__ grad, uint32_t n,
                                                                 const unsigned long long* __restrict__ mask,
                                                                 const uint32_t* __restrict__ prefix,
                                                                 T* __restrict__ compact, uint32_t nnz,
                                                                 uint32_t* __restrict__ status) {
    const unsigned long long i = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    if (i == n - 1) check_total(mask, prefix, (uint32_t)(((unsigned long long)n + 63) >> 6), nnz, status);
    const unsigned long long wd = mask[i >> 6];
    const uint32_t b = (uint32_t)i & 63u;
    if ((wd >> b) & 1ull) {
        const uint32_t slot = prefix[i >> 6] + popc64(wd & ((1ull << b) - 1ull));
        if (slot < nnz) compact[slot] = grad[i];
        else atomicOr(status, kDevMetaMismatch);
    }
}

// ---------------------------------------------------------------------------------- decompress
template <typename T>
__device__ __forceinline__ u32x4 gather_chunk(const T* p, uint32_t sub);
template <>
__device__ __forceinline__ u32x4 gather_chunk<uint32_t>(const uint32_t* p, uint32_t sub) {
    u32x4 o = (u32x4){0, 0, 0, 0};
    if (sub & 1u) { o.x = *p; ++p; }
    if (sub & 2u) { o.y = *p; ++p; }
    if (sub & 4u) { o.z = *p; ++p; }
    if (sub & 8u) { o.w = *p; }
    return o;
}
template <>
__device__ __forceinline__ u32x4 gather_chunk<uint16_t>(const uint16_t* p, uint32_t sub) {
    uint32_t d[4] = {0, 0, 0, 0};
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        if (sub & (1u << e)) {
            d[e >> 1] |= (uint32_t)(*p) << ((e & 1) * 16);
            ++p;
        }
    }
    return (u32x4){d[0], d[1], d[2], d[3]};
}

template <typename T, int U>
__global__ __launch_bounds__(kPackBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) void decompress_tile_kernel(const T* __restrict__ compact, uint32_t nnz,
                                                                     const unsigned long long* __restrict__ mask,
                                                                     const uint32_t* __restrict__ prefix,
                                                                     u32x4* __restrict__ dense, uint32_t n,
                                                                     uint32_t* __restrict__ status) {
    typedef Tile<T, U> G;
    constexpr uint32_t E = G::E;
    __shared__ __attribute__((aligned(16))) T stage[kPackWaves][G::kStage];

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t tile = blockIdx.x * kPackWaves + wave;
    if ((unsigned long long)tile * G::kElems >= n) return;
    const uint32_t n_chunks = n / E;
    const uint32_t words = (uint32_t)(((unsigned long long)n + 63) >> 6);
    const uint32_t chunk0 = tile * G::kChunks;

    unsigned long long word[U];
    uint32_t pre[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t q = chunk0 + (uint32_t)u * 64 + lane;
        word[u] = 0;
        pre[u] = 0;
        if (q < n_chunks) {
            const uint32_t w = (q * E) >> 6;
            word[u] = mask[w];
            pre[u] = prefix[w];
        }
    }

    const uint32_t w0 = tile * G::kWords;
    const uint32_t w1 = w0 + G::kWords;
    // both bounds in one round trip: the second index is clamped, not branched on
    const uint32_t s0 = prefix[w0];
    const uint32_t s1_read = prefix[w1 < words ? w1 : words - 1u];
    const uint32_t s1 = w1 < words ? s1_read : nnz;
    // Inconsistent metadata: read nothing, the tile's outputs become zero, the status word says so.
    const bool sane = s0 <= s1 && s1 <= nnz && s1 - s0 <= G::kElems;
    if (lane == 0) {
        if (!sane) atomicOr(status, kDevMetaMismatch);
        if (w1 >= words) check_total(mask, prefix, words, nnz, status);   // the tile that holds the end
    }
    const uint32_t count = sane ? s1 - s0 : 0u;
    const uint32_t ph = phase_of(compact + s0);
    T* my = stage[wave];

    // compact [s0, s1) -> LDS [ph, ph + count): an element-wise head and tail, 16-byte chunks between them.
    // All loads are issued before the first is used: a loop of load-then-store trips would cost one memory
    // round trip per trip (up to NB of them for a dense tile).
    if (count != 0) {
        constexpr int NB = U + 1;
        const T* gbase = compact + s0 - ph;
        const uint32_t a = ph, b = ph + count;
        uint32_t h_end = (a + E - 1u) & ~(E - 1u);
        if (h_end > b) h_end = b;
        uint32_t t0 = b & ~(E - 1u);
        if (t0 < h_end) t0 = h_end;
        const uint32_t c_begin = h_end / E, c_end = b / E;
        u32x4 r[NB];
        T head = 0, tail = 0;
        if (lane < h_end - a) head = gbase[a + lane];
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const uint32_t c = c_begin + lane + 64u * (uint32_t)i;
            r[i] = (u32x4){0, 0, 0, 0};
            if (c < c_end) r[i] = *reinterpret_cast<const u32x4*>(gbase + c * E);
        }
        if (lane < b - t0) tail = gbase[t0 + lane];
        if (lane < h_end - a) my[a + lane] = head;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const uint32_t c = c_begin + lane + 64u * (uint32_t)i;
            if (c < c_end) *reinterpret_cast<u32x4*>(my + c * E) = r[i];
        }
        if (lane < b - t0) my[t0 + lane] = tail;
    }
    wave_lds_sync();

#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t q = chunk0 + (uint32_t)u * 64 + lane;
        if (q < n_chunks) {
            const uint32_t bitoff = (q * E) & 63u;
            uint32_t sub = (uint32_t)(word[u] >> bitoff) & ((1u << E) - 1u);
            const uint32_t pos = pre[u] + popc64(word[u] & ((1ull << bitoff) - 1ull)) - s0 + ph;
            if (!sane || pos > ph + count || (uint32_t)__popc(sub) > ph + count - pos) sub = 0;
            __builtin_nontemporal_store(gather_chunk<T>(my + pos, sub), dense + q);
        }
    }
    if (tile == n_chunks / G::kChunks) {
        const uint32_t i = n_chunks * E + lane;
        if (lane < E && i < n) {
            const unsigned long long wd = mask[i >> 6];
            T val = 0;
            if ((wd >> (i & 63u)) & 1ull) {
                const uint32_t pos = prefix[i >> 6] + popc64(wd & ((1ull << (i & 63u)) - 1ull)) - s0 + ph;
                if (sane && pos < ph + count) val = my[pos];
            }
            reinterpret_cast<T*>(dense)[i] = val;
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void decompress_scalar_kernel(const T* __restrict__ compact, uint32_t nnz,
                                                                   const unsigned long long* __restrict__ mask,
                                                                   const uint32_t* __restrict__ prefix,
                                                                   T* __restrict__ dense, uint32_t n,
                                                                   uint32_t* __restrict__ status) {
    const unsigned long long i = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    if (i == n - 1) check_total(mask, prefix, (uint32_t)(((unsigned long long)n + 63) >> 6), nnz, status);
    const unsigned long long wd = mask[i >> 6];
    const uint32_t b = (uint32_t)i & 63u;
    T val = 0;
    if ((wd >> b) & 1ull) {
        const uint32_t slot = prefix[i >> 6] + popc64(wd & ((1ull << b) - 1ull));
        if (slot < nnz) val = compact[slot];
        else atomicOr(status, kDevMetaMismatch);
    }
    dense[i] = val;
}

// --------------------------------------------------------------- decompress + weight update
// Eq. 1 on the sparse model, fused into the scatter: the dense gradient is never written.  Same
// tile scheme as decompress with fp32 weight chunks (4 weights per lane and step): the tile's
// compact range goes through the wave's LDS staging area, every lane reads its chunk of weights,
// subtracts alpha * g where the mask bit is set (a multiply and a subtract, each rounded on its own)
// and stores +0 where it is not.
template <typename T>
__device__ __forceinline__ float widen(T v);
template <>
__device__ __forceinline__ float widen<uint32_t>(uint32_t v) { return __uint_as_float(v); }
template <>
__device__ __forceinline__ float widen<uint16_t>(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }

template <typename T, int U>
struct UpdateTile {
    static constexpr uint32_t E = 4;                      // weights per 16-byte chunk
    static constexpr uint32_t EC = 16 / sizeof(T);        // compact elements per 16 bytes
    static constexpr uint32_t kChunks = 64 * U;
    static constexpr uint32_t kElems = kChunks * E;
    static constexpr uint32_t kWords = kElems / 64;
    static constexpr uint32_t kStage = kElems + 2 * EC;
};

template <typename T, int U>
__global__ __launch_bounds__(kPackBlock) __attribute__((amdgpu_waves_per_eu(8, 8))) void update_tile_kernel(const T* __restrict__ compact, uint32_t nnz,
                                                                 const unsigned long long* __restrict__ mask,
                                                                 const uint32_t* __restrict__ prefix, float alpha,
                                                                 u32x4* __restrict__ weights, uint32_t n,
                                                                 uint32_t* __restrict__ status) {
    typedef UpdateTile<T, U> G;
    constexpr uint32_t E = G::E, EC = G::EC;
    __shared__ __attribute__((aligned(16))) T stage[kPackWaves][G::kStage];

    const uint32_t lane = threadIdx.x & 63u;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const uint32_t tile = blockIdx.x * kPackWaves + wave;
    if ((unsigned long long)tile * G::kElems >= n) return;
    const uint32_t n_chunks = n / E;
    const uint32_t words = (uint32_t)(((unsigned long long)n + 63) >> 6);
    const uint32_t chunk0 = tile * G::kChunks;

    u32x4 x[U];
    unsigned long long word[U];
    uint32_t pre[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t q = chunk0 + (uint32_t)u * 64 + lane;
        word[u] = 0;
        pre[u] = 0;
        x[u] = (u32x4){0, 0, 0, 0};
        if (q < n_chunks) {
            x[u] = __builtin_nontemporal_load(weights + q);
            const uint32_t w = (q * E) >> 6;
            word[u] = mask[w];
            pre[u] = prefix[w];
        }
    }

    const uint32_t w0 = tile * G::kWords;
    const uint32_t w1 = w0 + G::kWords;
    // both bounds in one round trip: the second index is clamped, not branched on
    const uint32_t s0 = prefix[w0];
    const uint32_t s1_read = prefix[w1 < words ? w1 : words - 1u];
    const uint32_t s1 = w1 < words ? s1_read : nnz;
    // Inconsistent metadata: read no compact value, kept weights of the tile stay as they are.
    const bool sane = s0 <= s1 && s1 <= nnz && s1 - s0 <= G::kElems;
    if (lane == 0) {
        if (!sane) atomicOr(status, kDevMetaMismatch);
        if (w1 >= words) check_total(mask, prefix, words, nnz, status);   // the tile that holds the end
    }
    const uint32_t count = sane ? s1 - s0 : 0u;
    const uint32_t ph = phase_of(compact + s0);
    T* my = stage[wave];

    // compact [s0, s1) -> LDS [ph, ph + count): an element-wise head and tail, 16-byte chunks between them.
    // All loads are issued before the first is used: a loop of load-then-store trips would cost one memory
    // round trip per trip (up to NB of them for a dense tile).
    if (count != 0) {
        constexpr int NB = (int)(G::kElems / EC / 64) + 1;
        const T* gbase = compact + s0 - ph;
        const uint32_t a = ph, b = ph + count;
        uint32_t h_end = (a + EC - 1u) & ~(EC - 1u);
        if (h_end > b) h_end = b;
        uint32_t t0 = b & ~(EC - 1u);
        if (t0 < h_end) t0 = h_end;
        const uint32_t c_begin = h_end / EC, c_end = b / EC;
        u32x4 r[NB];
        T head = 0, tail = 0;
        if (lane < h_end - a) head = gbase[a + lane];
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const uint32_t c = c_begin + lane + 64u * (uint32_t)i;
            r[i] = (u32x4){0, 0, 0, 0};
            if (c < c_end) r[i] = *reinterpret_cast<const u32x4*>(gbase + c * EC);
        }
        if (lane < b - t0) tail = gbase[t0 + lane];
        if (lane < h_end - a) my[a + lane] = head;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const uint32_t c = c_begin + lane + 64u * (uint32_t)i;
            if (c < c_end) *reinterpret_cast<u32x4*>(my + c * EC) = r[i];
        }
        if (lane < b - t0) my[t0 + lane] = tail;
    }
    wave_lds_sync();

    auto updated = [&](uint32_t xbits, bool kept, const T* p) -> uint32_t {
        if (!kept) return 0u;
        const float g = p ? widen<T>(*p) : 0.0f;
        return __float_as_uint(__fsub_rn(__uint_as_float(xbits), __fmul_rn(alpha, g)));
    };
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint32_t q = chunk0 + (uint32_t)u * 64 + lane;
        if (q < n_chunks) {
            const uint32_t bitoff = (q * E) & 63u;
            const uint32_t sub = (uint32_t)(word[u] >> bitoff) & 0xFu;
            const uint32_t pos = pre[u] + popc64(word[u] & ((1ull << bitoff) - 1ull)) - s0 + ph;
            // compact values this chunk may read: LDS [pos, pos + popc(sub)) inside [ph, ph + count)
            const bool readable = sane && pos <= ph + count && (uint32_t)__popc(sub) <= ph + count - pos;
            const T* p = my + pos;
            u32x4 o;
            o.x = updated(x[u].x, sub & 1u, readable ? p : nullptr); p += (sub & 1u);
            o.y = updated(x[u].y, sub & 2u, readable ? p : nullptr); p += (sub >> 1) & 1u;
            o.z = updated(x[u].z, sub & 4u, readable ? p : nullptr); p += (sub >> 2) & 1u;
            o.w = updated(x[u].w, sub & 8u, readable ? p : nullptr);
            __builtin_nontemporal_store(o, weights + q);
        }
    }
    if (tile == n_chunks / G::kChunks) {   // the elements after the last whole chunk
        const uint32_t i = n_chunks * E + lane;
        if (lane < E && i < n) {
            float* wts = reinterpret_cast<float*>(weights);
            const unsigned long long wd = mask[i >> 6];
            float val = 0.0f;
            if ((wd >> (i & 63u)) & 1ull) {
                const uint32_t pos = prefix[i >> 6] + popc64(wd & ((1ull << (i & 63u)) - 1ull)) - s0 + ph;
                const float g = (sane && pos < ph + count) ? widen<T>(my[pos]) : 0.0f;
                val = __fsub_rn(wts[i], __fmul_rn(alpha, g));
            }
            wts[i] = val;
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void update_scalar_kernel(const T* __restrict__ compact, uint32_t nnz,
                                                               const unsigned long long* __restrict__ mask,
                                                               const uint32_t* __restrict__ prefix, float alpha,
                                                               float* __restrict__ weights, uint32_t n,
                                                               uint32_t* __restrict__ status) {
    const unsigned long long i = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    if (i == n - 1) check_total(mask, prefix, (uint32_t)(((unsigned long long)n + 63) >> 6), nnz, status);
    const unsigned long long wd = mask[i >> 6];
    const uint32_t b = (uint32_t)i & 63u;
    float val = 0.0f;
    if ((wd >> b) & 1ull) {
        const uint32_t slot = prefix[i >> 6] + popc64(wd & ((1ull << b) - 1ull));
        if (slot >= nnz) atomicOr(status, kDevMetaMismatch);
        const float g = slot < nnz ? widen<T>(compact[slot]) : 0.0f;
        val = __fsub_rn(weights[i], __fmul_rn(alpha, g));
    }
    weights[i] = val;
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

__device__ __forceinline__ uint4 load_stream(const void* base, uint32_t q) {
    const u32x4 v = __builtin_nontemporal_load(static_cast<const u32x4*>(base) + q);   // read once, never reused
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <int DT>
__global__ __launch_bounds__(kBlock) void reduce_vec_kernel(WorkerPtrs bufs, uint32_t W, uint32_t nnz, void* out) {
    constexpr uint32_t E = DT == 0 ? 4 : 8;
    const uint32_t n_chunks = nnz / E;
    const uint32_t q = blockIdx.x * (uint32_t)kBlock + threadIdx.x;
    if (q < n_chunks) {
        Acc<DT> acc;
        acc.set(load_stream(bufs.p[0], q));
        uint32_t w = 1;
        for (; w + 4 <= W; w += 4) {   // four loads in flight, adds in worker order
            const uint4 v0 = load_stream(bufs.p[w], q);
            const uint4 v1 = load_stream(bufs.p[w + 1], q);
            const uint4 v2 = load_stream(bufs.p[w + 2], q);
            const uint4 v3 = load_stream(bufs.p[w + 3], q);
            acc.add(v0); acc.add(v1); acc.add(v2); acc.add(v3);
        }
        for (; w < W; ++w) acc.add(load_stream(bufs.p[w], q));
        const uint4 r = acc.get();
        static_cast<uint4*>(out)[q] = r;   // plain store: pac_decompress reads the sum next, from cache
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

// ------------------------------------------------------------------------- fused gather + sum
// compress for each of the W workers followed by the sum, without the W compact buffers in between:
// a lane keeps the running sums of its chunks' elements in registers - every element, kept or not; the
// adds are cheap next to the loads - walks the workers in order (worker 0's value first, then one IEEE
// single add per further worker: the order and the arithmetic of reduce_vec_kernel), and only the final
// sums of the kept elements go through the LDS staging area into the reduced buffer, as in
// compress_tile_kernel.  Mask words and prefix entries are read once per tile instead of once per worker.
// A lane takes U chunks and has the loads of G workers in flight together: bf16 2 chunks x 4 workers (tiles
// of 4096 elements), fp32 1 chunk x up to 16 workers (tiles of 1024 elements).
template <typename T>
struct FusedShape;
template <>
struct FusedShape<uint16_t> { static constexpr int U = 2, G = 4; };   // measured: 6.3 TB/s on 16 bf16 streams; 4 x 4 and 2 x 8 the same, 1 x 8 slower
template <>
struct FusedShape<uint32_t> { static constexpr int U = 1, G = 16; };  // measured on 8 fp32 streams: 1 x 16 5.8-6.2 TB/s; 1 x 8 2 % less; 4 x 4 and 2 x 4 up to 10 % less

template <typename T>
struct FusedAcc;
template <>
struct FusedAcc<uint32_t> {
    float a[4];
    __device__ __forceinline__ void set(const u32x4& v) {
        a[0] = __uint_as_float(v.x); a[1] = __uint_as_float(v.y); a[2] = __uint_as_float(v.z); a[3] = __uint_as_float(v.w);
    }
    __device__ __forceinline__ void add(const u32x4& v) {
        a[0] = __fadd_rn(a[0], __uint_as_float(v.x)); a[1] = __fadd_rn(a[1], __uint_as_float(v.y));
        a[2] = __fadd_rn(a[2], __uint_as_float(v.z)); a[3] = __fadd_rn(a[3], __uint_as_float(v.w));
    }
    __device__ __forceinline__ uint32_t get(int e) const { return __float_as_uint(a[e]); }
};
template <>
struct FusedAcc<uint16_t> {
    float a[8];
    __device__ __forceinline__ void set(const u32x4& v) {
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[2 * i] = __uint_as_float(d[i] << 16);
            a[2 * i + 1] = __uint_as_float(d[i] & 0xFFFF0000u);
        }
    }
    __device__ __forceinline__ void add(const u32x4& v) {
        const uint32_t d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[2 * i] = __fadd_rn(a[2 * i], __uint_as_float(d[i] << 16));
            a[2 * i + 1] = __fadd_rn(a[2 * i + 1], __uint_as_float(d[i] & 0xFFFF0000u));
        }
    }
    __device__ __forceinline__ uint16_t get(int e) const { return (uint16_t)f32_to_bf16_bits(a[e]); }
};

template <typename T>
__global__ __launch_bounds__(kCompressBlock) void fused_tile_kernel(WorkerPtrs grads, uint32_t W, uint32_t n,
                                                                    const unsigned long long* __restrict__ mask,
                                                                    const uint32_t* __restrict__ prefix,
                                                                    T* __restrict__ out, uint32_t nnz,
                                                                    uint32_t* __restrict__ status) {
    constexpr int U = FusedShape<T>::U, G = FusedShape<T>::G;
    typedef BlockTile<T, U> Geo;
    constexpr uint32_t E = Geo::E;
    constexpr int DT = sizeof(T) == 4 ? 0 : 1;
    __shared__ __attribute__((aligned(16))) T stage[Geo::kStage];

    const uint32_t tile = blockIdx.x;
    const uint32_t n_chunks = n / E;
    const uint32_t words = (uint32_t)(((unsigned long long)n + 63) >> 6);
    const uint32_t chunk0 = tile * Geo::kChunks;
    uint32_t q[U];
    bool live[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        q[u] = chunk0 + (uint32_t)u * kCompressBlock + threadIdx.x;
        live[u] = q[u] < n_chunks;
    }

    // the sums, workers in order, G workers' loads in flight
    FusedAcc<T> acc[U];
    {
        const u32x4* g0 = static_cast<const u32x4*>(grads.p[0]);
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u].set(live[u] ? __builtin_nontemporal_load(g0 + q[u]) : (u32x4){0, 0, 0, 0});
    }
    uint32_t w = 1;
    for (; w + G <= W; w += G) {
        u32x4 v[G][U];
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const u32x4* gp = static_cast<const u32x4*>(grads.p[w + g]);
#pragma unroll
            for (int u = 0; u < U; ++u) v[g][u] = live[u] ? __builtin_nontemporal_load(gp + q[u]) : (u32x4){0, 0, 0, 0};
        }
#pragma unroll
        for (int g = 0; g < G; ++g)
#pragma unroll
            for (int u = 0; u < U; ++u) acc[u].add(v[g][u]);
    }
    for (; w < W; ++w) {
        const u32x4* gp = static_cast<const u32x4*>(grads.p[w]);
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = live[u] ? __builtin_nontemporal_load(gp + q[u]) : (u32x4){0, 0, 0, 0};
#pragma unroll
        for (int u = 0; u < U; ++u) acc[u].add(v[u]);
    }

    // the kept sums into the tile's compact range, as in compress_tile_kernel
    const uint32_t w0 = tile * Geo::kWords;   // < words by the launch shape
    const uint32_t w1 = w0 + Geo::kWords;
    const uint32_t s0 = prefix[w0];
    const uint32_t s1 = w1 < words ? prefix[w1] : nnz;
    if (tile == gridDim.x - 1 && threadIdx.x == 0) check_total(mask, prefix, words, nnz, status);
    if (s0 > s1 || s1 > nnz || s1 - s0 > Geo::kElems) {   // same decision in every thread
        if (threadIdx.x == 0) atomicOr(status, kDevMetaMismatch);
        return;
    }
    const uint32_t count = s1 - s0;
    const uint32_t ph = phase_of(out + s0);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if (live[u]) {
            const uint32_t wd = (q[u] * E) >> 6;
            const unsigned long long word = mask[wd];
            const uint32_t bitoff = (q[u] * E) & 63u;
            uint32_t sub = (uint32_t)(word >> bitoff) & ((1u << E) - 1u);
            const uint32_t pos = prefix[wd] + popc64(word & ((1ull << bitoff) - 1ull)) - s0 + ph;
            if (pos > Geo::kStage - E) sub = 0;
            T* p = stage + pos;
#pragma unroll
            for (int e = 0; e < (int)E; ++e) {
                if (sub & (1u << e)) {
                    *p = acc[u].get(e);
                    ++p;
                }
            }
        }
    }
    // Elements after the last whole chunk (n not a multiple of E) belong to the tile they follow.
    if (tile == n_chunks / Geo::kChunks) {
        const uint32_t i = n_chunks * E + threadIdx.x;
        if (threadIdx.x < E && i < n) {
            const unsigned long long wd = mask[i >> 6];
            if ((wd >> (i & 63u)) & 1ull) {
                float a = load_scalar<DT>(grads.p[0], i);
                for (uint32_t ww = 1; ww < W; ++ww) a = __fadd_rn(a, load_scalar<DT>(grads.p[ww], i));
                const uint32_t pos = prefix[i >> 6] + popc64(wd & ((1ull << (i & 63u)) - 1ull)) - s0 + ph;
                if (pos < Geo::kStage) stage[pos] = DT == 0 ? (T)__float_as_uint(a) : (T)f32_to_bf16_bits(a);
            }
        }
    }
    __syncthreads();

    // LDS [ph, ph + count) -> out [s0, s1); (out + s0 - ph) is 16-byte aligned.
    T* gbase = out + s0 - ph;
    const uint32_t a = ph, b = ph + count;
    uint32_t h_end = (a + E - 1u) & ~(E - 1u);
    if (h_end > b) h_end = b;
    if (threadIdx.x < h_end - a) gbase[a + threadIdx.x] = stage[a + threadIdx.x];
    for (uint32_t c = h_end / E + threadIdx.x; c < b / E; c += kCompressBlock)
        *reinterpret_cast<u32x4*>(gbase + c * E) = *reinterpret_cast<const u32x4*>(stage + c * E);   // read next by pac_decompress
    uint32_t t0 = b & ~(E - 1u);
    if (t0 < h_end) t0 = h_end;
    if (threadIdx.x < b - t0) gbase[t0 + threadIdx.x] = stage[t0 + threadIdx.x];
}

// Any element alignment: one element per lane.
template <int DT, typename T>
__global__ __launch_bounds__(kBlock) void fused_scalar_kernel(WorkerPtrs grads, uint32_t W, uint32_t n,
                                                              const unsigned long long* __restrict__ mask,
                                                              const uint32_t* __restrict__ prefix, T* __restrict__ out,
                                                              uint32_t nnz, uint32_t* __restrict__ status) {
    const unsigned long long i = (unsigned long long)blockIdx.x * kBlock + threadIdx.x;
    if (i >= n) return;
    if (i == n - 1) check_total(mask, prefix, (uint32_t)(((unsigned long long)n + 63) >> 6), nnz, status);
    const unsigned long long wd = mask[i >> 6];
    const uint32_t b = (uint32_t)i & 63u;
    if ((wd >> b) & 1ull) {
        const uint32_t slot = prefix[i >> 6] + popc64(wd & ((1ull << b) - 1ull));
        if (slot < nnz) {
            float a = load_scalar<DT>(grads.p[0], (uint32_t)i);
            for (uint32_t w = 1; w < W; ++w) a = __fadd_rn(a, load_scalar<DT>(grads.p[w], (uint32_t)i));
            store_scalar<DT>(out, slot, a);
        } else {
            atomicOr(status, kDevMetaMismatch);
        }
    }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline uint32_t div_up(unsigned long long a, unsigned long long b) { return (uint32_t)((a + b - 1) / b); }

}  // namespace

hipError_t launch_compress(const void* d_grad, int dtype, uint32_t n, const unsigned long long* d_mask,
                           const uint32_t* d_prefix, void* d_compact, uint32_t nnz, uint32_t* d_status,
                           hipStream_t stream) {
    if (n == 0) return hipSuccess;
    if (aligned16(d_grad)) {
        if (dtype == 0) {
            const uint32_t tiles = div_up(n, BlockTile<uint32_t, kCompressU>::kElems);
            hipLaunchKernelGGL((compress_tile_kernel<uint32_t, kCompressU>), dim3(tiles), dim3(kCompressBlock), 0,
                               stream, static_cast<const u32x4*>(d_grad), n, d_mask, d_prefix,
                               static_cast<uint32_t*>(d_compact), nnz, d_status);
        } else {
            const uint32_t tiles = div_up(n, BlockTile<uint16_t, kCompressU>::kElems);
            hipLaunchKernelGGL((compress_tile_kernel<uint16_t, kCompressU>), dim3(tiles), dim3(kCompressBlock), 0,
                               stream, static_cast<const u32x4*>(d_grad), n, d_mask, d_prefix,
                               static_cast<uint16_t*>(d_compact), nnz, d_status);
        }
    } else {
        const uint32_t blocks = div_up(n, kBlock);
        if (dtype == 0)
            hipLaunchKernelGGL((compress_scalar_kernel<uint32_t>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint32_t*>(d_grad), n, d_mask, d_prefix,
                               static_cast<uint32_t*>(d_compact), nnz, d_status);
        else
            hipLaunchKernelGGL((compress_scalar_kernel<uint16_t>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint16_t*>(d_grad), n, d_mask, d_prefix,
                               static_cast<uint16_t*>(d_compact), nnz, d_status);
    }
    return hipGetLastError();
}

hipError_t launch_decompress(const void* d_compact, int dtype, uint32_t nnz, const unsigned long long* d_mask,
                             const uint32_t* d_prefix, void* d_dense, uint32_t n, uint32_t* d_status,
                             hipStream_t stream) {
    if (n == 0) return hipSuccess;
    if (aligned16(d_dense)) {
        if (dtype == 0) {
            const uint32_t tiles = div_up(n, Tile<uint32_t, kPackU>::kElems);
            hipLaunchKernelGGL((decompress_tile_kernel<uint32_t, kPackU>), dim3(div_up(tiles, kPackWaves)),
                               dim3(kPackBlock), 0, stream, static_cast<const uint32_t*>(d_compact), nnz, d_mask,
                               d_prefix, static_cast<u32x4*>(d_dense), n, d_status);
        } else {
            const uint32_t tiles = div_up(n, Tile<uint16_t, kPackU>::kElems);
            hipLaunchKernelGGL((decompress_tile_kernel<uint16_t, kPackU>), dim3(div_up(tiles, kPackWaves)),
                               dim3(kPackBlock), 0, stream, static_cast<const uint16_t*>(d_compact), nnz, d_mask,
                               d_prefix, static_cast<u32x4*>(d_dense), n, d_status);
        }
    } else {
        const uint32_t blocks = div_up(n, kBlock);
        if (dtype == 0)
            hipLaunchKernelGGL((decompress_scalar_kernel<uint32_t>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint32_t*>(d_compact), nnz, d_mask, d_prefix,
                               static_cast<uint32_t*>(d_dense), n, d_status);
        else
            hipLaunchKernelGGL((decompress_scalar_kernel<uint16_t>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint16_t*>(d_compact), nnz, d_mask, d_prefix,
                               static_cast<uint16_t*>(d_dense), n, d_status);
    }
    return hipGetLastError();
}

hipError_t launch_decompress_update(const void* d_compact, int dtype, uint32_t nnz, const unsigned long long* d_mask,
                                    const uint32_t* d_prefix, float alpha, float* d_weights, uint32_t n,
                                    uint32_t* d_status, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    if (aligned16(d_weights)) {
        const uint32_t tiles = div_up(n, UpdateTile<uint32_t, kPackU>::kElems);   // same for both payload types
        if (dtype == 0)
            hipLaunchKernelGGL((update_tile_kernel<uint32_t, kPackU>), dim3(div_up(tiles, kPackWaves)), dim3(kPackBlock),
                               0, stream, static_cast<const uint32_t*>(d_compact), nnz, d_mask, d_prefix, alpha,
                               reinterpret_cast<u32x4*>(d_weights), n, d_status);
        else
            hipLaunchKernelGGL((update_tile_kernel<uint16_t, kPackU>), dim3(div_up(tiles, kPackWaves)), dim3(kPackBlock),
                               0, stream, static_cast<const uint16_t*>(d_compact), nnz, d_mask, d_prefix, alpha,
                               reinterpret_cast<u32x4*>(d_weights), n, d_status);
    } else {
        const uint32_t blocks = div_up(n, kBlock);
        if (dtype == 0)
            hipLaunchKernelGGL((update_scalar_kernel<uint32_t>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint32_t*>(d_compact), nnz, d_mask, d_prefix, alpha, d_weights, n, d_status);
        else
            hipLaunchKernelGGL((update_scalar_kernel<uint16_t>), dim3(blocks), dim3(kBlock), 0, stream,
                               static_cast<const uint16_t*>(d_compact), nnz, d_mask, d_prefix, alpha, d_weights, n, d_status);
    }
    return hipGetLastError();
}

hipError_t launch_step_fused(const WorkerPtrs& grads, uint32_t W, int dtype, uint32_t n,
                             const unsigned long long* d_mask, const uint32_t* d_prefix, void* d_reduced, uint32_t nnz,
                             uint32_t* d_status, hipStream_t stream) {
    if (n == 0) return hipSuccess;
    bool vec = true;
    for (uint32_t w = 0; w < W; ++w) vec = vec && aligned16(grads.p[w]);
    if (vec) {
        if (dtype == 0) {
            const uint32_t tiles = div_up(n, BlockTile<uint32_t, FusedShape<uint32_t>::U>::kElems);
            hipLaunchKernelGGL((fused_tile_kernel<uint32_t>), dim3(tiles), dim3(kCompressBlock), 0, stream, grads, W, n,
                               d_mask, d_prefix, static_cast<uint32_t*>(d_reduced), nnz, d_status);
        } else {
            const uint32_t tiles = div_up(n, BlockTile<uint16_t, FusedShape<uint16_t>::U>::kElems);
            hipLaunchKernelGGL((fused_tile_kernel<uint16_t>), dim3(tiles), dim3(kCompressBlock), 0, stream, grads, W, n,
                               d_mask, d_prefix, static_cast<uint16_t*>(d_reduced), nnz, d_status);
        }
    } else {
        const uint32_t blocks = div_up(n, kBlock);
        if (dtype == 0)
            hipLaunchKernelGGL((fused_scalar_kernel<0, uint32_t>), dim3(blocks), dim3(kBlock), 0, stream, grads, W, n,
                               d_mask, d_prefix, static_cast<uint32_t*>(d_reduced), nnz, d_status);
        else
            hipLaunchKernelGGL((fused_scalar_kernel<1, uint16_t>), dim3(blocks), dim3(kBlock), 0, stream, grads, W, n,
                               d_mask, d_prefix, static_cast<uint16_t*>(d_reduced), nnz, d_status);
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
