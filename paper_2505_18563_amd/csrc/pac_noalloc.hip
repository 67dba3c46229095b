// pac_mask_from_nonzero_noalloc: pac_mask_from_nonzero for callers that cannot allocate (code under
// HIP graph capture, tight serving loops, harnesses that forbid hipMalloc).  It needs no context: the
// scratch of its prefix scan (tile states, the ticket counter, a status word) lives in a file-scope
// device array of this library instead of in memory a pac_create call allocated.
//
// Every GPU the library runs on holds its own copy of the array, at its own address, until the process
// ends.  Host code never uses the array's name as an address: the address is looked up once per device
// with hipGetSymbolAddress, with that device current, and kept.
#include "../../include/pactrain.h"

#include <mutex>

#include "pac_internal.h"

namespace {

// Layout of the array (bytes): [0, 16640) scan tile states, kScanMaxTiles + 1 words of 8 bytes, rounded
// up; [16640, 16672) the scan's counters; [16896, 16900) the status word.  The largest mask the scan
// takes (n = 2^32 - 1 elements) uses kScanMaxTiles tiles, so the array bounds n by nothing less.
constexpr size_t kTileStateOffset = 0;
constexpr size_t kGlobalsOffset = 16640;
constexpr size_t kStatusOffset = 16896;
constexpr size_t kScratchBytes = 32768;
static_assert((pac::kScanMaxTiles + 1) * sizeof(unsigned long long) <= kGlobalsOffset, "tile states fit");
static_assert(kGlobalsOffset + sizeof(pac::Globals) <= kStatusOffset && kStatusOffset + 4 <= kScratchBytes, "layout");

static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_lookup_mutex;
unsigned char* g_scratch_ptr[kMaxDevices];   // address of `scratch` on each device, once looked up

// The array's address on the current device `dev`; null with *err set if the lookup fails.
unsigned char* scratch_on_device(int dev, hipError_t* err) {
    std::lock_guard<std::mutex> lock(g_lookup_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        const hipError_t r = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (r != hipSuccess || p == nullptr) {
            *err = r != hipSuccess ? r : hipErrorInvalidSymbol;
            return nullptr;
        }
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    return g_scratch_ptr[dev];
}

bool aligned_to(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

}  // namespace

extern "C" pac_status pac_mask_from_nonzero_noalloc(const void* d_values, pac_dtype dtype, uint64_t n, uint64_t* d_mask,
                                                    uint32_t* d_prefix, uint64_t* d_nnz_out, uint32_t* d_flags_out,
                                                    void* hip_stream) {
    const char* who = "pac_mask_from_nonzero_noalloc";
    if (dtype != PAC_F32 && dtype != PAC_BF16) return pac::thread_fail(PAC_ERR_ARG, "%s: unknown dtype %d", who, (int)dtype);
    if (n >= (1ull << 32))
        return pac::thread_fail(PAC_ERR_RANGE, "%s: n=%llu exceeds the maximum of 2^32 - 1 elements", who, (unsigned long long)n);
    if (n > 0 && (!d_values || !d_mask || !d_prefix)) return pac::thread_fail(PAC_ERR_ARG, "%s: NULL device pointer", who);
    if (!aligned_to(d_values, dtype == PAC_F32 ? 4 : 2) || !aligned_to(d_mask, 8) || !aligned_to(d_prefix, 4) ||
        !aligned_to(d_nnz_out, 8) || !aligned_to(d_flags_out, 4))
        return pac::thread_fail(PAC_ERR_ALIGN, "%s: pointer not aligned to its element size", who);

    int dev = -1;
    hipError_t r = hipGetDevice(&dev);
    if (r != hipSuccess) return pac::thread_fail(PAC_ERR_HIP, "%s: hipGetDevice: %s", who, hipGetErrorString(r));
    if (dev < 0 || dev >= kMaxDevices) return pac::thread_fail(PAC_ERR_RANGE, "%s: device %d not below %d", who, dev, kMaxDevices);
    unsigned char* base = scratch_on_device(dev, &r);
    if (!base) return pac::thread_fail(PAC_ERR_HIP, "%s: hipGetSymbolAddress: %s", who, hipGetErrorString(r));

    pac::MaskScratch s{};
    s.tile_state = reinterpret_cast<unsigned long long*>(base + kTileStateOffset);
    s.glob = reinterpret_cast<pac::Globals*>(base + kGlobalsOffset);
    s.status = reinterpret_cast<uint32_t*>(base + kStatusOffset);
    s.scan_spin_limit = 1u << 22;

    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned long long* total = reinterpret_cast<unsigned long long*>(d_nnz_out);
    if (n == 0) {
        // an empty mask has no words; the count and the flags are still defined
        if (total) r = pac::launch_mask_diff(nullptr, nullptr, 0, total, nullptr, stream);   // writes 0
        if (r == hipSuccess) r = pac::launch_status_read(s.status, d_flags_out, true, stream);
    } else {
        r = pac::launch_nonzero_mask(d_values, (int)dtype, (uint32_t)n, reinterpret_cast<unsigned long long*>(d_mask), stream);
        // The array keeps the last call's contents: the scan's reset kernel clears the tile states, the
        // ticket and (here) the status word before the scan runs.
        if (r == hipSuccess)
            r = pac::launch_prefix_scan(s, reinterpret_cast<const unsigned long long*>(d_mask), (uint32_t)pac_mask_words(n),
                                        d_prefix, total, /*reset_status=*/true, stream);
        if (r == hipSuccess && d_flags_out) r = pac::launch_status_read(s.status, d_flags_out, false, stream);
    }
    if (r != hipSuccess) return pac::thread_fail(PAC_ERR_HIP, "%s: launch: %s", who, hipGetErrorString(r));
    return PAC_OK;
}
