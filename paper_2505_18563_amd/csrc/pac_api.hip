// C ABI of libpactrain: argument checks, scratch ownership, segment-table upload, launches.
#include "../../include/pactrain.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "pac_internal.h"

namespace {

constexpr int kTableSlots = (int)PAC_TABLE_SLOTS;   // scope tables kept resident on the device
constexpr uint32_t kMaxSegments = 65535;   // scopes index a grid dimension

static_assert(pac::kDevScanStalled == PAC_DEV_SCAN_STALLED && pac::kDevCountMismatch == PAC_DEV_COUNT_MISMATCH &&
              pac::kDevMetaMismatch == PAC_DEV_META_MISMATCH && pac::kDevRetryTaken == PAC_DEV_RETRY_TAKEN &&
              pac::kDevSlowPath == PAC_DEV_SLOW_PATH, "status bits of the kernels and of the header");

thread_local char g_create_error[256] = "";

// One scope table resident on the device, with what the kernels derive from it.
struct TableSlot {
    pac::SegDesc* d_seg = nullptr;        // [max_segments]
    uint32_t* d_tile_scope = nullptr;     // [tiles]
    pac::SegDesc* h_stage = nullptr;      // pinned: the upload reads it asynchronously
    hipEvent_t uploaded = nullptr;        // recorded behind the upload
    bool upload_recorded = false;
    bool valid = false;
    bool captured = false;                // baked into a graph: never replaced
    uint64_t last_use = 0;
    std::vector<pac::SegDesc> table;      // what d_seg holds
};

}  // namespace

struct pac_ctx {
    int device = 0;
    int num_cu = 0;
    uint64_t max_elems = 0;
    uint32_t max_segments = 0;
    pac::MaskScratch scratch{};           // seg / tile_scope are set per call from a table slot
    TableSlot slots[kTableSlots];
    uint64_t use_clock = 0;
    uint32_t* d_status_copy = nullptr;    // device word pac_device_status copies through
    uint32_t* h_status = nullptr;         // pinned
    char err[256] = "";
};

struct pac_tracker {
    pac_ctx* ctx = nullptr;
    unsigned long long* prev = nullptr;      // the previous iteration's mask (device)
    pac::TrackerState* state = nullptr;      // counters (device)
    uint64_t max_elems = 0;
    uint32_t patience = 1;
    bool has_prev = false;
    uint64_t prev_n = 0;
};

namespace {

pac_status fail(pac_ctx* ctx, pac_status code, const char* fmt, ...) {
    char* dst = ctx ? ctx->err : g_create_error;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 256, fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace

int32_t pac::thread_fail(int32_t code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_create_error, sizeof g_create_error, fmt, ap);
    va_end(ap);
    return code;
}

namespace {

// Makes the context's device current for the duration of a call and restores the caller's.
struct DeviceGuard {
    int prev = -1;
    bool switched = false;
    hipError_t status = hipSuccess;
    explicit DeviceGuard(int want) {
        status = hipGetDevice(&prev);
        if (status == hipSuccess && prev != want) {
            status = hipSetDevice(want);
            switched = status == hipSuccess;
        }
    }
    ~DeviceGuard() {
        if (switched) (void)hipSetDevice(prev);
    }
};

bool is_aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

uint32_t elem_size(pac_dtype dt) { return dt == PAC_F32 ? 4u : 2u; }

// Stride of the sampled histogram pass over one prune scope.  Scopes below 4M elements are counted in
// full (a table without sampled scopes also needs no retry round).  Larger ones are sampled, one
// 16384-element tile in `stride`, so that between half a million and a million elements are visited (at
// most one tile in 64): the sample only has to place the bracket - its rank error of about 1/sqrt(sample)
// decides how many elements stay undecided in the one full pass - while the pass over the sample costs
// one LDS atomic per element; with a hundred large scopes and four times this sample it was a quarter of
// the whole call.  0 marks a small scope.
uint32_t sample_stride(uint64_t len) {
    if (len <= pac::kSmallScope) return 0;   // small scope: resolved by one workgroup, outside the histogram passes
    if (len < (1ull << 22)) return 1;
    uint32_t stride = 1;
    while (stride < pac::kMaxSampleStride && len / (2ull * stride) >= (1ull << 19)) stride *= 2;
    return stride;
}

void free_scratch(pac_ctx* ctx) {
    pac::MaskScratch& s = ctx->scratch;
    (void)hipFree(s.status);
    (void)hipFree(ctx->d_status_copy);
    if (ctx->h_status) (void)hipHostFree(ctx->h_status);
    (void)hipFree(s.state);
    (void)hipFree(s.hist0);
    (void)hipFree(s.hist1);
    (void)hipFree(s.kept_above);
    (void)hipFree(s.tie_count);
    (void)hipFree(s.glob);
    (void)hipFree(s.rec);
    (void)hipFree(s.hdrs);
    (void)hipFree(s.match);
    (void)hipFree(s.match_count);
    (void)hipFree(s.tile_state);
    if (s.side_stream) (void)hipStreamDestroy(s.side_stream);
    if (s.fork_event) (void)hipEventDestroy(s.fork_event);
    if (s.join_event) (void)hipEventDestroy(s.join_event);
    for (TableSlot& t : ctx->slots) {
        (void)hipFree(t.d_seg);
        (void)hipFree(t.d_tile_scope);
        if (t.h_stage) (void)hipHostFree(t.h_stage);
        if (t.uploaded) (void)hipEventDestroy(t.uploaded);
    }
}

}  // namespace

extern "C" {

uint64_t pac_keep_count(uint64_t n, double sparsity) {
    if (!(sparsity >= 0.0 && sparsity <= 1.0)) return 0;
    const uint64_t kMillion = 1000000u;
    const uint64_t ppm = (uint64_t)std::llround(sparsity * 1e6);
    // n < 2^32 on every path that reaches the device; for larger n do the product in 128 bits.
    const unsigned __int128 num = (unsigned __int128)n * (kMillion - ppm) + (kMillion - 1);
    return (uint64_t)(num / kMillion);
}

uint64_t pac_mask_words(uint64_t n) { return n / 64 + (n % 64 != 0 ? 1 : 0); }

const char* pac_last_error(const pac_ctx* ctx) { return ctx ? ctx->err : g_create_error; }

pac_status pac_create(pac_ctx** out, int hip_device, uint64_t max_elems, uint32_t max_segments) {
    if (!out) return fail(nullptr, PAC_ERR_ARG, "pac_create: out is NULL");
    *out = nullptr;
    if (max_elems == 0 || max_elems >= (1ull << 32))
        return fail(nullptr, PAC_ERR_RANGE, "pac_create: max_elems must be in [1, 2^32)");
    if (max_segments == 0 || max_segments > kMaxSegments)
        return fail(nullptr, PAC_ERR_RANGE, "pac_create: max_segments must be in [1, %u]", kMaxSegments);

    int count = 0;
    hipError_t e = hipGetDeviceCount(&count);
    if (e != hipSuccess) return fail(nullptr, PAC_ERR_HIP, "pac_create: hipGetDeviceCount: %s", hipGetErrorString(e));
    if (hip_device < 0 || hip_device >= count)
        return fail(nullptr, PAC_ERR_ARG, "pac_create: device %d not in [0, %d)", hip_device, count);

    pac_ctx* ctx = new (std::nothrow) pac_ctx();
    if (!ctx) return fail(nullptr, PAC_ERR_NOMEM, "pac_create: host allocation failed");
    ctx->device = hip_device;
    ctx->max_elems = max_elems;
    ctx->max_segments = max_segments;

    DeviceGuard guard(hip_device);
    if (guard.status != hipSuccess) {
        delete ctx;
        return fail(nullptr, PAC_ERR_HIP, "pac_create: hipSetDevice: %s", hipGetErrorString(guard.status));
    }
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, hip_device);
    if (e != hipSuccess) {
        delete ctx;
        return fail(nullptr, PAC_ERR_HIP, "pac_create: hipGetDeviceProperties: %s", hipGetErrorString(e));
    }
    ctx->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    pac::MaskScratch& s = ctx->scratch;
    s.cand_cap = ~0ull;   // every tile record may use all of its slots
    const uint64_t emit_tiles = (max_elems + pac::kEmitTileElems - 1) / pac::kEmitTileElems;
    const size_t hist0_bytes = (size_t)max_segments * pac::kDigit0Bins * sizeof(uint32_t);
    const size_t hist1_bytes = (size_t)max_segments * pac::kDigit1Bins * sizeof(uint32_t);
    bool ok = true;
    pac_status code = PAC_OK;
    auto alloc = [&](void** p, size_t bytes) {
        if (!ok) return;
        hipError_t r = hipMalloc(p, bytes);
        if (r != hipSuccess) {
            ok = false;
            code = fail(nullptr, PAC_ERR_NOMEM, "pac_create: hipMalloc(%zu): %s", bytes, hipGetErrorString(r));
        }
    };
    alloc((void**)&s.status, sizeof(uint32_t));
    alloc((void**)&ctx->d_status_copy, sizeof(uint32_t));
    alloc((void**)&s.state, (size_t)max_segments * sizeof(pac::SegState));
    alloc((void**)&s.hist0, hist0_bytes);
    alloc((void**)&s.hist1, hist1_bytes);
    alloc((void**)&s.kept_above, (size_t)max_segments * sizeof(uint32_t));
    alloc((void**)&s.tie_count, (size_t)max_segments * sizeof(uint32_t));
    alloc((void**)&s.glob, sizeof(pac::Globals));
    alloc((void**)&s.rec, (size_t)emit_tiles * pac::kRecSlots * sizeof(unsigned long long));
    alloc((void**)&s.hdrs, (size_t)emit_tiles * sizeof(unsigned long long));
    alloc((void**)&s.match, (size_t)pac::kMatchSlots * sizeof(unsigned long long));
    alloc((void**)&s.match_count, (size_t)pac::kMatchBlocks * sizeof(uint32_t));
    alloc((void**)&s.tile_state, (size_t)(pac::kScanMaxTiles + 1) * sizeof(unsigned long long));
    for (TableSlot& t : ctx->slots) {
        alloc((void**)&t.d_seg, (size_t)max_segments * sizeof(pac::SegDesc));
        alloc((void**)&t.d_tile_scope, (size_t)emit_tiles * sizeof(uint32_t));
        if (!ok) break;
        hipError_t r = hipHostMalloc((void**)&t.h_stage, (size_t)max_segments * sizeof(pac::SegDesc), hipHostMallocDefault);
        if (r == hipSuccess) r = hipEventCreateWithFlags(&t.uploaded, hipEventDisableTiming);
        if (r != hipSuccess) {
            ok = false;
            code = fail(nullptr, PAC_ERR_NOMEM, "pac_create: pinned staging: %s", hipGetErrorString(r));
        }
    }
    if (ok) {
        hipError_t r = hipHostMalloc((void**)&ctx->h_status, sizeof(uint32_t), hipHostMallocDefault);
        if (r != hipSuccess) {
            ok = false;
            code = fail(nullptr, PAC_ERR_NOMEM, "pac_create: pinned status word: %s", hipGetErrorString(r));
        }
    }
    if (ok) {
        // default priority, not synchronising with the NULL stream
        hipError_t r = hipStreamCreateWithFlags(&s.side_stream, hipStreamNonBlocking);
        if (r == hipSuccess) r = hipEventCreateWithFlags(&s.fork_event, hipEventDisableTiming);
        if (r == hipSuccess) r = hipEventCreateWithFlags(&s.join_event, hipEventDisableTiming);
        if (r != hipSuccess) {
            ok = false;
            code = fail(nullptr, PAC_ERR_HIP, "pac_create: side stream: %s", hipGetErrorString(r));
        }
    }
    if (ok) {
        hipError_t r = pac::prepare_mask_kernels();
        if (r != hipSuccess) {
            ok = false;
            code = fail(nullptr, PAC_ERR_HIP, "pac_create: kernel attributes: %s", hipGetErrorString(r));
        }
        s.hist_blocks = pac::mask_hist_blocks(ctx->num_cu);
        s.scan_spin_limit = 1u << 22;
    }
    if (ok) {
        // The histograms are all-zero between calls: the kernels that read them clear them.
        hipError_t r = hipMemset(s.hist0, 0, hist0_bytes);
        if (r == hipSuccess) r = hipMemset(s.hist1, 0, hist1_bytes);
        if (r == hipSuccess) r = hipMemset(s.glob, 0, sizeof(pac::Globals));
        if (r == hipSuccess) r = hipMemset(s.status, 0, sizeof(uint32_t));
        if (r == hipSuccess) r = hipMemset(s.state, 0, (size_t)max_segments * sizeof(pac::SegState));
        if (r == hipSuccess) r = hipDeviceSynchronize();
        if (r != hipSuccess) {
            ok = false;
            code = fail(nullptr, PAC_ERR_HIP, "pac_create: clearing scratch: %s", hipGetErrorString(r));
        }
    }
    if (!ok) {
        free_scratch(ctx);
        delete ctx;
        return code;
    }
    *out = ctx;
    return PAC_OK;
}

pac_status pac_destroy(pac_ctx* ctx) {
    if (!ctx) return PAC_OK;
    DeviceGuard guard(ctx->device);
    (void)hipDeviceSynchronize();
    free_scratch(ctx);
    delete ctx;
    return PAC_OK;
}

pac_status pac_debug_set_candidate_capacity(pac_ctx* ctx, uint64_t capacity) {
    if (!ctx) return PAC_ERR_ARG;
    ctx->scratch.cand_cap = capacity;
    return PAC_OK;
}

pac_status pac_debug_set_scan_spin_limit(pac_ctx* ctx, uint32_t polls) {
    if (!ctx) return PAC_ERR_ARG;
    ctx->scratch.scan_spin_limit = polls;
    return PAC_OK;
}

pac_status pac_device_status(pac_ctx* ctx, uint32_t* d_flags_out, uint32_t* h_flags_out, int clear, void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    if (!d_flags_out && !h_flags_out && !clear) return PAC_OK;
    if (!is_aligned(d_flags_out, 4)) return fail(ctx, PAC_ERR_ALIGN, "pac_device_status: d_flags_out not 4-byte aligned");
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess)
        return fail(ctx, PAC_ERR_HIP, "pac_device_status: hipSetDevice: %s", hipGetErrorString(guard.status));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // One read serves both destinations, so that a clearing read loses nothing.
    uint32_t* d_dst = d_flags_out ? d_flags_out : (h_flags_out ? ctx->d_status_copy : nullptr);
    hipError_t r = pac::launch_status_read(ctx->scratch.status, d_dst, clear != 0, stream);
    if (r == hipSuccess && h_flags_out) {
        r = hipMemcpyAsync(ctx->h_status, d_dst, sizeof(uint32_t), hipMemcpyDeviceToHost, stream);
        if (r == hipSuccess) r = hipStreamSynchronize(stream);
        if (r == hipSuccess) *h_flags_out = *ctx->h_status;
    }
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "pac_device_status: %s", hipGetErrorString(r));
    return PAC_OK;
}

pac_status pac_build_mask(pac_ctx* ctx, const float* d_weights, uint64_t n, const uint64_t* h_seg_offsets,
                          uint32_t nseg, const double* h_sparsity, uint64_t* d_mask, uint32_t* d_prefix,
                          uint64_t* h_nnz_out, void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    if (!h_seg_offsets || !h_sparsity || nseg == 0)
        return fail(ctx, PAC_ERR_ARG, "pac_build_mask: segment table missing");
    if (n >= (1ull << 32) || n > ctx->max_elems)
        return fail(ctx, PAC_ERR_RANGE, "pac_build_mask: n=%llu exceeds the context capacity %llu",
                    (unsigned long long)n, (unsigned long long)ctx->max_elems);
    if (nseg > ctx->max_segments)
        return fail(ctx, PAC_ERR_RANGE, "pac_build_mask: nseg=%u exceeds the context capacity %u", nseg,
                    ctx->max_segments);
    if (h_seg_offsets[0] != 0 || h_seg_offsets[nseg] != n)
        return fail(ctx, PAC_ERR_ARG, "pac_build_mask: segment offsets must start at 0 and end at n");
    for (uint32_t s = 0; s < nseg; ++s) {
        if (h_seg_offsets[s] > h_seg_offsets[s + 1])
            return fail(ctx, PAC_ERR_ARG, "pac_build_mask: segment offsets not ascending at %u", s);
        if (!(h_sparsity[s] >= 0.0 && h_sparsity[s] <= 1.0))
            return fail(ctx, PAC_ERR_RANGE, "pac_build_mask: sparsity[%u] outside [0,1]", s);
    }
    if (n > 0) {
        if (!d_weights || !d_mask || !d_prefix) return fail(ctx, PAC_ERR_ARG, "pac_build_mask: NULL device pointer");
        if (!is_aligned(d_weights, 4) || !is_aligned(d_mask, 8) || !is_aligned(d_prefix, 4))
            return fail(ctx, PAC_ERR_ALIGN, "pac_build_mask: weights/prefix need 4-byte, mask 8-byte alignment");
    }

    // Keep counts: host arithmetic, so the total is known without waiting for the device.
    std::vector<pac::SegDesc> table(nseg);
    uint64_t total = 0;
    uint32_t slots0 = 0, slots1 = 0;   // work items of the sampled and of the full histogram pass
    bool any_sampled = false;
    uint32_t max_small = 0, max_tiny = 0;   // longest small scope of the table, and longest of the tiny class
    for (uint32_t s = 0; s < nseg; ++s) {
        const uint64_t b = h_seg_offsets[s], e = h_seg_offsets[s + 1];
        const uint64_t k = pac_keep_count(e - b, h_sparsity[s]);
        table[s] = pac::SegDesc{(uint32_t)b, (uint32_t)e, (uint32_t)k, sample_stride(e - b), slots0, slots1};
        total += k;
        if (table[s].stride > 1) any_sampled = true;
        if (table[s].stride != 0) {
            slots0 += pac::hist_slots((uint32_t)b, (uint32_t)e, table[s].stride);
            slots1 += pac::hist_slots((uint32_t)b, (uint32_t)e, 1);
        } else {
            if (e - b > max_small) max_small = (uint32_t)(e - b);
            if (e - b <= pac::kTinyScope && e - b > max_tiny) max_tiny = (uint32_t)(e - b);
        }
    }
    if (h_nnz_out) *h_nnz_out = total;
    if (n == 0) return PAC_OK;

    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess)
        return fail(ctx, PAC_ERR_HIP, "pac_build_mask: hipSetDevice: %s", hipGetErrorString(guard.status));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);

    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capture) != hipSuccess) {
        (void)hipGetLastError();
        capture = hipStreamCaptureStatusNone;
    }
    const bool capturing = capture != hipStreamCaptureStatusNone;

    // The table among the resident ones (steady state, also of a cyclic sparsity schedule): nothing to upload.
    TableSlot* slot = nullptr;
    for (TableSlot& t : ctx->slots) {
        if (t.valid && t.table.size() == table.size() &&
            std::memcmp(t.table.data(), table.data(), table.size() * sizeof(pac::SegDesc)) == 0) {
            slot = &t;
            break;
        }
    }
    const bool fresh = slot == nullptr;
    if (fresh) {
        if (capturing)
            return fail(ctx, PAC_ERR_ARG, "pac_build_mask: this scope table is not resident on the device and the stream "
                                          "is being captured; run the call once outside the capture first");
        // Replace a slot that holds nothing, else the least recently used one that no graph refers to.
        for (TableSlot& t : ctx->slots) {
            if (t.captured) continue;
            if (!slot || (!t.valid && slot->valid) || (t.valid == slot->valid && t.last_use < slot->last_use)) slot = &t;
        }
        if (!slot)
            return fail(ctx, PAC_ERR_RANGE, "pac_build_mask: all %d scope-table slots are held by captured graphs", kTableSlots);
        if (slot->upload_recorded) {
            // The pinned staging block may be rewritten only after the upload that last read it has run:
            // true long ago unless more than kTableSlots tables alternate faster than the device follows.
            hipError_t q = hipEventQuery(slot->uploaded);
            if (q == hipErrorNotReady) q = hipEventSynchronize(slot->uploaded);
            if (q != hipSuccess) return fail(ctx, PAC_ERR_HIP, "pac_build_mask: waiting for an earlier table upload: %s", hipGetErrorString(q));
        }
        slot->valid = false;
        std::memcpy(slot->h_stage, table.data(), table.size() * sizeof(pac::SegDesc));
        hipError_t r = hipMemcpyAsync(slot->d_seg, slot->h_stage, table.size() * sizeof(pac::SegDesc),
                                      hipMemcpyHostToDevice, stream);
        if (r == hipSuccess) r = hipEventRecord(slot->uploaded, stream);
        if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "pac_build_mask: scope table upload: %s", hipGetErrorString(r));
        slot->upload_recorded = true;
        slot->table.swap(table);
        slot->valid = true;
    }
    slot->last_use = ++ctx->use_clock;
    if (capturing) slot->captured = true;

    pac::MaskScratch call = ctx->scratch;
    call.seg = slot->d_seg;
    call.tile_scope = slot->d_tile_scope;
    hipError_t r = pac::launch_build_mask(call, d_weights, (uint32_t)n, nseg, slots0, slots1, any_sampled, max_tiny, max_small,
                                          fresh, reinterpret_cast<unsigned long long*>(d_mask), d_prefix, total, stream);
    if (r != hipSuccess) {
        if (fresh) slot->valid = false;   // its tile_scope may not have been filled
        return fail(ctx, PAC_ERR_HIP, "pac_build_mask: launch: %s", hipGetErrorString(r));
    }
    return PAC_OK;
}

static pac_status check_pack_args(pac_ctx* ctx, const char* who, const void* d_dense, const void* d_compact,
                                  pac_dtype dtype, uint64_t n, uint64_t nnz, const uint64_t* d_mask,
                                  const uint32_t* d_prefix) {
    if (dtype != PAC_F32 && dtype != PAC_BF16) return fail(ctx, PAC_ERR_ARG, "%s: unknown dtype %d", who, (int)dtype);
    if (n >= (1ull << 32)) return fail(ctx, PAC_ERR_RANGE, "%s: n=%llu must be below 2^32", who, (unsigned long long)n);
    if (nnz > n) return fail(ctx, PAC_ERR_COUNT, "%s: nnz=%llu exceeds n=%llu", who, (unsigned long long)nnz, (unsigned long long)n);
    if (n == 0) return PAC_OK;
    if (!d_dense || !d_mask || !d_prefix || (nnz > 0 && !d_compact)) return fail(ctx, PAC_ERR_ARG, "%s: NULL device pointer", who);
    const uint32_t es = elem_size(dtype);
    if (!is_aligned(d_dense, es) || !is_aligned(d_compact, es) || !is_aligned(d_mask, 8) || !is_aligned(d_prefix, 4))
        return fail(ctx, PAC_ERR_ALIGN, "%s: pointer not aligned to its element size", who);
    return PAC_OK;
}

pac_status pac_compress(pac_ctx* ctx, const void* d_grad, pac_dtype dtype, uint64_t n, const uint64_t* d_mask,
                        const uint32_t* d_prefix, void* d_compact, uint64_t nnz, void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    pac_status st = check_pack_args(ctx, "pac_compress", d_grad, d_compact, dtype, n, nnz, d_mask, d_prefix);
    if (st != PAC_OK || n == 0) return st;
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return fail(ctx, PAC_ERR_HIP, "pac_compress: hipSetDevice: %s", hipGetErrorString(guard.status));
    hipError_t r = pac::launch_compress(d_grad, (int)dtype, (uint32_t)n, reinterpret_cast<const unsigned long long*>(d_mask),
                                        d_prefix, d_compact, (uint32_t)nnz, ctx->scratch.status,
                                        static_cast<hipStream_t>(hip_stream));
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "pac_compress: launch: %s", hipGetErrorString(r));
    return PAC_OK;
}

pac_status pac_decompress(pac_ctx* ctx, const void* d_compact, pac_dtype dtype, uint64_t nnz, const uint64_t* d_mask,
                          const uint32_t* d_prefix, void* d_dense_out, uint64_t n, void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    pac_status st = check_pack_args(ctx, "pac_decompress", d_dense_out, d_compact, dtype, n, nnz, d_mask, d_prefix);
    if (st != PAC_OK || n == 0) return st;
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return fail(ctx, PAC_ERR_HIP, "pac_decompress: hipSetDevice: %s", hipGetErrorString(guard.status));
    hipError_t r = pac::launch_decompress(d_compact, (int)dtype, (uint32_t)nnz, reinterpret_cast<const unsigned long long*>(d_mask),
                                          d_prefix, d_dense_out, (uint32_t)n, ctx->scratch.status,
                                          static_cast<hipStream_t>(hip_stream));
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "pac_decompress: launch: %s", hipGetErrorString(r));
    return PAC_OK;
}

pac_status pac_reduce_local(pac_ctx* ctx, const void* const* h_d_compact, uint32_t W, pac_dtype dtype, uint64_t nnz,
                            void* d_out, void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    if (dtype != PAC_F32 && dtype != PAC_BF16) return fail(ctx, PAC_ERR_ARG, "pac_reduce_local: unknown dtype %d", (int)dtype);
    if (W < 1 || W > PAC_MAX_WORKERS) return fail(ctx, PAC_ERR_RANGE, "pac_reduce_local: W=%u not in [1, %u]", W, PAC_MAX_WORKERS);
    if (nnz >= (1ull << 32)) return fail(ctx, PAC_ERR_RANGE, "pac_reduce_local: nnz must be below 2^32");
    if (!h_d_compact) return fail(ctx, PAC_ERR_ARG, "pac_reduce_local: pointer table is NULL");
    if (nnz == 0) return PAC_OK;
    const uint32_t es = elem_size(dtype);
    pac::WorkerPtrs bufs;
    for (uint32_t w = 0; w < PAC_MAX_WORKERS; ++w) bufs.p[w] = nullptr;
    for (uint32_t w = 0; w < W; ++w) {
        if (!h_d_compact[w]) return fail(ctx, PAC_ERR_ARG, "pac_reduce_local: buffer %u is NULL", w);
        if (!is_aligned(h_d_compact[w], es)) return fail(ctx, PAC_ERR_ALIGN, "pac_reduce_local: buffer %u misaligned", w);
        bufs.p[w] = h_d_compact[w];
    }
    if (!d_out) return fail(ctx, PAC_ERR_ARG, "pac_reduce_local: d_out is NULL");
    if (!is_aligned(d_out, es)) return fail(ctx, PAC_ERR_ALIGN, "pac_reduce_local: d_out misaligned");
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return fail(ctx, PAC_ERR_HIP, "pac_reduce_local: hipSetDevice: %s", hipGetErrorString(guard.status));
    hipError_t r = pac::launch_reduce(bufs, W, (int)dtype, (uint32_t)nnz, d_out, static_cast<hipStream_t>(hip_stream));
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "pac_reduce_local: launch: %s", hipGetErrorString(r));
    return PAC_OK;
}

pac_status pac_step_fused(pac_ctx* ctx, const void* const* h_d_grads, uint32_t W, pac_dtype dtype, uint64_t n,
                          const uint64_t* d_mask, const uint32_t* d_prefix, void* d_reduced, uint64_t nnz,
                          void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    const char* who = "pac_step_fused";
    if (dtype != PAC_F32 && dtype != PAC_BF16) return fail(ctx, PAC_ERR_ARG, "%s: unknown dtype %d", who, (int)dtype);
    if (W < 1 || W > PAC_MAX_WORKERS) return fail(ctx, PAC_ERR_RANGE, "%s: W=%u not in [1, %u]", who, W, PAC_MAX_WORKERS);
    if (n >= (1ull << 32)) return fail(ctx, PAC_ERR_RANGE, "%s: n=%llu must be below 2^32", who, (unsigned long long)n);
    if (nnz > n) return fail(ctx, PAC_ERR_COUNT, "%s: nnz=%llu exceeds n=%llu", who, (unsigned long long)nnz, (unsigned long long)n);
    if (!h_d_grads) return fail(ctx, PAC_ERR_ARG, "%s: pointer table is NULL", who);
    if (n == 0) return PAC_OK;
    if (!d_mask || !d_prefix || (nnz > 0 && !d_reduced)) return fail(ctx, PAC_ERR_ARG, "%s: NULL device pointer", who);
    const uint32_t es = elem_size(dtype);
    if (!is_aligned(d_reduced, es) || !is_aligned(d_mask, 8) || !is_aligned(d_prefix, 4))
        return fail(ctx, PAC_ERR_ALIGN, "%s: pointer not aligned to its element size", who);
    pac::WorkerPtrs bufs;
    for (uint32_t w = 0; w < PAC_MAX_WORKERS; ++w) bufs.p[w] = nullptr;
    for (uint32_t w = 0; w < W; ++w) {
        if (!h_d_grads[w]) return fail(ctx, PAC_ERR_ARG, "%s: gradient %u is NULL", who, w);
        if (!is_aligned(h_d_grads[w], es)) return fail(ctx, PAC_ERR_ALIGN, "%s: gradient %u misaligned", who, w);
        bufs.p[w] = h_d_grads[w];
    }
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: hipSetDevice: %s", who, hipGetErrorString(guard.status));
    hipError_t r = pac::launch_step_fused(bufs, W, (int)dtype, (uint32_t)n, reinterpret_cast<const unsigned long long*>(d_mask),
                                          d_prefix, d_reduced, (uint32_t)nnz, ctx->scratch.status,
                                          static_cast<hipStream_t>(hip_stream));
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: launch: %s", who, hipGetErrorString(r));
    return PAC_OK;
}

// ---- Mask Tracker and weight update ----------------------------------------------------------

pac_status pac_mask_from_nonzero(pac_ctx* ctx, const void* d_values, pac_dtype dtype, uint64_t n, uint64_t* d_mask,
                                 uint32_t* d_prefix, uint64_t* d_nnz_out, void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    const char* who = "pac_mask_from_nonzero";
    if (dtype != PAC_F32 && dtype != PAC_BF16) return fail(ctx, PAC_ERR_ARG, "%s: unknown dtype %d", who, (int)dtype);
    if (n > ctx->max_elems) return fail(ctx, PAC_ERR_RANGE, "%s: n=%llu exceeds the context's max_elems=%llu", who,
                                        (unsigned long long)n, (unsigned long long)ctx->max_elems);
    if (n > 0 && (!d_values || !d_mask || !d_prefix)) return fail(ctx, PAC_ERR_ARG, "%s: NULL device pointer", who);
    if (!is_aligned(d_values, elem_size(dtype)) || !is_aligned(d_mask, 8) || !is_aligned(d_prefix, 4) ||
        !is_aligned(d_nnz_out, 8))
        return fail(ctx, PAC_ERR_ALIGN, "%s: pointer not aligned to its element size", who);
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: hipSetDevice: %s", who, hipGetErrorString(guard.status));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    unsigned long long* total = reinterpret_cast<unsigned long long*>(d_nnz_out);
    hipError_t r = hipSuccess;
    if (n == 0) {
        // an empty mask has no words; the count is still defined
        if (total) r = pac::launch_mask_diff(nullptr, nullptr, 0, total, nullptr, stream);   // writes 0
    } else {
        r = pac::launch_nonzero_mask(d_values, (int)dtype, (uint32_t)n, reinterpret_cast<unsigned long long*>(d_mask), stream);
        if (r == hipSuccess)
            r = pac::launch_prefix_scan(ctx->scratch, reinterpret_cast<const unsigned long long*>(d_mask),
                                        (uint32_t)pac_mask_words(n), d_prefix, total, /*reset_status=*/false, stream);
    }
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: launch: %s", who, hipGetErrorString(r));
    return PAC_OK;
}

pac_status pac_mask_equal(pac_ctx* ctx, const uint64_t* d_mask_a, const uint64_t* d_mask_b, uint64_t n,
                          uint64_t* d_diff_bits_out, void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    const char* who = "pac_mask_equal";
    if (n >= (1ull << 32)) return fail(ctx, PAC_ERR_RANGE, "%s: n=%llu must be below 2^32", who, (unsigned long long)n);
    if (!d_diff_bits_out || (n > 0 && (!d_mask_a || !d_mask_b))) return fail(ctx, PAC_ERR_ARG, "%s: NULL device pointer", who);
    if (!is_aligned(d_mask_a, 8) || !is_aligned(d_mask_b, 8) || !is_aligned(d_diff_bits_out, 8))
        return fail(ctx, PAC_ERR_ALIGN, "%s: pointer not aligned to 8 bytes", who);
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: hipSetDevice: %s", who, hipGetErrorString(guard.status));
    hipError_t r = pac::launch_mask_diff(reinterpret_cast<const unsigned long long*>(d_mask_a),
                                         reinterpret_cast<const unsigned long long*>(d_mask_b), (uint32_t)n,
                                         reinterpret_cast<unsigned long long*>(d_diff_bits_out), nullptr,
                                         static_cast<hipStream_t>(hip_stream));
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: launch: %s", who, hipGetErrorString(r));
    return PAC_OK;
}

pac_status pac_tracker_create(pac_ctx* ctx, uint64_t max_elems, uint32_t patience, pac_tracker** out) {
    if (!ctx) return PAC_ERR_ARG;
    if (!out) return fail(ctx, PAC_ERR_ARG, "pac_tracker_create: out is NULL");
    *out = nullptr;
    if (max_elems == 0 || max_elems >= (1ull << 32))
        return fail(ctx, PAC_ERR_RANGE, "pac_tracker_create: max_elems must be in [1, 2^32)");
    if (patience == 0) return fail(ctx, PAC_ERR_RANGE, "pac_tracker_create: patience must be at least 1");
    pac_tracker* t = new (std::nothrow) pac_tracker();
    if (!t) return fail(ctx, PAC_ERR_NOMEM, "pac_tracker_create: host allocation failed");
    t->ctx = ctx;
    t->max_elems = max_elems;
    t->patience = patience;
    DeviceGuard guard(ctx->device);
    hipError_t r = guard.status;
    if (r == hipSuccess) r = hipMalloc((void**)&t->prev, (size_t)pac_mask_words(max_elems) * 8);
    if (r == hipSuccess) r = hipMalloc((void**)&t->state, sizeof(pac::TrackerState));
    if (r == hipSuccess) r = hipMemset(t->state, 0, sizeof(pac::TrackerState));
    if (r == hipSuccess) r = hipDeviceSynchronize();
    if (r != hipSuccess) {
        (void)hipFree(t->prev);
        (void)hipFree(t->state);
        delete t;
        return fail(ctx, PAC_ERR_NOMEM, "pac_tracker_create: device allocation: %s", hipGetErrorString(r));
    }
    *out = t;
    return PAC_OK;
}

pac_status pac_tracker_update(pac_tracker* t, const uint64_t* d_mask, uint64_t n, uint32_t* d_state_out,
                              void* hip_stream) {
    if (!t) return PAC_ERR_ARG;
    pac_ctx* ctx = t->ctx;
    const char* who = "pac_tracker_update";
    if (n > t->max_elems) return fail(ctx, PAC_ERR_RANGE, "%s: n=%llu exceeds the tracker's max_elems=%llu", who,
                                      (unsigned long long)n, (unsigned long long)t->max_elems);
    if (n > 0 && !d_mask) return fail(ctx, PAC_ERR_ARG, "%s: d_mask is NULL", who);
    if (!is_aligned(d_mask, 8) || !is_aligned(d_state_out, 4)) return fail(ctx, PAC_ERR_ALIGN, "%s: misaligned pointer", who);
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: hipSetDevice: %s", who, hipGetErrorString(guard.status));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const unsigned long long* m = reinterpret_cast<const unsigned long long*>(d_mask);
    const bool fresh = !t->has_prev || t->prev_n != n;
    hipError_t r;
    if (fresh) {
        r = pac::launch_mask_copy(m, t->prev, (uint32_t)pac_mask_words(n), stream);
    } else {
        // compare with the previous mask and replace it in one pass
        r = pac::launch_mask_diff(t->prev, m, (uint32_t)n, &t->state->diff, t->prev, stream);
    }
    if (r == hipSuccess) r = pac::launch_tracker_finalize(t->state, t->patience, fresh ? 1u : 0u, d_state_out, stream);
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: launch: %s", who, hipGetErrorString(r));
    t->has_prev = true;
    t->prev_n = n;
    return PAC_OK;
}

pac_status pac_tracker_destroy(pac_tracker* t) {
    if (!t) return PAC_OK;
    DeviceGuard guard(t->ctx->device);
    (void)hipDeviceSynchronize();
    (void)hipFree(t->prev);
    (void)hipFree(t->state);
    delete t;
    return PAC_OK;
}

pac_status pac_decompress_update(pac_ctx* ctx, const void* d_reduced, pac_dtype dtype, uint64_t nnz,
                                 const uint64_t* d_mask, const uint32_t* d_prefix, float alpha, float* d_weights,
                                 uint64_t n, void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    const char* who = "pac_decompress_update";
    if (dtype != PAC_F32 && dtype != PAC_BF16) return fail(ctx, PAC_ERR_ARG, "%s: unknown dtype %d", who, (int)dtype);
    if (n >= (1ull << 32)) return fail(ctx, PAC_ERR_RANGE, "%s: n=%llu must be below 2^32", who, (unsigned long long)n);
    if (nnz > n) return fail(ctx, PAC_ERR_COUNT, "%s: nnz=%llu exceeds n=%llu", who, (unsigned long long)nnz, (unsigned long long)n);
    if (n == 0) return PAC_OK;
    if (!d_weights || !d_mask || !d_prefix || (nnz > 0 && !d_reduced)) return fail(ctx, PAC_ERR_ARG, "%s: NULL device pointer", who);
    if (!is_aligned(d_weights, 4) || !is_aligned(d_reduced, elem_size(dtype)) || !is_aligned(d_mask, 8) || !is_aligned(d_prefix, 4))
        return fail(ctx, PAC_ERR_ALIGN, "%s: pointer not aligned to its element size", who);
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: hipSetDevice: %s", who, hipGetErrorString(guard.status));
    hipError_t r = pac::launch_decompress_update(d_reduced, (int)dtype, (uint32_t)nnz,
                                                 reinterpret_cast<const unsigned long long*>(d_mask), d_prefix, alpha,
                                                 d_weights, (uint32_t)n, ctx->scratch.status,
                                                 static_cast<hipStream_t>(hip_stream));
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: launch: %s", who, hipGetErrorString(r));
    return PAC_OK;
}

// ---- ternary payload ---------------------------------------------------------------------------

pac_status pac_absmax(pac_ctx* ctx, const void* d_values, pac_dtype dtype, uint64_t count, int accumulate,
                      float* d_scale_inout, void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    const char* who = "pac_absmax";
    if (dtype != PAC_F32 && dtype != PAC_BF16) return fail(ctx, PAC_ERR_ARG, "%s: unknown dtype %d", who, (int)dtype);
    if (count >= (1ull << 32)) return fail(ctx, PAC_ERR_RANGE, "%s: count must be below 2^32", who);
    if (!d_scale_inout || (count > 0 && !d_values)) return fail(ctx, PAC_ERR_ARG, "%s: NULL device pointer", who);
    if (!is_aligned(d_values, elem_size(dtype)) || !is_aligned(d_scale_inout, 4))
        return fail(ctx, PAC_ERR_ALIGN, "%s: pointer not aligned to its element size", who);
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: hipSetDevice: %s", who, hipGetErrorString(guard.status));
    hipError_t r = pac::launch_absmax(d_values, (int)dtype, (uint32_t)count, accumulate != 0, d_scale_inout,
                                      static_cast<hipStream_t>(hip_stream));
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: launch: %s", who, hipGetErrorString(r));
    return PAC_OK;
}

pac_status pac_ternarize(pac_ctx* ctx, const void* d_values, pac_dtype dtype, uint64_t count, const float* d_scale,
                         uint64_t seed, uint64_t stream_id, uint8_t* d_packed_out, void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    const char* who = "pac_ternarize";
    if (dtype != PAC_F32 && dtype != PAC_BF16) return fail(ctx, PAC_ERR_ARG, "%s: unknown dtype %d", who, (int)dtype);
    if (count >= (1ull << 32)) return fail(ctx, PAC_ERR_RANGE, "%s: count must be below 2^32", who);
    if (count == 0) return PAC_OK;
    if (!d_values || !d_scale || !d_packed_out) return fail(ctx, PAC_ERR_ARG, "%s: NULL device pointer", who);
    if (!is_aligned(d_values, elem_size(dtype)) || !is_aligned(d_scale, 4) || !is_aligned(d_packed_out, 4))
        return fail(ctx, PAC_ERR_ALIGN, "%s: misaligned pointer (packed buffers need 4 bytes)", who);
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: hipSetDevice: %s", who, hipGetErrorString(guard.status));
    hipError_t r = pac::launch_ternarize(d_values, (int)dtype, (uint32_t)count, d_scale, seed, stream_id, d_packed_out,
                                         static_cast<hipStream_t>(hip_stream));
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: launch: %s", who, hipGetErrorString(r));
    return PAC_OK;
}

pac_status pac_ternary_reduce_local(pac_ctx* ctx, const uint8_t* const* h_d_packed, uint32_t W, uint64_t count,
                                    const float* d_scale, pac_dtype out_dtype, void* d_out, void* hip_stream) {
    if (!ctx) return PAC_ERR_ARG;
    const char* who = "pac_ternary_reduce_local";
    if (out_dtype != PAC_F32 && out_dtype != PAC_BF16) return fail(ctx, PAC_ERR_ARG, "%s: unknown dtype %d", who, (int)out_dtype);
    if (W < 1 || W > PAC_MAX_WORKERS) return fail(ctx, PAC_ERR_RANGE, "%s: W=%u not in [1, %u]", who, W, PAC_MAX_WORKERS);
    if (count >= (1ull << 32)) return fail(ctx, PAC_ERR_RANGE, "%s: count must be below 2^32", who);
    if (!h_d_packed) return fail(ctx, PAC_ERR_ARG, "%s: pointer table is NULL", who);
    if (count == 0) return PAC_OK;
    pac::WorkerPtrs bufs;
    for (uint32_t w = 0; w < PAC_MAX_WORKERS; ++w) bufs.p[w] = nullptr;
    for (uint32_t w = 0; w < W; ++w) {
        if (!h_d_packed[w]) return fail(ctx, PAC_ERR_ARG, "%s: buffer %u is NULL", who, w);
        if (!is_aligned(h_d_packed[w], 4)) return fail(ctx, PAC_ERR_ALIGN, "%s: buffer %u not 4-byte aligned", who, w);
        bufs.p[w] = h_d_packed[w];
    }
    if (!d_out || !d_scale) return fail(ctx, PAC_ERR_ARG, "%s: NULL device pointer", who);
    if (!is_aligned(d_out, elem_size(out_dtype)) || !is_aligned(d_scale, 4)) return fail(ctx, PAC_ERR_ALIGN, "%s: misaligned pointer", who);
    DeviceGuard guard(ctx->device);
    if (guard.status != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: hipSetDevice: %s", who, hipGetErrorString(guard.status));
    hipError_t r = pac::launch_ternary_reduce(bufs, W, (uint32_t)count, d_scale, (int)out_dtype, d_out,
                                              static_cast<hipStream_t>(hip_stream));
    if (r != hipSuccess) return fail(ctx, PAC_ERR_HIP, "%s: launch: %s", who, hipGetErrorString(r));
    return PAC_OK;
}

}  // extern "C"
