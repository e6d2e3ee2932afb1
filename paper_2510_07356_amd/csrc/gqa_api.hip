// C-ABI layer: argument validation, split planning, workspace carving, launches.
#include "../../include/gqa_decode.h"
#include "gqa_internal.h"

#include <atomic>
#include <cmath>
#include <new>

struct gqa_timer {
    int32_t max_calls;
    int32_t calls;
    hipEvent_t* events;      // 3 per call
};

namespace {

using gqa::KernelArgs;

constexpr int kVersion = 200;          // 0.2.0
constexpr int kMaxWorkgroups = 1024;   // bound of the persistent launch; the workspace is sized for it
constexpr int kMaxWorkers = kMaxWorkgroups * gqa::kMaxWorkersPerGroup;   // shares when none is fixed
constexpr int kMaxDevices = 64;

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline bool mult8(int64_t s) { return s % 8 == 0; }

struct Plan {
    int fixed_share_tiles;   // 0: one share per workgroup
    int64_t max_tiles;       // Hkv * B * ceil(max_kv_len / 32)
    int64_t slots;           // partial-result slots the workspace holds
    size_t header_bytes, prefix_bytes, ml_bytes, o_bytes;
    size_t total_bytes() const { return header_bytes + prefix_bytes + ml_bytes + o_bytes; }
};

// Scratch buffer of gqa_decode_attn_static: one copy per device, in the code object's
// zero-initialised data.  In host code the name is only a handle for hipGetSymbolAddress; the
// device address it yields (kept per device below) is what kernels and launches receive.
constexpr size_t kStaticScratchBytes = GQA_DECODE_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

int check_shape(const gqa_decode_params* p) {
    if (p == nullptr) return GQA_ERR_INVALID_ARG;
    if (p->batch < 1 || p->num_q_heads < 1 || p->num_kv_heads < 1 || p->max_kv_len < 0)
        return GQA_ERR_INVALID_ARG;
    if (p->num_q_heads % p->num_kv_heads != 0) return GQA_ERR_INVALID_ARG;
    if (p->page_size < 0 || p->chunk_tokens < 0) return GQA_ERR_INVALID_ARG;
    if (p->chunk_tokens % gqa::kChunkGranule != 0) return GQA_ERR_INVALID_ARG;
    if (p->kernel_variant != 0 && p->kernel_variant != 1) return GQA_ERR_INVALID_ARG;
    if (!std::isfinite(p->scale)) return GQA_ERR_INVALID_ARG;
    if (p->head_dim != gqa::kHeadDim) return GQA_ERR_UNSUPPORTED;
    const int group = p->num_q_heads / p->num_kv_heads;
    if (group > gqa::kMaxGroup) return GQA_ERR_UNSUPPORTED;
    if (p->kernel_variant == 1 && group > 8) return GQA_ERR_UNSUPPORTED;
    if (p->page_size != 0) {
        if (p->page_size < 16 || (p->page_size & (p->page_size - 1)) != 0) return GQA_ERR_UNSUPPORTED;
        if ((int64_t)p->block_table_stride * p->page_size < p->max_kv_len) return GQA_ERR_INVALID_ARG;
    }
    return GQA_OK;
}

// `workers` is the number of shares when none is fixed: kMaxWorkers for a workspace sized without
// looking at a device, the real number of persistent workers when the launch size is known.
int make_plan(const gqa_decode_params* p, Plan* plan, int64_t workers = kMaxWorkers) {
    const int rc = check_shape(p);
    if (rc != GQA_OK) return rc;
    const int group = p->num_q_heads / p->num_kv_heads;
    plan->fixed_share_tiles = p->chunk_tokens / gqa::kTileTokens;
    plan->max_tiles = (int64_t)p->num_kv_heads * p->batch * gqa::tiles_of(p->max_kv_len);
    if (plan->max_tiles > 0x3fffffffLL) return GQA_ERR_UNSUPPORTED;     // stream positions are int32
    int64_t shares = workers;
    if (plan->fixed_share_tiles > 0) {
        const int64_t fixed = (plan->max_tiles + plan->fixed_share_tiles - 1) / plan->fixed_share_tiles;
        if (fixed > shares) shares = fixed;
    }
    plan->slots = shares + (int64_t)p->batch * p->num_kv_heads;
    plan->header_bytes = 256;
    plan->prefix_bytes = align_up(sizeof(int32_t) * ((size_t)p->batch + 1), 256);
    plan->ml_bytes = align_up((size_t)plan->slots * group * 2 * sizeof(float), 256);
    plan->o_bytes = align_up((size_t)plan->slots * group * gqa::kHeadDim * sizeof(float), 256);
    return GQA_OK;
}

// Persistent launch size of the current device: CUs x resident workgroups per CU,
// looked up once per device and kernel variant.
int workgroups_for(int variant) {
    static std::atomic<int> cache[kMaxDevices][2];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 0;
    int n = cache[dev][variant].load(std::memory_order_acquire);
    if (n > 0) return n;
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) return 0;
    const int occ = variant == 1 ? gqa::partial_valu_occupancy() : gqa::partial_mfma_occupancy();
    n = cus * occ;
    if (n > kMaxWorkgroups) n = kMaxWorkgroups;
    cache[dev][variant].store(n, std::memory_order_release);
    return n;
}

// Persistent workgroups one call launches: the device's capacity, but no more than the stream can
// feed with shares of the minimum length.
int launch_workgroups(const gqa_decode_params* p, int64_t max_tiles) {
    int workgroups = workgroups_for(p->kernel_variant);
    if (workgroups < 1) return 0;
    const int per_group = p->kernel_variant == 1 ? 1 : gqa::partial_mfma_workers_per_group();
    const int64_t useful = (max_tiles + gqa::kMinShareTiles * per_group - 1) / (gqa::kMinShareTiles * per_group);
    if (useful < workgroups) workgroups = (int)(useful > 0 ? useful : 1);
    return workgroups;
}

// Device address of this device's copy of `scratch`, looked up once per device.
int static_scratch(void** out) {
    static std::atomic<void*> cache[kMaxDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GQA_ERR_LAUNCH;
    void* ptr = cache[dev].load(std::memory_order_acquire);
    if (ptr == nullptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return GQA_ERR_LAUNCH;
        cache[dev].store(ptr, std::memory_order_release);
    }
    *out = ptr;
    return GQA_OK;
}

// Host-side checks of the tensors of one call (the shape was checked by make_plan).
int check_tensors(const gqa_decode_params* p, const void* q, const void* k, const void* v,
                  const int32_t* kv_lens, const int32_t* block_table, const float* out) {
    if (!q || !k || !v || !kv_lens || !out) return GQA_ERR_INVALID_ARG;
    if ((p->page_size != 0) != (block_table != nullptr)) return GQA_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return GQA_ERR_INVALID_ARG;
    if (!mult8(p->q_stride_b) || !mult8(p->q_stride_h) || !mult8(p->k_stride_b) || !mult8(p->k_stride_h) ||
        !mult8(p->k_stride_t) || !mult8(p->v_stride_b) || !mult8(p->v_stride_h) || !mult8(p->v_stride_t))
        return GQA_ERR_INVALID_ARG;
    if (p->k_stride_t < gqa::kHeadDim || p->v_stride_t < gqa::kHeadDim || p->q_stride_h < gqa::kHeadDim)
        return GQA_ERR_INVALID_ARG;
    return GQA_OK;
}

int run(const gqa_decode_params* p, const Plan& plan, const void* q, const void* k, const void* v,
        const int32_t* kv_lens, const int32_t* block_table,
        float* out, float* lse, void* workspace, size_t workspace_bytes, void* stream,
        gqa_timer* timer) {
    const int rc = check_tensors(p, q, k, v, kv_lens, block_table, out);
    if (rc != GQA_OK) return rc;
    if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return GQA_ERR_INVALID_ARG;
    if (workspace_bytes < plan.total_bytes()) return GQA_ERR_WORKSPACE_TOO_SMALL;

    KernelArgs a{};
    a.q = static_cast<const uint16_t*>(q);
    a.k = static_cast<const uint16_t*>(k);
    a.v = static_cast<const uint16_t*>(v);
    a.kv_lens = kv_lens;
    a.block_table = block_table;
    char* ws = static_cast<char*>(workspace);
    a.header = reinterpret_cast<int32_t*>(ws);
    a.row_prefix = reinterpret_cast<int32_t*>(ws + plan.header_bytes);
    a.part_ml = reinterpret_cast<float*>(ws + plan.header_bytes + plan.prefix_bytes);
    a.part_o = reinterpret_cast<float*>(ws + plan.header_bytes + plan.prefix_bytes + plan.ml_bytes);
    a.out = out;
    a.lse = lse;
    a.batch = p->batch;
    a.num_q_heads = p->num_q_heads;
    a.num_kv_heads = p->num_kv_heads;
    a.group = p->num_q_heads / p->num_kv_heads;
    a.max_kv_len = p->max_kv_len;
    a.fixed_share_tiles = plan.fixed_share_tiles;
    a.page_size = p->page_size;
    a.page_shift = 0;
    while (p->page_size > 1 && (1 << a.page_shift) < p->page_size) ++a.page_shift;
    a.block_table_stride = p->block_table_stride;
    a.q_stride_b = p->q_stride_b; a.q_stride_h = p->q_stride_h;
    a.k_stride_b = p->k_stride_b; a.k_stride_h = p->k_stride_h; a.k_stride_t = p->k_stride_t;
    a.v_stride_b = p->v_stride_b; a.v_stride_h = p->v_stride_h; a.v_stride_t = p->v_stride_t;
    a.scale_log2e = p->scale * 1.4426950408889634f;

    const int workgroups = launch_workgroups(p, plan.max_tiles);
    if (workgroups < 1) return GQA_ERR_LAUNCH;

    hipStream_t s = static_cast<hipStream_t>(stream);
    hipEvent_t* ev = nullptr;
    if (timer != nullptr) {
        if (timer->calls >= timer->max_calls) return GQA_ERR_INVALID_ARG;
        ev = timer->events + 3 * (size_t)timer->calls;
    }
    int status = GQA_OK;
    if (ev && hipEventRecord(ev[0], s) != hipSuccess) status = GQA_ERR_LAUNCH;
    if (status == GQA_OK) {
        const hipError_t e = (p->kernel_variant == 1) ? gqa::launch_partial_valu(a, workgroups, s)
                                                      : gqa::launch_partial_mfma(a, workgroups, s);
        if (e != hipSuccess) status = GQA_ERR_LAUNCH;
    }
    if (status == GQA_OK && ev && hipEventRecord(ev[1], s) != hipSuccess) status = GQA_ERR_LAUNCH;
    if (status == GQA_OK && gqa::launch_combine(a, workgroups, s) != hipSuccess) status = GQA_ERR_LAUNCH;
    if (status == GQA_OK && ev && hipEventRecord(ev[2], s) != hipSuccess) status = GQA_ERR_LAUNCH;
    if (status == GQA_OK && timer != nullptr) ++timer->calls;
    return status;
}

}  // namespace

extern "C" {

int gqa_decode_version(void) { return kVersion; }

const char* gqa_decode_strerror(int status) {
    switch (status) {
        case GQA_OK: return "ok";
        case GQA_ERR_INVALID_ARG: return "invalid argument";
        case GQA_ERR_UNSUPPORTED: return "unsupported shape";
        case GQA_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case GQA_ERR_LAUNCH: return "HIP launch failed";
        case GQA_ERR_SCRATCH_LIMIT: return "problem too large for the built-in scratch buffer";
        default: return "unknown status";
    }
}

size_t gqa_decode_workspace_bytes(const gqa_decode_params* params) {
    Plan plan;
    if (make_plan(params, &plan) != GQA_OK) return 0;
    return plan.total_bytes();
}

int gqa_decode_plan_info(const gqa_decode_params* params, const int32_t* host_kv_lens,
                         int32_t* share_tokens, int32_t* workgroups, int64_t* partial_slots) {
    Plan plan;
    const int rc = make_plan(params, &plan);
    if (rc != GQA_OK) return rc;
    const int wgs = launch_workgroups(params, plan.max_tiles);     // 0 when no device is present
    const int per_group = params->kernel_variant == 1 ? 1 : gqa::partial_mfma_workers_per_group();
    if (workgroups) *workgroups = wgs;
    if (partial_slots) *partial_slots = plan.slots;
    if (share_tokens) {
        *share_tokens = plan.fixed_share_tiles * gqa::kTileTokens;
        if (plan.fixed_share_tiles == 0 && host_kv_lens != nullptr && wgs > 0) {
            int64_t total = 0;
            for (int b = 0; b < params->batch; ++b) {
                int64_t len = host_kv_lens[b];
                if (len < 0) len = 0;
                if (len > params->max_kv_len) len = params->max_kv_len;
                total += (int64_t)params->num_kv_heads * gqa::tiles_of((int)len);
            }
            *share_tokens = gqa::share_tiles_for(total, 0, wgs * per_group) * gqa::kTileTokens;
        }
    }
    return GQA_OK;
}

int gqa_decode_init(void) {
    if (workgroups_for(0) < 1 || workgroups_for(1) < 1) return GQA_ERR_LAUNCH;
    if (gqa::prepare_prefill() != hipSuccess) return GQA_ERR_LAUNCH;
    void* ptr = nullptr;
    return static_scratch(&ptr);
}

int gqa_decode_attn(const gqa_decode_params* params, const void* q, const void* k, const void* v,
                    const int32_t* kv_lens, const int32_t* block_table, const int32_t* host_kv_lens,
                    float* out, float* lse, void* workspace, size_t workspace_bytes, void* stream) {
    (void)host_kv_lens;      // the launch size does not depend on the lengths
    Plan plan;
    const int rc = make_plan(params, &plan);
    if (rc != GQA_OK) return rc;
    return run(params, plan, q, k, v, kv_lens, block_table, out, lse, workspace, workspace_bytes, stream, nullptr);
}

size_t gqa_decode_static_scratch_bytes(void) { return kStaticScratchBytes; }

int gqa_decode_attn_static(const gqa_decode_params* params, const void* q, const void* k, const void* v,
                           const int32_t* kv_lens, const int32_t* block_table,
                           float* out, float* lse, void* stream) {
    // sized for the launch this device will really get, not for the largest one the library knows
    Plan plan;
    int rc = make_plan(params, &plan);
    if (rc != GQA_OK) return rc;
    rc = check_tensors(params, q, k, v, kv_lens, block_table, out);
    if (rc != GQA_OK) return rc;
    const int workgroups = launch_workgroups(params, plan.max_tiles);
    if (workgroups < 1) return GQA_ERR_LAUNCH;
    const int per_group = params->kernel_variant == 1 ? 1 : gqa::partial_mfma_workers_per_group();
    rc = make_plan(params, &plan, (int64_t)workgroups * per_group);
    if (rc != GQA_OK) return rc;
    if (plan.total_bytes() > kStaticScratchBytes) return GQA_ERR_SCRATCH_LIMIT;
    void* ptr = nullptr;
    rc = static_scratch(&ptr);
    if (rc != GQA_OK) return rc;
    return run(params, plan, q, k, v, kv_lens, block_table, out, lse, ptr, kStaticScratchBytes, stream, nullptr);
}

int gqa_decode_attn_timed(const gqa_decode_params* params, const void* q, const void* k, const void* v,
                          const int32_t* kv_lens, const int32_t* block_table,
                          const int32_t* host_kv_lens, float* out, float* lse, void* workspace,
                          size_t workspace_bytes, void* stream, gqa_timer* timer) {
    (void)host_kv_lens;
    if (timer == nullptr) return GQA_ERR_INVALID_ARG;
    Plan plan;
    const int rc = make_plan(params, &plan);
    if (rc != GQA_OK) return rc;
    return run(params, plan, q, k, v, kv_lens, block_table, out, lse, workspace, workspace_bytes, stream, timer);
}

int gqa_timer_create(int32_t max_calls, gqa_timer** host_out) {
    if (host_out == nullptr || max_calls < 1 || max_calls > (1 << 20)) return GQA_ERR_INVALID_ARG;
    *host_out = nullptr;
    gqa_timer* t = new (std::nothrow) gqa_timer{max_calls, 0, nullptr};
    if (t == nullptr) return GQA_ERR_LAUNCH;
    t->events = new (std::nothrow) hipEvent_t[3 * (size_t)max_calls]();
    if (t->events == nullptr) { delete t; return GQA_ERR_LAUNCH; }
    for (size_t i = 0; i < 3 * (size_t)max_calls; ++i) {
        if (hipEventCreate(&t->events[i]) != hipSuccess) {
            for (size_t j = 0; j < i; ++j) (void)hipEventDestroy(t->events[j]);
            delete[] t->events;
            delete t;
            return GQA_ERR_LAUNCH;
        }
    }
    *host_out = t;
    return GQA_OK;
}

void gqa_timer_destroy(gqa_timer* timer) {
    if (timer == nullptr) return;
    for (size_t i = 0; i < 3 * (size_t)timer->max_calls; ++i) (void)hipEventDestroy(timer->events[i]);
    delete[] timer->events;
    delete timer;
}

int gqa_timer_read(gqa_timer* timer, int32_t* host_calls, float host_kernel_ms[2]) {
    if (timer == nullptr || host_kernel_ms == nullptr) return GQA_ERR_INVALID_ARG;
    host_kernel_ms[0] = host_kernel_ms[1] = 0.f;
    int status = GQA_OK;
    if (timer->calls > 0 &&
        hipEventSynchronize(timer->events[3 * (size_t)timer->calls - 1]) != hipSuccess)
        status = GQA_ERR_LAUNCH;
    for (int c = 0; c < timer->calls && status == GQA_OK; ++c)
        for (int i = 0; i < 2; ++i) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, timer->events[3 * (size_t)c + i],
                                    timer->events[3 * (size_t)c + i + 1]) != hipSuccess) {
                status = GQA_ERR_LAUNCH;
                break;
            }
            host_kernel_ms[i] += ms;
        }
    if (host_calls) *host_calls = timer->calls;
    timer->calls = 0;
    return status;
}

int gqa_timer_read_calls(gqa_timer* timer, int32_t capacity, int32_t* host_calls,
                         float* host_partial_ms, float* host_combine_ms) {
    if (timer == nullptr || capacity < 0 || timer->calls > capacity) return GQA_ERR_INVALID_ARG;
    int status = GQA_OK;
    if (timer->calls > 0 &&
        hipEventSynchronize(timer->events[3 * (size_t)timer->calls - 1]) != hipSuccess)
        status = GQA_ERR_LAUNCH;
    for (int c = 0; c < timer->calls && status == GQA_OK; ++c) {
        float* dst[2] = {host_partial_ms, host_combine_ms};
        for (int i = 0; i < 2; ++i) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, timer->events[3 * (size_t)c + i],
                                    timer->events[3 * (size_t)c + i + 1]) != hipSuccess) {
                status = GQA_ERR_LAUNCH;
                break;
            }
            if (dst[i] != nullptr) dst[i][c] = ms;
        }
    }
    if (host_calls) *host_calls = timer->calls;
    timer->calls = 0;
    return status;
}

namespace {

struct CascadePlan {
    int64_t max_cost;        // upper bound of the stream's length on the cost axis
    int64_t prefix_slots, suffix_slots;
    size_t header_bytes, entry_bytes, ml_prefix_bytes, o_prefix_bytes, ml_bytes, o_bytes;
    size_t total_bytes() const {
        return header_bytes + entry_bytes + ml_prefix_bytes + o_prefix_bytes + ml_bytes + o_bytes;
    }
};

int make_cascade_plan(const gqa_cascade_params* cp, CascadePlan* plan) {
    if (cp == nullptr) return GQA_ERR_INVALID_ARG;
    const gqa_decode_params* p = &cp->decode;
    const int rc = check_shape(p);
    if (rc != GQA_OK) return rc;
    if (p->kernel_variant != 0) return GQA_ERR_UNSUPPORTED;
    if (cp->num_groups < 1 || cp->num_groups > p->batch || cp->max_prefix_len < 0) return GQA_ERR_INVALID_ARG;
    const int64_t entries = (int64_t)cp->num_groups + p->batch;
    plan->max_cost = (int64_t)p->num_kv_heads *
        ((int64_t)cp->num_groups * gqa::tiles_of(cp->max_prefix_len) * 2 * gqa::kCascadeMaxTileCost +      // two reads at most
         (int64_t)p->batch * gqa::tiles_of(p->max_kv_len) * gqa::cascade_tile_cost(1));
    if (plan->max_cost > 0x3fffffffLL) return GQA_ERR_UNSUPPORTED;      // positions on the cost axis are int32
    int64_t shares = kMaxWorkers;
    const int fixed = p->chunk_tokens / gqa::kTileTokens;
    if (fixed > 0) {
        const int64_t sc = gqa::cascade_share_cost(0, fixed, 1);
        if ((plan->max_cost + sc - 1) / sc > shares) shares = (plan->max_cost + sc - 1) / sc;
    }
    // a piece of a prefix row goes to slot share + 2 (group * Hkv + g) + read, a piece of a suffix row to share + b * Hkv + g
    plan->prefix_slots = shares + 2 * (int64_t)cp->num_groups * p->num_kv_heads;
    plan->suffix_slots = shares + (int64_t)p->batch * p->num_kv_heads;
    plan->header_bytes = 256;
    plan->entry_bytes = align_up(sizeof(int32_t) * ((size_t)entries + 1), 256);
    plan->ml_prefix_bytes = align_up((size_t)plan->prefix_slots * 32 * 2 * sizeof(float), 256);
    plan->o_prefix_bytes = align_up((size_t)plan->prefix_slots * 32 * gqa::kHeadDim * sizeof(float), 256);
    plan->ml_bytes = align_up((size_t)plan->suffix_slots * 16 * 2 * sizeof(float), 256);
    plan->o_bytes = align_up((size_t)plan->suffix_slots * 16 * gqa::kHeadDim * sizeof(float), 256);
    return GQA_OK;
}

}  // namespace

size_t gqa_cascade_workspace_bytes(const gqa_cascade_params* params) {
    CascadePlan plan;
    if (make_cascade_plan(params, &plan) != GQA_OK) return 0;
    return plan.total_bytes();
}

int gqa_decode_attn_shared_prefix(const gqa_cascade_params* cp, const void* q, const void* k_prefix,
                                  const void* v_prefix, const int32_t* prefix_lens, const int32_t* group_start,
                                  const int32_t* host_group_start, const void* k, const void* v,
                                  const int32_t* kv_lens, const int32_t* block_table, float* out, float* lse,
                                  void* workspace, size_t workspace_bytes, void* stream) {
    CascadePlan plan;
    const int rc = make_cascade_plan(cp, &plan);
    if (rc != GQA_OK) return rc;
    const gqa_decode_params* p = &cp->decode;
    if (!q || !k_prefix || !v_prefix || !prefix_lens || !group_start || !host_group_start || !k || !v ||
        !kv_lens || !out || !workspace)
        return GQA_ERR_INVALID_ARG;
    if ((p->page_size != 0) != (block_table != nullptr)) return GQA_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(k_prefix) || !aligned16(v_prefix) ||
        !aligned16(out))
        return GQA_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return GQA_ERR_INVALID_ARG;
    if (!mult8(p->q_stride_b) || !mult8(p->q_stride_h) || !mult8(p->k_stride_b) || !mult8(p->k_stride_h) ||
        !mult8(p->k_stride_t) || !mult8(p->v_stride_b) || !mult8(p->v_stride_h) || !mult8(p->v_stride_t) ||
        !mult8(cp->kp_stride_g) || !mult8(cp->kp_stride_h) || !mult8(cp->kp_stride_t) ||
        !mult8(cp->vp_stride_g) || !mult8(cp->vp_stride_h) || !mult8(cp->vp_stride_t))
        return GQA_ERR_INVALID_ARG;
    if (p->k_stride_t < gqa::kHeadDim || p->v_stride_t < gqa::kHeadDim || p->q_stride_h < gqa::kHeadDim ||
        cp->kp_stride_t < gqa::kHeadDim || cp->vp_stride_t < gqa::kHeadDim)
        return GQA_ERR_INVALID_ARG;
    const int group = p->num_q_heads / p->num_kv_heads;
    if (host_group_start[0] != 0 || host_group_start[cp->num_groups] != p->batch) return GQA_ERR_INVALID_ARG;
    for (int j = 0; j < cp->num_groups; ++j) {
        const int64_t m = (int64_t)host_group_start[j + 1] - host_group_start[j];
        if (m < 0) return GQA_ERR_INVALID_ARG;
        if (m * group > gqa::kCascadeColumns) return GQA_ERR_UNSUPPORTED;
    }
    if (workspace_bytes < plan.total_bytes()) return GQA_ERR_WORKSPACE_TOO_SMALL;

    gqa::CascadeArgs ca{};
    KernelArgs& a = ca.base;
    a.q = static_cast<const uint16_t*>(q);
    a.k = static_cast<const uint16_t*>(k);
    a.v = static_cast<const uint16_t*>(v);
    a.kv_lens = kv_lens;
    a.block_table = block_table;
    char* ws = static_cast<char*>(workspace);
    a.header = reinterpret_cast<int32_t*>(ws);
    a.row_prefix = reinterpret_cast<int32_t*>(ws + plan.header_bytes);
    size_t at = plan.header_bytes + plan.entry_bytes;
    ca.part_ml_prefix = reinterpret_cast<float*>(ws + at); at += plan.ml_prefix_bytes;
    ca.part_o_prefix = reinterpret_cast<float*>(ws + at);  at += plan.o_prefix_bytes;
    a.part_ml = reinterpret_cast<float*>(ws + at);         at += plan.ml_bytes;
    a.part_o = reinterpret_cast<float*>(ws + at);
    a.out = out;
    a.lse = lse;
    a.batch = p->batch;
    a.num_q_heads = p->num_q_heads;
    a.num_kv_heads = p->num_kv_heads;
    a.group = group;
    a.max_kv_len = p->max_kv_len;
    a.fixed_share_tiles = p->chunk_tokens / gqa::kTileTokens;
    a.page_size = p->page_size;
    a.page_shift = 0;
    while (p->page_size > 1 && (1 << a.page_shift) < p->page_size) ++a.page_shift;
    a.block_table_stride = p->block_table_stride;
    a.q_stride_b = p->q_stride_b; a.q_stride_h = p->q_stride_h;
    a.k_stride_b = p->k_stride_b; a.k_stride_h = p->k_stride_h; a.k_stride_t = p->k_stride_t;
    a.v_stride_b = p->v_stride_b; a.v_stride_h = p->v_stride_h; a.v_stride_t = p->v_stride_t;
    a.scale_log2e = p->scale * 1.4426950408889634f;
    ca.kp = static_cast<const uint16_t*>(k_prefix);
    ca.vp = static_cast<const uint16_t*>(v_prefix);
    ca.prefix_lens = prefix_lens;
    ca.group_start = group_start;
    ca.num_groups = cp->num_groups;
    ca.max_prefix_len = cp->max_prefix_len;
    ca.kp_stride_g = cp->kp_stride_g; ca.kp_stride_h = cp->kp_stride_h; ca.kp_stride_t = cp->kp_stride_t;
    ca.vp_stride_g = cp->vp_stride_g; ca.vp_stride_h = cp->vp_stride_h; ca.vp_stride_t = cp->vp_stride_t;

    int workgroups = workgroups_for(0);
    if (workgroups < 1) return GQA_ERR_LAUNCH;
    // no more workgroups than the stream can feed with shares of the minimum cost
    const int64_t per_group_cost = (int64_t)gqa::cascade_share_cost(0, 0, 1) * gqa::partial_cascade_workers_per_group();
    const int64_t useful = (plan.max_cost + per_group_cost - 1) / per_group_cost;
    if (useful < workgroups) workgroups = (int)(useful > 0 ? useful : 1);
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (gqa::launch_partial_cascade(ca, workgroups, s) != hipSuccess) return GQA_ERR_LAUNCH;
    if (gqa::launch_combine_cascade(ca, s) != hipSuccess) return GQA_ERR_LAUNCH;
    return GQA_OK;
}

int gqa_prefill_attn(const gqa_prefill_params* p, const void* q, const void* k, const void* v, float* out,
                     float* lse, void* stream) {
    return gqa_prefill_attn_varlen(p, q, k, v, nullptr, out, lse, stream);
}

int gqa_prefill_attn_varlen(const gqa_prefill_params* p, const void* q, const void* k, const void* v,
                            const int32_t* seq_lens, float* out, float* lse, void* stream) {
    if (p == nullptr) return GQA_ERR_INVALID_ARG;
    if (p->batch < 1 || p->seq_len < 1 || p->num_q_heads < 1 || p->num_kv_heads < 1) return GQA_ERR_INVALID_ARG;
    if (p->num_q_heads % p->num_kv_heads != 0 || !std::isfinite(p->scale)) return GQA_ERR_INVALID_ARG;
    if (p->head_dim != gqa::kHeadDim) return GQA_ERR_UNSUPPORTED;
    const int group = p->num_q_heads / p->num_kv_heads;
    if (group > gqa::kMaxGroup) return GQA_ERR_UNSUPPORTED;
    if (!q || !k || !v || !out) return GQA_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return GQA_ERR_INVALID_ARG;
    if (!mult8(p->q_stride_b) || !mult8(p->q_stride_t) || !mult8(p->q_stride_h) || !mult8(p->k_stride_b) ||
        !mult8(p->k_stride_t) || !mult8(p->k_stride_h) || !mult8(p->v_stride_b) || !mult8(p->v_stride_t) ||
        !mult8(p->v_stride_h) || p->o_stride_b % 4 != 0 || p->o_stride_t % 4 != 0 || p->o_stride_h % 4 != 0)
        return GQA_ERR_INVALID_ARG;
    const int64_t blocks = ((int64_t)p->seq_len + 255) / 256;
    if (8 * blocks * group * ((p->num_kv_heads + 7) / 8) * p->batch > 0x7fffffffLL) return GQA_ERR_UNSUPPORTED;
    gqa::PrefillArgs a{};
    a.q = static_cast<const uint16_t*>(q);
    a.k = static_cast<const uint16_t*>(k);
    a.v = static_cast<const uint16_t*>(v);
    a.out = out;
    a.lse = lse;
    a.seq_lens = seq_lens;
    a.batch = p->batch; a.seq_len = p->seq_len;
    a.num_q_heads = p->num_q_heads; a.num_kv_heads = p->num_kv_heads; a.group = group;
    a.q_stride_b = p->q_stride_b; a.q_stride_t = p->q_stride_t; a.q_stride_h = p->q_stride_h;
    a.k_stride_b = p->k_stride_b; a.k_stride_t = p->k_stride_t; a.k_stride_h = p->k_stride_h;
    a.v_stride_b = p->v_stride_b; a.v_stride_t = p->v_stride_t; a.v_stride_h = p->v_stride_h;
    a.o_stride_b = p->o_stride_b; a.o_stride_t = p->o_stride_t; a.o_stride_h = p->o_stride_h;
    a.scale_log2e = p->scale * 1.4426950408889634f;
    return gqa::launch_prefill(a, static_cast<hipStream_t>(stream)) == hipSuccess ? GQA_OK : GQA_ERR_LAUNCH;
}

int gqa_decode_kv_append(const gqa_append_params* p, const void* q_in, void* q_out, const void* k_new,
                         const void* v_new, void* k_cache, void* v_cache, const int32_t* kv_lens,
                         const int32_t* block_table, const float* cos_sin, void* stream) {
    if (p == nullptr) return GQA_ERR_INVALID_ARG;
    if (p->batch < 1 || p->num_q_heads < 1 || p->num_kv_heads < 1 || p->max_kv_len < 0 || p->page_size < 0)
        return GQA_ERR_INVALID_ARG;
    if (p->head_dim != gqa::kHeadDim) return GQA_ERR_UNSUPPORTED;
    if (p->page_size != 0) {
        if (p->page_size < 16 || (p->page_size & (p->page_size - 1)) != 0) return GQA_ERR_UNSUPPORTED;
        if ((int64_t)p->block_table_stride * p->page_size < p->max_kv_len) return GQA_ERR_INVALID_ARG;
    }
    if (!q_in || !q_out || !k_new || !v_new || !k_cache || !v_cache || !kv_lens) return GQA_ERR_INVALID_ARG;
    if ((p->page_size != 0) != (block_table != nullptr)) return GQA_ERR_INVALID_ARG;
    if (cos_sin != nullptr && p->rope_positions < p->max_kv_len) return GQA_ERR_INVALID_ARG;
    if (p->k_stride_t < gqa::kHeadDim || p->v_stride_t < gqa::kHeadDim || p->q_stride_h < gqa::kHeadDim)
        return GQA_ERR_INVALID_ARG;
    gqa::AppendArgs a{};
    a.q_in = static_cast<const uint16_t*>(q_in);
    a.q_out = static_cast<uint16_t*>(q_out);
    a.k_new = static_cast<const uint16_t*>(k_new);
    a.v_new = static_cast<const uint16_t*>(v_new);
    a.k_cache = static_cast<uint16_t*>(k_cache);
    a.v_cache = static_cast<uint16_t*>(v_cache);
    a.kv_lens = kv_lens;
    a.block_table = block_table;
    a.cos_sin = cos_sin;
    a.batch = p->batch; a.num_q_heads = p->num_q_heads; a.num_kv_heads = p->num_kv_heads;
    a.max_kv_len = p->max_kv_len;
    a.page_size = p->page_size; a.block_table_stride = p->block_table_stride;
    a.q_stride_b = p->q_stride_b; a.q_stride_h = p->q_stride_h;
    a.k_stride_b = p->k_stride_b; a.k_stride_h = p->k_stride_h; a.k_stride_t = p->k_stride_t;
    a.v_stride_b = p->v_stride_b; a.v_stride_h = p->v_stride_h; a.v_stride_t = p->v_stride_t;
    return gqa::launch_kv_append(a, static_cast<hipStream_t>(stream)) == hipSuccess ? GQA_OK : GQA_ERR_LAUNCH;
}

int gqa_decode_stream_read(const void* src, size_t bytes, void* sink, int32_t workgroups, void* stream) {
    if (!src || !sink || workgroups < 1 || bytes % 16 != 0 || !aligned16(src)) return GQA_ERR_INVALID_ARG;
    return gqa::launch_stream_read(src, bytes, sink, workgroups, static_cast<hipStream_t>(stream)) == hipSuccess
               ? GQA_OK : GQA_ERR_LAUNCH;
}

int gqa_decode_stream_probe(const void* src, size_t bytes, void* sink, int32_t workgroups, int32_t mode, void* stream) {
    if (!src || !sink || workgroups < 1 || workgroups > 4096 || bytes < 16384 || bytes / 16384 > 0x7fffffffULL ||
        !aligned16(src) || mode < 0 || mode > 9)
        return GQA_ERR_INVALID_ARG;
    return gqa::launch_stream_probe(src, bytes, sink, workgroups, mode, static_cast<hipStream_t>(stream)) == hipSuccess
               ? GQA_OK : GQA_ERR_LAUNCH;
}

int gqa_decode_stream_copy(const void* src, void* dst, size_t bytes, int32_t workgroups, void* stream) {
    if (!src || !dst || workgroups < 1 || bytes % 16 != 0 || !aligned16(src) || !aligned16(dst))
        return GQA_ERR_INVALID_ARG;
    return gqa::launch_stream_copy(src, dst, bytes, workgroups, static_cast<hipStream_t>(stream)) == hipSuccess
               ? GQA_OK : GQA_ERR_LAUNCH;
}

}  // extern "C"
