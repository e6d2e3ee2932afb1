// Internal declarations shared by the translation units of libgqa_decode.so.
// Nothing here is visible across the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gqa {

constexpr int kHeadDim = 128;        // the only supported head size
constexpr int kMaxGroup = 16;        // query heads per KV head served by one K/V read
constexpr int kTileTokens = 64;      // granularity of chunk_tokens (one workgroup step)

// Device-side view of one call.  Strides are in bf16 elements.
struct KernelArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const int32_t* kv_lens;
    const int32_t* block_table;
    int32_t* chunk_offset;   // [batch + 1] running sum of per-sequence split counts
    int4* work_list;         // [split f] = (b, t_begin, t_end, 0), written by the plan kernel
    float* part_ml;          // [work item][G][2]  running max (log2 domain) and normaliser
    float* part_o;           // [work item][G][D]  unnormalised weighted value sum
    float* out;
    float* lse;
    int32_t batch, num_q_heads, num_kv_heads, group;
    int32_t max_kv_len;      // lengths read on the device are clamped to this bound
    int32_t chunk_tokens, page_size, page_shift, block_table_stride;
    int64_t q_stride_b, q_stride_h;
    int64_t k_stride_b, k_stride_h, k_stride_t;
    int64_t v_stride_b, v_stride_h, v_stride_t;
    float scale_log2e;       // scale * log2(e): the softmax runs on base-2 exponentials
};

// Work item w = (flat split index f, kv head g) with w = f * Hkv + g; f counts the
// splits of all sequences in order, chunk_offset[b] being the first split of b.
struct WorkItem {
    int b, g, t_begin, t_end;
    bool valid;
};

__device__ __forceinline__ WorkItem locate_work_item(const KernelArgs& a, int w) {
    WorkItem it;
    it.g = w % a.num_kv_heads;
    const int f = w / a.num_kv_heads;
    const int32_t* __restrict__ off = a.chunk_offset;
    it.valid = f < off[a.batch];
    it.b = 0; it.t_begin = 0; it.t_end = 0;
    if (!it.valid) return it;
    const int4 e = reinterpret_cast<const int4* __restrict__>(a.work_list)[f];
    it.b = e.x; it.t_begin = e.y; it.t_end = e.z;
    return it;
}

// Launchers (each checks nothing: the C-ABI layer validated the arguments).
hipError_t launch_plan(const KernelArgs& a, hipStream_t s);
hipError_t launch_partial_valu(const KernelArgs& a, int64_t work_items, hipStream_t s);
hipError_t launch_partial_mfma(const KernelArgs& a, int64_t work_items, hipStream_t s);
hipError_t launch_combine(const KernelArgs& a, hipStream_t s);
hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, int workgroups, hipStream_t s);

}  // namespace gqa
