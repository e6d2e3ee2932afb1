// Internal declarations shared by the translation units of libgqa_decode.so.
// Nothing here is visible across the C ABI.
//
// Work decomposition ("stream split").  A row is one (sequence b, kv head g)
// pair, r = b * Hkv + g, and owns tiles(b) = ceil(kv_len[b] / 32) tiles of 32
// tokens.  All rows are laid end to end, in order of r, into one stream of
// `total` tiles.  The stream is cut into shares of `share_tiles` tiles; share s
// covers stream positions [s * share_tiles, (s + 1) * share_tiles).  A share
// that crosses row boundaries consists of several pieces, one per row; each
// piece produces one partial result (running maximum, normaliser, weighted value
// sum) in slot s + r, which is unique because s + r grows along the stream.
// The combine kernel merges, for every row, the slots of the shares that touch
// it.  With one share per persistent worker (a wavefront of the matrix-core
// kernel, a workgroup of the vector-ALU kernel) every worker streams the same
// number of bytes whatever the mix of sequence lengths.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gqa {

constexpr int kHeadDim = 128;        // the only supported head size
constexpr int kMaxGroup = 16;        // query heads per KV head served by one K/V read
constexpr int kTileTokens = 32;      // one MFMA tile; the unit of the stream split
constexpr int kChunkGranule = 32;    // chunk_tokens must be a multiple of this
constexpr int kMinShareTiles = 2;    // shares are never shorter than this (64 tokens)
constexpr int kThreads = 256;        // workgroup size of the partial kernels

// Device-side view of one call.  Strides are in bf16 elements.
struct KernelArgs {
    const uint16_t* q;
    const uint16_t* k;
    const uint16_t* v;
    const int32_t* kv_lens;
    const int32_t* block_table;
    int32_t* header;         // [0] total tiles, [1] share_tiles, written by workgroup 0 of the partial kernel
    int32_t* row_prefix;     // [batch + 1] stream position of row (b, 0), written likewise
    float* part_ml;          // [slot][G][2]  running max (log2 domain) and normaliser
    float* part_o;           // [slot][G][D]  unnormalised weighted value sum
    float* out;
    float* lse;
    int32_t batch, num_q_heads, num_kv_heads, group;
    int32_t max_kv_len;      // lengths read on the device are clamped to [0, max_kv_len]
    int32_t fixed_share_tiles;   // > 0: shares of exactly this many tiles; 0: total / workers
    int32_t page_size, page_shift, block_table_stride;
    int64_t q_stride_b, q_stride_h;
    int64_t k_stride_b, k_stride_h, k_stride_t;
    int64_t v_stride_b, v_stride_h, v_stride_t;
    float scale_log2e;       // scale * log2(e): the softmax runs on base-2 exponentials
};

__device__ __forceinline__ int clamped_len(const KernelArgs& a, int b) {
    return min(max(a.kv_lens[b], 0), a.max_kv_len);
}

// Read-only int32 at a wavefront-uniform index through the scalar data path (constant address
// space): the value lands in an SGPR and the load is tracked by lgkmcnt, so it neither occupies a
// slot among the K/V vector loads in flight nor forces a wait on them.  Only for arrays the kernel
// never writes (kv_lens, block_table).
__device__ __forceinline__ int uniform_i32(const int32_t* base, int64_t index) {
    typedef const __attribute__((address_space(4))) int32_t* const_ptr;
    return reinterpret_cast<const_ptr>(reinterpret_cast<uintptr_t>(base))[index];
}
__device__ __forceinline__ int uniform_len(const KernelArgs& a, int b) {
    return min(max(uniform_i32(a.kv_lens, b), 0), a.max_kv_len);
}
__host__ __device__ __forceinline__ int tiles_of(int len) { return (len + kTileTokens - 1) / kTileTokens; }

__host__ __device__ __forceinline__ int share_tiles_for(int64_t total, int fixed, int workers) {
    if (fixed > 0) return fixed;
    const int64_t per = (total + workers - 1) / workers;
    return (int)(per < kMinShareTiles ? kMinShareTiles : per);
}

// Inclusive scan over the 256 threads of a workgroup (wave shuffles, one LDS hop).
// `scratch` holds at least 4 ints.  Also returns the workgroup total.
__device__ __forceinline__ int block_scan_256(int x, int* scratch, int& block_total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = x;
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(incl, o);
        if (lane >= o) incl += y;
    }
    __syncthreads();                       // scratch may still be read from a previous use
    if (lane == 63) scratch[wave] = incl;
    __syncthreads();
    int before = 0;
    for (int w = 0; w < 4; ++w) before += (w < wave) ? scratch[w] : 0;
    block_total = scratch[0] + scratch[1] + scratch[2] + scratch[3];
    return incl + before;
}

// Sum over all sequences of Hkv * tiles(b): the length of the stream.
__device__ __forceinline__ int stream_total(const KernelArgs& a, int* scratch) {
    int carry = 0;
    for (int base = 0; base < a.batch; base += kThreads) {
        const int b = base + (int)threadIdx.x;
        const int n = (b < a.batch) ? a.num_kv_heads * tiles_of(clamped_len(a, b)) : 0;
        int tot;
        (void)block_scan_256(n, scratch, tot);
        carry += tot;
    }
    return carry;
}

// Position in the stream -> (sequence, kv head, tile within the row).  Every thread
// of the workgroup must call it; the answer is broadcast through `found` (3 ints).
// If `prefix_out` is given, also writes the stream position of every sequence.
struct StreamPos { int b, g, tile, len; };

__device__ __forceinline__ StreamPos stream_locate(const KernelArgs& a, int pos, int* scratch, int* found,
                                                   int32_t* prefix_out) {
    int carry = 0;
    for (int base = 0; base < a.batch; base += kThreads) {
        const int b = base + (int)threadIdx.x;
        const int tb = (b < a.batch) ? tiles_of(clamped_len(a, b)) : 0;
        const int n = a.num_kv_heads * tb;
        int tot;
        const int excl = carry + block_scan_256(n, scratch, tot) - n;
        if (prefix_out != nullptr && b < a.batch) prefix_out[b] = excl;
        if (n > 0 && excl <= pos && pos < excl + n) {
            found[0] = b;
            found[1] = (pos - excl) / tb;
            found[2] = (pos - excl) % tb;
        }
        carry += tot;
    }
    if (prefix_out != nullptr && threadIdx.x == 0) prefix_out[a.batch] = carry;
    __syncthreads();
    StreamPos p;
    p.b = found[0]; p.g = found[1]; p.tile = found[2];
    p.len = clamped_len(a, p.b);
    return p;
}

// Wavefront-level versions (64 lanes, no barrier, no LDS): every lane of the
// calling wavefront must be active.
__device__ __forceinline__ int wave_scan_incl(int x) {
    const int lane = threadIdx.x & 63;
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(x, o);
        if (lane >= o) x += y;
    }
    return x;
}

__device__ __forceinline__ int wave_stream_total(const KernelArgs& a) {
    const int lane = threadIdx.x & 63;
    int carry = 0;
    for (int base = 0; base < a.batch; base += 64) {
        const int b = base + lane;
        const int n = (b < a.batch) ? a.num_kv_heads * tiles_of(clamped_len(a, b)) : 0;
        carry += __shfl(wave_scan_incl(n), 63);
    }
    return carry;
}

__device__ __forceinline__ StreamPos wave_stream_locate(const KernelArgs& a, int pos, int32_t* prefix_out) {
    const int lane = threadIdx.x & 63;
    int carry = 0;
    StreamPos p;
    p.b = 0; p.g = 0; p.tile = 0; p.len = 0;
    for (int base = 0; base < a.batch; base += 64) {
        const int b = base + lane;
        const int len = (b < a.batch) ? clamped_len(a, b) : 0;
        const int tb = tiles_of(len);
        const int n = a.num_kv_heads * tb;
        const int incl = wave_scan_incl(n);
        const int excl = carry + incl - n;
        if (prefix_out != nullptr && b < a.batch) prefix_out[b] = excl;
        const bool hit = n > 0 && excl <= pos && pos < excl + n;
        const unsigned long long mask = __builtin_amdgcn_ballot_w64(hit);
        if (mask != 0) {                                  // at most one lane hits
            const int src = __builtin_ctzll(mask);
            const int tbs = __shfl(tb, src), ex = __shfl(excl, src);
            p.b = base + src;
            p.g = (pos - ex) / tbs;
            p.tile = (pos - ex) % tbs;
            p.len = __shfl(len, src);
        }
        carry += __shfl(incl, 63);
    }
    if (prefix_out != nullptr && lane == 0) prefix_out[a.batch] = carry;
    return p;
}

// Device-side view of one shared-prefix ("cascade") call: `base` describes the queries, the
// per-sequence suffix caches (kv_lens = suffix lengths), the outputs and the suffix area of the
// partial results (16 columns per slot); the prefix of group j lives at
// kp + j*kp_stride_g + g*kp_stride_h + t*kp_stride_t and its pieces go to the prefix area (32
// columns per slot).  base.row_prefix holds entries + 1 ints (entries = num_groups prefixes, then
// batch suffixes): the position of every entry on the cost axis of the stream split.
constexpr int kCascadeColumns = 64;      // query rows (samples x heads of a KV group) a group may have
#ifndef GQA_CASCADE_COST_TILE            // cost of a tile with one column block (reading it dominates)
#define GQA_CASCADE_COST_TILE 8
#endif
#ifndef GQA_CASCADE_COST_BLOCK           // cost of every further column block served from the same read
#define GQA_CASCADE_COST_BLOCK 1
#endif
constexpr int kCascadeMaxTileCost = GQA_CASCADE_COST_TILE + GQA_CASCADE_COST_BLOCK;     // two column blocks per read
__host__ __device__ __forceinline__ int cascade_tile_cost(int nb) {
    return GQA_CASCADE_COST_TILE + GQA_CASCADE_COST_BLOCK * (nb - 1);
}
// Cost units per share: the total cut into equal parts (never below two plain tiles), or a fixed
// number of plain tiles; in both cases at least the largest tile cost, so that consecutive shares
// inside a row each own a tile of it.
__host__ __device__ __forceinline__ int cascade_share_cost(int64_t total, int fixed_tiles, int workers) {
    int64_t c = fixed_tiles > 0 ? (int64_t)fixed_tiles * GQA_CASCADE_COST_TILE : (total + workers - 1) / workers;
    const int64_t floor_cost = kMinShareTiles * GQA_CASCADE_COST_TILE > kCascadeMaxTileCost
                                   ? kMinShareTiles * GQA_CASCADE_COST_TILE : kCascadeMaxTileCost;
    if (c < floor_cost) c = floor_cost;
    return (int)c;
}
struct CascadeArgs {
    KernelArgs base;
    const uint16_t* kp;
    const uint16_t* vp;
    const int32_t* prefix_lens;      // [num_groups]
    const int32_t* group_start;      // [num_groups + 1], sequences of group j: [group_start[j], group_start[j+1])
    float* part_ml_prefix;           // [slot][32][2]
    float* part_o_prefix;            // [slot][32][D]
    int32_t num_groups, max_prefix_len;
    int64_t kp_stride_g, kp_stride_h, kp_stride_t;
    int64_t vp_stride_g, vp_stride_h, vp_stride_t;
};
hipError_t launch_partial_cascade(const CascadeArgs& ca, int workgroups, hipStream_t s);
hipError_t launch_combine_cascade(const CascadeArgs& ca, hipStream_t s);
int partial_cascade_workers_per_group();

// Device-side view of one causal prefill call.  Strides in elements (bf16 for q/k/v, fp32 for out).
struct PrefillArgs {
    const uint16_t* q;       // [batch, seq, Hq, D] via strides
    const uint16_t* k;       // [batch, seq, Hkv, D]
    const uint16_t* v;
    float* out;              // [batch, seq, Hq, D] via strides
    float* lse;              // [batch, seq, Hq] dense, may be null
    const int32_t* seq_lens; // [batch] tokens per sequence (clamped to [0, seq_len]), null: all have seq_len
    int32_t batch, seq_len, num_q_heads, num_kv_heads, group;   // seq_len: the padded length T of the tensors
    int64_t q_stride_b, q_stride_t, q_stride_h;
    int64_t k_stride_b, k_stride_t, k_stride_h;
    int64_t v_stride_b, v_stride_t, v_stride_h;
    int64_t o_stride_b, o_stride_t, o_stride_h;
    float scale_log2e;
};
hipError_t launch_prefill(const PrefillArgs& a, hipStream_t s);
hipError_t prepare_prefill();      // per-device set-up of the prefill kernel (idempotent)

// Device-side view of one append call.
struct AppendArgs {
    const uint16_t* q_in;
    uint16_t* q_out;
    const uint16_t* k_new;   // [batch, Hkv, D] dense
    const uint16_t* v_new;
    uint16_t* k_cache;
    uint16_t* v_cache;
    const int32_t* kv_lens;
    const int32_t* block_table;
    const float* cos_sin;    // [positions, D]: cos in columns [0, D/2), sin in [D/2, D); may be null
    int32_t batch, num_q_heads, num_kv_heads, max_kv_len;
    int32_t page_size, block_table_stride;
    int64_t q_stride_b, q_stride_h;
    int64_t k_stride_b, k_stride_h, k_stride_t;
    int64_t v_stride_b, v_stride_h, v_stride_t;
};
hipError_t launch_kv_append(const AppendArgs& a, hipStream_t s);

// Launchers (each checks nothing: the C-ABI layer validated the arguments).
hipError_t launch_partial_valu(const KernelArgs& a, int workgroups, hipStream_t s);
hipError_t launch_partial_mfma(const KernelArgs& a, int workgroups, hipStream_t s);
hipError_t launch_combine(const KernelArgs& a, int workgroups, hipStream_t s);
hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, int workgroups, hipStream_t s);
hipError_t launch_stream_copy(const void* src, void* dst, size_t bytes, int workgroups, hipStream_t s);
hipError_t launch_stream_probe(const void* src, size_t bytes, void* sink, int workgroups, int mode, hipStream_t s);
int partial_mfma_occupancy();   // resident workgroups per CU (from the HIP occupancy query)
int partial_valu_occupancy();
int partial_mfma_workers_per_group();     // independent wavefronts per workgroup of the matrix-core kernel
constexpr int kMaxWorkersPerGroup = 8;

}  // namespace gqa
