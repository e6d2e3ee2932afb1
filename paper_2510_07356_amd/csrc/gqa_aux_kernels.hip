// Log-sum-exp combine and the streaming-read probe.
#include "gqa_internal.h"

namespace gqa {

// ---------------------------------------------------------------------------
// Combine: for each output row (b, h) merge the partial results of the shares
// that touch row (b, g(h)) of the stream split (slots s + r for s from the share
// holding the row's first tile to the share holding its last):
//   M = max_c m_c,  w_c = 2^(m_c - M),
//   out = sum_c w_c o_c / sum_c w_c l_c,   lse = ln 2 * (M + log2 sum_c w_c l_c).
// One wavefront per row, two columns per lane; pieces are merged in stream order
// with a running maximum, eight at a time so that their loads are in flight
// together.  The stream geometry (header, row_prefix) was written by the
// partial kernel.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void combine_kernel(KernelArgs a) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.batch * a.num_q_heads) return;
    const int b = row / a.num_q_heads, h = row % a.num_q_heads;
    const int G = a.group, g = h / G, hh = h % G;
    const int32_t* __restrict__ hdr = a.header;
    const int32_t* __restrict__ pre = a.row_prefix;
    const int share_tiles = hdr[1];
    const int pb = pre[b];
    const int tiles_b = (pre[b + 1] - pb) / a.num_kv_heads;
    const int start = pb + g * tiles_b;
    const int r = b * a.num_kv_heads + g;
    int s_first = 0, n = 0;
    if (tiles_b > 0) {
        s_first = start / share_tiles;
        n = (start + tiles_b - 1) / share_tiles - s_first + 1;
    }
    const float2* __restrict__ ml = reinterpret_cast<const float2*>(a.part_ml);
    const float2* __restrict__ po = reinterpret_cast<const float2*>(a.part_o);
    constexpr int kBatch = 8;
    float M = -INFINITY, den = 0.f;
    float2 acc = make_float2(0.f, 0.f);
    for (int c0 = 0; c0 < n; c0 += kBatch) {
        float2 mlv[kBatch], ov[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int c = min(c0 + u, n - 1);
            const int64_t w = ((int64_t)(s_first + c) + r) * G + hh;
            mlv[u] = ml[w];
            ov[u] = po[w * (kHeadDim / 2) + lane];
        }
        float bm = M;
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (c0 + u >= n) mlv[u].x = -INFINITY;       // duplicates of the last piece count once
            bm = fmaxf(bm, mlv[u].x);
        }
        const float ms = (bm == -INFINITY) ? 0.f : bm;   // keeps (-inf) - (-inf) out
        const float sa = exp2f(M - ms);
        den *= sa; acc.x *= sa; acc.y *= sa;
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const float wgt = exp2f(mlv[u].x - ms);      // an empty or absent piece gets weight 0
            den = fmaf(wgt, mlv[u].y, den);
            acc.x = fmaf(wgt, ov[u].x, acc.x);
            acc.y = fmaf(wgt, ov[u].y, acc.y);
        }
        M = bm;
    }
    const float inv = den > 0.f ? 1.f / den : 0.f;
    reinterpret_cast<float2*>(a.out)[(int64_t)row * (kHeadDim / 2) + lane] = make_float2(acc.x * inv, acc.y * inv);
    if (a.lse != nullptr && lane == 0)
        a.lse[row] = den > 0.f ? 0.6931471805599453f * (M + log2f(den)) : -INFINITY;
}

hipError_t launch_combine(const KernelArgs& a, int /*workgroups*/, hipStream_t s) {
    const int rows = a.batch * a.num_q_heads;
    hipLaunchKernelGGL(combine_kernel, dim3((rows + 3) / 4), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Streaming read probe: grid-stride non-temporal 128-bit loads, xor-folded.
// ---------------------------------------------------------------------------
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ src, size_t n16,
                                                          uint32_t* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    u32x4 acc = {0, 0, 0, 0};
    size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x;
    for (; i + 3 * 256 < n16; i += stride) {             // four independent non-temporal loads in flight
        const u32x4 x0 = __builtin_nontemporal_load(src + i), x1 = __builtin_nontemporal_load(src + i + 256);
        const u32x4 x2 = __builtin_nontemporal_load(src + i + 512), x3 = __builtin_nontemporal_load(src + i + 768);
        acc ^= x0 ^ x1 ^ x2 ^ x3;
    }
    for (; i < n16; i += 256) acc ^= __builtin_nontemporal_load(src + i);   // ragged end of the last full stride
    uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    for (int o = 32; o > 0; o >>= 1) r ^= __shfl_xor(r, o);
    __shared__ uint32_t red[4];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = r;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = red[0] ^ red[1] ^ red[2] ^ red[3];
}

hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, int workgroups, hipStream_t s) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(256), 0, s,
                       (const u32x4*)src, bytes / 16, (uint32_t*)sink);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Plain copy of n16 16-byte words (grid-stride): the known-size kernel against
// which the HBM byte counters of a profile are scaled.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stream_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                          size_t n16) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

hipError_t launch_stream_copy(const void* src, void* dst, size_t bytes, int workgroups, hipStream_t s) {
    hipLaunchKernelGGL(stream_copy_kernel, dim3(workgroups), dim3(256), 0, s,
                       (const uint4*)src, (uint4*)dst, bytes / 16);
    return hipGetLastError();
}

}  // namespace gqa
