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
        for (int u = 0; u < kBatch; ++u) {
            const int c = min(c0 + u, n - 1);
            const int64_t w = ((int64_t)(s_first + c) + r) * G + hh;
            mlv[u] = ml[w];
            ov[u] = po[w * (kHeadDim / 2) + lane];
        }
        for (int u = 0; u < kBatch; ++u) {
            if (c0 + u >= n) break;
            const float m = mlv[u].x;
            if (m == -INFINITY) continue;            // an empty piece contributes nothing
            const float Mn = fmaxf(M, m);
            const float sa = exp2f(M - Mn), sb = exp2f(m - Mn);
            den = den * sa + mlv[u].y * sb;
            acc.x = acc.x * sa + ov[u].x * sb;
            acc.y = acc.y * sa + ov[u].y * sb;
            M = Mn;
        }
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
// Streaming read probe: grid-stride 128-bit loads, xor-folded.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src, size_t n16,
                                                          uint32_t* __restrict__ sink) {
    const size_t stride = (size_t)gridDim.x * 256 * 4;
    uint4 acc = make_uint4(0, 0, 0, 0);
    size_t i = (size_t)blockIdx.x * 256 * 4 + threadIdx.x;
    for (; i + 3 * 256 < n16; i += stride) {             // four independent loads in flight
        const uint4 x0 = src[i], x1 = src[i + 256], x2 = src[i + 512], x3 = src[i + 768];
        acc.x ^= x0.x ^ x1.x ^ x2.x ^ x3.x;
        acc.y ^= x0.y ^ x1.y ^ x2.y ^ x3.y;
        acc.z ^= x0.z ^ x1.z ^ x2.z ^ x3.z;
        acc.w ^= x0.w ^ x1.w ^ x2.w ^ x3.w;
    }
    for (; i < n16; i += 256) {                          // ragged end of the last full stride
        const uint4 x = src[i];
        acc.x ^= x.x; acc.y ^= x.y; acc.z ^= x.z; acc.w ^= x.w;
    }
    uint32_t r = acc.x ^ acc.y ^ acc.z ^ acc.w;
    for (int o = 32; o > 0; o >>= 1) r ^= __shfl_xor(r, o);
    __shared__ uint32_t red[4];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = r;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = red[0] ^ red[1] ^ red[2] ^ red[3];
}

hipError_t launch_stream_read(const void* src, size_t bytes, void* sink, int workgroups, hipStream_t s) {
    hipLaunchKernelGGL(stream_read_kernel, dim3(workgroups), dim3(256), 0, s,
                       (const uint4*)src, bytes / 16, (uint32_t*)sink);
    return hipGetLastError();
}

}  // namespace gqa
