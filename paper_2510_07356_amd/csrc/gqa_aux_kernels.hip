// Plan, log-sum-exp combine and the streaming-read probe.
#include "gqa_internal.h"

namespace gqa {

// ---------------------------------------------------------------------------
// Plan: chunk_offset[b] = sum_{b' < b} ceil(kv_lens[b'] / chunk_tokens), one
// workgroup, any batch size (tiles of 256 sequences with a running carry).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void plan_kernel(KernelArgs a) {
    __shared__ int scan[256];
    __shared__ int carry;
    const int tid = threadIdx.x;
    if (tid == 0) carry = 0;
    __syncthreads();
    for (int base = 0; base < a.batch; base += 256) {
        const int b = base + tid;
        int n = 0;
        if (b < a.batch) {
            const int len = min(max(a.kv_lens[b], 0), a.max_kv_len);
            n = (len + a.chunk_tokens - 1) / a.chunk_tokens;
        }
        scan[tid] = n;
        __syncthreads();
        for (int d = 1; d < 256; d <<= 1) {          // inclusive Hillis-Steele scan
            const int x = (tid >= d) ? scan[tid - d] : 0;
            __syncthreads();
            scan[tid] += x;
            __syncthreads();
        }
        const int incl = scan[tid];
        const int c = carry;
        if (b < a.batch) a.chunk_offset[b] = c + incl - n;
        __syncthreads();
        if (tid == 255) carry = c + incl;
        __syncthreads();
    }
    if (tid == 0) a.chunk_offset[a.batch] = carry;
}

hipError_t launch_plan(const KernelArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(256), 0, s, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Combine: for each (b, h) merge the partial results of the splits of (b, g(h)):
//   M = max_c m_c,  w_c = 2^(m_c - M),  out = sum_c w_c o_c / sum_c w_c l_c,
//   lse = ln 2 * (M + log2 sum_c w_c l_c).
// One workgroup of 128 threads (one per output column) per (b, g).
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(128) void combine_kernel(KernelArgs a) {
    const int b = blockIdx.x / a.num_kv_heads;
    const int g = blockIdx.x % a.num_kv_heads;
    const int d = threadIdx.x;
    const int G = a.group;
    const int32_t* __restrict__ off = a.chunk_offset;
    const int first = off[b];
    const int n = off[b + 1] - first;
    const float* __restrict__ ml = a.part_ml;
    const float* __restrict__ po = a.part_o;
    for (int h = 0; h < G; ++h) {
        float M = -INFINITY;
        for (int c = 0; c < n; ++c) {
            const int64_t w = (int64_t)(first + c) * a.num_kv_heads + g;
            M = fmaxf(M, ml[(w * G + h) * 2]);
        }
        float acc = 0.f, den = 0.f;
        if (M > -INFINITY) {
            for (int c = 0; c < n; ++c) {
                const int64_t w = (int64_t)(first + c) * a.num_kv_heads + g;
                const float m = ml[(w * G + h) * 2];
                const float l = ml[(w * G + h) * 2 + 1];
                const float wgt = exp2f(m - M);          // m = -inf gives 0
                den = fmaf(wgt, l, den);
                acc = fmaf(wgt, po[(w * G + h) * kHeadDim + d], acc);
            }
        }
        const int64_t row = (int64_t)b * a.num_q_heads + (int64_t)g * G + h;
        a.out[row * kHeadDim + d] = den > 0.f ? acc / den : 0.f;
        if (a.lse != nullptr && d == 0)
            a.lse[row] = den > 0.f ? 0.6931471805599453f * (M + log2f(den)) : -INFINITY;
    }
}

hipError_t launch_combine(const KernelArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(combine_kernel, dim3(a.batch * a.num_kv_heads), dim3(128), 0, s, a);
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
