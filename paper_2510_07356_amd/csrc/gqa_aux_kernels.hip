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
// Access-pattern probe: persistent wavefronts stream 16 KB tiles (the K or V part of one 32-token
// tile of the attention kernel: 64 rows of 256 bytes) the way a design candidate of the partial
// kernel would, with the arithmetic replaced by an xor fold.  It prices the choices of the
// partial kernel in achieved HBM bandwidth:
//   PATTERN 0  row-coalesced: one load instruction = 4 whole rows, 1 KB contiguous (the V path)
//   PATTERN 1  matrix-operand-shaped: lane (i, kb) reads 16 bytes of row 16 hf + i at byte
//              64 j + 16 kb, so a load instruction covers 16 rows x 64 bytes (the K path)
//   PATTERN 2  row-coalesced, then through LDS: written with ds_write_b128, read back in the
//              operand shape (what staging K in LDS would add)
//   NT         non-temporal loads or ordinary ones
//   TILES      tiles in flight per wavefront: 1 (registers refilled as soon as they are consumed)
//              or 2 (double-buffered)
// Every wavefront owns an equal, contiguous run of tiles, as in the stream split.
// ---------------------------------------------------------------------------
template <bool NT>
__device__ __forceinline__ u32x4 probe_load(const u32x4* p) {
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

template <int PATTERN, bool NT>
__device__ __forceinline__ void probe_request(const u32x4* tile, int lane, u32x4 (&r)[16]) {
    if (PATTERN == 1) {
        const int i = lane & 15, kb = lane >> 4;
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                r[4 * hf + j] = probe_load<NT>(tile + (16 * hf + i) * 16 + 4 * j + kb);            // rows 0..31
                r[8 + 4 * hf + j] = probe_load<NT>(tile + 512 + (16 * hf + i) * 16 + 4 * j + kb);  // rows 32..63
            }
    } else if (PATTERN == 3) {
        // the attention kernel's own mix: rows 0..31 operand-shaped (K), rows 32..63 row-coalesced (V)
        const int i = lane & 15, kb = lane >> 4;
#pragma unroll
        for (int j = 0; j < 8; ++j) r[8 + j] = probe_load<NT>(tile + 512 + 64 * j + lane);
#pragma unroll
        for (int hf = 0; hf < 2; ++hf)
#pragma unroll
            for (int j = 0; j < 4; ++j) r[4 * hf + j] = probe_load<NT>(tile + (16 * hf + i) * 16 + 4 * j + kb);
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) r[j] = probe_load<NT>(tile + 64 * j + lane);
    }
}

template <int PATTERN>
__device__ __forceinline__ u32x4 probe_consume(u32x4 (&r)[16], u32x4* lds_wave, int lane) {
    u32x4 acc = {0, 0, 0, 0};
    if (PATTERN == 2) {
        // one 16 KB tile through this wavefront's own LDS region: 1 KB per store instruction in, operand-shaped out
        const int i = lane & 15, kb = lane >> 4;
#pragma unroll
        for (int j = 0; j < 16; ++j) lds_wave[64 * j + lane] = r[j];
#pragma unroll
        for (int hf = 0; hf < 4; ++hf)
#pragma unroll
            for (int j = 0; j < 4; ++j) acc ^= lds_wave[(16 * hf + i) * 16 + 4 * j + kb];
    } else {
#pragma unroll
        for (int j = 0; j < 16; ++j) acc ^= r[j];
    }
    return acc;
}

// INTERLEAVE 0: every wavefront owns a contiguous run of tiles.  1: a workgroup owns a contiguous run and
// its 4 wavefronts take the tiles of it in turn.  2: all wavefronts take tiles in turn (the whole chip
// sweeps through memory together).
template <int PATTERN, bool NT, int TILES, int INTERLEAVE = 0>
__global__ __launch_bounds__(256, 1) void stream_probe_kernel(const u32x4* __restrict__ src, int n_tiles,
                                                              uint32_t* __restrict__ sink) {
    extern __shared__ u32x4 probe_lds[];                 // PATTERN 2: 16 KB per wavefront
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int worker = blockIdx.x * 4 + wave, workers = gridDim.x * 4;
    if (INTERLEAVE != 0) {
        // tile index of step k: base + k * step, for k < count
        int base, step, count;
        if (INTERLEAVE == 1) {
            const int per_group = (n_tiles + (int)gridDim.x - 1) / (int)gridDim.x;
            const int g0 = min((int)blockIdx.x * per_group, n_tiles), g1 = min(g0 + per_group, n_tiles);
            base = g0 + wave; step = 4; count = (g1 - base + 3) / 4;
        } else {
            base = worker; step = workers; count = (n_tiles - base + workers - 1) / workers;
        }
        u32x4 acc = {0, 0, 0, 0};
        u32x4 ra[16];
        if (count > 0) {
            probe_request<PATTERN, NT>(src + (size_t)base * 1024, lane, ra);
            for (int k = 0; k < count; ++k) {
                acc ^= probe_consume<PATTERN>(ra, probe_lds, lane);
                probe_request<PATTERN, NT>(src + (size_t)(base + min(k + 1, count - 1) * step) * 1024, lane, ra);
            }
            acc ^= probe_consume<PATTERN>(ra, probe_lds, lane);
        }
        uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
        for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o);
        if (lane == 0) sink[worker] = x;
        return;
    }
    const int share = (n_tiles + workers - 1) / workers;
    const int first = min(worker * share, n_tiles), last = min(first + share, n_tiles);
    u32x4* lds_wave = probe_lds + (PATTERN == 2 ? wave * 1024 : 0);
    u32x4 acc = {0, 0, 0, 0};
    u32x4 ra[16], rb[16];
    if (first < last) {
        probe_request<PATTERN, NT>(src + (size_t)first * 1024, lane, ra);
        if (TILES == 2) probe_request<PATTERN, NT>(src + (size_t)min(first + 1, last - 1) * 1024, lane, rb);
        for (int t = first; t < last; t += TILES) {
            // the refill is unconditional (the last tiles are requested again) so that the number of
            // loads in flight is the same on every iteration
            acc ^= probe_consume<PATTERN>(ra, lds_wave, lane);
            probe_request<PATTERN, NT>(src + (size_t)min(t + TILES, last - 1) * 1024, lane, ra);
            if (TILES == 2) {
                if (t + 1 < last) acc ^= probe_consume<PATTERN>(rb, lds_wave, lane);
                probe_request<PATTERN, NT>(src + (size_t)min(t + 3, last - 1) * 1024, lane, rb);
            }
        }
        // drain what is still in flight
        acc ^= probe_consume<PATTERN>(ra, lds_wave, lane);
        if (TILES == 2) acc ^= probe_consume<PATTERN>(rb, lds_wave, lane);
    }
    uint32_t x = acc.x ^ acc.y ^ acc.z ^ acc.w;
    for (int o = 32; o > 0; o >>= 1) x ^= __shfl_xor(x, o);
    if (lane == 0) sink[worker] = x;
}

hipError_t launch_stream_probe(const void* src, size_t bytes, void* sink, int workgroups, int mode, hipStream_t s) {
    const int n_tiles = (int)(bytes / 16384);
    const u32x4* p = (const u32x4*)src;
    uint32_t* k = (uint32_t*)sink;
    const dim3 g(workgroups), b(256);
    switch (mode) {
        case 0: hipLaunchKernelGGL((stream_probe_kernel<0, true, 1>), g, b, 0, s, p, n_tiles, k); break;
        case 1: hipLaunchKernelGGL((stream_probe_kernel<1, true, 1>), g, b, 0, s, p, n_tiles, k); break;
        case 2: hipLaunchKernelGGL((stream_probe_kernel<2, true, 1>), g, b, 65536, s, p, n_tiles, k); break;
        case 3: hipLaunchKernelGGL((stream_probe_kernel<1, false, 1>), g, b, 0, s, p, n_tiles, k); break;
        case 4: hipLaunchKernelGGL((stream_probe_kernel<1, true, 2>), g, b, 0, s, p, n_tiles, k); break;
        case 5: hipLaunchKernelGGL((stream_probe_kernel<0, true, 2>), g, b, 0, s, p, n_tiles, k); break;
        case 6: hipLaunchKernelGGL((stream_probe_kernel<3, true, 1>), g, b, 0, s, p, n_tiles, k); break;
        case 7: hipLaunchKernelGGL((stream_probe_kernel<3, false, 1>), g, b, 0, s, p, n_tiles, k); break;
        case 8: hipLaunchKernelGGL((stream_probe_kernel<3, true, 1, 1>), g, b, 0, s, p, n_tiles, k); break;
        case 9: hipLaunchKernelGGL((stream_probe_kernel<3, true, 1, 2>), g, b, 0, s, p, n_tiles, k); break;
        default: return hipErrorInvalidValue;
    }
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
