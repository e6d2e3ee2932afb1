// KV append with optional rotary embedding: the step that precedes attention in a decode layer.
//
// For every sequence b with L = kv_lens[b] > 0 the new token sits at position L - 1: its key row
// (rotated if a cos/sin table is given) and its value row are written into the contiguous or
// paged cache there, and the query rows are rotated by the same position.  Rotate-half pairing:
// column d < 64 pairs with column d + 64,
//     x' = x cos - y sin,   y' = y cos + x sin.
// The products of a bf16 value and an fp32 table entry are exact in fp64, so the rotation is done
// in fp64 (the difference or sum of the two exact products is its only rounding) and the fp64
// result is rounded to bf16, nearest-even, over the whole bf16 range: normal results, sub-normal
// results (fixed spacing 2^-133), signed zeros, overflow to infinity; a NaN result is stored as
// the quiet NaN 0x7FC0.  One workgroup per sequence, one thread per column pair; the work is a few KB per
// sequence, so the kernel is launch-bound and nothing here is tuned.
#include "gqa_internal.h"

namespace gqa {

namespace {

__device__ __forceinline__ double widen(uint16_t bits) { return (double)__uint_as_float((uint32_t)bits << 16); }

// Nearest-even rounding of a double to bf16.
__device__ __forceinline__ uint16_t round_bf16(double x) {
    if (x != x) return 0x7FC0u;
    unsigned long long u = __double_as_longlong(x);
    const double ax = fabs(x);
    if (ax < 0x1p-126) {
        // zero or below the smallest normal bf16: the grid is q * 2^-133, q = 0 .. 128 (q = 128 is the
        // smallest normal number, whose bit pattern 0x0080 is again q); the scaling is exact in fp64
        const unsigned q = (unsigned)rint(ax * 0x1p133);
        return (uint16_t)((unsigned)(u >> 48) & 0x8000u) | (uint16_t)q;
    }
    const unsigned long long lsb = (u >> 45) & 1ull;
    u += (1ull << 44) - 1ull + lsb;            // carries into the exponent when the mantissa overflows
    u &= ~((1ull << 45) - 1ull);
    const float f = (float)__longlong_as_double(u);      // exact (8 significant bits), or infinity beyond the range
    return (uint16_t)(__float_as_uint(f) >> 16);
}

__global__ __launch_bounds__(256) void kv_append_kernel(AppendArgs a) {
    const int b = blockIdx.x;
    const int pos = min(a.kv_lens[b], a.max_kv_len) - 1;
    const int pair = threadIdx.x & 63;
    const int half = kHeadDim / 2;
    const bool rotate = a.cos_sin != nullptr && pos >= 0;
    double c = 1.0, s = 0.0;
    if (rotate) {
        c = (double)a.cos_sin[(int64_t)pos * kHeadDim + pair];
        s = (double)a.cos_sin[(int64_t)pos * kHeadDim + half + pair];
    }
    // query rows
    for (int h = threadIdx.x >> 6; h < a.num_q_heads; h += 4) {
        const int64_t off = (int64_t)b * a.q_stride_b + (int64_t)h * a.q_stride_h;
        const uint16_t xb = a.q_in[off + pair], yb = a.q_in[off + half + pair];
        uint16_t xo = xb, yo = yb;
        if (rotate) {
            const double x = widen(xb), y = widen(yb);
            xo = round_bf16(x * c - y * s);
            yo = round_bf16(y * c + x * s);
        }
        a.q_out[off + pair] = xo;
        a.q_out[off + half + pair] = yo;
    }
    if (pos < 0) return;
    int64_t krow, vrow;
    if (a.page_size == 0) {
        krow = (int64_t)b * a.k_stride_b + (int64_t)pos * a.k_stride_t;
        vrow = (int64_t)b * a.v_stride_b + (int64_t)pos * a.v_stride_t;
    } else {
        const int64_t blk = a.block_table[(int64_t)b * a.block_table_stride + pos / a.page_size];
        const int slot = pos % a.page_size;
        krow = blk * a.k_stride_b + (int64_t)slot * a.k_stride_t;
        vrow = blk * a.v_stride_b + (int64_t)slot * a.v_stride_t;
    }
    for (int g = threadIdx.x >> 6; g < a.num_kv_heads; g += 4) {
        const int64_t src = ((int64_t)b * a.num_kv_heads + g) * kHeadDim;
        const uint16_t xb = a.k_new[src + pair], yb = a.k_new[src + half + pair];
        uint16_t xo = xb, yo = yb;
        if (rotate) {
            const double x = widen(xb), y = widen(yb);
            xo = round_bf16(x * c - y * s);
            yo = round_bf16(y * c + x * s);
        }
        uint16_t* kd = a.k_cache + krow + (int64_t)g * a.k_stride_h;
        uint16_t* vd = a.v_cache + vrow + (int64_t)g * a.v_stride_h;
        kd[pair] = xo;
        kd[half + pair] = yo;
        vd[pair] = a.v_new[src + pair];
        vd[half + pair] = a.v_new[src + half + pair];
    }
}

}  // namespace

hipError_t launch_kv_append(const AppendArgs& a, hipStream_t s) {
    hipLaunchKernelGGL(kv_append_kernel, dim3(a.batch), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace gqa
