// Split-KV partial kernel, vector-ALU variant (kernel_variant = 1).
//
// Kept as the plain fp32 path next to the matrix-core kernel: same stream-split
// work decomposition (see gqa_internal.h) and outputs, no bf16 rounding of the
// probabilities, group sizes up to 8.  The 4 wavefronts of a workgroup share each piece.
//
// Data path: each global_load_dwordx4 of a wavefront fetches 4 whole K (or V)
// rows: lane l reads the 16-byte piece (l % 16) of token (l / 16), so a load is
// one contiguous KB in the head-major layout.  A lane therefore owns 8 of the
// 128 columns; q.k is finished by a 16-lane DPP butterfly, and each of the four
// 16-lane rows of a wavefront runs its own online softmax over its own tokens.
// The 16 row states of the workgroup are merged at the end.
#include "gqa_internal.h"

namespace gqa {

namespace {

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ void unpack8(const uint4& r, float* f) {
    f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x); f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
    f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z); f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
}

// Sum over the 16 lanes of a DPP row; every lane ends with the total.
__device__ __forceinline__ float row16_sum(float x) {
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));  // row_half_mirror
    x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));  // row_mirror
    return x;
}

constexpr int kUnroll = 4;     // token quads in flight per wavefront

template <int G>
__global__ __launch_bounds__(kThreads) void partial_valu_kernel(KernelArgs a) {
    __shared__ float s_o[4][G][kHeadDim];
    __shared__ float s_m[4][G], s_l[4][G];
    __shared__ int s_scan[4];
    __shared__ int s_found[3];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int sub = lane >> 4;        // which of the 4 rows of a load
    const int piece16 = lane & 15;    // which 16-byte piece of the row
    const int32_t* __restrict__ bt = a.block_table;

    const int total = stream_total(a, s_scan);
    const int share_tiles = share_tiles_for(total, a.fixed_share_tiles, gridDim.x);
    const int n_shares = (total + share_tiles - 1) / share_tiles;
    if (blockIdx.x == 0) {
        if (tid == 0) { a.header[0] = total; a.header[1] = share_tiles; }
        if (total == 0) (void)stream_locate(a, 0, s_scan, s_found, a.row_prefix);
    }

    for (int share = blockIdx.x; share < n_shares; share += gridDim.x) {
        int pos = share * share_tiles;
        const int end = min(pos + share_tiles, total);
        const StreamPos sp = stream_locate(a, pos, s_scan, s_found, share == 0 ? a.row_prefix : nullptr);
        int b = sp.b, g = sp.g, tile0 = sp.tile;
        while (pos < end) {
            const int len = clamped_len(a, b);
            const int n = min(tiles_of(len) - tile0, end - pos);
            if (n <= 0) {                       // an empty sequence between two rows of the share
                tile0 = 0; g = 0; ++b;
                continue;
            }
            const int t_begin = kTileTokens * tile0;
            const int t_end = min(len, kTileTokens * (tile0 + n));

            float qf[G][8];
            for (int h = 0; h < G; ++h) {
                const uint16_t* qrow = a.q + (int64_t)b * a.q_stride_b + (int64_t)(g * G + h) * a.q_stride_h;
                const uint4 r = *reinterpret_cast<const uint4*>(qrow + piece16 * 8);
                unpack8(r, qf[h]);
                for (int e = 0; e < 8; ++e) qf[h][e] *= a.scale_log2e;
            }
            float m[G], l[G], o[G][8];
            for (int h = 0; h < G; ++h) {
                m[h] = -INFINITY; l[h] = 0.f;
                for (int e = 0; e < 8; ++e) o[h][e] = 0.f;
            }
            const int64_t kbase = (int64_t)g * a.k_stride_h + piece16 * 8;
            const int64_t vbase = (int64_t)g * a.v_stride_h + piece16 * 8;

            // the workgroup advances 16 tokens per step: wave w, row `sub` takes token 16*i + 4*w + sub
            for (int t0 = t_begin; t0 < t_end; t0 += 16 * kUnroll) {
                uint4 kr[kUnroll], vr[kUnroll];
                bool ok[kUnroll];
                for (int u = 0; u < kUnroll; ++u) {
                    const int t = t0 + 16 * u + 4 * wave + sub;
                    ok[u] = t < t_end;
                    kr[u] = make_uint4(0, 0, 0, 0);
                    vr[u] = make_uint4(0, 0, 0, 0);
                    if (ok[u]) {
                        int64_t ko, vo;
                        if (a.page_size == 0) {
                            ko = (int64_t)b * a.k_stride_b + (int64_t)t * a.k_stride_t;
                            vo = (int64_t)b * a.v_stride_b + (int64_t)t * a.v_stride_t;
                        } else {
                            const int64_t blk = bt[(int64_t)b * a.block_table_stride + (t >> a.page_shift)];
                            const int slot = t & (a.page_size - 1);
                            ko = blk * a.k_stride_b + (int64_t)slot * a.k_stride_t;
                            vo = blk * a.v_stride_b + (int64_t)slot * a.v_stride_t;
                        }
                        kr[u] = *reinterpret_cast<const uint4*>(a.k + kbase + ko);
                        vr[u] = *reinterpret_cast<const uint4*>(a.v + vbase + vo);
                    }
                }
                for (int u = 0; u < kUnroll; ++u) {
                    float kf[8], vf[8];
                    unpack8(kr[u], kf);
                    unpack8(vr[u], vf);
                    for (int h = 0; h < G; ++h) {
                        float s = 0.f;
                        for (int e = 0; e < 8; ++e) s = fmaf(qf[h][e], kf[e], s);
                        s = row16_sum(s);
                        s = ok[u] ? s : -INFINITY;
                        const float mn = fmaxf(m[h], s);
                        const float ms = (mn == -INFINITY) ? 0.f : mn;   // keeps (-inf) - (-inf) out
                        const float alpha = exp2f(m[h] - ms);
                        const float pr = exp2f(s - ms);
                        m[h] = mn;
                        l[h] = fmaf(l[h], alpha, pr);
                        for (int e = 0; e < 8; ++e) o[h][e] = fmaf(pr, vf[e], o[h][e] * alpha);
                    }
                }
            }

            // merge the 4 rows of the wavefront (lanes l, l^16, l^32, l^48 hold the same columns)
            for (int h = 0; h < G; ++h) {
                for (int step = 16; step <= 32; step <<= 1) {
                    const float m2 = __shfl_xor(m[h], step);
                    const float l2 = __shfl_xor(l[h], step);
                    const float mn = fmaxf(m[h], m2);
                    const float ms = (mn == -INFINITY) ? 0.f : mn;
                    const float w1 = exp2f(m[h] - ms), w2 = exp2f(m2 - ms);
                    for (int e = 0; e < 8; ++e) {
                        const float o2 = __shfl_xor(o[h][e], step);
                        o[h][e] = o[h][e] * w1 + o2 * w2;
                    }
                    l[h] = l[h] * w1 + l2 * w2;
                    m[h] = mn;
                }
            }

            // merge the 4 wavefronts through LDS and emit the partial result of this piece
            __syncthreads();                    // the buffers may still be read for the previous piece
            if (sub == 0) {
                for (int h = 0; h < G; ++h) {
                    for (int e = 0; e < 8; ++e) s_o[wave][h][piece16 * 8 + e] = o[h][e];
                    if (piece16 == 0) { s_m[wave][h] = m[h]; s_l[wave][h] = l[h]; }
                }
            }
            __syncthreads();
            const int64_t slot = (int64_t)share + (int64_t)b * a.num_kv_heads + g;
            for (int idx = tid; idx < G * kHeadDim; idx += kThreads) {
                const int h = idx / kHeadDim, d = idx % kHeadDim;
                const float mn = fmaxf(fmaxf(s_m[0][h], s_m[1][h]), fmaxf(s_m[2][h], s_m[3][h]));
                const float ms = (mn == -INFINITY) ? 0.f : mn;
                float acc = 0.f, den = 0.f;
                for (int x = 0; x < 4; ++x) {
                    const float wgt = exp2f(s_m[x][h] - ms);
                    acc = fmaf(wgt, s_o[x][h][d], acc);
                    den = fmaf(wgt, s_l[x][h], den);
                }
                a.part_o[(slot * G + h) * kHeadDim + d] = acc;
                if (d == 0) {
                    a.part_ml[(slot * G + h) * 2] = mn;
                    a.part_ml[(slot * G + h) * 2 + 1] = den;
                }
            }
            pos += n;
            tile0 = 0;
            if (++g == a.num_kv_heads) { g = 0; ++b; }
        }
    }
}

template <int G>
hipError_t launch_g(const KernelArgs& a, int workgroups, hipStream_t s) {
    hipLaunchKernelGGL(partial_valu_kernel<G>, dim3(workgroups), dim3(kThreads), 0, s, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_partial_valu(const KernelArgs& a, int workgroups, hipStream_t s) {
    switch (a.group) {
        case 1: return launch_g<1>(a, workgroups, s);
        case 2: return launch_g<2>(a, workgroups, s);
        case 3: return launch_g<3>(a, workgroups, s);
        case 4: return launch_g<4>(a, workgroups, s);
        case 5: return launch_g<5>(a, workgroups, s);
        case 6: return launch_g<6>(a, workgroups, s);
        case 7: return launch_g<7>(a, workgroups, s);
        case 8: return launch_g<8>(a, workgroups, s);
        default: return hipErrorInvalidValue;
    }
}

int partial_valu_occupancy() {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, partial_valu_kernel<8>, kThreads, 0) != hipSuccess || n < 1)
        n = 1;
    return n;
}

}  // namespace gqa
