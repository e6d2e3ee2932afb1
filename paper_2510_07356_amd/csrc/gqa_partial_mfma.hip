// Split-KV partial kernel, matrix-core variant (kernel_variant = 0, the default).
//
// One workgroup (4 wavefronts) per work item (b, g, split).  A wavefront walks
// 32-token tiles (tile index wave, wave + 4, ...).  For one tile:
//
//   S^T[tok, head] = K[tok, :] . Q[head, :]      v_mfma_f32_16x16x32_bf16, A = K, B = Q^T
//   online softmax per head in fp32 (base-2 exponentials), P rounded to bf16
//   O^T[d, head]  += V^T[d, tok] P^T[tok, head]   v_mfma_f32_16x16x32_bf16, A = V^T, B = P^T
//
// The G query heads of the KV group occupy the first G of the 16 MFMA columns,
// so every K and V byte is read once and serves all heads of the group.
//
// Operand layouts (lane l, i = l % 16, kb = l / 16; 16x16x32 MFMA: A[i][8kb+e],
// B[8kb+e][i], D[4kb+r][i]):
//   * K as A: lane holds 8 consecutive columns of token i.  The contraction
//     index is free to permute, so MFMA step j uses columns 8*(4j+kb)+e; Q is
//     loaded with the same map.
//   * S^T as D: lane holds head i, tokens 4kb+r of each 16-token half.  The
//     same lane feeds P^T as B of the second MFMA if contraction slot (kb, e)
//     stands for token 16*(e/4) + 4kb + e%4 -- no cross-lane movement.
//   * V^T as A: lane (c = i, kb) loads the 16-byte piece c of the 8 token rows
//     of its contraction slots (coalesced: 16 lanes cover one 256-byte row) and
//     transposes the 8x8 block in registers with v_perm_b32.  Row c of M-tile
//     x is then column d = 8c + x, and accumulator register r of M-tile x holds
//     O[head i][32kb + 8r + x].
#include "gqa_internal.h"

namespace gqa {

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// K and V are streamed once: non-temporal loads keep them from displacing anything in the caches.
__device__ __forceinline__ uint4 load_stream16(const uint16_t* p) {
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));   // round to nearest even
}
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ f32x4 mfma16(const uint4& a, const uint4& b, const f32x4& c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

struct Tile {            // one 32-token tile in registers
    uint4 k[2][4];       // [half][mfma step]
    uint4 v[8];          // [contraction slot e]
};

template <bool PAGED>
__device__ __forceinline__ void load_tile(const KernelArgs& a, int b, int g, int tile0, int t_end,
                                          int i, int kb, Tile& t) {
    const int last = t_end - 1;
    int64_t krow[2], vrow[2];
    for (int hf = 0; hf < 2; ++hf) {
        if (PAGED) {
            const int tu = min(tile0 + 16 * hf, last);        // wave-uniform: one page per 16-token half
            const int64_t blk = __builtin_amdgcn_readfirstlane(
                a.block_table[(int64_t)b * a.block_table_stride + (tu >> a.page_shift)]);
            krow[hf] = blk * a.k_stride_b + (int64_t)g * a.k_stride_h;
            vrow[hf] = blk * a.v_stride_b + (int64_t)g * a.v_stride_h;
        } else {
            krow[hf] = (int64_t)b * a.k_stride_b + (int64_t)g * a.k_stride_h;
            vrow[hf] = (int64_t)b * a.v_stride_b + (int64_t)g * a.v_stride_h;
        }
    }
    const int tmask = PAGED ? (a.page_size - 1) : 0x7fffffff;
    for (int hf = 0; hf < 2; ++hf) {
        const int tk = min(tile0 + 16 * hf + i, last);        // masked rows re-read the last valid row
        const uint16_t* kp = a.k + krow[hf] + (int64_t)(tk & tmask) * a.k_stride_t + 8 * kb;
        for (int j = 0; j < 4; ++j) t.k[hf][j] = load_stream16(kp + 32 * j);
        for (int e4 = 0; e4 < 4; ++e4) {
            const int tv = min(tile0 + 16 * hf + 4 * kb + e4, last);
            const uint16_t* vp = a.v + vrow[hf] + (int64_t)(tv & tmask) * a.v_stride_t + 8 * i;
            t.v[4 * hf + e4] = load_stream16(vp);
        }
    }
}

template <bool PAGED>
__global__ __launch_bounds__(256, 2) void partial_mfma_kernel(KernelArgs a) {
    const WorkItem it = locate_work_item(a, blockIdx.x);
    if (!it.valid) return;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int i = lane & 15, kb = lane >> 4;
    const int b = it.b, g = it.g, G = a.group;

    f32x4 acc[8];
    for (int x = 0; x < 8; ++x) acc[x] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float m = -INFINITY, l = 0.f;
    const float c = a.scale_log2e;

    const int n_tiles = (it.t_end - it.t_begin + 31) >> 5;
    Tile cur, nxt;
    if (wave < n_tiles) load_tile<PAGED>(a, b, g, it.t_begin + 32 * wave, it.t_end, i, kb, cur);

    // Q^T as the B operand: head i, columns 8*(4j+kb)+e; zero beyond the group
    uint4 qf[4];
    for (int j = 0; j < 4; ++j) qf[j] = make_uint4(0, 0, 0, 0);
    if (i < G) {
        const uint16_t* qrow = a.q + (int64_t)b * a.q_stride_b + (int64_t)(g * G + i) * a.q_stride_h;
        for (int j = 0; j < 4; ++j) qf[j] = *reinterpret_cast<const uint4*>(qrow + 8 * (4 * j + kb));
    }

    for (int tile = wave; tile < n_tiles; tile += 4) {
        const int tile0 = it.t_begin + 32 * tile;
        if (tile + 4 < n_tiles) load_tile<PAGED>(a, b, g, tile0 + 128, it.t_end, i, kb, nxt);

        // scores: two 16-token halves, contraction over the 128 columns in 4 steps
        f32x4 s[2];
        for (int hf = 0; hf < 2; ++hf) {
            s[hf] = (f32x4){0.f, 0.f, 0.f, 0.f};
            for (int j = 0; j < 4; ++j) s[hf] = mfma16(cur.k[hf][j], qf[j], s[hf]);
        }
        float sv[8];
        float tmax = -INFINITY;
        for (int hf = 0; hf < 2; ++hf)
            for (int r = 0; r < 4; ++r) {
                const int t = tile0 + 16 * hf + 4 * kb + r;
                const float x = (t < it.t_end) ? s[hf][r] * c : -INFINITY;
                sv[4 * hf + r] = x;
                tmax = fmaxf(tmax, x);
            }
        tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
        tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
        const float mn = fmaxf(m, tmax);          // finite: every tile holds at least one valid token
        if (__builtin_amdgcn_ballot_w64(mn > m) != 0) {
            const float alpha = exp2f(m - mn);    // first tile: 2^(-inf) = 0
            l *= alpha;
            for (int x = 0; x < 8; ++x) acc[x] *= alpha;
            m = mn;
        }
        uint4 pb;
        {
            float p[8];
            for (int e = 0; e < 8; ++e) p[e] = exp2f(sv[e] - m);
            pb.x = pack_bf16(p[0], p[1]); pb.y = pack_bf16(p[2], p[3]);
            pb.z = pack_bf16(p[4], p[5]); pb.w = pack_bf16(p[6], p[7]);
            // the normaliser sums the rounded weights, so the rounding cancels in O / l
            l += (bf16_lo(pb.x) + bf16_hi(pb.x)) + (bf16_lo(pb.y) + bf16_hi(pb.y)) +
                 (bf16_lo(pb.z) + bf16_hi(pb.z)) + (bf16_lo(pb.w) + bf16_hi(pb.w));
        }
        // V^T operands: 8x8 transpose of 16-bit elements, then one MFMA per M-tile
        for (int x2 = 0; x2 < 4; ++x2) {
            const uint32_t* v0 = reinterpret_cast<const uint32_t*>(&cur.v[0]);
            uint4 even, odd;
            uint32_t* pe = reinterpret_cast<uint32_t*>(&even);
            uint32_t* po = reinterpret_cast<uint32_t*>(&odd);
            for (int p2 = 0; p2 < 4; ++p2) {
                const uint32_t lo = v0[(2 * p2) * 4 + x2];       // slot 2*p2, columns 2*x2, 2*x2+1
                const uint32_t hi = v0[(2 * p2 + 1) * 4 + x2];   // slot 2*p2+1
                pe[p2] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                po[p2] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);
            }
            acc[2 * x2] = mfma16(even, pb, acc[2 * x2]);
            acc[2 * x2 + 1] = mfma16(odd, pb, acc[2 * x2 + 1]);
        }
        cur = nxt;
    }

    // the normaliser is spread over the 4 lanes (kb) of a head
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);

    __shared__ float s_o[4][kMaxGroup][kHeadDim];
    __shared__ float s_m[4][kMaxGroup], s_l[4][kMaxGroup];
    if (i < G) {
        for (int x = 0; x < 8; ++x)
            for (int r = 0; r < 4; ++r) s_o[wave][i][32 * kb + 8 * r + x] = acc[x][r];
        if (kb == 0) { s_m[wave][i] = m; s_l[wave][i] = l; }
    }
    __syncthreads();
    const int64_t w = blockIdx.x;
    for (int idx = tid; idx < G * kHeadDim; idx += 256) {
        const int h = idx / kHeadDim, d = idx % kHeadDim;
        const float mn = fmaxf(fmaxf(s_m[0][h], s_m[1][h]), fmaxf(s_m[2][h], s_m[3][h]));
        const float ms = (mn == -INFINITY) ? 0.f : mn;
        float o = 0.f, den = 0.f;
        for (int x = 0; x < 4; ++x) {
            const float wgt = exp2f(s_m[x][h] - ms);
            o = fmaf(wgt, s_o[x][h][d], o);
            den = fmaf(wgt, s_l[x][h], den);
        }
        a.part_o[(w * G + h) * kHeadDim + d] = o;
        if (d == 0) {
            a.part_ml[(w * G + h) * 2] = mn;
            a.part_ml[(w * G + h) * 2 + 1] = den;
        }
    }
}

}  // namespace

hipError_t launch_partial_mfma(const KernelArgs& a, int64_t work_items, hipStream_t s) {
    if (a.page_size == 0)
        hipLaunchKernelGGL(partial_mfma_kernel<false>, dim3((unsigned)work_items), dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(partial_mfma_kernel<true>, dim3((unsigned)work_items), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace gqa
