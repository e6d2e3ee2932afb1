// Tile-level building blocks of the matrix-core partial kernels: streaming loads, the two MFMA
// contractions of one 32-token tile and the online-softmax update between them.  The operand
// layouts are described at the top of gqa_partial_mfma.hip.
#pragma once

#include "gqa_internal.h"

#ifndef GQA_STREAM_NT                // 1: K and V are read with non-temporal loads
#define GQA_STREAM_NT 1
#endif

namespace gqa {
namespace tile {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// K and V are streamed once: non-temporal loads keep them from displacing anything in the caches.
__device__ __forceinline__ uint4 load_stream16(const uint16_t* p) {
#if GQA_STREAM_NT
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
#else
    return *reinterpret_cast<const uint4*>(p);
#endif
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

// Makes the compiler wait for Q here, outside the tile loop: otherwise the wait for the (rarely
// reloaded) Q registers lands on the loop's first MFMA and also waits for the K/V tile just requested.
__device__ __forceinline__ void settle_q(uint4 (&qf)[4]) {
    for (int j = 0; j < 4; ++j)
        asm volatile("" : "+v"(qf[j].x), "+v"(qf[j].y), "+v"(qf[j].z), "+v"(qf[j].w));
}

struct SoftmaxState {
    f32x4 acc[8];        // O^T: M-tile x, register r -> O[head i][32kb + 8r + x]
    float m, l;          // running maximum (log2 domain) and this lane's share of the normaliser
};

__device__ __forceinline__ void reset(SoftmaxState& st) {
    for (int x = 0; x < 8; ++x) st.acc[x] = (f32x4){0.f, 0.f, 0.f, 0.f};
    st.m = -INFINITY;
    st.l = 0.f;
}

// scores of one tile: two 16-token halves, contraction over the 128 columns in 4 steps
__device__ __forceinline__ void scores(const uint4 (&k)[2][4], const uint4 (&qf)[4], f32x4 (&s)[2]) {
    for (int hf = 0; hf < 2; ++hf) {
        s[hf] = (f32x4){0.f, 0.f, 0.f, 0.f};
        for (int j = 0; j < 4; ++j) s[hf] = mfma16(k[hf][j], qf[j], s[hf]);
    }
}

// online softmax update; returns the bf16 probabilities as the B operand of P.V
__device__ __forceinline__ uint4 softmax_update(const f32x4 (&s)[2], SoftmaxState& st, int tok0, int len, int kb, float c) {
    float sv[8];
    float tmax = -INFINITY;
    for (int hf = 0; hf < 2; ++hf)
        for (int r = 0; r < 4; ++r) {
            const int tok = tok0 + 16 * hf + 4 * kb + r;
            const float x = (tok < len) ? s[hf][r] * c : -INFINITY;
            sv[4 * hf + r] = x;
            tmax = fmaxf(tmax, x);
        }
    tmax = fmaxf(tmax, __shfl_xor(tmax, 16));
    tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
    const float mn = fmaxf(st.m, tmax);           // finite: every tile holds at least one valid token
    if (__builtin_amdgcn_ballot_w64(mn > st.m) != 0) {
        const float alpha = exp2f(st.m - mn);     // first tile: 2^(-inf) = 0
        st.l *= alpha;
        for (int x = 0; x < 8; ++x) st.acc[x] *= alpha;
        st.m = mn;
    }
    float pr[8];
    for (int e = 0; e < 8; ++e) pr[e] = exp2f(sv[e] - st.m);
    uint4 pb;
    pb.x = pack_bf16(pr[0], pr[1]); pb.y = pack_bf16(pr[2], pr[3]);
    pb.z = pack_bf16(pr[4], pr[5]); pb.w = pack_bf16(pr[6], pr[7]);
    // the normaliser sums the rounded weights, so the rounding cancels in O / l
    st.l += (bf16_lo(pb.x) + bf16_hi(pb.x)) + (bf16_lo(pb.y) + bf16_hi(pb.y)) +
            (bf16_lo(pb.z) + bf16_hi(pb.z)) + (bf16_lo(pb.w) + bf16_hi(pb.w));
    return pb;
}

// V^T operands of the 8 M-tiles: 8x8 transpose of 16-bit elements in registers.  vt[2*x2] holds the
// even column of each pair, vt[2*x2+1] the odd one (M-tile x <-> column d = 8c + x of piece c).
__device__ __forceinline__ void transpose_values(const uint4 (&v)[8], uint4 (&vt)[8]) {
    const uint32_t* v0 = reinterpret_cast<const uint32_t*>(&v[0]);
    for (int x2 = 0; x2 < 4; ++x2) {
        uint32_t* pe = reinterpret_cast<uint32_t*>(&vt[2 * x2]);
        uint32_t* po = reinterpret_cast<uint32_t*>(&vt[2 * x2 + 1]);
        for (int p2 = 0; p2 < 4; ++p2) {
            const uint32_t lo = v0[(2 * p2) * 4 + x2];       // slot 2*p2, columns 2*x2, 2*x2+1
            const uint32_t hi = v0[(2 * p2 + 1) * 4 + x2];   // slot 2*p2+1
            pe[p2] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            po[p2] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);
        }
    }
}

// O^T += V^T P^T from already transposed operands: one MFMA per M-tile
__device__ __forceinline__ void weighted_values_t(const uint4 (&vt)[8], const uint4& pb, SoftmaxState& st) {
    for (int x = 0; x < 8; ++x) st.acc[x] = mfma16(vt[x], pb, st.acc[x]);
}

// O^T += V^T P^T: 8x8 transpose of 16-bit elements in registers, then one MFMA per M-tile
__device__ __forceinline__ void weighted_values(const uint4 (&v)[8], const uint4& pb, SoftmaxState& st) {
    const uint32_t* v0 = reinterpret_cast<const uint32_t*>(&v[0]);
    for (int x2 = 0; x2 < 4; ++x2) {
        uint4 even, odd;
        uint32_t* pe = reinterpret_cast<uint32_t*>(&even);
        uint32_t* po = reinterpret_cast<uint32_t*>(&odd);
        for (int p2 = 0; p2 < 4; ++p2) {
            const uint32_t lo = v0[(2 * p2) * 4 + x2];       // slot 2*p2, columns 2*x2, 2*x2+1
            const uint32_t hi = v0[(2 * p2 + 1) * 4 + x2];   // slot 2*p2+1
            pe[p2] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
            po[p2] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);
        }
        st.acc[2 * x2] = mfma16(even, pb, st.acc[2 * x2]);
        st.acc[2 * x2 + 1] = mfma16(odd, pb, st.acc[2 * x2 + 1]);
    }
}

}  // namespace tile
}  // namespace gqa
