// Causal prefill attention (forward): every token t of a sequence attends over tokens 0..t.
//
// This is the compute-bound sibling of the decode kernels: the prompt is prefilled once before a
// trace is generated, and fine-tuning on the traces runs full sequences of up to 32,768 tokens
// through the same attention (Section 4.1 of the paper).  Row t of the result is by definition
// the decode attention of query t over the first t + 1 keys.
//
// Decomposition.  One workgroup (8 wavefronts, two per SIMD) owns 256 consecutive query rows of one
// query head, 32 rows per wavefront, and walks the key/value tokens 0 .. (last row) in tiles of 128.
// K and V tiles are staged in LDS row-major (K rows of 272 bytes, V rows of 320 bytes: the paddings
// that make the fragment reads bank-conflict free), both double-buffered with one barrier per tile.
// V^T fragments come out of the transposing LDS load ds_read_b64_tr_b16, which hands every lane four
// consecutive tokens of one column, so V is never transposed in registers.  The two halves of the
// next tile travel in turn, so that only one of them holds registers: K is requested at the start of
// a tile and stored after its second 32-token step, V is requested then and stored at the end.
//
// LDS fragments are requested ahead of the matrix instructions that use them: the V^T fragments of
// a 32-token step and the K fragments of the next step are requested right after the step's score
// products, so their latency passes behind the softmax.
//
// Per wavefront and 32 tokens (v_mfma_f32_32x32x16_bf16; lane l: n = l % 32, kb = l / 32;
// A[m][8kb+e], B[8kb+e][n], D[8(r/4) + 4kb + r%4][n] in register r):
//   S^T[tok, q]  = K Q^T      A = K rows from LDS, B = Q^T kept in registers for the whole kernel
//   online softmax per query row (= per lane column), base-2 exponentials, P rounded to bf16; the
//                             accumulators are rescaled only when a score exceeds the reference by 2^8
//   O^T[d, q]   += V^T P^T    A = V^T from LDS, B = P^T: with contraction slot (kb, e) of step s
//                             standing for token 16s + 4kb + e (e < 4) or 16s + 8 + 4kb + e - 4,
//                             the D registers 8s .. 8s+7 of S^T are exactly the B operand, so P
//                             never moves between lanes.
//
// Scheduling across the chip: blockIdx % 8 is the XCD a workgroup lands on; KV head g is served
// by XCD g % 8 only, so the five query heads of a KV group and all their row blocks share that
// XCD's L2, and the row blocks are taken from the last (longest) to the first.
#include "gqa_internal.h"
#include "gqa_mfma_tile.h"

#include <atomic>

namespace gqa {

namespace {

using namespace tile;

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef short v4i16 __attribute__((ext_vector_type(4)));

constexpr int kBM = 256;               // query rows per workgroup
constexpr int kWaveRows = 32;          // query rows per wavefront (one MFMA column block)
constexpr int kPrefillThreads = 64 * (kBM / kWaveRows);
constexpr int kBN = 128;               // key tokens per LDS tile
constexpr int kKStride = kHeadDim + 8; // bf16 elements per K row in LDS (272 B: conflict-free b128 reads)
constexpr int kVStride = kHeadDim + 32; // bf16 elements per V row in LDS (320 B: the 8 rows x 64 B a transposing read touches fall in distinct banks; measured full rate, 288 B half)
constexpr float kSlack = 8.f;             // log2 of the largest softmax weight before the accumulators are rescaled
constexpr int kKTile = kBN * kKStride;         // elements
constexpr int kVTile = kBN * kVStride;         // elements

__device__ __forceinline__ f32x16 mfma32(const uint4& a, const uint4& b, const f32x16& c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                   c, 0, 0, 0);
}

// acc + lo + hi of a packed bf16 pair, exact products with 1.0, fp32 accumulation
__device__ __forceinline__ float pair_sum(uint32_t pair, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), __builtin_bit_cast(bf16x2, 0x3F803F80u),
                                           acc, false);
}

// max of a value and the one held by lane ^ 32: v_permlane32_swap exchanges the upper half of its first
// operand with the lower half of its second, so both results hold one half broadcast to both halves
__device__ __forceinline__ float max_across_halves(float x) {
    const unsigned u = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    return fmaxf(__builtin_bit_cast(float, (unsigned)r[0]), __builtin_bit_cast(float, (unsigned)r[1]));
}

// 8 bytes of LDS through the transposing load: within each group of 16 lanes, result lane j receives
// element j % 4 of the 8-byte pieces addressed by lanes j / 4, 4 + j / 4, 8 + j / 4, 12 + j / 4
__device__ __forceinline__ uint2 lds_read_tr(const uint16_t* p) {
    const v4i16 r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4i16*)p);
    return __builtin_bit_cast(uint2, r);
}

// One K (V) tile on its way from global memory to LDS, per thread.  The two halves are staged in
// turn so that only one of them occupies registers at a time: K of the next tile travels during the
// first half of the work on the current tile, V during the second.
struct StagingK { uint4 r0, r1, r2, r3; };   // token (tid / 16) + 32 i, 16-byte piece tid % 16
struct StagingV { uint4 r0, r1, r2, r3; };   // tokens 4 * (tid / 16) + i, 16-byte piece tid % 16

__device__ __forceinline__ void load_k_tile(const PrefillArgs& a, const uint16_t* kbase, int tok0, int len, StagingK& st) {
    const int tid = threadIdx.x;
    const int piece = tid & 15, grp = tid >> 4;
    if (tok0 + kBN <= len) {
        // whole tile inside the sequence: one per-thread pointer, wave-uniform row offsets
        const uint16_t* kp = kbase + (int64_t)tok0 * a.k_stride_t + ((int64_t)grp * a.k_stride_t + 8 * piece);
        const int64_t k32 = 32 * a.k_stride_t;
        st.r0 = *reinterpret_cast<const uint4*>(kp);
        st.r1 = *reinterpret_cast<const uint4*>(kp + k32);
        st.r2 = *reinterpret_cast<const uint4*>(kp + 2 * k32);
        st.r3 = *reinterpret_cast<const uint4*>(kp + 3 * k32);
    } else {
        const int last = max(len - 1, 0);               // rows beyond the sequence re-read the last row
        auto row = [&](int i) {
            return *reinterpret_cast<const uint4*>(kbase + (int64_t)min(tok0 + grp + 32 * i, last) * a.k_stride_t + 8 * piece);
        };
        st.r0 = row(0); st.r1 = row(1); st.r2 = row(2); st.r3 = row(3);
    }
}

__device__ __forceinline__ void load_v_tile(const PrefillArgs& a, const uint16_t* vbase, int tok0, int len, StagingV& st) {
    const int tid = threadIdx.x;
    const int piece = tid & 15, grp = tid >> 4;
    if (tok0 + kBN <= len) {
        const uint16_t* vp = vbase + (int64_t)tok0 * a.v_stride_t + ((int64_t)(4 * grp) * a.v_stride_t + 8 * piece);
        st.r0 = *reinterpret_cast<const uint4*>(vp);
        st.r1 = *reinterpret_cast<const uint4*>(vp + a.v_stride_t);
        st.r2 = *reinterpret_cast<const uint4*>(vp + 2 * a.v_stride_t);
        st.r3 = *reinterpret_cast<const uint4*>(vp + 3 * a.v_stride_t);
    } else {
        const int last = max(len - 1, 0);
        auto row = [&](int i) {
            return *reinterpret_cast<const uint4*>(vbase + (int64_t)min(tok0 + 4 * grp + i, last) * a.v_stride_t + 8 * piece);
        };
        st.r0 = row(0); st.r1 = row(1); st.r2 = row(2); st.r3 = row(3);
    }
}

__device__ __forceinline__ void store_k_tile(const StagingK& st, uint16_t* ks) {
    const int tid = threadIdx.x;
    const int piece = tid & 15, grp = tid >> 4;
    *reinterpret_cast<uint4*>(ks + (grp + 0) * kKStride + 8 * piece) = st.r0;
    *reinterpret_cast<uint4*>(ks + (grp + 32) * kKStride + 8 * piece) = st.r1;
    *reinterpret_cast<uint4*>(ks + (grp + 64) * kKStride + 8 * piece) = st.r2;
    *reinterpret_cast<uint4*>(ks + (grp + 96) * kKStride + 8 * piece) = st.r3;
}

__device__ __forceinline__ void store_v_tile(const StagingV& st, uint16_t* vs) {
    const int tid = threadIdx.x;
    const int piece = tid & 15, grp = tid >> 4;
    *reinterpret_cast<uint4*>(vs + (4 * grp + 0) * kVStride + 8 * piece) = st.r0;
    *reinterpret_cast<uint4*>(vs + (4 * grp + 1) * kVStride + 8 * piece) = st.r1;
    *reinterpret_cast<uint4*>(vs + (4 * grp + 2) * kVStride + 8 * piece) = st.r2;
    *reinterpret_cast<uint4*>(vs + (4 * grp + 3) * kVStride + 8 * piece) = st.r3;
}

__global__ __launch_bounds__(kPrefillThreads, 1) __attribute__((amdgpu_waves_per_eu(2, 2))) void prefill_kernel(PrefillArgs a) {
    extern __shared__ uint16_t lds[];           // [2][K tile] then [2][V^T tile]
    uint16_t* const k_lds = lds;
    uint16_t* const v_lds = lds + 2 * kKTile;

    // task: XCD x serves KV heads x, x + 8, ...; row blocks from the last to the first
    const int G = a.group;
    const int n_qb = (a.seq_len + kBM - 1) / kBM;
    const int xcd = blockIdx.x & 7;
    int s = blockIdx.x >> 3;
    const int hh = s % G; s /= G;
    const int qb = n_qb - 1 - (s % n_qb); s /= n_qb;
    const int heads_per_xcd = (a.num_kv_heads + 7) >> 3;
    const int g = xcd + 8 * (s % heads_per_xcd); s /= heads_per_xcd;
    const int b = s;
    if (g >= a.num_kv_heads) return;
    // tokens of this sequence; a.seq_len is the padded length the tensors and the grid are laid out for
    const int len = a.seq_lens != nullptr ? min(max(uniform_i32(a.seq_lens, b), 0), a.seq_len) : a.seq_len;
    const int h = g * G + hh;
    if (qb * kBM >= len) return;                              // a row block beyond the end of its sequence (whole workgroup)

    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n = lane & 31, kb = lane >> 5;
    const int q0 = qb * kBM + wave * kWaveRows;              // first query row of this wavefront
    const int q_last = min(q0 + kWaveRows, len) - 1;   // may be < q0: wavefront without rows
    const float c = fabsf(a.scale_log2e);                    // a negative scale is applied by negating Q (exact)
    const uint32_t qsign = a.scale_log2e < 0.f ? 0x80008000u : 0u;

    const uint16_t* qbase = a.q + (int64_t)b * a.q_stride_b + (int64_t)h * a.q_stride_h;
    const uint16_t* kbase = a.k + (int64_t)b * a.k_stride_b + (int64_t)g * a.k_stride_h;
    const uint16_t* vbase = a.v + (int64_t)b * a.v_stride_b + (int64_t)g * a.v_stride_h;

    // Q^T as B operands: column n of block nt is query row q0 + 32 nt + n, step st covers columns 16 st + 8 kb + e
    uint4 qf[8];
    {
        const int qr = min(q0 + n, max(len - 1, 0));
        const uint16_t* qrow = qbase + (int64_t)qr * a.q_stride_t;
#pragma unroll
        for (int st = 0; st < 8; ++st) {
            uint4 x = *reinterpret_cast<const uint4*>(qrow + 16 * st + 8 * kb);
            x.x ^= qsign; x.y ^= qsign; x.z ^= qsign; x.w ^= qsign;
            qf[st] = x;
        }
    }

    f32x16 acc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[dt][r] = 0.f;
    float m = -INFINITY, l = 0.f;          // reference of the exponents, a raw score within 2^kSlack of the running maximum (times |scale| log2 e in the exponent)
    const int qrow = q0 + n;
    // this lane's source piece of the transposing V reads: token row 4 kb + e (e = (lane % 16) / 4), columns
    // 16 ((lane / 16) % 2) + 4 (lane % 4) of a 32-column block; the 16 lanes of a group then receive columns
    // 0..15 of that half, four consecutive tokens each
    const int v_lane = (4 * kb + ((lane & 15) >> 2)) * kVStride + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    const int kv_end = min(qb * kBM + kBM, len);        // keys this workgroup needs: [0, kv_end)
    const int n_tiles = (kv_end + kBN - 1) / kBN;

    {
        StagingK k0;
        StagingV v0;
        load_k_tile(a, kbase, 0, len, k0);
        load_v_tile(a, vbase, 0, len, v0);
        store_k_tile(k0, k_lds);
        store_v_tile(v0, v_lds);
    }
    __syncthreads();

    for (int tile = 0; tile < n_tiles; ++tile) {
        const int buf = tile & 1;
        const bool more = tile + 1 < n_tiles;
        const int next_tok = (more ? tile + 1 : tile) * kBN;   // the last iteration re-reads its own tile (never stored)
        StagingK stk;
        load_k_tile(a, kbase, next_tok, len, stk);

        const uint16_t* ks = k_lds + buf * kKTile;
        const uint16_t* vs = v_lds + buf * kVTile;
        // K fragments of the first 32-token tile; afterwards they are requested one tile ahead
        uint4 kf[8];
#pragma unroll
        for (int st = 0; st < 8; ++st)
            kf[st] = *reinterpret_cast<const uint4*>(ks + n * kKStride + 16 * st + 8 * kb);
        // one 32-token step; false once the step lies entirely above the diagonal for this wavefront
        auto step = [&](int tt) -> bool {
            const int tok0 = tile * kBN + 32 * tt;
            if (tok0 > q_last) return false;
            f32x16 sc;
#pragma unroll
            for (int r = 0; r < 16; ++r) sc[r] = 0.f;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int st = 0; st < 8; ++st) sc = mfma32(kf[st], qf[st], sc);
            __builtin_amdgcn_sched_barrier(0);
            // requests that do not depend on the softmax: V^T of this tile, K of the next one
            uint2 vf[16];
            int v_step = v_lane + 32 * tt * kVStride;         // one base register per step; the rest are immediates
            asm volatile("" : "+v"(v_step));
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int ks2 = 0; ks2 < 2; ++ks2) {
                    const uint16_t* vp = vs + v_step + 16 * ks2 * kVStride + 32 * dt;
                    vf[4 * dt + 2 * ks2] = lds_read_tr(vp);                         // tokens 16 ks2 + 4 kb + 0..3
                    vf[4 * dt + 2 * ks2 + 1] = lds_read_tr(vp + 8 * kVStride);      // tokens 16 ks2 + 8 + 4 kb + 0..3
                }
            {
                const int tn = min(tt + 1, kBN / 32 - 1);
#pragma unroll
                for (int st = 0; st < 8; ++st)
                    kf[st] = *reinterpret_cast<const uint4*>(ks + (32 * tn + n) * kKStride + 16 * st + 8 * kb);
            }
            __builtin_amdgcn_sched_barrier(0);
            // online softmax on the raw scores (the scale is folded into the exponent: 2^(s c - m c));
            // only tiles that touch the diagonal pay for the mask
            const bool diagonal = tok0 + 31 > q0;             // some (token, row) pair of this tile is masked
            unsigned hidden = 0;                              // bit r: register r holds a token beyond this lane's row
            if (diagonal) {
                const int ahead = tok0 + 4 * kb - qrow;       // register r holds token qrow + ahead + 8 (r / 4) + r % 4
#pragma unroll
                for (int r = 0; r < 16; ++r) hidden |= (ahead + 8 * (r >> 2) + (r & 3) > 0 ? 1u : 0u) << r;
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if ((hidden >> r) & 1u) sc[r] = -INFINITY;
            }
            float tmax = sc[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) tmax = fmaxf(tmax, sc[r]);
            tmax = max_across_halves(tmax);
            const float mn = fmaxf(m, tmax);                  // finite: token 0 is visible to every row
            // the reference m only has to stay within 2^kSlack of the true maximum: weights up to 2^kSlack are
            // as exact in bf16 and fp32 as weights up to 1, and the accumulators are rescaled far less often
            if (__builtin_amdgcn_ballot_w64(!((tmax - m) * c <= kSlack)) != 0) {   // also the first step (m = -inf), whatever c
                // first tile: nothing accumulated yet (and -inf * 0 would not be a number for a zero scale)
                const float alpha = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((m - mn) * c);
                l *= alpha;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) acc[dt] *= alpha;
                m = mn;
            }
            const float mc = -m * c;
            float p[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) p[r] = __builtin_amdgcn_exp2f(fmaf(sc[r], c, mc));
            if (diagonal) {                                   // also covers a zero scale, where -inf * 0 is not a number
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if ((hidden >> r) & 1u) p[r] = 0.f;
            }
            uint4 pb[2];                                      // P^T operands of the two k-steps
#pragma unroll
            for (int ks2 = 0; ks2 < 2; ++ks2) {
                uint4 w;
                w.x = pack_bf16(p[8 * ks2 + 0], p[8 * ks2 + 1]); w.y = pack_bf16(p[8 * ks2 + 2], p[8 * ks2 + 3]);
                w.z = pack_bf16(p[8 * ks2 + 4], p[8 * ks2 + 5]); w.w = pack_bf16(p[8 * ks2 + 6], p[8 * ks2 + 7]);
                pb[ks2] = w;
                // the normaliser sums the rounded weights: one v_dot2 with (1, 1) per packed pair
                l = pair_sum(w.w, pair_sum(w.z, pair_sum(w.y, pair_sum(w.x, l))));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int ks2 = 0; ks2 < 2; ++ks2) {
                    const uint2 lo = vf[4 * dt + 2 * ks2], hi = vf[4 * dt + 2 * ks2 + 1];
                    acc[dt] = mfma32(make_uint4(lo.x, lo.y, hi.x, hi.y), pb[ks2], acc[dt]);
                }
            return true;
        };
        bool live = true;
#pragma unroll 1
        for (int tt = 0; tt < 2 && live; ++tt) live = step(tt);
        if (more) store_k_tile(stk, k_lds + (buf ^ 1) * kKTile);
        StagingV stv;
        load_v_tile(a, vbase, next_tok, len, stv);
#pragma unroll 1
        for (int tt = 2; tt < 4 && live; ++tt) live = step(tt);
        if (more) store_v_tile(stv, v_lds + (buf ^ 1) * kVTile);
        __syncthreads();
    }

    // epilogue: normalise and store; lane holds query row q0 + n, columns 32 dt + 8 (r/4) + 4 kb + r%4
    {
        float lt = l;
        lt += __shfl_xor(lt, 32);
        if (qrow < len) {
            const float inv = lt > 0.f ? 1.f / lt : 0.f;
            float* orow = a.out + (int64_t)b * a.o_stride_b + (int64_t)qrow * a.o_stride_t + (int64_t)h * a.o_stride_h;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int r4 = 0; r4 < 4; ++r4) {
                    float4 o;
                    o.x = acc[dt][4 * r4 + 0] * inv; o.y = acc[dt][4 * r4 + 1] * inv;
                    o.z = acc[dt][4 * r4 + 2] * inv; o.w = acc[dt][4 * r4 + 3] * inv;
                    *reinterpret_cast<float4*>(orow + 32 * dt + 8 * r4 + 4 * kb) = o;
                }
            if (a.lse != nullptr && kb == 0)
                a.lse[((int64_t)b * a.seq_len + qrow) * a.num_q_heads + h] =
                    lt > 0.f ? 0.6931471805599453f * (m * c + log2f(lt)) : -INFINITY;
        }
    }
}

constexpr size_t kPrefillLds = (size_t)(2 * kKTile + 2 * kVTile) * sizeof(uint16_t);

}  // namespace

// More than the default 64 KB of LDS: the limit is a per-device attribute of the kernel, raised
// once per device (gqa_decode_init, or the first prefill call on that device).
hipError_t prepare_prefill() {
    constexpr int kMaxDevices = 64;
    static std::atomic<bool> done[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (done[dev].load(std::memory_order_acquire)) return hipSuccess;
    e = hipFuncSetAttribute(reinterpret_cast<const void*>(prefill_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)kPrefillLds);
    if (e == hipSuccess) done[dev].store(true, std::memory_order_release);
    return e;
}

hipError_t launch_prefill(const PrefillArgs& a, hipStream_t s) {
    const hipError_t ready = prepare_prefill();
    if (ready != hipSuccess) return ready;
    const int n_qb = (a.seq_len + kBM - 1) / kBM;
    const int heads_per_xcd = (a.num_kv_heads + 7) / 8;
    const int64_t grid = 8LL * a.group * n_qb * heads_per_xcd * a.batch;
    hipLaunchKernelGGL(prefill_kernel, dim3((unsigned)grid), dim3(kPrefillThreads), kPrefillLds, s, a);
    return hipGetLastError();
}

}  // namespace gqa
