// Split-KV partial kernel, matrix-core variant (kernel_variant = 0, the default).
//
// Every wavefront is an independent persistent worker: it owns one share of the
// stream split described in gqa_internal.h (or takes shares in turn when the
// share length is fixed) and walks its 32-token tiles in order.  One tile (16
// loads of 16 bytes per lane) is in flight per wavefront: the K registers are
// refilled with the next tile's K as soon as the scores are computed, the V
// registers after P.V, so the load stream never drains and never holds more
// than one tile per wavefront (measured: deeper prefetch lowers the achieved
// HBM bandwidth on this chip).  No LDS, no barrier: the partial result of a
// piece goes from the accumulators straight to the workspace.
// For one tile:
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
#include "gqa_mfma_tile.h"

// Compile-time tunables (defaults are the measured best on MI355X: one wavefront per SIMD;
// more resident wavefronts put more requests in flight and lower the achieved HBM bandwidth).
#ifndef GQA_MFMA_WGS_PER_CU          // persistent workgroups launched per CU (register budget follows)
#define GQA_MFMA_WGS_PER_CU 1
#endif
#ifndef GQA_MFMA_WAVES               // wavefronts (independent workers) per workgroup
#define GQA_MFMA_WAVES 4
#endif
#ifndef GQA_MFMA_EARLY_K             // 1: request the next K tile right after the scores, 0: after P.V
#define GQA_MFMA_EARLY_K 1
#endif
#ifndef GQA_MFMA_EARLY_V             // 1: transpose V first and request the next V tile before the scores
#define GQA_MFMA_EARLY_V 1
#endif

namespace gqa {

namespace {

using namespace tile;

struct Piece {           // the part of a share inside one (b, g) row; uniform over the wavefront
    int b, g, tile0, n, len;
};

// Physical blocks of the two 16-token halves of a tile (paged caches): each half lies inside one
// page, so the ids are wave-uniform and come through the scalar path.
__device__ __forceinline__ void tile_blocks(const KernelArgs& a, const Piece& p, int tile, bool idle, int (&blk)[2]) {
    const int tok0 = kTileTokens * (p.tile0 + tile);
    const int last = idle ? tok0 : p.len - 1;
    for (int hf = 0; hf < 2; ++hf) {
        const int tu = min(tok0 + 16 * hf, last);
        blk[hf] = uniform_i32(a.block_table, (int64_t)p.b * a.block_table_stride + (tu >> a.page_shift));
    }
}

// K as the A operand: lane (i, kb) holds columns 8*(4j+kb)+e of token 16*hf + i.
template <bool PAGED>
__device__ __forceinline__ void load_k(const KernelArgs& a, const Piece& p, int tile, bool idle, const int (&blk)[2],
                                       int i, int kb, uint4 (&k)[2][4]) {
    const int tok0 = kTileTokens * (p.tile0 + tile);
    const int last = idle ? tok0 : p.len - 1;     // idle: every lane re-reads row tok0, one cache line per load
    const int tmask = PAGED ? (a.page_size - 1) : 0x7fffffff;
    for (int hf = 0; hf < 2; ++hf) {
        const int64_t row = (PAGED ? (int64_t)blk[hf] : (int64_t)p.b) * a.k_stride_b + (int64_t)p.g * a.k_stride_h;
        const int tk = min(tok0 + 16 * hf + i, last);         // masked rows re-read the last valid row
        const uint16_t* kp = a.k + row + (int64_t)(tk & tmask) * a.k_stride_t + (idle ? 0 : 8 * kb);
        for (int j = 0; j < 4; ++j) k[hf][j] = load_stream16(kp + (idle ? 0 : 32 * j));
    }
}

// V rows of the lane's contraction slots: slot e <-> token 16*(e/4) + 4kb + e%4, 16-byte piece i.
template <bool PAGED>
__device__ __forceinline__ void load_v(const KernelArgs& a, const Piece& p, int tile, bool idle, const int (&blk)[2],
                                       int i, int kb, uint4 (&v)[8]) {
    const int tok0 = kTileTokens * (p.tile0 + tile);
    const int last = idle ? tok0 : p.len - 1;
    const int tmask = PAGED ? (a.page_size - 1) : 0x7fffffff;
    for (int hf = 0; hf < 2; ++hf) {
        const int64_t row = (PAGED ? (int64_t)blk[hf] : (int64_t)p.b) * a.v_stride_b + (int64_t)p.g * a.v_stride_h;
        for (int e4 = 0; e4 < 4; ++e4) {
            const int tv = min(tok0 + 16 * hf + 4 * kb + e4, last);
            v[4 * hf + e4] = load_stream16(a.v + row + (int64_t)(tv & tmask) * a.v_stride_t + (idle ? 0 : 8 * i));
        }
    }
}

// Q^T as the B operand: head i, columns 8*(4j+kb)+e; zero beyond the group
__device__ __forceinline__ void load_q(const KernelArgs& a, const Piece& p, int i, int kb, uint4 (&qf)[4]) {
    for (int j = 0; j < 4; ++j) qf[j] = make_uint4(0, 0, 0, 0);
    if (i < a.group) {
        const uint16_t* qrow = a.q + (int64_t)p.b * a.q_stride_b + (int64_t)(p.g * a.group + i) * a.q_stride_h;
        for (int j = 0; j < 4; ++j) qf[j] = *reinterpret_cast<const uint4*>(qrow + 8 * (4 * j + kb));
    }
}

// Partial result of a finished piece: accumulators and (m, l) go to slot share + row.
__device__ __forceinline__ void emit_piece(const KernelArgs& a, const Piece& p, int share, SoftmaxState& st,
                                           int i, int kb) {
    float l = st.l;
    l += __shfl_xor(l, 16);          // the normaliser is spread over the 4 lanes (kb) of a head
    l += __shfl_xor(l, 32);
    const int G = a.group;
    if (i < G) {
        const int64_t slot = (int64_t)share + (int64_t)p.b * a.num_kv_heads + p.g;
        float* dst = a.part_o + (slot * G + i) * kHeadDim + 32 * kb;
        for (int r = 0; r < 4; ++r) {
            float4 lo4, hi4;
            lo4.x = st.acc[0][r]; lo4.y = st.acc[1][r]; lo4.z = st.acc[2][r]; lo4.w = st.acc[3][r];
            hi4.x = st.acc[4][r]; hi4.y = st.acc[5][r]; hi4.z = st.acc[6][r]; hi4.w = st.acc[7][r];
            *reinterpret_cast<float4*>(dst + 8 * r) = lo4;
            *reinterpret_cast<float4*>(dst + 8 * r + 4) = hi4;
        }
        if (kb == 0) *reinterpret_cast<float2*>(a.part_ml + (slot * G + i) * 2) = make_float2(st.m, l);
    }
}

// The piece that follows p inside a share that still has `left` tiles after p.
__device__ __forceinline__ Piece next_piece(const KernelArgs& a, const Piece& p, int left) {
    Piece q = p;
    q.tile0 = 0;
    q.g = p.g + 1;
    if (q.g == a.num_kv_heads) {
        q.g = 0;
        do { ++q.b; q.len = uniform_len(a, q.b); } while (q.len == 0 && q.b + 1 < a.batch);
    }
    q.n = min(tiles_of(q.len), left);
    return q;
}

template <bool PAGED>
__global__ __launch_bounds__(64 * GQA_MFMA_WAVES, GQA_MFMA_WGS_PER_CU) void partial_mfma_kernel(KernelArgs a) {
    const int lane = threadIdx.x & 63;
    const int i = lane & 15, kb = lane >> 4;
    const float c = a.scale_log2e;
    const int worker = __builtin_amdgcn_readfirstlane(blockIdx.x * GQA_MFMA_WAVES + (threadIdx.x >> 6));
    const int workers = gridDim.x * GQA_MFMA_WAVES;

    const int total = __builtin_amdgcn_readfirstlane(wave_stream_total(a));
    const int share_tiles = share_tiles_for(total, a.fixed_share_tiles, workers);
    const int n_shares = (total + share_tiles - 1) / share_tiles;
    if (worker == 0) {
        if (lane == 0) { a.header[0] = total; a.header[1] = share_tiles; }
        if (total == 0) (void)wave_stream_locate(a, 0, a.row_prefix);     // all-zero prefix for the combine
    }

    for (int share = worker; share < n_shares; share += workers) {
        int pos = share * share_tiles;
        const int end = min(pos + share_tiles, total);
        const StreamPos sp = wave_stream_locate(a, pos, share == 0 ? a.row_prefix : nullptr);
        Piece p;
        p.b = __builtin_amdgcn_readfirstlane(sp.b);
        p.g = __builtin_amdgcn_readfirstlane(sp.g);
        p.tile0 = __builtin_amdgcn_readfirstlane(sp.tile);
        p.len = __builtin_amdgcn_readfirstlane(sp.len);
        p.n = min(tiles_of(p.len) - p.tile0, end - pos);

        uint4 kreg[2][4], vreg[8], qf[4];
        SoftmaxState st;
        int blk[2] = {0, 0}, blk_ahead[2] = {0, 0};      // paged: blocks of the tile being requested / the one after
        bool ahead_valid = false;
        if (PAGED) tile_blocks(a, p, 0, false, blk);
        load_k<PAGED>(a, p, 0, false, blk, i, kb, kreg);
        load_v<PAGED>(a, p, 0, false, blk, i, kb, vreg);
        load_q(a, p, i, kb, qf);
        reset(st);
        bool has_next = pos + p.n < end;
        Piece q = has_next ? next_piece(a, p, end - pos - p.n) : p;
        int t = 0;                       // tile of p held (or arriving) in kreg / vreg
        settle_q(qf);

        while (true) {
            // the tile after (p, t); when nothing follows, one row of the current tile is requested
            // again by all lanes (a single cache line) so that the number of loads in flight is
            // the same on every path and the waits in the loop never cover the tile just requested
            const bool last_of_piece = t + 1 == p.n;
            const bool cross = last_of_piece && has_next;
            const bool idle = last_of_piece && !has_next;
            Piece ld;
            ld.b = cross ? q.b : p.b;
            ld.g = cross ? q.g : p.g;
            ld.tile0 = cross ? q.tile0 : p.tile0;
            ld.len = cross ? q.len : p.len;
            ld.n = 0;
            const int ldt = cross ? 0 : (last_of_piece ? t : t + 1);

            if (PAGED) {
                // block ids of the tile requested now: fetched one step ahead inside a piece
                if (ahead_valid && !last_of_piece) { blk[0] = blk_ahead[0]; blk[1] = blk_ahead[1]; }
                else tile_blocks(a, ld, ldt, idle, blk);
                ahead_valid = t + 2 < p.n;
                if (ahead_valid) tile_blocks(a, p, t + 2, false, blk_ahead);
            }

#if GQA_MFMA_EARLY_V
            uint4 vt[8];
            transpose_values(vreg, vt);
            load_v<PAGED>(a, ld, ldt, idle, blk, i, kb, vreg);    // the V registers are free again
#endif
            f32x4 s[2];
            scores(kreg, qf, s);
#if GQA_MFMA_EARLY_K
            load_k<PAGED>(a, ld, ldt, idle, blk, i, kb, kreg);    // the K registers are free again
#endif
            const uint4 pb = softmax_update(s, st, kTileTokens * (p.tile0 + t), p.len, kb, c);
#if GQA_MFMA_EARLY_V
            weighted_values_t(vt, pb, st);
#else
            weighted_values(vreg, pb, st);
#endif
#if !GQA_MFMA_EARLY_K
            load_k<PAGED>(a, ld, ldt, idle, blk, i, kb, kreg);
#endif
#if !GQA_MFMA_EARLY_V
            load_v<PAGED>(a, ld, ldt, idle, blk, i, kb, vreg);
#endif

            if (!last_of_piece) { ++t; continue; }
            emit_piece(a, p, share, st, i, kb);
            if (!has_next) break;
            pos += p.n;
            p = q;
            t = 0;
            load_q(a, p, i, kb, qf);
            reset(st);
            has_next = pos + p.n < end;
            if (has_next) q = next_piece(a, p, end - pos - p.n);
            ahead_valid = false;
            settle_q(qf);
        }
    }
}

}  // namespace

hipError_t launch_partial_mfma(const KernelArgs& a, int workgroups, hipStream_t s) {
    if (a.page_size == 0)
        hipLaunchKernelGGL(partial_mfma_kernel<false>, dim3(workgroups), dim3(64 * GQA_MFMA_WAVES), 0, s, a);
    else
        hipLaunchKernelGGL(partial_mfma_kernel<true>, dim3(workgroups), dim3(64 * GQA_MFMA_WAVES), 0, s, a);
    return hipGetLastError();
}

int partial_mfma_occupancy() {
    int n = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&n, partial_mfma_kernel<false>, 64 * GQA_MFMA_WAVES, 0) != hipSuccess || n < 1)
        n = 1;
    return n < GQA_MFMA_WGS_PER_CU ? n : GQA_MFMA_WGS_PER_CU;
}

int partial_mfma_workers_per_group() { return GQA_MFMA_WAVES; }

}  // namespace gqa
