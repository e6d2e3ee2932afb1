// Shared-prefix ("cascade") decode attention: split-KV partial kernel and combine kernel.
//
// The sequences of a batch come in groups -- the samples drawn for one prompt -- and all
// sequences of a group share the prompt's keys and values, which are stored once.  Each sequence
// attends over [shared prefix of its group ; its own suffix].  The prefix of a group is read ONCE
// per KV head and serves all M * G query rows of the group (M samples, G query heads per KV
// head): up to 64 rows = 4 MFMA column blocks per K/V tile, so this part is a real dense
// contraction.  The suffixes are handled exactly as in gqa_partial_mfma.hip.
//
// Stream split (see gqa_internal.h) over entries instead of sequences: entry e < num_groups is the
// prefix of group e, entry num_groups + b the suffix of sequence b; every entry has Hkv rows, one
// per KV head, of ceil(len / 32) tiles.  Row r = e * Hkv + g; a piece of share s writes its
// partial results to slot s + r, 64 columns per slot (column f = m * G + head-in-group for a
// prefix row, the head-in-group for a suffix row).  The combine kernel merges, for output row
// (b, h), the pieces of the prefix row of b's group and of b's suffix row.
#include "gqa_internal.h"
#include "gqa_mfma_tile.h"

#ifndef GQA_MFMA_WAVES
#define GQA_MFMA_WAVES 4
#endif

namespace gqa {

namespace {

using namespace tile;

constexpr int kMaxCb = kCascadeColumns / 16;      // MFMA column blocks a prefix row may need

__device__ __forceinline__ int entry_len_vec(const CascadeArgs& ca, int e) {      // per-lane loads
    const KernelArgs& a = ca.base;
    if (e < ca.num_groups) {
        const int m = ca.group_start[e + 1] - ca.group_start[e];
        return m > 0 ? min(max(ca.prefix_lens[e], 0), ca.max_prefix_len) : 0;
    }
    return clamped_len(a, e - ca.num_groups);
}

__device__ __forceinline__ int entry_len_uniform(const CascadeArgs& ca, int e) {  // scalar-path loads
    const KernelArgs& a = ca.base;
    if (e < ca.num_groups) {
        const int m = uniform_i32(ca.group_start, e + 1) - uniform_i32(ca.group_start, e);
        return m > 0 ? min(max(uniform_i32(ca.prefix_lens, e), 0), ca.max_prefix_len) : 0;
    }
    return uniform_len(a, e - ca.num_groups);
}

__device__ __forceinline__ int cascade_total(const CascadeArgs& ca, int entries) {
    const int lane = threadIdx.x & 63;
    int carry = 0;
    for (int base = 0; base < entries; base += 64) {
        const int e = base + lane;
        const int n = (e < entries) ? ca.base.num_kv_heads * tiles_of(entry_len_vec(ca, e)) : 0;
        carry += __shfl(wave_scan_incl(n), 63);
    }
    return carry;
}

// stream position -> (entry, kv head, tile, length); optionally writes every entry's position
__device__ __forceinline__ StreamPos cascade_locate(const CascadeArgs& ca, int entries, int pos, int32_t* prefix_out) {
    const int lane = threadIdx.x & 63;
    int carry = 0;
    StreamPos p;
    p.b = 0; p.g = 0; p.tile = 0; p.len = 0;
    for (int base = 0; base < entries; base += 64) {
        const int e = base + lane;
        const int len = (e < entries) ? entry_len_vec(ca, e) : 0;
        const int tb = tiles_of(len);
        const int n = ca.base.num_kv_heads * tb;
        const int incl = wave_scan_incl(n);
        const int excl = carry + incl - n;
        if (prefix_out != nullptr && e < entries) prefix_out[e] = excl;
        const bool hit = n > 0 && excl <= pos && pos < excl + n;
        const unsigned long long mask = __builtin_amdgcn_ballot_w64(hit);
        if (mask != 0) {
            const int src = __builtin_ctzll(mask);
            const int tbs = __shfl(tb, src), ex = __shfl(excl, src);
            p.b = base + src;
            p.g = (pos - ex) / tbs;
            p.tile = (pos - ex) % tbs;
            p.len = __shfl(len, src);
        }
        carry += __shfl(incl, 63);
    }
    if (prefix_out != nullptr && lane == 0) prefix_out[entries] = carry;
    return p;
}

struct CPiece {          // the part of a share inside one row; everything wave-uniform
    int e, g, tile0, n, len;
    bool prefix;         // row of a group's shared prefix
    int idx;             // group index (prefix) or sequence index (suffix)
    int b0;              // first sequence whose queries this row serves
    int ncols;           // query rows served: M * G (prefix) or G (suffix)
    int ncb;             // MFMA column blocks: ceil(ncols / 16)
};

__device__ __forceinline__ void describe(const CascadeArgs& ca, CPiece& p) {
    const int G = ca.base.group;
    p.prefix = p.e < ca.num_groups;
    if (p.prefix) {
        p.idx = p.e;
        p.b0 = uniform_i32(ca.group_start, p.e);
        const int m = uniform_i32(ca.group_start, p.e + 1) - p.b0;
        p.ncols = min(m * G, kCascadeColumns);
    } else {
        p.idx = p.e - ca.num_groups;
        p.b0 = p.idx;
        p.ncols = G;
    }
    p.ncb = (p.ncols + 15) >> 4;
}

__device__ __forceinline__ void tile_blocks(const CascadeArgs& ca, const CPiece& p, int tile, bool idle, int (&blk)[2]) {
    const KernelArgs& a = ca.base;
    const int tok0 = kTileTokens * (p.tile0 + tile);
    const int last = idle ? tok0 : p.len - 1;
    for (int hf = 0; hf < 2; ++hf) {
        const int tu = min(tok0 + 16 * hf, last);
        blk[hf] = uniform_i32(a.block_table, (int64_t)p.idx * a.block_table_stride + (tu >> a.page_shift));
    }
}

template <bool PAGED>
__device__ __forceinline__ void load_k(const CascadeArgs& ca, const CPiece& p, int tile, bool idle, const int (&blk)[2],
                                       int i, int kb, uint4 (&k)[2][4]) {
    const KernelArgs& a = ca.base;
    const int tok0 = kTileTokens * (p.tile0 + tile);
    const int last = idle ? tok0 : p.len - 1;
    const bool paged = PAGED && !p.prefix;
    const int tmask = paged ? (a.page_size - 1) : 0x7fffffff;
    const uint16_t* base = p.prefix ? ca.kp : a.k;
    const int64_t sb = p.prefix ? ca.kp_stride_g : a.k_stride_b;
    const int64_t sh = p.prefix ? ca.kp_stride_h : a.k_stride_h;
    const int64_t st = p.prefix ? ca.kp_stride_t : a.k_stride_t;
    for (int hf = 0; hf < 2; ++hf) {
        const int64_t row = (paged ? (int64_t)blk[hf] : (int64_t)p.idx) * sb + (int64_t)p.g * sh;
        const int tk = min(tok0 + 16 * hf + i, last);
        const uint16_t* kp = base + row + (int64_t)(tk & tmask) * st + (idle ? 0 : 8 * kb);
        for (int j = 0; j < 4; ++j) k[hf][j] = load_stream16(kp + (idle ? 0 : 32 * j));
    }
}

template <bool PAGED>
__device__ __forceinline__ void load_v(const CascadeArgs& ca, const CPiece& p, int tile, bool idle, const int (&blk)[2],
                                       int i, int kb, uint4 (&v)[8]) {
    const KernelArgs& a = ca.base;
    const int tok0 = kTileTokens * (p.tile0 + tile);
    const int last = idle ? tok0 : p.len - 1;
    const bool paged = PAGED && !p.prefix;
    const int tmask = paged ? (a.page_size - 1) : 0x7fffffff;
    const uint16_t* base = p.prefix ? ca.vp : a.v;
    const int64_t sb = p.prefix ? ca.vp_stride_g : a.v_stride_b;
    const int64_t sh = p.prefix ? ca.vp_stride_h : a.v_stride_h;
    const int64_t st = p.prefix ? ca.vp_stride_t : a.v_stride_t;
    for (int hf = 0; hf < 2; ++hf) {
        const int64_t row = (paged ? (int64_t)blk[hf] : (int64_t)p.idx) * sb + (int64_t)p.g * sh;
        for (int e4 = 0; e4 < 4; ++e4) {
            const int tv = min(tok0 + 16 * hf + 4 * kb + e4, last);
            v[4 * hf + e4] = load_stream16(base + row + (int64_t)(tv & tmask) * st + (idle ? 0 : 8 * i));
        }
    }
}

// Q^T operands of all column blocks: column f = 16 cb + i serves sample f / G, head-in-group f % G
__device__ __forceinline__ void load_q(const CascadeArgs& ca, const CPiece& p, int i, int kb, uint4 (&qf)[kMaxCb][4]) {
    const KernelArgs& a = ca.base;
    const int G = a.group;
#pragma unroll
    for (int cb = 0; cb < kMaxCb; ++cb) {
        for (int j = 0; j < 4; ++j) qf[cb][j] = make_uint4(0, 0, 0, 0);
        const int f = 16 * cb + i;
        if (f < p.ncols) {
            const int m = f / G, hh = f - m * G;
            const uint16_t* qrow = a.q + (int64_t)(p.b0 + m) * a.q_stride_b + (int64_t)(p.g * G + hh) * a.q_stride_h;
            for (int j = 0; j < 4; ++j) qf[cb][j] = *reinterpret_cast<const uint4*>(qrow + 8 * (4 * j + kb));
        }
    }
}

__device__ __forceinline__ void settle_all_q(uint4 (&qf)[kMaxCb][4]) {
#pragma unroll
    for (int cb = 0; cb < kMaxCb; ++cb) settle_q(qf[cb]);
}

__device__ __forceinline__ void emit_piece(const CascadeArgs& ca, const CPiece& p, int share, SoftmaxState (&st)[kMaxCb],
                                           int i, int kb) {
    const KernelArgs& a = ca.base;
    const int64_t slot = (int64_t)share + (int64_t)p.e * a.num_kv_heads + p.g;
#pragma unroll
    for (int cb = 0; cb < kMaxCb; ++cb) {
        if (cb >= p.ncb) continue;
        float l = st[cb].l;
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);
        const int f = 16 * cb + i;
        if (f < p.ncols) {
            float* dst = a.part_o + (slot * kCascadeColumns + f) * kHeadDim + 32 * kb;
            for (int r = 0; r < 4; ++r) {
                float4 lo4, hi4;
                lo4.x = st[cb].acc[0][r]; lo4.y = st[cb].acc[1][r]; lo4.z = st[cb].acc[2][r]; lo4.w = st[cb].acc[3][r];
                hi4.x = st[cb].acc[4][r]; hi4.y = st[cb].acc[5][r]; hi4.z = st[cb].acc[6][r]; hi4.w = st[cb].acc[7][r];
                *reinterpret_cast<float4*>(dst + 8 * r) = lo4;
                *reinterpret_cast<float4*>(dst + 8 * r + 4) = hi4;
            }
            if (kb == 0)
                *reinterpret_cast<float2*>(a.part_ml + (slot * kCascadeColumns + f) * 2) = make_float2(st[cb].m, l);
        }
    }
}

__device__ __forceinline__ CPiece next_piece(const CascadeArgs& ca, const CPiece& p, int left, int entries) {
    CPiece q = p;
    q.tile0 = 0;
    q.g = p.g + 1;
    if (q.g == ca.base.num_kv_heads) {
        q.g = 0;
        do { ++q.e; q.len = entry_len_uniform(ca, q.e); } while (q.len == 0 && q.e + 1 < entries);
        describe(ca, q);
    }
    q.n = min(tiles_of(q.len), left);
    return q;
}

template <bool PAGED>
__global__ __launch_bounds__(64 * GQA_MFMA_WAVES, 1) void partial_cascade_kernel(CascadeArgs ca) {
    const KernelArgs& a = ca.base;
    const int lane = threadIdx.x & 63;
    const int i = lane & 15, kb = lane >> 4;
    const float c = a.scale_log2e;
    const int entries = ca.num_groups + a.batch;
    const int worker = __builtin_amdgcn_readfirstlane(blockIdx.x * GQA_MFMA_WAVES + (threadIdx.x >> 6));
    const int workers = gridDim.x * GQA_MFMA_WAVES;

    const int total = __builtin_amdgcn_readfirstlane(cascade_total(ca, entries));
    const int share_tiles = share_tiles_for(total, a.fixed_share_tiles, workers);
    const int n_shares = (total + share_tiles - 1) / share_tiles;
    if (worker == 0) {
        if (lane == 0) { a.header[0] = total; a.header[1] = share_tiles; }
        if (total == 0) (void)cascade_locate(ca, entries, 0, a.row_prefix);
    }

    for (int share = worker; share < n_shares; share += workers) {
        int pos = share * share_tiles;
        const int end = min(pos + share_tiles, total);
        const StreamPos sp = cascade_locate(ca, entries, pos, share == 0 ? a.row_prefix : nullptr);
        CPiece p;
        p.e = __builtin_amdgcn_readfirstlane(sp.b);
        p.g = __builtin_amdgcn_readfirstlane(sp.g);
        p.tile0 = __builtin_amdgcn_readfirstlane(sp.tile);
        p.len = __builtin_amdgcn_readfirstlane(sp.len);
        p.n = min(tiles_of(p.len) - p.tile0, end - pos);
        describe(ca, p);

        uint4 kreg[2][4], vreg[8], qf[kMaxCb][4];
        SoftmaxState st[kMaxCb];
        int blk[2] = {0, 0};
        if (PAGED && !p.prefix) tile_blocks(ca, p, 0, false, blk);
        load_k<PAGED>(ca, p, 0, false, blk, i, kb, kreg);
        load_v<PAGED>(ca, p, 0, false, blk, i, kb, vreg);
        load_q(ca, p, i, kb, qf);
#pragma unroll
        for (int cb = 0; cb < kMaxCb; ++cb) reset(st[cb]);
        bool has_next = pos + p.n < end;
        CPiece q = has_next ? next_piece(ca, p, end - pos - p.n, entries) : p;
        int t = 0;
        settle_all_q(qf);

        while (true) {
            const bool last_of_piece = t + 1 == p.n;
            const bool cross = last_of_piece && has_next;
            const bool idle = last_of_piece && !has_next;
            const CPiece& ld = cross ? q : p;
            const int ldt = cross ? 0 : (last_of_piece ? t : t + 1);
            if (PAGED && !ld.prefix) tile_blocks(ca, ld, ldt, idle, blk);

            f32x4 s[kMaxCb][2];
#pragma unroll
            for (int cb = 0; cb < kMaxCb; ++cb)
                if (cb < p.ncb) scores(kreg, qf[cb], s[cb]);
            load_k<PAGED>(ca, ld, ldt, idle, blk, i, kb, kreg);          // the K registers are free again
            uint4 pb[kMaxCb];
#pragma unroll
            for (int cb = 0; cb < kMaxCb; ++cb)
                if (cb < p.ncb) pb[cb] = softmax_update(s[cb], st[cb], kTileTokens * (p.tile0 + t), p.len, kb, c);
            {   // O^T += V^T P^T for every column block: the transposed V operands are built once
                const uint32_t* v0 = reinterpret_cast<const uint32_t*>(&vreg[0]);
#pragma unroll
                for (int x2 = 0; x2 < 4; ++x2) {
                    uint4 even, odd;
                    uint32_t* pe = reinterpret_cast<uint32_t*>(&even);
                    uint32_t* po = reinterpret_cast<uint32_t*>(&odd);
                    for (int p2 = 0; p2 < 4; ++p2) {
                        const uint32_t lo = v0[(2 * p2) * 4 + x2];
                        const uint32_t hi = v0[(2 * p2 + 1) * 4 + x2];
                        pe[p2] = __builtin_amdgcn_perm(hi, lo, 0x05040100u);
                        po[p2] = __builtin_amdgcn_perm(hi, lo, 0x07060302u);
                    }
#pragma unroll
                    for (int cb = 0; cb < kMaxCb; ++cb)
                        if (cb < p.ncb) {
                            st[cb].acc[2 * x2] = mfma16(even, pb[cb], st[cb].acc[2 * x2]);
                            st[cb].acc[2 * x2 + 1] = mfma16(odd, pb[cb], st[cb].acc[2 * x2 + 1]);
                        }
                }
            }
            load_v<PAGED>(ca, ld, ldt, idle, blk, i, kb, vreg);

            if (!last_of_piece) { ++t; continue; }
            emit_piece(ca, p, share, st, i, kb);
            if (!has_next) break;
            pos += p.n;
            p = q;
            t = 0;
            load_q(ca, p, i, kb, qf);
#pragma unroll
            for (int cb = 0; cb < kMaxCb; ++cb) reset(st[cb]);
            has_next = pos + p.n < end;
            if (has_next) q = next_piece(ca, p, end - pos - p.n, entries);
            settle_all_q(qf);
        }
    }
}

// ---------------------------------------------------------------------------
// Combine for the cascade: output row (b, h) merges column f = (b - b0) * G + hh of the pieces
// of its group's prefix row and column hh of the pieces of its own suffix row.
// ---------------------------------------------------------------------------
struct Merge { float M, den; float2 acc; };

__device__ __forceinline__ void merge_row(const KernelArgs& a, int start, int tiles, int share_tiles, int r, int col,
                                          int lane, Merge& mg) {
    if (tiles <= 0) return;
    const int s_first = start / share_tiles;
    const int n = (start + tiles - 1) / share_tiles - s_first + 1;
    const float2* __restrict__ ml = reinterpret_cast<const float2*>(a.part_ml);
    const float2* __restrict__ po = reinterpret_cast<const float2*>(a.part_o);
    constexpr int kBatch = 8;
    for (int c0 = 0; c0 < n; c0 += kBatch) {
        float2 mlv[kBatch], ov[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int cc = min(c0 + u, n - 1);
            const int64_t w = ((int64_t)(s_first + cc) + r) * kCascadeColumns + col;
            mlv[u] = ml[w];
            ov[u] = po[w * (kHeadDim / 2) + lane];
        }
        float bm = mg.M;
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            if (c0 + u >= n) mlv[u].x = -INFINITY;
            bm = fmaxf(bm, mlv[u].x);
        }
        const float ms = (bm == -INFINITY) ? 0.f : bm;
        const float sa = exp2f(mg.M - ms);
        mg.den *= sa; mg.acc.x *= sa; mg.acc.y *= sa;
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const float wgt = exp2f(mlv[u].x - ms);
            mg.den = fmaf(wgt, mlv[u].y, mg.den);
            mg.acc.x = fmaf(wgt, ov[u].x, mg.acc.x);
            mg.acc.y = fmaf(wgt, ov[u].y, mg.acc.y);
        }
        mg.M = bm;
    }
}

__global__ __launch_bounds__(256) void combine_cascade_kernel(CascadeArgs ca) {
    const KernelArgs& a = ca.base;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.batch * a.num_q_heads) return;
    const int b = row / a.num_q_heads, h = row % a.num_q_heads;
    const int G = a.group, g = h / G, hh = h % G;
    const int32_t* __restrict__ gs = ca.group_start;
    const int32_t* __restrict__ pre = a.row_prefix;
    const int share_tiles = a.header[1];
    int lo = 0, hi = ca.num_groups;                 // group j with gs[j] <= b < gs[j + 1]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (gs[mid] <= b) lo = mid; else hi = mid;
    }
    const int j = lo;
    Merge mg;
    mg.M = -INFINITY; mg.den = 0.f; mg.acc = make_float2(0.f, 0.f);
    if (ca.num_groups > 0 && gs[j] <= b && b < gs[j + 1]) {
        const int col = (b - gs[j]) * G + hh;
        if (col < kCascadeColumns) {
            const int tiles = (pre[j + 1] - pre[j]) / a.num_kv_heads;
            merge_row(a, pre[j] + g * tiles, tiles, share_tiles, j * a.num_kv_heads + g, col, lane, mg);
        }
    }
    {
        const int e = ca.num_groups + b;
        const int tiles = (pre[e + 1] - pre[e]) / a.num_kv_heads;
        merge_row(a, pre[e] + g * tiles, tiles, share_tiles, e * a.num_kv_heads + g, hh, lane, mg);
    }
    const float inv = mg.den > 0.f ? 1.f / mg.den : 0.f;
    reinterpret_cast<float2*>(a.out)[(int64_t)row * (kHeadDim / 2) + lane] = make_float2(mg.acc.x * inv, mg.acc.y * inv);
    if (a.lse != nullptr && lane == 0)
        a.lse[row] = mg.den > 0.f ? 0.6931471805599453f * (mg.M + log2f(mg.den)) : -INFINITY;
}

}  // namespace

hipError_t launch_partial_cascade(const CascadeArgs& ca, int workgroups, hipStream_t s) {
    if (ca.base.page_size == 0)
        hipLaunchKernelGGL(partial_cascade_kernel<false>, dim3(workgroups), dim3(64 * GQA_MFMA_WAVES), 0, s, ca);
    else
        hipLaunchKernelGGL(partial_cascade_kernel<true>, dim3(workgroups), dim3(64 * GQA_MFMA_WAVES), 0, s, ca);
    return hipGetLastError();
}

hipError_t launch_combine_cascade(const CascadeArgs& ca, hipStream_t s) {
    const int rows = ca.base.batch * ca.base.num_q_heads;
    hipLaunchKernelGGL(combine_cascade_kernel, dim3((rows + 3) / 4), dim3(256), 0, s, ca);
    return hipGetLastError();
}

int partial_cascade_workers_per_group() { return GQA_MFMA_WAVES; }

}  // namespace gqa
