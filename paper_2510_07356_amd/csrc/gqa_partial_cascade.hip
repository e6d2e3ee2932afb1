// Shared-prefix ("cascade") decode attention: split-KV partial kernel and combine kernel.
//
// The sequences of a batch come in groups -- the samples drawn for one prompt -- and all
// sequences of a group share the prompt's keys and values, which are stored once.  Each sequence
// attends over [shared prefix of its group ; its own suffix].  One read of a prefix tile serves 16
// query rows (one MFMA column block) taken from the M * G query rows of the group (M samples, G
// query heads per KV head); a group with more than 16 such rows reads its prefix once per block of
// 16, i.e. ceil(M * G / 16) times instead of M times.  Every tile of the stream, prefix or suffix,
// then costs the same, which keeps the equal-share split balanced (a variant that served all 64
// rows from one read made prefix tiles 4x as expensive and the kernel as slow as its slowest
// wavefront).  The suffixes are handled exactly as in gqa_partial_mfma.hip.
//
// Stream split (see gqa_internal.h) over entries instead of sequences: entry e < num_groups is the
// prefix of group e with Hkv * ceil(M*G/16) rows (row index = g * blocks + block), entry
// num_groups + b the suffix of sequence b with Hkv rows; a row has ceil(len / 32) tiles.  Rows are
// numbered in stream order; a piece of share s writes its partial results to slot s + row, 16
// columns per slot.  The combine kernel merges, for output row (b, h), the pieces of the prefix
// row that holds its column and of b's suffix row.
#include "gqa_internal.h"
#include "gqa_mfma_tile.h"

#ifndef GQA_MFMA_WAVES
#define GQA_MFMA_WAVES 4
#endif

namespace gqa {

namespace {

using namespace tile;

struct EntryShape { int len, rows; };    // tokens per row, rows of the entry

__device__ __forceinline__ int blocks_of(int samples, int G) { return (min(samples * G, kCascadeColumns) + 15) >> 4; }

__device__ __forceinline__ EntryShape entry_shape_vec(const CascadeArgs& ca, int e) {      // per-lane loads
    const KernelArgs& a = ca.base;
    EntryShape s;
    if (e < ca.num_groups) {
        const int m = max(ca.group_start[e + 1] - ca.group_start[e], 0);
        s.rows = a.num_kv_heads * blocks_of(m, a.group);
        s.len = m > 0 ? min(max(ca.prefix_lens[e], 0), ca.max_prefix_len) : 0;
    } else {
        s.rows = a.num_kv_heads;
        s.len = clamped_len(a, e - ca.num_groups);
    }
    return s;
}

__device__ __forceinline__ EntryShape entry_shape_uniform(const CascadeArgs& ca, int e) {  // scalar-path loads
    const KernelArgs& a = ca.base;
    EntryShape s;
    if (e < ca.num_groups) {
        const int m = max(uniform_i32(ca.group_start, e + 1) - uniform_i32(ca.group_start, e), 0);
        s.rows = a.num_kv_heads * blocks_of(m, a.group);
        s.len = m > 0 ? min(max(uniform_i32(ca.prefix_lens, e), 0), ca.max_prefix_len) : 0;
    } else {
        s.rows = a.num_kv_heads;
        s.len = uniform_len(a, e - ca.num_groups);
    }
    return s;
}

__device__ __forceinline__ int cascade_total(const CascadeArgs& ca, int entries) {
    const int lane = threadIdx.x & 63;
    int carry = 0;
    for (int base = 0; base < entries; base += 64) {
        const int e = base + lane;
        int n = 0;
        if (e < entries) {
            const EntryShape s = entry_shape_vec(ca, e);
            n = s.rows * tiles_of(s.len);
        }
        carry += __shfl(wave_scan_incl(n), 63);
    }
    return carry;
}

struct CascadePos { int e, row_in_entry, tile, len, rows, first_row; };

// stream position -> entry, row within it, tile, row length, rows of the entry, number of its first row;
// optionally writes every entry's stream position and first row number
__device__ __forceinline__ CascadePos cascade_locate(const CascadeArgs& ca, int entries, int pos,
                                                     int32_t* tile_prefix_out, int32_t* row_prefix_out) {
    const int lane = threadIdx.x & 63;
    int carry = 0, row_carry = 0;
    CascadePos p;
    p.e = 0; p.row_in_entry = 0; p.tile = 0; p.len = 0; p.rows = 1; p.first_row = 0;
    for (int base = 0; base < entries; base += 64) {
        const int e = base + lane;
        EntryShape s;
        s.len = 0; s.rows = 0;
        if (e < entries) s = entry_shape_vec(ca, e);
        const int tb = tiles_of(s.len);
        const int n = s.rows * tb;
        const int incl = wave_scan_incl(n);
        const int excl = carry + incl - n;
        const int rincl = wave_scan_incl(s.rows);
        const int rexcl = row_carry + rincl - s.rows;
        if (tile_prefix_out != nullptr && e < entries) { tile_prefix_out[e] = excl; row_prefix_out[e] = rexcl; }
        const bool hit = n > 0 && excl <= pos && pos < excl + n;
        const unsigned long long mask = __builtin_amdgcn_ballot_w64(hit);
        if (mask != 0) {
            const int src = __builtin_ctzll(mask);
            const int tbs = __shfl(tb, src), ex = __shfl(excl, src);
            p.e = base + src;
            p.row_in_entry = (pos - ex) / tbs;
            p.tile = (pos - ex) % tbs;
            p.len = __shfl(s.len, src);
            p.rows = __shfl(s.rows, src);
            p.first_row = __shfl(rexcl, src);
        }
        carry += __shfl(incl, 63);
        row_carry += __shfl(rincl, 63);
    }
    if (tile_prefix_out != nullptr && lane == 0) { tile_prefix_out[entries] = carry; row_prefix_out[entries] = row_carry; }
    return p;
}

struct CPiece {          // the part of a share inside one row; everything wave-uniform
    int e, row_in_entry, rows, first_row;   // entry, row within it, rows of the entry, number of its first row
    int tile0, n, len;
    bool prefix;         // row of a group's shared prefix
    int idx;             // group index (prefix) or sequence index (suffix)
    int g;               // kv head
    int b0;              // first sequence whose queries this row serves
    int col0, ncols;     // query rows served: flat columns [col0, col0 + ncols) of the group (sample * G + head)
};

__device__ __forceinline__ void describe(const CascadeArgs& ca, CPiece& p) {
    const int G = ca.base.group;
    p.prefix = p.e < ca.num_groups;
    if (p.prefix) {
        const int blocks = p.rows / ca.base.num_kv_heads;
        p.idx = p.e;
        p.g = p.row_in_entry / blocks;
        p.b0 = uniform_i32(ca.group_start, p.e);
        const int m = uniform_i32(ca.group_start, p.e + 1) - p.b0;
        p.col0 = 16 * (p.row_in_entry - p.g * blocks);
        p.ncols = min(min(m * G, kCascadeColumns) - p.col0, 16);
    } else {
        p.idx = p.e - ca.num_groups;
        p.g = p.row_in_entry;
        p.b0 = p.idx;
        p.col0 = 0;
        p.ncols = G;
    }
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

// Q^T operand: MFMA column i serves flat column f = col0 + i of the row: sample f / G, head-in-group f % G
__device__ __forceinline__ void load_q(const CascadeArgs& ca, const CPiece& p, int i, int kb, uint4 (&qf)[4]) {
    const KernelArgs& a = ca.base;
    const int G = a.group;
    for (int j = 0; j < 4; ++j) qf[j] = make_uint4(0, 0, 0, 0);
    if (i < p.ncols) {
        const int f = p.col0 + i;
        const int m = f / G, hh = f - m * G;
        const uint16_t* qrow = a.q + (int64_t)(p.b0 + m) * a.q_stride_b + (int64_t)(p.g * G + hh) * a.q_stride_h;
        for (int j = 0; j < 4; ++j) qf[j] = *reinterpret_cast<const uint4*>(qrow + 8 * (4 * j + kb));
    }
}

__device__ __forceinline__ void emit_piece(const CascadeArgs& ca, const CPiece& p, int share, SoftmaxState& st,
                                           int i, int kb) {
    const KernelArgs& a = ca.base;
    float l = st.l;
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (i < p.ncols) {
        const int64_t slot = (int64_t)share + p.first_row + p.row_in_entry;
        float* dst = a.part_o + (slot * 16 + i) * kHeadDim + 32 * kb;
        for (int r = 0; r < 4; ++r) {
            float4 lo4, hi4;
            lo4.x = st.acc[0][r]; lo4.y = st.acc[1][r]; lo4.z = st.acc[2][r]; lo4.w = st.acc[3][r];
            hi4.x = st.acc[4][r]; hi4.y = st.acc[5][r]; hi4.z = st.acc[6][r]; hi4.w = st.acc[7][r];
            *reinterpret_cast<float4*>(dst + 8 * r) = lo4;
            *reinterpret_cast<float4*>(dst + 8 * r + 4) = hi4;
        }
        if (kb == 0) *reinterpret_cast<float2*>(a.part_ml + (slot * 16 + i) * 2) = make_float2(st.m, l);
    }
}

// The piece that follows p inside a share that still has `left` tiles after p.
__device__ __forceinline__ CPiece next_piece(const CascadeArgs& ca, const CPiece& p, int left, int entries) {
    CPiece q = p;
    q.tile0 = 0;
    q.row_in_entry = p.row_in_entry + 1;
    if (q.row_in_entry == p.rows) {
        q.row_in_entry = 0;
        int first = p.first_row + p.rows;
        EntryShape s;
        do {
            ++q.e;
            s = entry_shape_uniform(ca, q.e);
            if (s.len == 0) first += s.rows;          // rows of an empty entry still take numbers
        } while (s.len == 0 && q.e + 1 < entries);
        q.len = s.len;
        q.rows = s.rows;
        q.first_row = first;
    }
    describe(ca, q);
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
    int32_t* const row_numbers = a.row_prefix + entries + 1;       // first row number of every entry

    const int total = __builtin_amdgcn_readfirstlane(cascade_total(ca, entries));
    const int share_tiles = share_tiles_for(total, a.fixed_share_tiles, workers);
    const int n_shares = (total + share_tiles - 1) / share_tiles;
    if (worker == 0) {
        if (lane == 0) { a.header[0] = total; a.header[1] = share_tiles; }
        if (total == 0) (void)cascade_locate(ca, entries, 0, a.row_prefix, row_numbers);
    }

    for (int share = worker; share < n_shares; share += workers) {
        int pos = share * share_tiles;
        const int end = min(pos + share_tiles, total);
        const CascadePos sp = cascade_locate(ca, entries, pos, share == 0 ? a.row_prefix : nullptr, row_numbers);
        CPiece p;
        p.e = __builtin_amdgcn_readfirstlane(sp.e);
        p.row_in_entry = __builtin_amdgcn_readfirstlane(sp.row_in_entry);
        p.rows = __builtin_amdgcn_readfirstlane(sp.rows);
        p.first_row = __builtin_amdgcn_readfirstlane(sp.first_row);
        p.tile0 = __builtin_amdgcn_readfirstlane(sp.tile);
        p.len = __builtin_amdgcn_readfirstlane(sp.len);
        p.n = min(tiles_of(p.len) - p.tile0, end - pos);
        describe(ca, p);

        uint4 kreg[2][4], vreg[8], qf[4];
        SoftmaxState st;
        int blk[2] = {0, 0};
        if (PAGED && !p.prefix) tile_blocks(ca, p, 0, false, blk);
        load_k<PAGED>(ca, p, 0, false, blk, i, kb, kreg);
        load_v<PAGED>(ca, p, 0, false, blk, i, kb, vreg);
        load_q(ca, p, i, kb, qf);
        reset(st);
        bool has_next = pos + p.n < end;
        CPiece q = has_next ? next_piece(ca, p, end - pos - p.n, entries) : p;
        int t = 0;
        settle_q(qf);

        while (true) {
            // as in gqa_partial_mfma.hip: the next tile is requested unconditionally (one cache line
            // when nothing follows), V first (its registers are free after the transpose), K after the scores
            const bool last_of_piece = t + 1 == p.n;
            const bool cross = last_of_piece && has_next;
            const bool idle = last_of_piece && !has_next;
            const CPiece& ld = cross ? q : p;
            const int ldt = cross ? 0 : (last_of_piece ? t : t + 1);
            if (PAGED && !ld.prefix) tile_blocks(ca, ld, ldt, idle, blk);

            uint4 vt[8];
            transpose_values(vreg, vt);
            load_v<PAGED>(ca, ld, ldt, idle, blk, i, kb, vreg);
            f32x4 s[2];
            scores(kreg, qf, s);
            load_k<PAGED>(ca, ld, ldt, idle, blk, i, kb, kreg);
            const uint4 pb = softmax_update(s, st, kTileTokens * (p.tile0 + t), p.len, kb, c);
            weighted_values_t(vt, pb, st);

            if (!last_of_piece) { ++t; continue; }
            emit_piece(ca, p, share, st, i, kb);
            if (!has_next) break;
            pos += p.n;
            p = q;
            t = 0;
            load_q(ca, p, i, kb, qf);
            reset(st);
            has_next = pos + p.n < end;
            if (has_next) q = next_piece(ca, p, end - pos - p.n, entries);
            settle_q(qf);
        }
    }
}

// ---------------------------------------------------------------------------
// Combine for the cascade: output row (b, h), flat column f = (b - b0) * G + hh of its group,
// merges column f % 16 of the pieces of prefix row (g, f / 16) and column hh of the pieces of
// b's suffix row g.
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
            const int64_t w = ((int64_t)(s_first + cc) + r) * 16 + col;
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
    const int entries = ca.num_groups + a.batch;
    const int32_t* __restrict__ gs = ca.group_start;
    const int32_t* __restrict__ pre = a.row_prefix;                 // stream position of every entry
    const int32_t* __restrict__ num = a.row_prefix + entries + 1;   // first row number of every entry
    const int share_tiles = a.header[1];
    int lo = 0, hi = ca.num_groups;                 // group j with gs[j] <= b < gs[j + 1]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (gs[mid] <= b) lo = mid; else hi = mid;
    }
    const int j = lo;
    Merge mg;
    mg.M = -INFINITY; mg.den = 0.f; mg.acc = make_float2(0.f, 0.f);
    if (gs[j] <= b && b < gs[j + 1]) {
        const int f = (b - gs[j]) * G + hh;
        const int rows = num[j + 1] - num[j];
        const int blocks = rows / a.num_kv_heads;
        if (f < kCascadeColumns && rows > 0) {
            const int tiles = (pre[j + 1] - pre[j]) / rows;
            const int idx = g * blocks + (f >> 4);
            merge_row(a, pre[j] + idx * tiles, tiles, share_tiles, num[j] + idx, f & 15, lane, mg);
        }
    }
    {
        const int e = ca.num_groups + b;
        const int tiles = (pre[e + 1] - pre[e]) / a.num_kv_heads;
        merge_row(a, pre[e] + g * tiles, tiles, share_tiles, num[e] + g, hh, lane, mg);
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
