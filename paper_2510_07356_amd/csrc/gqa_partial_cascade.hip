// Shared-prefix ("cascade") decode attention: split-KV partial kernel and combine kernel.
//
// The sequences of a batch come in groups -- the samples drawn for one prompt -- and all
// sequences of a group share the prompt's keys and values, which are stored once.  Each sequence
// attends over [shared prefix of its group ; its own suffix].  One read of a prefix tile serves
// 32 of the group's M * G query rows (M samples, G query heads per KV head): two MFMA column
// blocks of 16 take their turns while the K and V^T operands of the tile stay in registers.  A
// group of up to 32 query rows (5 samples x 5 heads) therefore reads its prefix once instead of
// M times, a group of up to 64 (10 x 5) twice instead of 10 times.  (Four blocks per read do not
// fit the register file without spilling.)  The suffixes are handled exactly as in
// gqa_partial_mfma.hip (one block of G columns).
//
// Stream split by cost.  An entry is a group's prefix (entry e < num_groups) or a sequence's
// suffix (entry num_groups + b).  A suffix entry has one row per KV head; a prefix entry has, per
// KV head, one row per 32 query rows (read 0, and read 1 if the group has more than 32).  A row
// has ceil(len / 32) tiles; a tile of a row with nb column blocks costs
// kCostTile + kCostBlock * (nb - 1) units: reading it dominates, the second block adds its
// arithmetic.  All rows are laid end to end on a cost axis (entry, KV head, read), which is cut
// into equal shares, one per persistent wavefront; share s owns the tiles whose START lies in
// [s * share_cost, (s + 1) * share_cost).  With share_cost at least the largest tile cost, every
// share between the first and the last tile start of a row owns at least one tile of it, which
// is what the combine kernel relies on.
//
// Partial results: a piece (the tiles of one row inside one share) of a prefix row writes one
// partial per column block to the prefix area, slot share + 2 (e * Hkv + g) + read, 32 columns
// per slot; a piece of a suffix row writes to the suffix area, slot share + (b * Hkv + g), 16
// columns per slot.  share + row number grows strictly along the stream, so slots are unique.
#include "gqa_internal.h"
#include "gqa_mfma_tile.h"

#ifndef GQA_MFMA_WAVES
#define GQA_MFMA_WAVES 4
#endif

namespace gqa {

namespace {

using namespace tile;

struct EntryShape { int len, cols; };    // tokens per row (0: the entry has no work), query rows served

// column blocks of read r of an entry that serves `cols` query rows (32 per read)
__device__ __forceinline__ int blocks_of_read(int cols, int r) { return min(max(cols - 32 * r, 1), 32) > 16 ? 2 : 1; }
__device__ __forceinline__ int reads_of(int cols) { return cols > 32 ? 2 : 1; }
// cost of one tile position of one KV head of the entry, over all its reads, and of read 0 alone
__device__ __forceinline__ int head_tile_cost(int cols) {
    return cascade_tile_cost(blocks_of_read(cols, 0)) + (cols > 32 ? cascade_tile_cost(blocks_of_read(cols, 1)) : 0);
}

// Shape of entry e.  UNIFORM: e is wave-uniform and the loads go through the scalar path.  Otherwise
// e differs per lane (any value is allowed; the result for e >= entries is an entry without work)
// and all four loads are issued at once, from clamped indices, before anything is selected: a
// version that branches on the kind of entry makes the wavefront wait for up to three dependent
// round trips where this one waits for one.
template <bool UNIFORM>
__device__ __forceinline__ EntryShape entry_shape(const CascadeArgs& ca, int e) {
    const KernelArgs& a = ca.base;
    EntryShape s;
    if (UNIFORM) {
        if (e < ca.num_groups) {
            const int m = max(uniform_i32(ca.group_start, e + 1) - uniform_i32(ca.group_start, e), 0);
            s.cols = min(m * a.group, kCascadeColumns);
            s.len = m > 0 ? min(max(uniform_i32(ca.prefix_lens, e), 0), ca.max_prefix_len) : 0;
        } else {
            s.cols = a.group;
            s.len = uniform_len(a, e - ca.num_groups);
        }
        return s;
    }
    const int ng = ca.num_groups;
    const int j = min(e, ng - 1), b = min(max(e - ng, 0), a.batch - 1);
    const int g0 = ca.group_start[j], g1 = ca.group_start[j + 1];
    const int pl = ca.prefix_lens[j], kl = a.kv_lens[b];
    const int m = max(g1 - g0, 0);
    const bool prefix = e < ng;
    s.cols = prefix ? min(m * a.group, kCascadeColumns) : a.group;
    const int plen = m > 0 ? min(max(pl, 0), ca.max_prefix_len) : 0;
    const int slen = e < ng + a.batch ? min(max(kl, 0), a.max_kv_len) : 0;
    s.len = prefix ? plen : slen;
    return s;
}

__device__ __forceinline__ int cascade_total(const CascadeArgs& ca, int entries) {
    const int lane = threadIdx.x & 63;
    int carry = 0;
    for (int base = 0; base < entries; base += 64) {
        const int e = base + lane;
        const EntryShape s = entry_shape<false>(ca, e);
        const int n = ca.base.num_kv_heads * tiles_of(s.len) * head_tile_cost(s.cols);
        carry += __shfl(wave_scan_incl(n), 63);
    }
    return carry;
}

// The row whose cost range holds `pos`, and the first tile of it that starts at or after `pos`
// (tile == tiles of the row when no tile of the row does).  Optionally writes every entry's
// position on the cost axis.
struct CascadePos { int e, g, r, tile, len, cols, row_start; };

__device__ __forceinline__ CascadePos cascade_locate(const CascadeArgs& ca, int entries, int pos, int32_t* prefix_out) {
    const int lane = threadIdx.x & 63;
    int carry = 0;
    CascadePos p;
    p.e = 0; p.g = 0; p.r = 0; p.tile = 0; p.len = 0; p.cols = 1; p.row_start = 0;
    for (int base = 0; base < entries; base += 64) {
        const int e = base + lane;
        const EntryShape s = entry_shape<false>(ca, e);
        const int head_cost = tiles_of(s.len) * head_tile_cost(s.cols);
        const int n = ca.base.num_kv_heads * head_cost;
        const int incl = wave_scan_incl(n);
        const int excl = carry + incl - n;
        if (prefix_out != nullptr && e < entries) prefix_out[e] = excl;
        const bool hit = n > 0 && excl <= pos && pos < excl + n;
        const unsigned long long mask = __builtin_amdgcn_ballot_w64(hit);
        if (mask != 0) {                                  // at most one lane hits
            const int src = __builtin_ctzll(mask);
            const int hc = __shfl(head_cost, src), ex = __shfl(excl, src);
            p.e = base + src;
            p.len = __shfl(s.len, src);
            p.cols = __shfl(s.cols, src);
            p.g = (pos - ex) / hc;
            p.row_start = ex + p.g * hc;
            const int first_read = tiles_of(p.len) * cascade_tile_cost(blocks_of_read(p.cols, 0));
            p.r = (pos - p.row_start >= first_read) ? 1 : 0;
            p.row_start += p.r * first_read;
            const int w = cascade_tile_cost(blocks_of_read(p.cols, p.r));
            p.tile = (pos - p.row_start + w - 1) / w;
        }
        carry += __shfl(incl, 63);
    }
    if (prefix_out != nullptr && lane == 0) prefix_out[entries] = carry;
    return p;
}

struct CPiece {          // the part of a share inside one row; everything wave-uniform
    int e, g, r;         // entry, kv head, read (which 32 query rows of a prefix entry)
    int len, cols;       // tokens of the row, query rows the ENTRY serves
    int nb;              // column blocks of this row
    int row_start;       // position of the row's first tile on the cost axis
    int tile0, n;        // first tile and number of tiles of the piece
    int prefix;          // 1: row of a group's shared prefix (an int keeps the struct free of padding)
    int idx;             // group index (prefix) or sequence index (suffix)
    int b0;              // first sequence whose queries the entry serves
};

__device__ __forceinline__ void describe(const CascadeArgs& ca, CPiece& p) {
    p.prefix = p.e < ca.num_groups ? 1 : 0;
    p.idx = p.prefix ? p.e : p.e - ca.num_groups;
    p.b0 = p.prefix ? uniform_i32(ca.group_start, p.e) : p.idx;
    p.nb = blocks_of_read(p.cols, p.r);
}

// tiles of a row (first tile at row_start on the cost axis) that start before `share_end`
__device__ __forceinline__ int tiles_before(int row_start, int nb, int tiles, int share_end) {
    const int w = cascade_tile_cost(nb);
    return min(tiles, (share_end - row_start + w - 1) / w);
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

// Q^T operand of column block `block` of the row: MFMA column i serves flat column
// f = 32 read + 16 block + i of the entry: sample f / G, head-in-group f % G
__device__ __forceinline__ void load_q(const CascadeArgs& ca, const CPiece& p, int block, int i, int kb, uint4 (&qf)[4]) {
    const KernelArgs& a = ca.base;
    const int G = a.group;
    for (int j = 0; j < 4; ++j) qf[j] = make_uint4(0, 0, 0, 0);
    const int f = 32 * p.r + 16 * block + i;
    if (f < p.cols) {
        const int m = f / G, hh = f - m * G;
        const uint16_t* qrow = a.q + (int64_t)(p.b0 + m) * a.q_stride_b + (int64_t)(p.g * G + hh) * a.q_stride_h;
        for (int j = 0; j < 4; ++j) qf[j] = *reinterpret_cast<const uint4*>(qrow + 8 * (4 * j + kb));
    }
}

// Partial result of column block `block` of a finished piece
__device__ __forceinline__ void emit_block(const CascadeArgs& ca, const CPiece& p, int share, int block, SoftmaxState& st,
                                           int i, int kb) {
    const KernelArgs& a = ca.base;
    float l = st.l;
    l += __shfl_xor(l, 16);
    l += __shfl_xor(l, 32);
    if (32 * p.r + 16 * block + i < p.cols) {
        const int64_t row = (int64_t)p.idx * a.num_kv_heads + p.g;
        const int64_t col = p.prefix ? ((int64_t)share + 2 * row + p.r) * 32 + 16 * block + i : ((int64_t)share + row) * 16 + i;
        float* dst = (p.prefix ? ca.part_o_prefix : a.part_o) + col * kHeadDim + 32 * kb;
        for (int r = 0; r < 4; ++r) {
            float4 lo4, hi4;
            lo4.x = st.acc[0][r]; lo4.y = st.acc[1][r]; lo4.z = st.acc[2][r]; lo4.w = st.acc[3][r];
            hi4.x = st.acc[4][r]; hi4.y = st.acc[5][r]; hi4.z = st.acc[6][r]; hi4.w = st.acc[7][r];
            *reinterpret_cast<float4*>(dst + 8 * r) = lo4;
            *reinterpret_cast<float4*>(dst + 8 * r + 4) = hi4;
        }
        if (kb == 0)
            *reinterpret_cast<float2*>((p.prefix ? ca.part_ml_prefix : a.part_ml) + col * 2) = make_float2(st.m, l);
    }
}

// The row after p's, if its first tile starts before share_end: fills q and returns true.
__device__ __forceinline__ bool next_piece(const CascadeArgs& ca, const CPiece& p, int share_end, int entries, CPiece& q) {
    const int row_end = p.row_start + tiles_of(p.len) * cascade_tile_cost(p.nb);
    if (row_end >= share_end) return false;              // share_end <= total: a row starts at row_end
    q = p;
    q.row_start = row_end;
    q.tile0 = 0;
    if (p.r + 1 < reads_of(p.cols)) {
        q.r = p.r + 1;
    } else {
        q.r = 0;
        q.g = p.g + 1;
        if (q.g == ca.base.num_kv_heads) {
            q.g = 0;
            EntryShape s;
            do {                                          // entries without work take no room on the cost axis
                ++q.e;
                s = entry_shape<true>(ca, q.e);
            } while (s.len == 0 && q.e + 1 < entries);
            q.len = s.len;
            q.cols = s.cols;
        }
    }
    describe(ca, q);
    q.n = tiles_before(q.row_start, q.nb, tiles_of(q.len), share_end);
    return true;
}

// All tiles of piece p with NB column blocks per tile.  On entry kreg / vreg hold (or await) the
// piece's first tile; on exit they hold the first tile of `next` if there is one.  The next tile is
// requested unconditionally (one cache line when nothing follows), V first (its registers are free
// after the transpose), K after the scores of all blocks, as in gqa_partial_mfma.hip.
template <int NB, bool PAGED>
__device__ __forceinline__ void run_piece(const CascadeArgs& ca, const CPiece& p, bool has_next, const CPiece& next,
                                          int share, int i, int kb, float c, uint4 (&kreg)[2][4], uint4 (&vreg)[8]) {
    uint4 qf[NB][4];
    SoftmaxState st[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        load_q(ca, p, b, i, kb, qf[b]);
        reset(st[b]);
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) settle_q(qf[b]);
    int blk[2] = {0, 0};
    for (int t = 0; t < p.n; ++t) {
        const bool last_of_piece = t + 1 == p.n;
        const bool cross = last_of_piece && has_next;
        const bool idle = last_of_piece && !has_next;
        const CPiece& ld = cross ? next : p;
        const int ldt = cross ? 0 : (last_of_piece ? t : t + 1);
        if (PAGED && !ld.prefix) tile_blocks(ca, ld, ldt, idle, blk);

        uint4 vt[8];
        transpose_values(vreg, vt);
        load_v<PAGED>(ca, ld, ldt, idle, blk, i, kb, vreg);
        f32x4 s[NB][2];
#pragma unroll
        for (int b = 0; b < NB; ++b) scores(kreg, qf[b], s[b]);
        load_k<PAGED>(ca, ld, ldt, idle, blk, i, kb, kreg);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const uint4 pb = softmax_update(s[b], st[b], kTileTokens * (p.tile0 + t), p.len, kb, c);
            weighted_values_t(vt, pb, st[b]);
        }
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) emit_block(ca, p, share, b, st[b], i, kb);
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
    const int share_cost = cascade_share_cost(total, a.fixed_share_tiles, workers);
    const int n_shares = (total + share_cost - 1) / share_cost;
    if (worker == 0) {
        if (lane == 0) { a.header[0] = total; a.header[1] = share_cost; }
        if (total == 0) (void)cascade_locate(ca, entries, 0, a.row_prefix);
    }

    for (int share = worker; share < n_shares; share += workers) {
        const int begin = share * share_cost;
        const int end = min(begin + share_cost, total);
        CascadePos sp = cascade_locate(ca, entries, begin, share == 0 ? a.row_prefix : nullptr);
        if (sp.tile == tiles_of(sp.len)) {
            // no tile of that row starts inside the share: the share begins with the next row, if that starts in time
            const int row_end = sp.row_start + tiles_of(sp.len) * cascade_tile_cost(blocks_of_read(sp.cols, sp.r));
            if (row_end >= end) continue;
            sp = cascade_locate(ca, entries, row_end, nullptr);
        }
        CPiece p;
        p.e = __builtin_amdgcn_readfirstlane(sp.e);
        p.g = __builtin_amdgcn_readfirstlane(sp.g);
        p.r = __builtin_amdgcn_readfirstlane(sp.r);
        p.len = __builtin_amdgcn_readfirstlane(sp.len);
        p.cols = __builtin_amdgcn_readfirstlane(sp.cols);
        p.row_start = __builtin_amdgcn_readfirstlane(sp.row_start);
        p.tile0 = __builtin_amdgcn_readfirstlane(sp.tile);
        describe(ca, p);
        p.n = tiles_before(p.row_start, p.nb, tiles_of(p.len), end) - p.tile0;

        uint4 kreg[2][4], vreg[8];
        {
            int blk[2] = {0, 0};
            if (PAGED && !p.prefix) tile_blocks(ca, p, 0, false, blk);
            load_k<PAGED>(ca, p, 0, false, blk, i, kb, kreg);
            load_v<PAGED>(ca, p, 0, false, blk, i, kb, vreg);
        }
        while (true) {
            CPiece q;
            const bool has_next = next_piece(ca, p, end, entries, q);
            if (!has_next) q = p;
            if (p.nb == 1) run_piece<1, PAGED>(ca, p, has_next, q, share, i, kb, c, kreg, vreg);
            else run_piece<2, PAGED>(ca, p, has_next, q, share, i, kb, c, kreg, vreg);
            if (!has_next) break;
            p = q;
        }
    }
}

// ---------------------------------------------------------------------------
// Combine for the cascade: output row (b, h), flat column f = (b - b0) * G + hh of its group,
// merges column f % 32 of the pieces of prefix row (group, g, read f / 32) and column hh of the
// pieces of b's suffix row g.
// ---------------------------------------------------------------------------
// The pieces of one row: shares s_first .. s_first + n - 1; the piece of share s sits at column
// (s + row) * stride + col of its area.
struct RowPieces {
    const float2* ml;
    const float2* o;
    int s_first, n, row, stride, col;
};

__device__ __forceinline__ RowPieces row_pieces(const float* part_ml, const float* part_o, int row_start, int tiles, int w,
                                                int share_cost, int row, int stride, int col) {
    RowPieces r;
    r.ml = reinterpret_cast<const float2*>(part_ml);
    r.o = reinterpret_cast<const float2*>(part_o);
    r.s_first = tiles > 0 ? row_start / share_cost : 0;
    r.n = tiles > 0 ? (row_start + (tiles - 1) * w) / share_cost - r.s_first + 1 : 0;
    r.row = row; r.stride = stride; r.col = col;
    return r;
}

__global__ __launch_bounds__(256) void combine_cascade_kernel(CascadeArgs ca) {
    const KernelArgs& a = ca.base;
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= a.batch * a.num_q_heads) return;
    const int b = row / a.num_q_heads, h = row % a.num_q_heads;
    const int G = a.group, g = h / G, hh = h % G;
    const int32_t* __restrict__ gs = ca.group_start;
    const int32_t* __restrict__ pre = a.row_prefix;                 // position of every entry on the cost axis
    const int share_cost = a.header[1];
    // Everything the row needs to know about its group and its sequence is requested at once, so that the
    // wavefront waits for one round trip before it asks for the pieces: lane i holds group i's start, prefix
    // length and position on the cost axis, and the group of b is picked out of the lanes afterwards.
    // The last group j with gs[j] <= b holds b: gs rises, so the lanes whose entry is <= b form a prefix.
    const int e = ca.num_groups + b;
    const int pre_e = pre[e];
    const int len_b = clamped_len(a, b);
    int j, g0, g1, plen_j, pre_j;
    if (ca.num_groups < 64) {
        const int ig = min(lane, ca.num_groups - 1);
        const int v = gs[min(lane, ca.num_groups)];          // gs has num_groups + 1 entries
        const int pl = ca.prefix_lens[ig];
        const int pj = pre[ig];
        const int count = __builtin_popcountll(__builtin_amdgcn_ballot_w64(lane < ca.num_groups && v <= b));
        j = max(count - 1, 0);
        g0 = __shfl(v, j); g1 = __shfl(v, j + 1);
        plen_j = __shfl(pl, j); pre_j = __shfl(pj, j);
    } else {
        int count = 0;
        for (int base = 0; base < ca.num_groups; base += 64) {
            const int idx = base + lane;
            const int v = idx < ca.num_groups ? gs[idx] : 0x7fffffff;
            count += __builtin_popcountll(__builtin_amdgcn_ballot_w64(v <= b));
        }
        j = max(count - 1, 0);
        g0 = gs[j]; g1 = gs[j + 1];
        plen_j = ca.prefix_lens[j]; pre_j = pre[j];
    }
    // pieces of the prefix row (group j, g, read f / 32), then of b's suffix row g
    RowPieces rp[2];
    {
        const int m = max(g1 - g0, 0);                       // the shape of entry j, as entry_shape computes it
        const int cols = min(m * G, kCascadeColumns);
        const int plen = m > 0 ? min(max(plen_j, 0), ca.max_prefix_len) : 0;
        const int f = (b - g0) * G + hh;
        const bool served = g0 <= b && b < g1 && f < kCascadeColumns;
        const int tiles = served ? tiles_of(plen) : 0, r = (f >> 5) & 1;
        const int w = cascade_tile_cost(blocks_of_read(cols, r));
        const int row_start = pre_j + g * tiles * head_tile_cost(cols) + r * tiles * cascade_tile_cost(blocks_of_read(cols, 0));
        rp[0] = row_pieces(ca.part_ml_prefix, ca.part_o_prefix, row_start, tiles, w, share_cost,
                           2 * (j * a.num_kv_heads + g) + r, 32, f & 31);
        const int ws = cascade_tile_cost(1), stiles = tiles_of(len_b);
        rp[1] = row_pieces(a.part_ml, a.part_o, pre_e + g * stiles * ws, stiles, ws, share_cost, b * a.num_kv_heads + g, 16, hh);
    }
    // one list of n pieces, merged in order with a running maximum, eight at a time so that their
    // loads are in flight together (prefix and suffix pieces in the same batch)
    const int n0 = rp[0].n, n = n0 + rp[1].n;
    constexpr int kBatch = 8;
    float M = -INFINITY, den = 0.f;
    float2 acc = make_float2(0.f, 0.f);
    for (int c0 = 0; c0 < n; c0 += kBatch) {
        float2 mlv[kBatch], ov[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int cc = min(c0 + u, n - 1);
            const RowPieces& r = cc < n0 ? rp[0] : rp[1];
            const int64_t wi = ((int64_t)(r.s_first + (cc < n0 ? cc : cc - n0)) + r.row) * r.stride + r.col;
            mlv[u] = r.ml[wi];
            ov[u] = r.o[wi * (kHeadDim / 2) + lane];
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
            const float wgt = exp2f(mlv[u].x - ms);
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
