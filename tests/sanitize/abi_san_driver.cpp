// Exercises the host side of the C ABI (argument validation, workspace sizing, plan reporting,
// status strings) so that tests/test_sanitizers.py can run it under AddressSanitizer and
// UndefinedBehaviorSanitizer on the host.  Every call here either is a pure host function or is
// rejected before anything is launched; no device is needed.  Prints "abi ok" at the end.
#include "../../include/gqa_decode.h"
#include "../../include/concur_curation.h"

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#define EXPECT(cond) do { if (!(cond)) { std::printf("FAILED line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

static gqa_decode_params shape(int B, int Hq, int Hkv, int L, int page) {
    gqa_decode_params p;
    std::memset(&p, 0, sizeof p);
    p.batch = B; p.num_q_heads = Hq; p.num_kv_heads = Hkv; p.head_dim = 128; p.max_kv_len = L;
    p.page_size = page; p.block_table_stride = page ? (L + page - 1) / page : 0;
    p.scale = 0.088388f;
    p.q_stride_b = (int64_t)Hq * 128; p.q_stride_h = 128;
    p.k_stride_b = (int64_t)Hkv * (page ? page : L) * 128; p.k_stride_h = (int64_t)(page ? page : L) * 128; p.k_stride_t = 128;
    p.v_stride_b = p.k_stride_b; p.v_stride_h = p.k_stride_h; p.v_stride_t = p.k_stride_t;
    return p;
}

int main() {
    EXPECT(gqa_decode_version() >= 100);
    for (int code = -8; code <= 1; ++code) EXPECT(gqa_decode_strerror(code) != nullptr && std::strlen(gqa_decode_strerror(code)) > 0);

    gqa_decode_params p = shape(64, 40, 8, 16384, 0);
    const size_t need = gqa_decode_workspace_bytes(&p);
    EXPECT(need > 0 && need % 256 == 0);
    EXPECT(gqa_decode_workspace_bytes(nullptr) == 0);
    gqa_decode_params bad = p; bad.head_dim = 64;      EXPECT(gqa_decode_workspace_bytes(&bad) == 0);
    bad = p; bad.num_q_heads = 41;                    EXPECT(gqa_decode_workspace_bytes(&bad) == 0);
    bad = p; bad.num_q_heads = 8 * 17;                EXPECT(gqa_decode_workspace_bytes(&bad) == 0);
    bad = p; bad.chunk_tokens = 48;                   EXPECT(gqa_decode_workspace_bytes(&bad) == 0);
    bad = p; bad.page_size = 24; bad.block_table_stride = 1024; EXPECT(gqa_decode_workspace_bytes(&bad) == 0);
    bad = p; bad.batch = 1 << 20; bad.max_kv_len = 1 << 20;     EXPECT(gqa_decode_workspace_bytes(&bad) == 0);   // stream positions would overflow

    std::vector<int32_t> lens(64, 5000);
    int32_t share = -1, wgs = -1; int64_t slots = -1;
    EXPECT(gqa_decode_plan_info(&p, lens.data(), &share, &wgs, &slots) == GQA_OK && slots > 0 && wgs >= 0);
    EXPECT(gqa_decode_plan_info(&p, nullptr, nullptr, nullptr, nullptr) == GQA_OK);
    bad = p; bad.kernel_variant = 7;
    EXPECT(gqa_decode_plan_info(&bad, nullptr, &share, &wgs, &slots) == GQA_ERR_INVALID_ARG);

    // argument errors come back before anything touches a device; pointers are never dereferenced on the host
    alignas(256) static char fake[4096];
    void* dev = fake;
    EXPECT(gqa_decode_attn(&p, nullptr, dev, dev, (const int32_t*)dev, nullptr, nullptr, (float*)dev, nullptr, dev, need, nullptr) == GQA_ERR_INVALID_ARG);
    EXPECT(gqa_decode_attn(&p, dev, dev, dev, (const int32_t*)dev, nullptr, nullptr, (float*)dev, nullptr, dev, need - 1, nullptr) == GQA_ERR_WORKSPACE_TOO_SMALL);
    EXPECT(gqa_decode_attn(&p, fake + 2, dev, dev, (const int32_t*)dev, nullptr, nullptr, (float*)dev, nullptr, dev, need, nullptr) == GQA_ERR_INVALID_ARG);
    EXPECT(gqa_decode_attn(&p, dev, dev, dev, (const int32_t*)dev, nullptr, nullptr, (float*)dev, nullptr, fake + 16, need, nullptr) == GQA_ERR_INVALID_ARG);
    EXPECT(gqa_decode_attn(&p, dev, dev, dev, (const int32_t*)dev, (const int32_t*)dev, nullptr, (float*)dev, nullptr, dev, need, nullptr) == GQA_ERR_INVALID_ARG);
    bad = p; bad.k_stride_t = 132;
    EXPECT(gqa_decode_attn(&bad, dev, dev, dev, (const int32_t*)dev, nullptr, nullptr, (float*)dev, nullptr, dev, need, nullptr) == GQA_ERR_INVALID_ARG);
    EXPECT(gqa_decode_attn_static(&p, nullptr, dev, dev, (const int32_t*)dev, nullptr, (float*)dev, nullptr, nullptr) == GQA_ERR_INVALID_ARG);
    EXPECT(gqa_decode_attn_timed(&p, dev, dev, dev, (const int32_t*)dev, nullptr, nullptr, (float*)dev, nullptr, dev, need, nullptr, nullptr) == GQA_ERR_INVALID_ARG);
    EXPECT(gqa_decode_static_scratch_bytes() == GQA_DECODE_STATIC_SCRATCH_BYTES);

    gqa_cascade_params cp;
    std::memset(&cp, 0, sizeof cp);
    cp.decode = shape(10, 40, 8, 4096, 16);
    cp.num_groups = 2; cp.max_prefix_len = 2048;
    cp.kp_stride_g = 8 * 2048 * 128; cp.kp_stride_h = 2048 * 128; cp.kp_stride_t = 128;
    cp.vp_stride_g = cp.kp_stride_g; cp.vp_stride_h = cp.kp_stride_h; cp.vp_stride_t = 128;
    const size_t cneed = gqa_cascade_workspace_bytes(&cp);
    EXPECT(cneed > 0);
    const int32_t gs_decreasing[3] = {0, 12, 10};      // the second group would hold -2 sequences
    EXPECT(gqa_decode_attn_shared_prefix(&cp, dev, dev, dev, (const int32_t*)dev, (const int32_t*)dev, gs_decreasing, dev, dev,
                                         (const int32_t*)dev, (const int32_t*)dev, (float*)dev, nullptr, dev, cneed, nullptr) == GQA_ERR_INVALID_ARG);
    cp.decode.batch = 20;
    const int32_t gs20[3] = {0, 0, 20};
    EXPECT(gqa_decode_attn_shared_prefix(&cp, dev, dev, dev, (const int32_t*)dev, (const int32_t*)dev, gs20, dev, dev,
                                         (const int32_t*)dev, (const int32_t*)dev, (float*)dev, nullptr, dev, cneed * 4, nullptr) == GQA_ERR_UNSUPPORTED);

    gqa_prefill_params pp;
    std::memset(&pp, 0, sizeof pp);
    pp.batch = 1; pp.seq_len = 100; pp.num_q_heads = 40; pp.num_kv_heads = 8; pp.head_dim = 128; pp.scale = 0.1f;
    pp.q_stride_t = 40 * 128; pp.q_stride_h = 128; pp.k_stride_t = 8 * 128; pp.k_stride_h = 128;
    pp.v_stride_t = 8 * 128; pp.v_stride_h = 128; pp.o_stride_t = 40 * 128; pp.o_stride_h = 128;
    EXPECT(gqa_prefill_attn(&pp, nullptr, dev, dev, (float*)dev, nullptr, nullptr) == GQA_ERR_INVALID_ARG);
    pp.head_dim = 96;
    EXPECT(gqa_prefill_attn(&pp, dev, dev, dev, (float*)dev, nullptr, nullptr) == GQA_ERR_UNSUPPORTED);

    gqa_append_params ap;
    std::memset(&ap, 0, sizeof ap);
    ap.batch = 2; ap.num_q_heads = 40; ap.num_kv_heads = 8; ap.head_dim = 128; ap.max_kv_len = 100; ap.rope_positions = 50;
    ap.q_stride_b = 40 * 128; ap.q_stride_h = 128; ap.k_stride_b = 8 * 100 * 128; ap.k_stride_h = 100 * 128; ap.k_stride_t = 128;
    ap.v_stride_b = ap.k_stride_b; ap.v_stride_h = ap.k_stride_h; ap.v_stride_t = 128;
    EXPECT(gqa_decode_kv_append(&ap, dev, dev, dev, dev, dev, dev, (const int32_t*)dev, nullptr, (const float*)dev, nullptr) == GQA_ERR_INVALID_ARG);   // table shorter than the bound

    EXPECT(gqa_decode_stream_read(dev, 100, dev, 4, nullptr) == GQA_ERR_INVALID_ARG);
    gqa_timer* t = nullptr;
    EXPECT(gqa_timer_create(0, &t) == GQA_ERR_INVALID_ARG && t == nullptr);
    gqa_timer_destroy(nullptr);

    // host-only curation utilities on a small table
    const int64_t task[6] = {1, 1, 2, 2, 2, 3};
    const double sp[6] = {2.0, 0.0, 6.0, 1.5, 0.0, 0.0};
    const int32_t len[6] = {100, 50, 900, 400, 100, 10};
    const uint8_t single[6] = {0, 0, 1, 1, 0, 1};
    uint8_t flags[6]; int64_t counts[3];
    EXPECT(concur_select(6, task, sp, len, single, 5.0, 2, flags, counts) >= 0);
    EXPECT(concur_fast_p(6, sp, 1.0) == 0.5);
    std::printf("abi ok\n");
    return 0;
}
