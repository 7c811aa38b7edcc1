// Host-only driver for the sanitizer build of libst3's sources (tests/test_host_sanitizers.py):
// walks the argument validation of every entry point with pointers that are never dereferenced on
// an error path, and runs the host-only helpers on real arrays.  No kernel is launched; the program
// runs on a box without a GPU.  Prints one line per check and exits non-zero on the first surprise.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "st3.h"

static int failures = 0;
#define EXPECT(call, want)                                                                       \
    do {                                                                                         \
        const int got_ = (int)(call);                                                            \
        if (got_ != (int)(want)) { std::printf("FAIL %s: got %d, want %d\n", #call, got_, (int)(want)); ++failures; } \
        else std::printf("ok   %s\n", #call);                                                    \
    } while (0)

int main() {
    void* const fake = reinterpret_cast<void*>(0x1000);
    float* const ffake = reinterpret_cast<float*>(0x1000);
    int32_t* const ifake = reinterpret_cast<int32_t*>(0x1000);
    st3_attn_shape sh{1, 4, 64, ST3_F32, 0.0f};
    st3_attn_shape bad{1, 4, 80, ST3_F32, 0.0f};
    st3_kv_layer kv{fake, fake, 4 * 128 * 64, 128 * 64, 64, 128, ST3_KV_PLAIN, nullptr, nullptr};
    st3_segments seg{8, 64, 100, ifake, ifake, nullptr, 0, 0};
    const size_t big = (size_t)1 << 30;

    EXPECT(st3_version() >> 8 >= 1, 1);
    EXPECT(std::strcmp(st3_status_string(ST3_OK), "ok") == 0, 1);
    EXPECT(st3_workspace_bytes(&bad, 100, 64, 1), 0);
    EXPECT(st3_workspace_bytes(&sh, 100, 64, 1) > 0, 1);
    EXPECT(st3_workspace_bytes(nullptr, 100, 64, 1), 0);
    EXPECT(st3_workspace_init(&sh, 128, nullptr, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_workspace_init(&sh, 128, fake, 16, nullptr), ST3_ERR_WORKSPACE_TOO_SMALL);

    EXPECT(st3_decode_attention(&bad, fake, &kv, &seg, fake, nullptr, 0, fake, big, nullptr), ST3_ERR_UNSUPPORTED);
    EXPECT(st3_decode_attention(&sh, nullptr, &kv, &seg, fake, nullptr, 0, fake, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_decode_attention(&sh, fake, &kv, &seg, fake, nullptr, 0, fake, 16, nullptr), ST3_ERR_WORKSPACE_TOO_SMALL);
    EXPECT(st3_decode_attention(&sh, fake, nullptr, &seg, fake, nullptr, 0, fake, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_decode_attention(&sh, fake, &kv, nullptr, fake, nullptr, 0, fake, big, nullptr), ST3_ERR_INVALID_ARG);
    st3_segments seg_big = seg; seg_big.max_kv_len = 129;
    EXPECT(st3_decode_attention(&sh, fake, &kv, &seg_big, fake, nullptr, 0, fake, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_decode_attention(&sh, fake, &kv, &seg, fake, ffake, 10, fake, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_decode_attention_noalloc(&sh, nullptr, &kv, &seg, fake, nullptr, 0, nullptr), ST3_ERR_INVALID_ARG);
    st3_attn_shape huge{64, 40, 128, ST3_BF16, 0.0f};
    st3_kv_layer kv_huge{fake, fake, (int64_t)40 * 4096 * 128, 4096 * 128, 128, 4096, ST3_KV_PLAIN, nullptr, nullptr};
    EXPECT(st3_decode_attention_noalloc(&huge, fake, &kv_huge, &seg, fake, nullptr, 0, nullptr), ST3_ERR_WORKSPACE_TOO_SMALL);
    EXPECT(st3_decode_attention_inherit(&sh, &kv, &seg, nullptr, big, 128, fake, fake, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_decode_attention_inherit(&sh, &kv, &seg, fake, 16, 128, fake, fake, big, nullptr), ST3_ERR_WORKSPACE_TOO_SMALL);

    st3_segments seg_full = seg; seg_full.max_kv_len = 128;
    EXPECT(st3_kv_append(&sh, &kv, &seg_full, fake, fake, nullptr), ST3_ERR_INVALID_ARG);
    st3_kv_layer kv_mis = kv; kv_mis.k = reinterpret_cast<void*>(0x1004);
    EXPECT(st3_kv_append(&sh, &kv_mis, &seg, fake, fake, nullptr), ST3_ERR_INVALID_ARG);
    st3_kv_layer kv_fp8 = kv; kv_fp8.format = ST3_KV_E4M3;
    EXPECT(st3_kv_append(&sh, &kv_fp8, &seg, fake, fake, nullptr), ST3_ERR_UNSUPPORTED);     // E4M3 needs bf16 I/O

    EXPECT(st3_select_topk(ffake, 10, nullptr, 0, 1, nullptr, 10, 11, nullptr, ifake, 11, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_select_topk(ffake, 20000, nullptr, 0, 1, nullptr, 20000, 5, nullptr, ifake, 5, nullptr), ST3_ERR_UNSUPPORTED);
    EXPECT(st3_select_topk(ffake, 10, nullptr, 0, 1, nullptr, 0, 0, nullptr, ifake, 0, nullptr), ST3_OK);   // n = 0: nothing to do
    EXPECT(st3_compact_rows(fake, 1, 1, 0, 0, 8, 6, ifake, 4, 4, 8, 0, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_compact_rows(fake, 1, 1, 0, 0, 8, 8, ifake, 4, 0, 8, 0, nullptr), ST3_OK);                   // nothing kept, no tail
    st3_gather_pair gp{fake, 1024, 256, 16, fake, 1024, 256, 16};
    EXPECT(st3_gather_rows(&gp, 1, 1, 1, 16, 0, ifake, 4, 4, 8, 0, nullptr), ST3_ERR_INVALID_ARG);          // src overlaps dst
    EXPECT(st3_gather_rows(&gp, 5, 1, 1, 16, 0, ifake, 4, 4, 8, 0, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_select_compact_layer(&sh, &kv, &seg, ffake, ifake, 64, 10, 7, fake, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_select_compact_layer(&sh, &kv, &seg, ffake, ifake, 64, -1, 0, fake, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_select_compact_layer(&sh, &kv, &seg, ffake, ifake, 10, 5, 0, fake, big, nullptr), ST3_ERR_INVALID_ARG);

    st3_tensor4 t4{fake, 4 * 128 * 64, 128 * 64, 64};
    EXPECT(st3_prefill_attention(&sh, &t4, &t4, &t4, 100, 50, 60, 1, &t4, nullptr, 0, fake, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_prefill_attention(&sh, &t4, &t4, &t4, 100, 8, 64, 17, &t4, nullptr, 0, fake, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_prefill_attention(&sh, &t4, &t4, &t4, 40000, 8, 64, 1, &t4, nullptr, 0, fake, big, nullptr), ST3_ERR_UNSUPPORTED);
    EXPECT(st3_prefill_attention(&sh, nullptr, &t4, &t4, 100, 8, 64, 1, &t4, nullptr, 0, fake, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_quantize_rows(&sh, &t4, &kv_fp8, 0, 10, nullptr), ST3_ERR_UNSUPPORTED);
    EXPECT(st3_quantize_rows(&sh, &t4, &kv, 2, 10, nullptr), ST3_ERR_INVALID_ARG);

    // fused steps: the whole-step array with a lazy layer that asks for a mass its source does not produce
    const size_t ws_bytes = st3_workspace_bytes(&sh, 128, 64, 1);
    std::vector<st3_layer_step> steps(3);
    for (int i = 0; i < 3; ++i) {
        st3_layer_step& s = steps[i];
        std::memset(&s, 0, sizeof(s));
        s.kv = kv; if (i) s.kv.k = nullptr;
        s.seg = seg;
        s.score_col = reinterpret_cast<float*>(0x100000 + 0x1000 * i);
        s.id_col = reinterpret_cast<int32_t*>(0x200000 + 0x1000 * i);
        s.col_stride = 64; s.keep_after = 60; s.inherit_from = i == 0 ? -1 : 0;
        s.q = s.k_new = s.v_new = fake; s.out = fake;
        s.vis_mass = i == 0 ? nullptr : ffake; s.mass_stride = 64;
        s.workspace = reinterpret_cast<void*>(0x10000000 * (i + 1)); s.workspace_bytes = ws_bytes;
    }
    EXPECT(st3_decode_step(&sh, 3, steps.data(), ST3_HOLE_FILL, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_decode_plans(&sh, 3, steps.data(), ST3_HOLE_FILL, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_decode_layer_attend(&sh, 3, steps.data(), 1, ST3_HOLE_FILL, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_decode_layer_attend(&sh, 3, steps.data(), 3, ST3_HOLE_FILL, nullptr), ST3_ERR_INVALID_ARG);
    steps[2].inherit_from = 2;
    EXPECT(st3_decode_step(&sh, 3, steps.data(), ST3_HOLE_FILL, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_decode_step(&sh, 0, steps.data(), ST3_HOLE_FILL, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_decode_layer_step(&sh, &kv, &seg_full, ffake, ifake, 64, 60, ST3_HOLE_FILL, fake, fake, fake, fake, nullptr, 0,
                                 fake, big, nullptr), ST3_ERR_INVALID_ARG);
    EXPECT(st3_decode_layer_step(&sh, &kv, &seg, ffake, ifake, 64, 60, 9, fake, fake, fake, fake, nullptr, 0, fake, big, nullptr),
           ST3_ERR_INVALID_ARG);

    // diagnostics on mass vectors
    EXPECT(st3_overlap_topk(ffake, ifake, 10, nullptr, 10, ffake, ifake, 10, nullptr, 10, 1, 5, 20000, ifake, ifake, nullptr),
           ST3_ERR_UNSUPPORTED);
    EXPECT(st3_cosine_similarity(nullptr, nullptr, 10, nullptr, 10, ffake, nullptr, 10, nullptr, 10, 1, 16, ffake, nullptr),
           ST3_ERR_INVALID_ARG);

    // host-only helpers on real arrays of exactly the documented sizes (the sanitizer watches their bounds)
    {
        const int L = 40, T = 512, nv = 576;
        std::vector<int32_t> keep_l(L), keep_lt((size_t)L * (T + 1));
        EXPECT(st3_schedule_pvtp(L, nv, 3, 4, 5000, 500, keep_l.data()), ST3_OK);
        EXPECT(keep_l[2] == nv && keep_l[3] == nv / 2 && keep_l[L - 1] == nv * 500 / 10000, 1);
        EXPECT(st3_schedule_linear(L, nv, 2, 1000, keep_l.data()), ST3_OK);
        EXPECT(keep_l[0] == nv && keep_l[L - 1] == 57, 1);
        for (int kind = ST3_ANNEAL_COS; kind <= ST3_ANNEAL_NONE; ++kind)
            EXPECT(st3_schedule_anneal(kind, kind == ST3_ANNEAL_DROP ? 4.0 : (double)T, T, keep_l.data(), L, keep_lt.data()), ST3_OK);
        EXPECT(st3_schedule_anneal(ST3_ANNEAL_COS, 0.0, 4, keep_l.data(), 2, keep_lt.data()), ST3_ERR_INVALID_ARG);
        EXPECT(st3_schedule_pvtp(32, 576, 3, 0, 5000, 100, keep_l.data()), ST3_ERR_INVALID_ARG);
        EXPECT(st3_schedule_linear(1, 576, 0, 1000, keep_l.data()), ST3_OK);       // a single layer: no span to fall over
        std::vector<int32_t> lens(L, 631);
        EXPECT(st3_kv_bytes(16, 40, 128, ST3_BF16, lens.data(), L) == (int64_t)16 * 631 * L * 2 * 40 * 128 * 2, 1);
        EXPECT(st3_kv_bytes(16, 40, 128, ST3_BF16, nullptr, L), -1);
    }
    EXPECT(st3_debug_set_attend_tile(4), st3_debug_enabled() ? ST3_OK : ST3_ERR_UNSUPPORTED);
    EXPECT(st3_profile_read(nullptr, nullptr, nullptr, nullptr), st3_debug_enabled() ? ST3_OK : ST3_ERR_UNSUPPORTED);
    std::printf("%d failures\n", failures);
    return failures == 0 ? 0 : 1;
}
