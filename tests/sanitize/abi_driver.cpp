// Host-only driver for a sanitizer build of the C ABI's argument layer: every call below is rejected by
// the host-side checks or is host-only arithmetic, so nothing is launched and no GPU is needed.  The process
// runs under AddressSanitizer and UndefinedBehaviorSanitizer; a report makes it exit non-zero.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/loma.h"

static int failures = 0;
#define EXPECT(call, want)                                                                     \
    do {                                                                                       \
        const long long got_ = (long long)(call);                                              \
        if (got_ != (long long)(want)) { std::printf("FAIL %s = %lld, want %lld\n", #call, got_, (long long)(want)); ++failures; } \
    } while (0)

int main() {
    void* P = reinterpret_cast<void*>(0x10000);      // non-null, 16-byte aligned, never dereferenced on the host
    void* P2 = reinterpret_cast<void*>(0x20000);
    void* odd = reinterpret_cast<void*>(0x10004);
    // status strings for every code and an unknown one
    for (int code = 1; code >= -6; --code) if (loma_status_string(code) == nullptr) ++failures;
    EXPECT(loma_abi_version() >= 1, 1);
    // mask pass and its gradients
    EXPECT(loma_mask_attn_fwd(nullptr, P, P, P, nullptr, 1, 1, 128, 16, 4, 2, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_mask_attn_fwd(P, odd, P, P, nullptr, 1, 1, 128, 16, 4, 2, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_mask_attn_fwd(P, P, P, P, nullptr, 1, 1, 128, 16, 4, 1 << 28, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_UNSUPPORTED);
    EXPECT(loma_mask_attn_fwd(P, P, P, P, nullptr, 1, 1, 100, 16, 4, 2, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_UNSUPPORTED);
    EXPECT(loma_mask_attn_fwd(P, P, P, P, nullptr, 0x7fffffff, 0x7fffffff, 128, 16, 4, 2, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_UNSUPPORTED);
    EXPECT(loma_mask_attn_fwd(P, P, P, P, nullptr, 1, 1, 128, 0x7fffffff, 0x7fffffff, 2, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_UNSUPPORTED);
    EXPECT(loma_mask_attn_bwd_workspace_bytes(2, 32, 128, 16, 4, 28, LOMA_BF16) > 0, 1);
    EXPECT(loma_mask_attn_bwd_workspace_bytes(1, 32, 128, 32, 8, 60, LOMA_BF16) > 0, 1);
    EXPECT(loma_mask_attn_bwd_workspace_bytes(1, 1, 64, 4, 4, 4, LOMA_F32), 8 * 144);
    EXPECT(loma_mask_attn_bwd_workspace_bytes(1, 1, 64, 0, 4, 4, LOMA_F32), 0);
    EXPECT(loma_mask_attn_bwd(P, P, P, P, (const float*)P, P, P2, P2, P2, 1, 1, 128, 16, 4, 2, 0.1f, LOMA_BF16, P, 1 << 20, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_mask_attn_bwd(P, P, P, P, (const float*)P, P, P2, (char*)P2 + 4096, (char*)P2 + 8192, 1, 1, 128, 16, 4, 2, 0.1f, LOMA_BF16, P, 8, nullptr), LOMA_ERR_WORKSPACE);
    // compression
    EXPECT(loma_compress_step(P, P, P, P, P, P, P, P, 1, 1, 128, 16, 4, 4, 64, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_compress_step(P, P, P, P, P, nullptr, P, P, 1, 1, 128, 16, 4, 2, 64, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_compress_step(P, P, P, P, P, P, P, P, 1, 1, 128, 16, 4, 0x7fffffff, 64, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_compress_step_rope(P, P, P, P, P, P, P, P2, 1, 1, 128, 16, 4, 2, 64, 0.1f, LOMA_BF16, -1, 4, 1e4f, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_compress_step_rope(P, P, P, P, P, P, P, P, 1, 1, 128, 16, 4, 2, 64, 0.1f, LOMA_BF16, 3, 4, 1e4f, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_compress_step_rope(P, P, P, P, P, P, P, P2, 1, 1, 96, 16, 4, 2, 64, 0.1f, LOMA_BF16, 3, 4, 1e4f, nullptr), LOMA_ERR_UNSUPPORTED);
    // decode in its four forms
    EXPECT(loma_decode_workspace_bytes(1, 8, 128, 16, 4, 4, LOMA_BF16) > 0, 1);
    EXPECT(loma_decode_workspace_bytes(8, 32, 128, 16, 4, 65, LOMA_BF16), 0);
    EXPECT(loma_decode_workspace_bytes(64, 32, 128, 16, 16, 513, LOMA_BF16) > 0, 1);
    EXPECT(loma_decode_workspace_bytes(1, 8, 128, 0x7fffffff, 4, 4, LOMA_BF16), 0);
    EXPECT(loma_decode_attn(P, P, P, P, P, P, P, P, 8, 32, 128, 16, 4, 4, 64, 64, 0.1f, LOMA_BF16, P, 1 << 30, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_decode_attn(P, P, nullptr, P, P, P, P, P, 8, 32, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, P, 1 << 30, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_decode_attn(P, P, P, P, P, P, P, P, 1, 8, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, nullptr, 0, nullptr), LOMA_ERR_WORKSPACE);
    EXPECT(loma_decode_attn_static(P, P, P, P, P, P, P, P, 4095, 1, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_UNSUPPORTED);
    EXPECT(loma_decode_attn_static(P, P, P, nullptr, P, P, P, P, 1, 8, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_decode_static_scratch_bytes(), 4u << 20);
    EXPECT(loma_decode_attn_rope(P, P, P, P, P, P, P, P, 1, 8, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, -2, 1e4f, P, 1 << 30, nullptr), LOMA_ERR_INVALID_ARG);
    const void* const* T = reinterpret_cast<const void* const*>(P);
    void* const* Tw = reinterpret_cast<void* const*>(P);
    EXPECT(loma_decode_attn_layers(T, T, T, T, T, Tw, Tw, Tw, 0, 1, 8, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, P, 1 << 30, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_decode_attn_layers(T, T, T, T, T, Tw, Tw, Tw, 4, 1, 8, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, nullptr, 0, nullptr), LOMA_ERR_WORKSPACE);
    EXPECT(loma_decode_layers_workspace_bytes(4, 1, 8, 128, 16, 4, 4, LOMA_BF16), 4 * loma_decode_workspace_bytes(1, 8, 128, 16, 4, 4, LOMA_BF16));
    // grouped-query decode
    EXPECT(loma_decode_attn_gqa(P, P, P, P, P, P, P, P, 1, 8, 3, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, P, 1 << 30, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_decode_attn_gqa(P, P, P, P, P, P, P, P, 1, 6, 2, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, P, 1 << 30, nullptr), LOMA_ERR_UNSUPPORTED);
    EXPECT(loma_decode_attn_gqa(P, P, P, P, P, P, P, P, 1, 8, 2, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, nullptr, 0, nullptr), LOMA_ERR_WORKSPACE);
    EXPECT(loma_decode_gqa_workspace_bytes(1, 8, 3, 128, LOMA_BF16), 0u);
    EXPECT(loma_decode_attn_gqa_layers(T, T, T, T, T, Tw, Tw, Tw, 0, 1, 8, 2, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, P, 1 << 30, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_decode_attn_gqa_layers(T, T, T, T, T, Tw, Tw, Tw, 3, 1, 8, 2, 128, 16, 4, 4, 64, 3, 0.1f, LOMA_BF16, nullptr, 0, nullptr), LOMA_ERR_WORKSPACE);
    // prompt form
    EXPECT(loma_prefill_attn(P, P, P, P, P, P, P, P, nullptr, 1, 8, 128, 16, 4, 4, 64, 60, 5, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_INVALID_ARG);
    EXPECT(loma_prefill_attn(P, nullptr, P, P, P, P, P, P, nullptr, 1, 8, 128, 16, 4, 4, 64, 0, 5, 0.1f, LOMA_BF16, nullptr), LOMA_ERR_INVALID_ARG);
    // the tile schedule, walked in full for two shapes: every item written into a 6-int array
    for (int shape = 0; shape < 2; ++shape) {
        const int t = shape ? 5 : 16, c = shape ? 7 : 4, n = shape ? 3 : 28, B = shape ? 1 : 2, H = shape ? 3 : 32;
        const long long nblk = loma_mask_schedule_size(B, H, 128, t, c, n, LOMA_BF16);
        EXPECT(nblk > 0, 1);
        long long rows = 0;
        for (long long b = 0; b < nblk; ++b) {
            std::vector<int> item(6, -1);             // heap array: an overrun is a sanitizer report
            if (loma_mask_schedule_item(B, H, 128, t, c, n, LOMA_BF16, b, item.data()) == 1) rows += item[4];
        }
        EXPECT(rows, (long long)B * H * n * t * (2 * c + 1));
        std::vector<int> item(6);
        EXPECT(loma_mask_schedule_item(B, H, 128, t, c, n, LOMA_BF16, nblk, item.data()), LOMA_ERR_INVALID_ARG);
        EXPECT(loma_mask_schedule_item(B, H, 128, t, c, n, LOMA_BF16, 0, nullptr), LOMA_ERR_INVALID_ARG);
    }
    EXPECT(loma_mask_schedule_size(1, 1, 128, 4096, 1, 258, LOMA_BF16), 0);
    // position ids into exactly sized heap arrays
    for (int type = 0; type < 2; ++type) {
        std::vector<int> mem(16), all(28 * 16 * 9);
        EXPECT(loma_memory_position_ids(16, 4, 63, type, mem.data()), LOMA_OK);
        EXPECT(loma_sample_position_ids(16, 4, 28, type, all.data()), LOMA_OK);
        EXPECT(all[27 * 144 + 64 + 15], type == LOMA_POS_INTERMITTENT ? 27 * 64 + 63 : 27 * 16 + 15);
    }
    EXPECT(loma_memory_position_ids(16, 16, 1 << 24, 0, (int*)P), LOMA_ERR_UNSUPPORTED);
    if (failures) { std::printf("%d check(s) failed\n", failures); return 1; }
    std::printf("abi driver ok\n");
    return 0;
}
