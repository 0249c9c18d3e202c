// Calls every entry point of the C ABI with arguments that its host-side validation must refuse (or with empty
// inputs that are no-ops), and every workspace query, in a build whose HOST code carries
// -fsanitize=address,undefined: the launch planning (splits, tile lists, workspace sizes) and the validation run,
// nothing reaches a GPU.  Prints "ok" when every call returned what it should.
#include <cstdint>
#include <cstdio>
#include <limits>

#include "../../include/dd.h"

static int fails = 0;
#define EXPECT(call, want)                                                          \
    do {                                                                            \
        const long got_ = (long)(call);                                             \
        if (got_ != (long)(want)) {                                                 \
            std::printf("line %d: got %ld, want %ld\n", __LINE__, got_, (long)(want)); \
            ++fails;                                                                \
        }                                                                           \
    } while (0)

int main()
{
    void *const P = reinterpret_cast<void *>(0x1000);      // non-NULL, aligned, never dereferenced
    void *const P2 = reinterpret_cast<void *>(0x9000);
    const float *const S = reinterpret_cast<const float *>(0x2000);
    // ---- attention
    EXPECT(dd_bidir_attention(nullptr, P, P, P, 1, 4, 2, 64, 128, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_NULL);
    EXPECT(dd_bidir_attention(P, P, P, P, 0, 4, 2, 64, 128, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_bidir_attention(P, P, P, P, 1, 3, 2, 64, 128, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_bidir_attention(P, P, P, P, 1, 4, 2, 64, 96, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_bidir_attention(P, P, P, P, 1 << 20, 1 << 10, 1 << 10, 1 << 20, 128, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_bidir_attention(P, P, P, P, 1, 4, 2, 64, 128, DD_FP8_E4M3, DD_BF16, nullptr, S, nullptr, 0, nullptr), DD_ERR_NULL);
    EXPECT(dd_bidir_attention(P, P, P, P, 1, 4, 2, 64, 128, DD_BF16, DD_F32, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_DTYPE);
    EXPECT(dd_bidir_attention_workspace_bytes(8, 32, 32, 1024, 128, DD_BF16, DD_BF16), 0);
    const int shapes[][6] = {{1, 32, 32, 4096, 128, 64}, {16, 32, 8, 2048, 128, 64}, {1, 4, 1, 4097, 128, 128}, {3, 6, 2, 77, 64, 5},
                             {1, 1, 1, 1, 64, 1}, {2, 2, 1, 65536, 128, 64}, {8, 32, 32, 1024, 128, 64}, {1, 32, 32, 512, 128, 32}};
    for (const auto &s : shapes) {
        const dd_dtype types[3][2] = {{DD_BF16, DD_BF16}, {DD_FP8_E4M3, DD_BF16}, {DD_F32, DD_F32}};
        for (const auto &t : types) {
            const size_t need = dd_block_attention_cached_workspace_bytes(s[5], s[0], s[1], s[2], s[3], s[4], t[0], t[1]);
            EXPECT(dd_block_attention_refresh_workspace_bytes(s[5], s[0], s[1], s[2], s[3], s[4], t[0], t[1]), need);
            EXPECT(dd_block_attention_batched_workspace_bytes(s[5], s[0], s[1], s[2], s[3], s[4], t[0], t[1]), need);
            EXPECT(dd_block_attention_window_workspace_bytes(s[5], s[3], s[0], s[1], s[2], s[3], s[4], t[0], t[1]), need);
            // a block that runs past the end, a missing workspace when one is needed
            EXPECT(dd_block_attention_cached(P, P, P, P, s[3] - s[5] + 1, s[5], nullptr, nullptr, s[0], s[1], s[2], s[3], s[4],
                                             t[0], t[1], S, S, nullptr, 0, nullptr), DD_ERR_SHAPE);
        }
    }
    {   // the split plan of this shape needs a workspace whatever the block position
        const size_t need = dd_block_attention_cached_workspace_bytes(64, 1, 32, 32, 4096, 128, DD_BF16, DD_BF16);
        EXPECT(need > 0, 1);
        EXPECT(dd_block_attention_cached(P, P, P, P, 0, 64, nullptr, nullptr, 1, 32, 32, 4096, 128, DD_BF16, DD_BF16, nullptr, nullptr,
                                         P, need - 1, nullptr), DD_ERR_WORKSPACE);
        EXPECT(dd_block_attention_cached(P, P, P, P, 0, 64, nullptr, nullptr, 1, 32, 32, 4096, 128, DD_BF16, DD_BF16, nullptr, nullptr,
                                         reinterpret_cast<void *>(0x1010), need, nullptr), DD_ERR_WORKSPACE);
    }
    EXPECT(dd_block_attention_cached(P, P, P, P, -1, 16, nullptr, nullptr, 1, 4, 2, 64, 128, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_block_attention_cached(P, P, P, P, std::numeric_limits<int>::max() - 3, 16, nullptr, nullptr, 1, 4, 2, 64, 128, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_block_attention_cached(P, P, P, P, 0, 16, P, nullptr, 1, 4, 2, 64, 128, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_NULL);
    EXPECT(dd_block_attention_refresh(P, P, P, P, 0, 16, nullptr, nullptr, 1, 4, 2, 64, 128, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_NULL);
    EXPECT(dd_block_attention_window(P, P, P, P, 16, 16, 17, 40, nullptr, nullptr, 1, 4, 2, 64, 128, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_block_attention_window(P, P, P, P, 16, 16, 0, std::numeric_limits<int>::max(), nullptr, nullptr, 1, 4, 2, 64, 128, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_block_attention_batched(P, P, P, P, nullptr, 16, P, P, 1, 4, 2, 64, 128, DD_BF16, DD_BF16, nullptr, nullptr, nullptr, 0, nullptr), DD_ERR_NULL);
    EXPECT(dd_cache_insert_rows(P, P, P, P, nullptr, 4, 2, 2, 64, 128, DD_BF16, DD_BF16, nullptr), DD_ERR_NULL);
    EXPECT(dd_cache_insert_rows(nullptr, nullptr, nullptr, nullptr, nullptr, 0, 2, 2, 64, 128, DD_BF16, DD_BF16, nullptr), DD_OK);
    // ---- verification
    const uint8_t *const M = reinterpret_cast<const uint8_t *>(0x3000);
    uint8_t *const OM = reinterpret_cast<uint8_t *>(0x7000);
    int32_t *const OT = reinterpret_cast<int32_t *>(0x4000);
    float *const OS = reinterpret_cast<float *>(0x5000);
    const int vshapes[][3] = {{1, 64, 1024}, {1, 256, 126464}, {8, 512, 126464}, {16, 512, 152064}, {2, 5, 8}, {1, 191, 8200}, {0, 7, 16}};
    for (const auto &v : vshapes) {
        const size_t need = dd_verify_remask_workspace_bytes(v[0], v[1], v[2], DD_BF16);
        EXPECT(dd_unmask_workspace_bytes(v[0], v[1], v[2], DD_BF16), need);
        EXPECT(dd_verify_scores_workspace_bytes(v[0] * v[1], v[2], DD_BF16), need);
        EXPECT(need <= 128u * 1024u, 1);
        if (need > 0) {
            EXPECT(dd_verify_remask(P, P2, M, DD_KL_THRESH, 0.3f, 0, OM, OT, OS, v[0], v[1], v[2], DD_BF16, nullptr, 0, nullptr), DD_ERR_WORKSPACE);
            EXPECT(dd_unmask(P, M, DD_UNMASK_THRESH, 0.5f, nullptr, OM, OT, OS, v[0], v[1], v[2], DD_BF16, P, need - 1, nullptr), DD_ERR_WORKSPACE);
        }
    }
    EXPECT(dd_verify_remask(P, P2, M, (dd_mode)9, 0.3f, 0, OM, OT, OS, 2, 8, 1024, DD_BF16, nullptr, 0, nullptr), DD_ERR_MODE);
    EXPECT(dd_verify_remask(P, P2, M, DD_KL_TOPK, -1.f, 0, OM, OT, OS, 2, 8, 1024, DD_BF16, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_verify_remask(P, P2, M, DD_KL_TOPK, 2.f, 0, const_cast<uint8_t *>(M), OT, OS, 2, 8, 1024, DD_BF16, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_verify_remask(P, P2, M, DD_KL_THRESH, 0.3f, 0, const_cast<uint8_t *>(M) + 3, OT, OS, 2, 8, 1024, DD_BF16, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_verify_remask(P, P2, M, DD_KL_THRESH, 0.3f, 0, OM, OT, OS, 46341, 46341, 1024, DD_BF16, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_verify_remask(P, P2, M, DD_KL_THRESH, 0.3f, 0, OM, OT, OS, 2, 8, 1001, DD_BF16, nullptr, 0, nullptr), DD_ERR_ALIGN);
    EXPECT(dd_verify_remask(P, P2, M, DD_KL_THRESH, 0.3f, 0, OM, OT, OS, 0, 8, 1024, DD_BF16, nullptr, 0, nullptr), DD_OK);
    EXPECT(dd_verify_remask_static(nullptr, P2, M, DD_KL_THRESH, 0.3f, 0, OM, OT, OS, 2, 8, 1024, DD_BF16, nullptr), DD_ERR_NULL);
    EXPECT(dd_verify_remask_static(P, P2, M, (dd_mode)-1, 0.3f, 0, OM, OT, OS, 2, 8, 1024, DD_BF16, nullptr), DD_ERR_MODE);
    EXPECT(dd_verify_remask_static(P, P2, M, DD_TRUST, 0.f, 0, OM, OT, OS, 0, 8, 1024, DD_BF16, nullptr), DD_OK);
    EXPECT(dd_unmask(P, M, (dd_unmask_mode)5, 0.5f, nullptr, OM, OT, OS, 2, 8, 1024, DD_BF16, nullptr, 0, nullptr), DD_ERR_MODE);
    EXPECT(dd_unmask(P, M, DD_UNMASK_THRESH, 0.5f, nullptr, const_cast<uint8_t *>(M) + 15, OT, OS, 2, 8, 1024, DD_BF16, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_verify_scores(P, P2, OS, OS, OT, nullptr, nullptr, -1, 1024, DD_BF16, nullptr, 0, nullptr), DD_ERR_SHAPE);
    EXPECT(dd_verify_scores(P, P2, OS, OS, OT, nullptr, nullptr, 0, 1024, DD_BF16, nullptr, 0, nullptr), DD_OK);
    for (int code = -9; code <= 1; ++code) EXPECT(dd_strerror(code) != nullptr, 1);
    EXPECT(dd_version() >= 100, 1);
    if (fails) return 1;
    std::printf("ok\n");
    return 0;
}
