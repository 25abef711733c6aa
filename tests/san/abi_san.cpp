// Sanitizer driver for the boundary: the argument checks of every entry point of include/sparsek.h, compiled with
// -fsanitize=address,undefined on the host side and called with the arguments a careless caller passes -- null
// pointers, sizes of zero, negative, huge and overflowing, wrong enums, short workspaces.  Every call must come
// back with its error code before anything touches a GPU (none is needed), and without undefined arithmetic.
#include <climits>
#include <cstdio>
#include <cstdlib>
#include <initializer_list>

#include "../../include/sparsek.h"

static int fails = 0;
#define EXPECT(call, want)                                                                  \
    do {                                                                                    \
        const long long got_ = (long long)(call);                                           \
        if (got_ != (long long)(want)) {                                                    \
            std::fprintf(stderr, "abi_san: %s = %lld, expected %lld\n", #call, got_, (long long)(want)); \
            fails++;                                                                        \
        }                                                                                   \
    } while (0)

int main()
{
    void* one = (void*)256;  // never dereferenced: validation fails first
    void* null = nullptr;
    const int big[] = {INT_MAX, INT_MAX - 1, 1 << 30, (1 << 28) + 1};
    sparsek_cfg ok = {1, 2, 1, 16, 64, 4, 4, SPARSEK_BF16, 0, 1.0f};
    EXPECT(sparsek_mask_workspace_bytes(&ok) > 0, 1);
    EXPECT(sparsek_mask_workspace_bytes(nullptr), 0);
    EXPECT(sparsek_mask(&ok, (const float*)null, (float*)one, (int32_t*)one, one, 1 << 20, null), SPARSEK_ERR_INVALID_ARG);
    EXPECT(sparsek_mask(&ok, (const float*)one, (float*)one, (int32_t*)one, one, 8, null), SPARSEK_ERR_WORKSPACE);
    EXPECT(sparsek_mask_static(&ok, (const float*)null, (float*)one, (int32_t*)one, null), SPARSEK_ERR_INVALID_ARG);
    int32_t flag = 0;
    EXPECT(sparsek_mask_status(&ok, null, 1 << 20, &flag, null), SPARSEK_ERR_INVALID_ARG);
    for (int v : big) {
        sparsek_cfg c = ok;
        c.k = v;
        EXPECT(sparsek_mask_workspace_bytes(&c), 0);
        EXPECT(sparsek_attn_fwd_workspace_bytes(&c), 0);
        EXPECT(sparsek_attn_fwd(&c, one, one, one, (const float*)one, (const float*)one, (const int32_t*)one, one,
                                (float*)one, one, (size_t)1 << 40, null), SPARSEK_ERR_UNSUPPORTED);
        c = ok;
        c.w = v;
        c.k = v;
        EXPECT(sparsek_bwd_workspace_bytes(&c), 0);
        EXPECT(sparsek_mask_static(&c, (const float*)one, (float*)one, (int32_t*)one, null), SPARSEK_ERR_UNSUPPORTED);
        c = ok;
        c.n = v;
        EXPECT(sparsek_mask_workspace_bytes(&c), 0);
        c = ok;
        c.B = v;
        c.H = v;
        c.Gu = v;
        EXPECT(sparsek_attn_bwd_workspace_bytes(&c), 0);
        sparsek_decode_cfg d = {1, 2, 1, 64, v, v, 0, SPARSEK_BF16, 0, 1.0f};
        EXPECT(sparsek_decode_state_bytes(&d), 0);
        d = {v, v, v, 64, 8, 8, v, SPARSEK_BF16, 0, 1.0f};
        EXPECT(sparsek_decode_state_bytes(&d), 0);
        sparsek_chunk_cfg ch = {1, 2, 1, 64, v, v, v, v, SPARSEK_BF16, 0, 1.0f};
        EXPECT(sparsek_chunk_state_bytes(&ch), 0);
        EXPECT(sparsek_chunk_workspace_bytes(&ch), 0);
        sparsek_scores_cfg sc = {v, v, v, SPARSEK_BF16, 1, 0.0f, 1e-5f};
        EXPECT(sparsek_scores_workspace_bytes(&sc), 0);
    }
    for (int neg : {-1, INT_MIN}) {
        sparsek_cfg c = ok;
        c.k = neg;
        EXPECT(sparsek_mask_workspace_bytes(&c), 0);
        c = ok;
        c.w = neg;
        EXPECT(sparsek_attn_fwd_workspace_bytes(&c), 0);
        c = ok;
        c.n = neg;
        EXPECT(sparsek_mask_bwd_workspace_bytes(&c), 0);
        c = ok;
        c.d = neg;
        EXPECT(sparsek_attn_fwd_workspace_bytes(&c), 0);
        c = ok;
        c.gate_mode = neg;
        EXPECT(sparsek_attn_fwd_workspace_bytes(&c), 0);
        EXPECT(sparsek_materialize(&ok, (const float*)one, (const float*)one, (const int32_t*)one, neg, 4, (int32_t*)one,
                                   (float*)one, null), SPARSEK_ERR_INVALID_ARG);
    }
    {   // legitimate large configurations: sizes are computed in size_t, nothing wraps
        sparsek_cfg c = {1, 32, 32, 1 << 20, 128, 1024, 1024, SPARSEK_BF16, 0, 1.0f};
        EXPECT(sparsek_attn_fwd_workspace_bytes(&c) > ((size_t)1 << 32), 1);
        EXPECT(sparsek_bwd_workspace_bytes(&c) > sparsek_attn_bwd_workspace_bytes(&c), 1);
        EXPECT(sparsek_mask_static(&c, (const float*)one, (float*)one, (int32_t*)one, null) == SPARSEK_ERR_TOO_LARGE ||
               sparsek_mask_workspace_bytes(&c) <= SPARSEK_MASK_STATIC_MAX_BYTES, 1);
    }
    sparsek_cfg bad = ok;
    bad.softmax_scale = 0.0f;
    EXPECT(sparsek_attn_fwd_workspace_bytes(&bad), 0);
    bad = ok;
    bad.Gu = 3;
    EXPECT(sparsek_mask(&bad, (const float*)one, (float*)one, (int32_t*)one, one, 1 << 20, null), SPARSEK_ERR_INVALID_ARG);
    sparsek_decode_cfg dc = {1, 2, 1, 64, 8, 8, 0, SPARSEK_BF16, 0, 1.0f};
    EXPECT(sparsek_decode_init(&dc, null, 1 << 20, null), SPARSEK_ERR_INVALID_ARG);
    EXPECT(sparsek_decode_init(&dc, one, 8, null), SPARSEK_ERR_WORKSPACE);
    EXPECT(sparsek_decode_step(&dc, one, null, one, one, (const float*)one, one, null), SPARSEK_ERR_INVALID_ARG);
    sparsek_chunk_cfg cc = {1, 2, 1, 64, 8, 8, 0, 256, SPARSEK_BF16, 0, 1.0f};
    EXPECT(sparsek_chunk_prefill(&cc, one, sparsek_chunk_state_bytes(&cc), 0, one, one, one, (const float*)one, one, one,
                                 sparsek_chunk_workspace_bytes(&cc), null), SPARSEK_ERR_INVALID_ARG);
    EXPECT(sparsek_chunk_to_decode(&cc, one, sparsek_chunk_state_bytes(&cc), 15, one, sparsek_chunk_workspace_bytes(&cc), &dc,
                                   one, sparsek_decode_state_bytes(&dc), null), SPARSEK_ERR_UNSUPPORTED);
    sparsek_scores_cfg sc = {2, 100, 768, SPARSEK_BF16, 1, 0.0f, 0.0f};
    EXPECT(sparsek_scores(&sc, one, (const float*)one, (float*)one, one, 1 << 20, null), SPARSEK_ERR_INVALID_ARG);
    if (fails) return 1;
    std::printf("abi_san ok\n");
    return 0;
}
