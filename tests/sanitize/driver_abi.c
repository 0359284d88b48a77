/* Host side of the C ABI under -fsanitize=address,undefined: workspace sizing and every argument check of the MoE entry
 * points, all of which return before the first HIP call, so no GPU is needed.  Pointers are fake (aligned, never
 * dereferenced by a correct library).  Exit code 0 = clean. */
#include <stdint.h>
#include <stdio.h>

#include "moe_ffn.h"
#include "moe_ffn_backward.h"

#define EXPECT(call, want) do { int got_ = (int)(call); if (got_ != (want)) { fprintf(stderr, "%s -> %d, expected %d\n", #call, got_, (want)); return 1; } } while (0)

int main(void) {
    void *p[14];
    for (int i = 0; i < 14; ++i) p[i] = (void *)(uintptr_t)(0x10000 * (i + 1));
    static const int shapes[][7] = {      /* T, H, E, K, I, dtype, renormalize */
        {64, 2048, 128, 8, 768, 0, 1}, {16384, 2048, 128, 8, 768, 0, 1}, {4, 64, 8, 2, 32, 1, 1}, {0, 64, 4, 2, 32, 0, 1},
        {1500, 256, 70, 4, 64, 0, 0}, {600, 64, 1024, 16, 16, 1, 1}, {1 << 20, 2048, 128, 8, 768, 0, 1}, {1, 8, 1, 1, 8, 0, 1},
    };
    for (size_t i = 0; i < sizeof shapes / sizeof shapes[0]; ++i) {
        moe_shape_t s = {shapes[i][0], shapes[i][1], shapes[i][2], shapes[i][3], shapes[i][4], shapes[i][5], shapes[i][6]};
        size_t need = 0, need_bw = 0;
        EXPECT(moe_workspace_bytes(&s, &need), MOE_OK);
        EXPECT(moe_backward_workspace_bytes(&s, &need_bw), MOE_OK);
        if (need % 256 || need_bw % 256 || need_bw <= need) { fprintf(stderr, "workspace sizes %zu %zu\n", need, need_bw); return 1; }
        /* a workspace one byte short is refused before anything else happens */
        EXPECT(moe_forward(&s, p[0], p[1], NULL, p[2], p[3], p[4], p[5], NULL, NULL, p[6], need - 1, NULL), MOE_ERR_WORKSPACE);
        EXPECT(moe_route_topk(&s, p[0], p[1], NULL, (int32_t *)p[2], (float *)p[3], p[6], need - 1, NULL), MOE_ERR_WORKSPACE);
        EXPECT(moe_permute(&s, (int32_t *)p[0], NULL, (int32_t *)p[1], (int32_t *)p[2], (int32_t *)p[3], NULL, p[6], need - 1, NULL), MOE_ERR_WORKSPACE);
        EXPECT(moe_grouped_swiglu(&s, p[0], (int32_t *)p[1], p[2], p[3], p[4], p[5], p[6], need - 1, NULL), MOE_ERR_WORKSPACE);
        EXPECT(moe_backward(&s, p[0], p[1], NULL, p[2], p[3], p[4], p[5], p[6], (float *)p[7], NULL, (float *)p[8], (float *)p[9],
                            (float *)p[10], p[11], need_bw - 1, NULL), MOE_ERR_WORKSPACE);
        EXPECT(moe_forward(&s, NULL, p[1], NULL, p[2], p[3], p[4], p[5], NULL, NULL, p[6], need, NULL), MOE_ERR_NULL);
        EXPECT(moe_forward(&s, (char *)p[0] + 4, p[1], NULL, p[2], p[3], p[4], p[5], NULL, NULL, p[6], need, NULL), MOE_ERR_ALIGN);
        EXPECT(moe_combine(&s, p[0], (int32_t *)p[1], (float *)p[2], NULL, NULL), MOE_ERR_NULL);
        if (need > MOE_NOALLOC_SCRATCH_BYTES)
            EXPECT(moe_forward_noalloc(&s, p[0], p[1], NULL, p[2], p[3], p[4], p[5], NULL, NULL, NULL), MOE_ERR_STATIC_LIMIT);
    }
    moe_shape_t bad = {4, 60, 8, 2, 32, 0, 1};
    size_t n = 0;
    EXPECT(moe_workspace_bytes(&bad, &n), MOE_ERR_SHAPE);
    EXPECT(moe_workspace_bytes(NULL, &n), MOE_ERR_NULL);
    bad.H = 64; bad.dtype = 9;
    EXPECT(moe_backward_workspace_bytes(&bad, &n), MOE_ERR_DTYPE);
    if (!moe_status_string(MOE_ERR_STATIC_LIMIT) || !moe_status_string((moe_status_t)99)) return 1;
    puts("ABI host side clean under the sanitizers");
    return 0;
}
