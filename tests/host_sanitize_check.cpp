// Sanitizer run of the library's host layer (no GPU needed): built by tests/test_sanitizers.py together with
// csrc/cks_api.hip, host code compiled with -fsanitize=address,undefined.  Drives everything the entry
// points do before a launch -- argument checks, workspace sizes, tile / segment planning, the work-list
// arithmetic of every kernel family -- through cks_plan_hw and the size queries, over a grid of geometries
// and pointer alignments.  Exits 0 and prints the number of plans, or 1 on an unexpected status.
#include "../include/cks.h"

#include <cstdio>
#include <cstring>

int main()
{
    static const int shapes[][7] = {   // N, C, H, W, OC, FH, FW
        {2, 4, 8, 8, 4, 3, 3},       {128, 64, 32, 32, 64, 3, 3},  {128, 128, 16, 16, 256, 3, 3}, {256, 512, 7, 7, 512, 3, 3},
        {64, 128, 32, 32, 256, 4, 4}, {64, 3, 224, 224, 64, 7, 7},  {33, 5, 9, 7, 7, 3, 3},        {37, 3, 24, 224, 64, 7, 7},
        {40, 16, 9, 10, 70, 3, 3},   {32, 32, 16, 15, 64, 4, 4},   {64, 256, 16, 16, 256, 3, 3},  {33, 130, 16, 16, 98, 5, 5},
        {1, 1, 1, 1, 1, 1, 1},       {9, 64, 1024, 1024, 16, 3, 3}, {6, 3, 21, 22, 16, 3, 3},      {10, 8, 9, 9, 32, 1, 1},
        {3, 2, 15, 18, 60, 6, 6},    {300, 20, 4, 4, 24, 3, 3},    {5, 1, 10, 11, 70, 5, 3},      {70, 50, 9, 8, 64, 3, 3},
    };
    char text[2048];
    long plans = 0;
    int bad = 0;
    for (const auto &s : shapes)
        for (int sh = 1; sh <= 4; ++sh)
            for (int sw = 1; sw <= 3; sw += (sh == 2 ? 1 : 2))
                for (int ph = 0; ph <= 7; ph += (ph < 3 ? 1 : 4))
                    for (int pw = ph; pw <= ph + 2; pw += 2) {
                        const bool valid = s[2] + 2 * ph >= s[5] && s[3] + 2 * pw >= s[6];
                        for (int op = 0; op <= CKS_OP_WGRAD_UNTRIMMED; ++op)
                            for (unsigned mask = 0; mask < 16; mask += 5) {
                                const int rc = cks_plan_hw(op, s[0], s[1], s[2], s[3], s[4], s[5], s[6], sh, sw, ph, pw, mask, text, sizeof text);
                                // the forward pass on the transposed filter exists for whole 32-channel chunks, aligned pointers and
                                // tile rows within 2 GiB only: on a valid geometry it may also answer that it has no kernel
                                if (valid && op >= CKS_OP_CONV2D_FWD_TRANSPOSED && rc == CKS_ERR_UNSUPPORTED) { ++plans; continue; }
                                if (valid ? (rc != CKS_OK || !strchr(text, '[')) : rc != CKS_ERR_SHAPE) {
                                    printf("op %d shape %d,%d,%d,%d,%d,%d,%d s %d,%d p %d,%d mask %u: status %d\n", op, s[0], s[1], s[2], s[3],
                                           s[4], s[5], s[6], sh, sw, ph, pw, mask, rc);
                                    bad = 1;
                                }
                                ++plans;
                            }
                        const size_t w1 = cks_deconv2d_workspace_hw(s[0], s[1], s[2], s[3], s[4], s[5], s[6], sh, sw, ph, pw);
                        const size_t w2 = cks_dilated_conv2d_wgrad_workspace_hw(s[0], s[1], s[2], s[3], s[4], s[5], s[6], sh, sw, ph, pw);
                        const int gz = cks_dilated_conv2d_wgrad_segments_hw(s[0], s[1], s[2], s[3], s[4], s[5], s[6], sh, sw, ph, pw);
                        const long long macs = cks_useful_macs_hw(s[0], s[1], s[2], s[3], s[4], s[5], s[6], sh, sw, ph, pw);
                        if (valid ? (gz < 1 || macs < 0 || (gz > 1) != (w2 > 0) || w1 < cks_kernel_split_bytes_hw(s[1], s[4], s[5], s[6], sh, sw))
                                  : (gz != 0 || macs != -1 || w1 != 0 || w2 != 0)) {
                            printf("queries disagree on shape %d,%d,%d,%d,%d,%d,%d s %d,%d p %d,%d\n", s[0], s[1], s[2], s[3], s[4], s[5], s[6], sh, sw, ph, pw);
                            bad = 1;
                        }
                    }
    // entry points refuse bad arguments before any device call
    float *fake = reinterpret_cast<float *>(0x1000);
    bad |= cks_conv2d_fwd(nullptr, fake, fake, 2, 4, 8, 8, 4, 3, 3, 1, 1, nullptr, 0, nullptr) != CKS_ERR_NULL;
    bad |= cks_deconv2d(fake, fake, fake, 2, 4, 8, 8, 4, 3, 3, 1, 1, nullptr, 0, nullptr) != CKS_ERR_WORKSPACE;
    bad |= cks_dilated_conv2d_wgrad(fake, fake, fake, 128, 64, 32, 32, 64, 3, 3, 1, 1, nullptr, 0, nullptr) != CKS_ERR_WORKSPACE;
    bad |= cks_dilated_conv2d_wgrad_noalloc_hw(fake, fake, fake, 256, 512, 7, 7, 512, 3, 3, 1, 1, 1, 1, nullptr) != CKS_ERR_SCRATCH;
    bad |= cks_plan_hw(0, 128, 64, 32, 32, 64, 3, 3, 1, 1, 1, 1, 0, text, 8) != CKS_ERR_WORKSPACE;
    printf("%ld plans %s\n", plans, bad ? "FAILED" : "ok");
    return bad;
}
