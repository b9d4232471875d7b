/* Host-side walk through the argument validation of libechoattn, meant to be linked against the library built
 * with -fsanitize=address,undefined on its host code and run without a GPU: every call here must stop at a
 * host check (nothing is launched), and the sanitizers must stay silent.  Prints "ok" at the end. */
#include <stdio.h>
#include <string.h>

#include "echoattn.h"
#include "echodropout.h"
#include "echolstm.h"

#define EXPECT(call, want)                                                                     \
    do {                                                                                       \
        int got_ = (int)(call);                                                                \
        if (got_ != (int)(want)) {                                                             \
            fprintf(stderr, "%s:%d: %s returned %d, expected %d\n", __FILE__, __LINE__, #call, got_, (int)(want)); \
            return 1;                                                                          \
        }                                                                                      \
    } while (0)

int main(void) {
    void *A = (void *)0x10000;              /* aligned, never dereferenced */
    void *M = (void *)0x10004;              /* misaligned */
    echo_attn_desc_t d = {4, 6, 7, 16, 16, ECHO_F32};
    echo_attn_desc_t bad = d, unfused = d, big = d, step = d;
    bad.B = 0;
    unfused.H = 18;
    big.B = 512; big.Tq = 300; big.Tk = 300; big.H = 64; big.Dv = 64;
    step.Tq = 1;

    if (echo_attn_fwd_workspace_bytes(&d) != 0) return 2;
    if (echo_attn_fwd_workspace_bytes(&unfused) < (size_t)4 * 6 * 7 * 4) return 2;
    if (echo_attn_bwd_workspace_bytes(&d) == 0 || echo_attn_bwd_workspace_bytes(&bad) != 0) return 2;
    if (echo_attn_bwd_workspace_bytes(NULL) != 0 || echo_attn_stash_bytes(&d) != (size_t)4 * 6 * 7 * 16 * 4) return 2;
    if (echo_attn_fwd_stash_workspace_bytes(&d) < (size_t)4 * 6 * 7 * 4) return 2;

    EXPECT(echo_attn_fwd(NULL, A, A, A, A, (const int32_t *)A, (float *)A, (float *)A, A, 1, NULL), ECHO_ERR_NULL);
    EXPECT(echo_attn_fwd(&d, NULL, A, A, A, (const int32_t *)A, (float *)A, (float *)A, NULL, 0, NULL), ECHO_ERR_NULL);
    EXPECT(echo_attn_fwd(&d, M, A, A, A, (const int32_t *)A, (float *)A, (float *)A, NULL, 0, NULL), ECHO_ERR_ALIGN);
    EXPECT(echo_attn_fwd(&bad, A, A, A, A, (const int32_t *)A, (float *)A, (float *)A, A, 1, NULL), ECHO_ERR_SHAPE);
    EXPECT(echo_attn_fwd(&unfused, A, A, A, A, (const int32_t *)A, (float *)A, (float *)A, A, 16, NULL), ECHO_ERR_WORKSPACE);
    EXPECT(echo_attn_bwd(&d, (const float *)A, (const float *)A, A, A, A, A, (const int32_t *)A, (float *)A, (float *)A,
                         (float *)A, NULL, A, (size_t)1 << 40, NULL), ECHO_ERR_NULL);
    EXPECT(echo_attn_bwd(&d, (const float *)A, (const float *)A, A, A, A, A, (const int32_t *)A, (float *)A, (float *)A,
                         (float *)A, (float *)A, A, 8, NULL), ECHO_ERR_WORKSPACE);
    EXPECT(echo_attn_bwd_accumulate(&d, (const float *)A, (const float *)A, A, A, A, A, (const int32_t *)A, (float *)A,
                                    (float *)M, (float *)A, (float *)A, A, (size_t)1 << 40, NULL), ECHO_ERR_ALIGN);
    EXPECT(echo_attn_bwd_static(&big, (const float *)A, (const float *)A, A, A, A, A, (const int32_t *)A, (float *)A,
                                (float *)A, (float *)A, (float *)A, NULL), ECHO_ERR_WORKSPACE);
    if (strstr(echo_last_error_detail(), "bytes") == NULL) return 3;
    EXPECT(echo_attn_fwd_stash(&d, A, A, A, A, (const int32_t *)A, (float *)A, (float *)A, NULL, A, (size_t)1 << 40, NULL),
           ECHO_ERR_NULL);
    EXPECT(echo_attn_bwd_stash(&d, (const float *)A, (const float *)A, NULL, A, A, (const int32_t *)A, (float *)A,
                               (float *)A, (float *)A, (float *)A, A, (size_t)1 << 40, NULL), ECHO_ERR_NULL);
    EXPECT(echo_attn_step_fwd(&d, A, A, A, A, (const int32_t *)A, (float *)A, (float *)A, NULL), ECHO_ERR_SHAPE);
    EXPECT(echo_attn_step_fwd(&step, A, A, A, A, (const int32_t *)A, (float *)A, NULL, NULL), ECHO_ERR_NULL);
    EXPECT(echo_attn_step_bwd(&step, (const float *)A, (const float *)A, A, A, A, A, (const int32_t *)A, (float *)A,
                              (float *)A, (float *)A, NULL, NULL), ECHO_ERR_NULL);
    EXPECT(echo_attn_step_finish(&step, NULL, (float *)A, NULL), ECHO_ERR_NULL);
    {
        double work = 0.0;
        EXPECT(echo_attn_calibrate(ECHO_CAL_FMA, 0, 1, NULL, A, 1024, &work, NULL), ECHO_ERR_SHAPE);
        EXPECT(echo_attn_calibrate(99, 1, 1, NULL, A, 1 << 20, &work, NULL), ECHO_ERR_DTYPE);
    }
    echo_attn_profile_enable(1);
    {
        const char *names[4];
        int launches[4];
        float ms[4];
        if (echo_attn_profile_read(names, launches, ms, 4) != 0) return 4;
    }
    echo_attn_profile_enable(0);
    for (int s = 0; s < 8; ++s)
        if (echo_status_string((echo_status_t)s) == NULL) return 5;
    if (strstr(echo_version(), "gfx950") == NULL) return 5;

    if (echo_dropout_mask_words(33) != 2) return 6;
    EXPECT(echo_dropout_fwd(NULL, 8, 0.5f, 1, 0, (float *)A, (uint32_t *)A, NULL), ECHO_ERR_NULL);
    EXPECT(echo_dropout_fwd((const float *)A, 8, 1.0f, 1, 0, (float *)A, (uint32_t *)A, NULL), ECHO_ERR_SHAPE);
    EXPECT(echo_dropout_bwd((const float *)A, NULL, 8, 0.5f, (float *)A, NULL), ECHO_ERR_NULL);
    if (echo_lstm_cell_kept_bytes(128, 512, 0) != (size_t)5 * 128 * 512 * 4) return 7;
    EXPECT(echo_lstm_cell_fwd(0, 8, (const float *)A, (const float *)A, (const float *)A, (float *)A, (float *)A, (float *)A,
                              NULL), ECHO_ERR_SHAPE);
    EXPECT(echo_lstm_cell_bwd(4, 8, NULL, (const float *)A, (const float *)A, (const float *)A, (float *)A, (float *)A,
                              NULL), ECHO_ERR_NULL);
    puts("ok");
    return 0;
}
