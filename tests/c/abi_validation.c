/*
 * A plain C11 user of include/comp_ams.h: proves that the header is C (not only C++), and drives the
 * host-side argument validation of the library - the part that answers before any device call - so
 * that it can run under AddressSanitizer / UBSan on a machine without a GPU.
 * Returns 0 when every call answered as the header says.
 */
#include "comp_ams.h"
#include "comp_ams_tuning.h"

#include <math.h>
#include <stdio.h>
#include <string.h>

#define EXPECT(call, want)                                                            \
    do {                                                                              \
        int got__ = (call);                                                           \
        if (got__ != (want)) {                                                        \
            printf("%s: got %d, expected %d\n", #call, got__, (int)(want));           \
            ++failures;                                                               \
        }                                                                             \
    } while (0)

int main(void)
{
    int failures = 0;
    comp_ams_t *h = NULL;
    float buf[8] = {0};
    uint16_t half[8] = {0};
    uint64_t bytes = 0;

    /* comp_ams_create: ranges of the problem statement and of the hyper-parameters */
    EXPECT(comp_ams_create(NULL, 10, 1, COMP_AMS_TOPK, 1, 0.9f, 0.999f, 1e-8f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, 0, 1, COMP_AMS_TOPK, 1, 0.9f, 0.999f, 1e-8f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, (int64_t)1 << 31, 1, COMP_AMS_TOPK, 1, 0.9f, 0.999f, 1e-8f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, 10, 0, COMP_AMS_TOPK, 1, 0.9f, 0.999f, 1e-8f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, 10, 1, 9, 1, 0.9f, 0.999f, 1e-8f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, 10, 1, COMP_AMS_TOPK, 0, 0.9f, 0.999f, 1e-8f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, 10, 1, COMP_AMS_TOPK, 11, 0.9f, 0.999f, 1e-8f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, 10, 1, COMP_AMS_RANDK, 11, 0.9f, 0.999f, 1e-8f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, 10, 1, COMP_AMS_BLOCKSIGN, 0, 0.9f, 0.999f, 1e-8f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, 10, 1, COMP_AMS_TOPK, 1, 1.0f, 0.999f, 1e-8f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, 10, 1, COMP_AMS_TOPK, 1, 0.9f, NAN, 1e-8f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, 10, 1, COMP_AMS_TOPK, 1, 0.9f, 0.999f, 0.0f, 1e-3f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_create(&h, 10, 1, COMP_AMS_TOPK, 1, 0.9f, 0.999f, 1e-8f, INFINITY), COMP_AMS_EINVAL);
    if (h != NULL) {
        printf("a failed create wrote its output\n");
        ++failures;
    }
    if (strlen(comp_ams_last_error(NULL)) == 0) {
        printf("no message for the failed create\n");
        ++failures;
    }

    /* every entry point answers a NULL handle with EINVAL and touches nothing */
    EXPECT(comp_ams_step(NULL, buf, NULL), COMP_AMS_EINVAL);
    EXPECT(comp_ams_step_bf16(NULL, half, NULL), COMP_AMS_EINVAL);
    EXPECT(comp_ams_step_f16(NULL, half, NULL), COMP_AMS_EINVAL);
    EXPECT(comp_ams_set_blocks(NULL, NULL, 1), COMP_AMS_EINVAL);
    EXPECT(comp_ams_set_theta(NULL, buf, 0), COMP_AMS_EINVAL);
    EXPECT(comp_ams_set_lr(NULL, 0.1f), COMP_AMS_EINVAL);
    EXPECT(comp_ams_set_eps_mode(NULL, 1), COMP_AMS_EINVAL);
    EXPECT(comp_ams_set_method(NULL, COMP_AMS_METHOD_CD), COMP_AMS_EINVAL);
    EXPECT(comp_ams_set_rand(NULL, 1u, 0u), COMP_AMS_EINVAL);
    EXPECT(comp_ams_get_theta(NULL, buf, 0), COMP_AMS_EINVAL);
    EXPECT(comp_ams_get_error(NULL, 0, buf, 0), COMP_AMS_EINVAL);
    EXPECT(comp_ams_get_selected(NULL, 0, NULL, buf), COMP_AMS_EINVAL);
    EXPECT(comp_ams_get_scales(NULL, buf), COMP_AMS_EINVAL);
    EXPECT(comp_ams_message_bytes(NULL, &bytes), COMP_AMS_EINVAL);
    EXPECT(comp_ams_message_bits(NULL, &bytes, &bytes), COMP_AMS_EINVAL);
    EXPECT(comp_ams_pack_message(NULL, 0, buf, sizeof buf, &bytes), COMP_AMS_EINVAL);
    EXPECT(comp_ams_n_blocks(NULL), COMP_AMS_EINVAL);
    EXPECT(comp_ams_sync(NULL), COMP_AMS_EINVAL);
    EXPECT(comp_ams_probe_copy(NULL, buf, 4, NULL), COMP_AMS_EINVAL);
    EXPECT(comp_ams_probe_copy(buf, buf, 3, NULL), COMP_AMS_EINVAL);
    EXPECT(comp_ams_probe_update(NULL, buf, 1, 4, NULL), COMP_AMS_EINVAL);
    EXPECT(comp_ams_probe_update(buf, buf, 1, 6, NULL), COMP_AMS_EINVAL);
    comp_ams_destroy(NULL);

    /* valid arguments: a handle on a machine with a GPU, a device error (not a crash) without one */
    {
        int rc = comp_ams_create(&h, 100, 2, COMP_AMS_BLOCKSIGN, 16, 0.9f, 0.999f, 1e-8f, 1e-3f);
        if (rc == COMP_AMS_OK) {
            EXPECT(comp_ams_set_lr(h, -1.0f), COMP_AMS_EINVAL);
            EXPECT(comp_ams_set_eps_mode(h, 2), COMP_AMS_EINVAL);
            EXPECT(comp_ams_get_selected(h, 0, NULL, NULL), COMP_AMS_ESTATE);
            comp_ams_destroy(h);
        } else if (rc != COMP_AMS_EDEVICE) {
            printf("valid create: got %d\n", rc);
            ++failures;
        }
    }
    printf("abi validation: %d failures\n", failures);
    return failures != 0;
}
