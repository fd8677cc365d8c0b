/* The header must be plain C, and the entry points must be callable from C without a GPU for
 * everything that is decided on the host: version, status names, argument checks. */
#include <stdio.h>
#include <string.h>

#include "dhq.h"

#define CHECK(cond)                                                         \
    do {                                                                    \
        if (!(cond)) {                                                      \
            fprintf(stderr, "c_abi_check: line %d: %s\n", __LINE__, #cond); \
            return 1;                                                       \
        }                                                                   \
    } while (0)

int main(void)
{
    CHECK(dhq_version() >= 100);
    CHECK(strcmp(dhq_strerror(DHQ_OK), "ok") == 0);
    CHECK(strlen(dhq_strerror(DHQ_ENOSCALE)) > 0 && strlen(dhq_strerror(-99)) > 0);

    static float w0[4 * 2], b0[4], w1[1 * 4], b1[1];
    const float *W[2] = {w0, w1}, *B[2] = {b0, b1};
    int32_t dims[3] = {2, 4, 1};
    dhq_net_desc d = {2, dims, 30.0f, 8, 8};
    dhq_model *m = (dhq_model *)0x1;

    CHECK(dhq_quantize_weights(NULL, W, B, &m) == DHQ_EINVAL);
    d.bits_w = 5;
    CHECK(dhq_quantize_weights(&d, W, B, &m) == DHQ_EINVAL && m == NULL);
    d.bits_w = 8;
    dims[1] = 513;
    CHECK(dhq_quantize_weights(&d, W, B, &m) == DHQ_EUNSUPPORTED);
    dims[1] = 4;
    CHECK(dhq_quantize_weights_mode(&d, 7u, W, B, &m) == DHQ_EINVAL);
    CHECK(dhq_quantize_weights_mode(&d, DHQ_ROTATE_BOTH | DHQ_W8A32, W, B, &m) == DHQ_EUNSUPPORTED);
    /* wavelet networks: the spread and omega0 are checked on the host */
    m = (dhq_model *)0x1;
    CHECK(dhq_quantize_weights_wavelet(&d, DHQ_ROTATE_IN, -1.0f, W, B, &m) == DHQ_EINVAL && m == NULL);
    CHECK(dhq_quantize_weights_wavelet(&d, DHQ_ROTATE_IN, 1.0f / 0.0f, W, B, &m) == DHQ_EINVAL);
    CHECK(dhq_quantize_weights_wavelet(NULL, DHQ_ROTATE_IN, 10.0f, W, B, &m) == DHQ_EINVAL);
    CHECK(dhq_quantize_weights_wavelet(&d, 7u, 10.0f, W, B, &m) == DHQ_EINVAL);
    d.omega0 = 0.0f;
    CHECK(dhq_quantize_weights_wavelet(&d, DHQ_ROTATE_IN, 10.0f, W, B, &m) == DHQ_EINVAL);
    d.omega0 = 30.0f;
    w0[3] = 1.0f / 0.0f;
    CHECK(dhq_quantize_weights(&d, W, B, &m) == DHQ_EINVAL);
    CHECK(dhq_quantize_weights_wavelet(&d, DHQ_ROTATE_IN, 10.0f, W, B, &m) == DHQ_EINVAL);

    CHECK(dhq_forward(NULL, NULL, 0, NULL, NULL, DHQ_AUTO) == DHQ_EINVAL);
    CHECK(dhq_set_act_scales(NULL, NULL) == DHQ_EINVAL);
    CHECK(dhq_has_fused(NULL) == DHQ_EINVAL);
    dhq_free(NULL);
    printf("c_abi_check ok\n");
    return 0;
}
