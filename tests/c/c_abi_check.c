/* The header must be plain C, and the entry points must be callable from C without a GPU for
 * everything that is decided on the host: version, status names, argument checks.  Called with
 * the argument "forward" (on a machine with a GPU) the program also quantizes a tiny network,
 * calibrates it and runs it through dhq_forward and dhq_forward_noalloc, all from plain C. */
#include <math.h>
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

/* the four HIP runtime calls the forward part needs, declared by hand: the runtime's own header
 * is not written for -std=c99 -pedantic (status and copy direction are enums, i.e. ints) */
extern int hipMalloc(void **ptr, size_t size);
extern int hipFree(void *ptr);
extern int hipMemcpy(void *dst, const void *src, size_t size, int kind); /* 1: host to device, 2: device to host */
extern int hipDeviceSynchronize(void);

static int forward_from_c(void)
{
    /* 2 -> 4 -> 1: the first layer's weights are zero, so its outputs are sin(omega0 b0[j]) whatever
     * the coordinates, and the network's value is sum_j w1[j] sin(omega0 b0[j]) + b1 up to quantization */
    static float w0[4 * 2];
    float b0[4] = {0.01f, 0.02f, -0.03f, 0.04f}, w1[4] = {0.5f, -0.25f, 0.125f, 1.0f}, b1[1] = {0.3f};
    const float *W[2], *B[2];
    int32_t dims[3] = {2, 4, 1};
    dhq_net_desc d;
    dhq_model *m = NULL;
    float coords[8 * 2], out[8], out2[8], s_w[2], s_a[2];
    void *coords_dev = NULL, *out_dev = NULL;
    double expect = 0.3;
    int i;
    W[0] = w0; W[1] = w1; B[0] = b0; B[1] = b1;
    d.n_layers = 2; d.dims = dims; d.omega0 = 30.0f; d.bits_w = 8; d.bits_a = 8;
    for (i = 0; i < 4; ++i) expect += (double)w1[i] * sin(30.0 * (double)b0[i]);
    for (i = 0; i < 16; ++i) coords[i] = (float)(i - 8) / 8.0f;
    CHECK(dhq_quantize_weights(&d, W, B, &m) == DHQ_OK && m != NULL);
    CHECK(hipMalloc(&coords_dev, sizeof(coords)) == 0 && hipMalloc(&out_dev, sizeof(out)) == 0);
    CHECK(hipMemcpy(coords_dev, coords, sizeof(coords), 1) == 0);
    CHECK(dhq_forward(m, (const float *)coords_dev, 8, (float *)out_dev, NULL, DHQ_AUTO) == DHQ_ENOSCALE);
    CHECK(dhq_calibrate(m, (const float *)coords_dev, 8, NULL) == DHQ_OK);
    CHECK(dhq_get_scales(m, s_w, s_a) == DHQ_OK && s_a[0] > 0.0f && s_a[1] > 0.0f && s_w[0] == 1.0f);
    CHECK(dhq_forward(m, (const float *)coords_dev, 8, (float *)out_dev, NULL, DHQ_AUTO) == DHQ_OK);
    CHECK(hipDeviceSynchronize() == 0 && hipMemcpy(out, out_dev, sizeof(out), 2) == 0);
    for (i = 0; i < 8; ++i) CHECK(fabs((double)out[i] - expect) < 0.02);
    /* scales measured on line, on the model's buffers and on the library's fixed one: the same bits */
    CHECK(dhq_forward(m, (const float *)coords_dev, 8, (float *)out_dev, NULL, DHQ_AUTO | DHQ_DYNAMIC) == DHQ_OK);
    CHECK(hipDeviceSynchronize() == 0 && hipMemcpy(out, out_dev, sizeof(out), 2) == 0);
    CHECK(dhq_noalloc_max_rows(m) >= 8);
    CHECK(dhq_forward_noalloc(m, (const float *)coords_dev, 8, (float *)out_dev, NULL, DHQ_AUTO) == DHQ_OK);
    CHECK(hipDeviceSynchronize() == 0 && hipMemcpy(out2, out_dev, sizeof(out2), 2) == 0);
    CHECK(memcmp(out, out2, sizeof(out)) == 0);
    for (i = 0; i < 8; ++i) CHECK(fabs((double)out[i] - expect) < 0.02);
    CHECK(dhq_forward_noalloc(m, (const float *)coords_dev, dhq_noalloc_max_rows(m) + 1, (float *)out_dev, NULL, DHQ_AUTO) == DHQ_ETOOBIG);
    dhq_free(m);
    CHECK(hipFree(coords_dev) == 0 && hipFree(out_dev) == 0);
    printf("c_abi_check forward ok (value %.6f, expected %.6f)\n", (double)out[0], expect);
    return 0;
}

int main(int argc, char **argv)
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
    CHECK(dhq_reserve_dynamic(NULL, 1) == DHQ_EINVAL);
    CHECK(dhq_forward_noalloc(NULL, NULL, 0, NULL, NULL, DHQ_AUTO) == DHQ_EINVAL);
    CHECK(dhq_noalloc_max_rows(NULL) == 0);
    CHECK(dhq_forward_debug_fused(NULL, NULL, 0, 0, NULL, NULL, NULL, NULL) == DHQ_EINVAL);
    dhq_free(NULL);
    if (argc > 1 && strcmp(argv[1], "forward") == 0 && forward_from_c() != 0) return 1;
    printf("c_abi_check ok\n");
    return 0;
}
