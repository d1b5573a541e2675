/* Host-side sanitizer run of the C ABI's argument validation: linked against a build of the library
 * whose host code is compiled with -fsanitize=address,undefined (tests/test_sanitizers.py).  Every entry
 * point is called with arguments it must reject before its first HIP call, so this runs without a GPU. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include "imunpack.h"

#define EXPECT(call, code) do { int rc__ = (call); if (rc__ != (code)) { printf("%s -> %d, expected %d\n", #call, rc__, (code)); ++failures; } } while (0)

int main(void) {
    int failures = 0;
    float *fake = (float *)0x1000;      /* non-null, never dereferenced */
    int32_t *ifake = (int32_t *)0x1000;
    int8_t *bfake = (int8_t *)0x1000;
    imunpack_plan_t *plan = NULL;
    int64_t shape[6], dims[12];
    double ratios[4];
    uint64_t bound[2];
    size_t sz;
    int ba, bb;
    EXPECT(imunpack_quantize(NULL, 4, 4, 4, 1, 1.0f, 8, ifake, 4, NULL, NULL, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_quantize(fake, 4, 4, 4, 1, 1.0f, 9, ifake, 4, NULL, NULL, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_quantize(fake, 4, 4, 4, 1, 0.0f, 8, ifake, 4, NULL, NULL, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_quantize(fake, 4, 4, 4, 1, NAN, 8, ifake, 4, NULL, NULL, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_quantize(fake, 4, 4, 0, 1, 1.0f, 8, ifake, 4, NULL, NULL, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_scan(NULL, 4, 4, 4, 8, NULL, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_percentile(fake, 4, 4, 4, 1, 0.0, fake, NULL, fake, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_percentile_static(fake, 4, 4, 4, 1, 101.0, fake, NULL, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_percentile_static(fake, (int64_t)1 << 16, (int64_t)1 << 16, (int64_t)1 << 16, 1, 95.0, fake, NULL, NULL), IMUNPACK_ERANGE);
    EXPECT(imunpack_plan(ifake, 4, 4, 4, ifake, 4, 4, 8, 3, 0, NULL, NULL, &plan, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_plan(ifake, 4, 4, 3, ifake, 4, 4, 8, 0, 0, NULL, NULL, &plan, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_plan(ifake, 4, 4, 4, ifake, 4, 4, 8, 0, 0, NULL, NULL, NULL, NULL), IMUNPACK_EINVAL);
    EXPECT(plan != NULL, 0);
    EXPECT(imunpack_plan_dims(NULL, dims, dims, dims, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_plan_export(NULL, ifake, ifake, ifake, ifake, ifake, ifake, ifake, ifake, dims), IMUNPACK_EINVAL);
    EXPECT(imunpack_plan_layout(NULL, shape), IMUNPACK_EINVAL);
    EXPECT(imunpack_unpacked_bytes(NULL, &sz, &sz, &sz), IMUNPACK_EINVAL);
    EXPECT(imunpack_unpack(NULL, ifake, 4, ifake, 4, bfake, bfake, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_unpack_canonical(NULL, bfake, bfake, bfake, bfake, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_gemm(NULL, bfake, bfake, NULL, NULL, fake, 4, 1.0f, 1.0f, 1, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_recombine(NULL, fake, 1.0f, 1.0f, NULL, fake, 4, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_plan_bounds(NULL, bound), IMUNPACK_EINVAL);
    EXPECT(imunpack_plan_fusable(NULL), 0);
    EXPECT(imunpack_price(NULL, 4, NULL, 4, 4, 8, fake, dims, ratios, &ba, &bb, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_plan_destroy(NULL), IMUNPACK_OK);
    EXPECT(imunpack_diag_mfma_peak(0, 10, NULL, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_diag_copy(NULL, fake, 1 << 20, NULL), IMUNPACK_EINVAL);
    EXPECT(imunpack_strerror(IMUNPACK_ERANGE) == NULL, 0);
    printf("C ABI sanitizer walk: %d failures\n", failures);
    return failures != 0;
}
