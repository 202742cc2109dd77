/* A plain C caller of the library: builds the cfg0-style chain with the one-shot
 * call and with the builders, evaluates both on the host and checks them against
 * the chain written out as loops.  Exercises include/amap.h from C (no C++,
 * no Python); touches no device entry point. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "amap.h"

#define CHECK(x)                                                          \
    do {                                                                  \
        amap_status st_ = (x);                                            \
        if (st_ != AMAP_OK) {                                             \
            printf("FAIL %s: %s\n", #x, amap_status_str(st_));            \
            return 1;                                                     \
        }                                                                 \
    } while (0)

int main(void)
{
    /* [2,4,3,5] -> transpose (0,2,3,1) -> [2,3,5,4] -> reshape [2,15,4] -> slice rows 2..12 -> pad last dim by 2 */
    const int64_t shape[4] = {2, 4, 3, 5};
    const int64_t perm[4] = {0, 2, 3, 1};
    const int64_t r2[3] = {2, 15, 4};
    const int64_t sl[3] = {2, 12, 1};
    const int64_t lo[3] = {0, 0, 0}, hi[3] = {0, 0, 2};
    amap_src_desc src = {4, shape, AMAP_B32};
    amap_op ops[4];
    memset(ops, 0, sizeof(ops));
    ops[0].kind = AMAP_TRANSPOSE; ops[0].n = 4; ops[0].a = perm;
    ops[1].kind = AMAP_RESHAPE;   ops[1].n = 3; ops[1].a = r2;
    ops[2].kind = AMAP_SLICE;     ops[2].axis = 1; ops[2].n = 3; ops[2].a = sl;
    ops[3].kind = AMAP_PAD;       ops[3].n = 3; ops[3].a = lo; ops[3].b = hi; ops[3].fill_bits = 0xABCD1234u;
    amap_t *m = NULL;
    CHECK(amap_compose(&src, 1, ops, 4, &m));

    amap_t *s0 = NULL, *t = NULL, *r = NULL, *c = NULL, *p = NULL;
    const int32_t perm32[4] = {0, 2, 3, 1};
    CHECK(amap_source(0, 4, shape, AMAP_B32, &s0));
    CHECK(amap_transpose(s0, perm32, &t));
    CHECK(amap_reshape(t, 3, r2, &r));
    CHECK(amap_slice(r, 1, 2, 12, 1, &c));
    CHECK(amap_pad(c, lo, hi, 0xABCD1234u, &p));

    amap_info info;
    CHECK(amap_describe(m, &info));
    if (info.rank != 3 || info.shape[0] != 2 || info.shape[1] != 10 || info.shape[2] != 6 || !info.strided) {
        printf("FAIL describe\n");
        return 1;
    }
    uint32_t in[2 * 4 * 3 * 5], out1[2 * 10 * 6], out2[2 * 10 * 6], want[2 * 10 * 6];
    for (int i = 0; i < 120; ++i) in[i] = 1000u + (uint32_t)i;
    for (int b = 0; b < 2; ++b)
        for (int row = 0; row < 10; ++row)
            for (int col = 0; col < 6; ++col) {
                uint32_t v = 0xABCD1234u;
                if (col < 4) {
                    const int hw = row + 2, h = hw / 5, w = hw % 5; /* row of the [2,15,4] view = h*5 + w */
                    v = in[((b * 4 + col) * 3 + h) * 5 + w];
                }
                want[(b * 10 + row) * 6 + col] = v;
            }
    const void *srcs[1] = {in};
    CHECK(amap_eval_host(m, srcs, out1, 0));
    CHECK(amap_eval_host(p, srcs, out2, 1));
    if (memcmp(out1, want, sizeof(want)) || memcmp(out2, want, sizeof(want))) {
        printf("FAIL values\n");
        return 1;
    }
    int64_t un = -1, over = -1, errs = -1;
    CHECK(amap_check_cover(m, &un, &over));
    CHECK(amap_plan_selfcheck(m, -1, &errs));
    if (un || over || errs) {
        printf("FAIL cover %lld %lld %lld\n", (long long)un, (long long)over, (long long)errs);
        return 1;
    }
    if (amap_slice(m, 7, 0, 1, 1, &t) != AMAP_E_INVALID) { /* t must stay untouched on error */
        printf("FAIL error path\n");
        return 1;
    }
    amap_free(m); amap_free(s0); amap_free(t); amap_free(r); amap_free(c); amap_free(p);
    printf("OK\n");
    return 0;
}
