/* Plain C translation unit against include/tpo.h: proves the header is C (not C++), that the
 * library links from C, and that argument validation answers before any device is touched.
 * Returns 0 when every status is the documented one. */
#include <stdio.h>
#include <string.h>

#include "tpo.h"
#include "tpo_bench.h"

int main(void)
{
    static double buf[6][4 * 4 * 4 * 2];
    int bad = 0;
    bad += strcmp(tpo_status_string(TPO_OK), "ok") != 0;
    bad += tpo_ihelm_apply(buf[0], buf[1], buf[2], buf[3], buf[4], buf[5], 0, 2, TPO_F64, NULL)
           != TPO_ERR_INVALID_ARG;
    bad += tpo_ihelm_apply(buf[0], buf[1], buf[2], buf[3], buf[4], buf[5], TPO_MAX_N + 1, 2, TPO_F64,
                           NULL) != TPO_ERR_UNSUPPORTED;
    bad += tpo_ihelm_apply(buf[0], buf[1], buf[2], buf[3], buf[4], buf[4], 4, 2, TPO_F64, NULL)
           != TPO_ERR_ALIAS;
    bad += tpo_ihelm_apply(buf[0], buf[1], buf[2], buf[3], buf[4], buf[5], 4, 0, TPO_F64, NULL)
           != TPO_OK;
    bad += tpo_transform_apply(buf[0], buf[1], buf[2], buf[3], buf[5], 4, 2, TPO_F64, 7, NULL)
           != TPO_ERR_INVALID_ARG;
    bad += tpo_ihelm_apply_sep(buf[0], buf[1], buf[2], buf[3], buf[4], buf[4], buf[4], NULL, buf[5],
                               4, 2, TPO_F64, NULL) != TPO_ERR_INVALID_ARG;
    bad += tpo_ihelm_apply_variant(buf[0], buf[1], buf[2], buf[3], buf[4], buf[5], 4, 2, TPO_F64,
                                   NULL, 99) != TPO_ERR_INVALID_ARG;
    bad += tpo_ihelm_apply_sep_variant(buf[0], buf[1], buf[2], buf[3], buf[4], buf[4], buf[4],
                                       buf[4], buf[5], 4, -1, TPO_F64, NULL, TPO_VARIANT_AUTO)
           != TPO_ERR_INVALID_ARG;
    bad += tpo_ihelm_apply_aniso(buf[0], buf[1], buf[2], buf[3], buf[4], buf[5], 2, 3, 17, 2,
                                 TPO_F64, NULL) != TPO_ERR_UNSUPPORTED;
    bad += tpo_ihelm_apply_aniso(buf[0], buf[1], buf[2], buf[3], buf[4], buf[5], 2, 3, 4, 0,
                                 TPO_F64, NULL) != TPO_OK;
    bad += tpo_convection_apply(buf[0], buf[1], buf[2], buf[3], NULL, 3, 4, 1, TPO_F64, NULL)
           != TPO_ERR_INVALID_ARG;
    bad += tpo_stream_scale(buf[0] + 1, buf[1], buf[2], 4, TPO_F64, NULL) != TPO_ERR_INVALID_ARG;
    bad += tpo_ihelm_has_variant(11, TPO_F64, TPO_VARIANT_MFMA) != 1;
    bad += tpo_ihelm_has_variant(11, TPO_F64, TPO_VARIANT_PENCIL_MM) != 0;
    bad += tpo_ihelm_sep_has_variant(13, TPO_F32, TPO_VARIANT_PENCIL_MM) != 1;
    bad += tpo_ihelm_sep_variant_for(13, TPO_F32) != TPO_VARIANT_PENCIL_MM;
    {   /* with a device the pair succeeds; without one create reports it and destroy has
           nothing to drop */
        const int rc = tpo_create();
        bad += rc != TPO_OK && rc != TPO_ERR_DEVICE;
        bad += tpo_destroy() != (rc == TPO_OK ? TPO_OK : TPO_ERR_NOT_INITIALIZED);
    }
    bad += tpo_convection_has_shape(8, 12, TPO_F64) != 1;
    bad += tpo_ihelm_variant_for(11, TPO_F64, 1) != TPO_VARIANT_PENCIL;
    bad += tpo_ihelm_variant_for_batch(16, TPO_F64, 1, 1 << 20) != TPO_VARIANT_MFMA;
    bad += tpo_ihelm_variant_for_batch(16, TPO_F64, 1, -1) != TPO_ERR_INVALID_ARG;
    bad += tpo_ihelm_sep_variant_for_batch(16, TPO_F64, 1, 1 << 20) != TPO_VARIANT_MFMA;
    printf("abi_check: %d unexpected status(es)\n", bad);
    return bad;
}
