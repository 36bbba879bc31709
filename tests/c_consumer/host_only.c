/* A plain C99 consumer of the library's header: host-side helpers only (no GPU needed). */
#include <stdio.h>
#include <string.h>

#include "iptq.h"

int main(void)
{
    iptq_softmax_params_t sp;
    iptq_gelu_params_t gp;
    int32_t m = 0, s = 0;
    int rc;

    if (iptq_version() <= 0) return 1;
    rc = iptq_make_dyadic(0.3, &m, &s);
    if (rc != IPTQ_OK || m <= 0 || m >= 32768 || s < 0 || s > 62) return 2;
    rc = iptq_softmax_prepare(1.0 / 128.0, 197, IPTQ_SOFTMAX_EFFICIENT_BITEXP, 0, &sp);
    if (rc != IPTQ_OK || sp.i0 != 128 || sp.variant != IPTQ_SOFTMAX_EFFICIENT_BITEXP) return 3;
    rc = iptq_gelu_prepare(1.0 / 16.0, 1.0 / 32.0, 0, 0, IPTQ_GELU_POLY4_DATA_AWARE, 255, &gp);
    if (rc != IPTQ_OK || gp.q_b >= 0 || gp.q_c >= 0) return 4;
    /* errors come back as codes with a message, never as a crash */
    rc = iptq_softmax_prepare(-1.0, 197, 0, 0, &sp);
    if (rc == IPTQ_OK || strlen(iptq_strerror(rc)) == 0) return 5;
    if (iptq_softmax_i32(NULL, NULL, 0, NULL, 4, 197, &sp, NULL) != IPTQ_ERR_NULL) return 6;
    /* the windowed forms check their arguments on the host as well: nothing is launched here */
    rc = iptq_softmax_prepare(1.0 / 128.0, 49, IPTQ_SOFTMAX_BITEXP_DEGREE2, 0, &sp);
    if (rc != IPTQ_OK || sp.variant != IPTQ_SOFTMAX_BITEXP_DEGREE2) return 7;
    if (iptq_softmax_i32_windowed_bits(NULL, NULL, 0, (const uint64_t *)8, 0, 1, NULL, 49, 49, &sp, NULL) != IPTQ_ERR_SHAPE) return 8;
    if (iptq_pack_window_mask(NULL, 2, 49, NULL, NULL) != IPTQ_ERR_NULL) return 9;
    if (iptq_pack_window_mask(NULL, 0, 49, NULL, NULL) != IPTQ_OK) return 10;
    {
        double x[4] = {100.0, -100.0, 100.0, -100.0}, xh[4] = {110.0, -110.0, 110.0, -110.0};
        iptq_metric_t mt;
        /* power 10^4 against an error power of 100: 20 dB (the worked example of Section 4.5) */
        if (iptq_unified_metric(x, xh, 4, 18.0, IPTQ_METRIC_PER_ELEMENT, &mt) != IPTQ_OK) return 11;
        if (mt.q_db < 19.999 || mt.q_db > 20.001) return 12;
    }
    printf("ok %d %d %d %d\n", iptq_version(), (int)m, (int)s, (int)sp.i0);
    return 0;
}
