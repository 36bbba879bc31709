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
    printf("ok %d %d %d %d\n", iptq_version(), (int)m, (int)s, (int)sp.i0);
    return 0;
}
