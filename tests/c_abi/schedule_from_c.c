/* The boundary is a C ABI: this file is plain C99, includes the public header and links against the shared library.
 * It schedules the 5-layer instance on which Algorithm 2's "optimal hiding" is not optimal (backward times 1,1,8,1,2,
 * communication times 2,5,2,1,9, H = 2) with both policies, evaluates Eq. (8) and Eq. (7) for the results, and prints
 * everything for the test to compare. */
#include <stdint.h>
#include <stdio.h>

#include "dreamddp.h"

int main(void) {
    const int64_t bp[5] = {1, 1, 8, 1, 2}, comm[5] = {2, 5, 2, 1, 9};
    const int policies[2] = {DDP_SCHED_ALG2, DDP_SCHED_OPT};
    int p;
    for (p = 0; p < 2; ++p) {
        int32_t slot[5], set_ptr[3], set_layers[5];
        int64_t cost = -1, cost2 = -1, iter[2], exposed[2], period = -1;
        int rc = ddp_schedule(policies[p], 5, 2, NULL, bp, comm, slot, set_ptr, set_layers, &cost);
        int j;
        if (rc != DDP_OK) {
            printf("ddp_schedule failed: %d %s\n", rc, ddp_last_error(NULL));
            return 1;
        }
        rc = ddp_schedule_cost(5, 2, bp, comm, set_ptr, set_layers, &cost2);
        if (rc != DDP_OK || cost2 != cost) return 2;
        rc = ddp_schedule_time_model(5, 2, NULL, bp, comm, set_ptr, set_layers, iter, exposed, &period);
        if (rc != DDP_OK) return 3;
        printf("policy %d cost %lld sets", policies[p], (long long)cost);
        for (j = 0; j < 5; ++j) printf("%s%d", j == set_ptr[1] ? " | " : " ", (int)set_layers[j]);
        printf(" period %lld\n", (long long)period);
    }
    /* an argument error comes back as a code and a message, never as a crash */
    if (ddp_schedule(DDP_SCHED_OPT, 0, 2, NULL, bp, comm, NULL, NULL, NULL, NULL) != DDP_EINVAL) return 4;
    printf("error: %s\n", ddp_last_error(NULL));
    return 0;
}
