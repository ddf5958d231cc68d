/* The public header must be plain C: this file is compiled with a C compiler (C99, pedantic, no warnings
 * allowed) and linked against the built library by tests/test_lib_host.py, then run: it plans one problem
 * and queries one Bloom set through the C ABI, host side only. */
#include <stdio.h>
#include "streamk.h"

int main(void) {
    sk_plan_t* plan = NULL;
    sk_plan_header h;
    sk_bloom_t* bloom = NULL;
    sk_bloom_record rec = {3840u, 4224u, 4096u, 0x41u};
    uint32_t mask = 0;
    int64_t times[3] = {100, 120, 121};
    if (sk_plan(3840, 4224, 4096, SK_POLICY_SK1_DP, NULL, &plan) != SK_OK) return 1;
    if (sk_plan_info(plan, &h) != SK_OK || h.tiles < 1 || h.grid != 256) return 2;
    if (sk_workspace_bytes(plan) > SK_STATIC_WORKSPACE_MAX_BYTES) return 3;
    sk_plan_destroy(plan);
    if (bloom_build(&rec, 1, NULL, &bloom) != SK_OK) return 4;
    if (bloom_query(bloom, 3840, 4224, 4096, &mask) != SK_OK || (mask & 0x41u) != 0x41u) return 5;
    bloom_destroy(bloom);
    if (bloom_winner_mask(times, 3, 200u, &mask) != SK_OK || mask != 3u) return 6;
    printf("%s\n", sk_status_str(SK_OK));
    return 0;
}
