/* Plain C99 client of the C ABI (no HIP, no C++): plans the tiny GPT reshard host-side and prints its
 * statistics.  Built and run by tests/test_c_abi.py to show that include/liver.h is valid C and that the
 * library can be driven without Python. */
#include <stdio.h>
#include <string.h>

#include "liver.h"

int main(void) {
    liver_model_spec_t spec;
    liver_layout_t src, dst;
    liver_plan_t* plan = NULL;
    liver_plan_info_t info;
    liver_desc_t d;
    size_t bytes = 0;
    int rc;
    memset(&spec, 0, sizeof spec);
    memset(&src, 0, sizeof src);
    memset(&dst, 0, sizeof dst);
    spec.n_layers = 2, spec.hidden = 256, spec.n_q_heads = 4, spec.n_kv_heads = 4, spec.ffn = 1024, spec.vocab = 1024;
    spec.max_pos = 512, spec.flags = LIVER_NORM_BIAS | LIVER_LINEAR_BIAS | LIVER_TIED_EMBED;
    src.tp = 2, src.pp = 1, src.dp = 2, src.pad_multiple = 128, src.only_tp = src.only_pp = src.only_dp = -1;
    dst.tp = 1, dst.pp = 2, dst.dp = 2, dst.pad_multiple = 128, dst.only_tp = dst.only_pp = dst.only_dp = -1;
    rc = liver_plan_create(&spec, &src, &dst, (size_t)1 << 20, &plan);
    if (rc != LIVER_OK) {
        printf("plan_create failed: %s\n", liver_strerror(rc));
        return 1;
    }
    if (liver_plan_info(plan, &info) != LIVER_OK || liver_plan_buffer_bytes(plan, 1, 0, LIVER_MASTER_F32, &bytes) != LIVER_OK ||
        liver_plan_desc(plan, LIVER_LIST_DIRECT, 0, &d) != LIVER_OK)
        return 2;
    printf("chunks %lld descriptors %lld stream_bytes %lld dst0_master_bytes %zu first_op %d\n", (long long)info.n_chunks,
           (long long)info.n_desc, (long long)info.stream_bytes, bytes, d.op);
    rc = liver_plan_create(&spec, &src, &dst, 100, &plan); /* bad chunk size */
    printf("bad chunk_bytes -> %d (%s)\n", rc, liver_strerror(rc));
    liver_plan_destroy(plan);
    liver_plan_destroy(NULL);
    return rc == LIVER_E_INVALID_ARG ? 0 : 3;
}
