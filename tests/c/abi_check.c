/* A plain C99 program against include/dream.h: the header must compile as C, and the host-only entry points must
 * work without a GPU.  Built and run by tests/test_abi.py. */
#include <stdio.h>
#include <string.h>
#include "dream.h"

int main(void)
{
    int32_t parent[5] = {-1, 0, 0, 1, 3};
    int32_t depth = -1;
    if (dream_tree_validate_host(parent, 5, &depth) != DREAM_OK || depth != 3) {
        printf("validate: depth %d, %s\n", (int)depth, dream_last_error());
        return 1;
    }
    parent[2] = 2;   /* a node that is its own parent */
    if (dream_tree_validate_host(parent, 5, &depth) == DREAM_OK || strlen(dream_last_error()) == 0) {
        printf("a malformed tree was accepted\n");
        return 2;
    }
    dream_attn_desc desc;
    memset(&desc, 0, sizeof desc);
    desc.batch = 1; desc.n_q_heads = 32; desc.n_kv_heads = 32; desc.head_dim = 128; desc.dtype = DREAM_BF16; desc.s_max = 764;
    char plan[256];
    if (dream_attn_plan_describe(&desc, 60, 764, plan, sizeof plan) != DREAM_OK) {
        printf("plan: %s\n", dream_last_error());
        return 3;
    }
    if (dream_tree_verify_attn_workspace(&desc, 60, 764) < DREAM_WORKSPACE_MIN_BYTES)
        return 4;
    /* a NULL tensor is an argument error found on the host: nothing is launched */
    if (dream_tree_verify_attn(&desc, NULL, NULL, NULL, NULL, 60, NULL, NULL, 764, NULL, NULL, NULL, 0, NULL) != DREAM_ERR_INVALID_ARG)
        return 5;
    dream_proj_job job;
    memset(&job, 0, sizeof job);
    if (dream_project_rows_multi(&desc, &job, 0, 10, 4096, NULL) != DREAM_ERR_INVALID_ARG)
        return 6;
    printf("%s\n", plan);
    return 0;
}
