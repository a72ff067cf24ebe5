// Prefill / mixed path: LDS-tiled bf16 MFMA GEMM (placeholder until the kernels land: never eligible).
#include "common.h"

bool elora::gemm_eligible(const elora_linear_desc_t &d, int max_rank)
{
    (void)d;
    (void)max_rank;
    return false;
}

void elora::gemm_plan(const elora_linear_desc_t &d, elora_plan_t *plan)
{
    (void)d;
    plan->n_launches = 0;
    plan->grid = 0;
}

int elora::launch_gemm(const LinearArgs &a, const elora_plan_t &plan, hipStream_t stream)
{
    (void)a;
    (void)plan;
    (void)stream;
    return ELORA_E_DTYPE;
}
