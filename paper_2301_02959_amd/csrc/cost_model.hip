// fs_cost_model / fs_tier_traffic: the paper's analytical per-GPU costs (Section 3.2, the memory
// and communication cost tables) and the traffic the tiers of a routed batch imply.  Host
// arithmetic in double precision; nothing here touches the GPU.
#include "fs_common.h"

extern "C" fs_status fs_cost_model(const fs_cost_params* p, int32_t strategy, double* out)
{
    if (!p || !out) return FS_ERR_NULL;
    if (!(p->E >= 0) || !(p->D > 0) || !(p->dtype_bytes > 0) || !(p->L >= 0) || !(p->W >= 1) || !(p->N >= 1) ||
        !(p->B >= 1) || !(p->a2a_global > 0) || !(p->a2a_intra > 0) || !(p->ar_global > 0) || !(p->ar_cross > 0) ||
        !(p->dp_multiplier > 0))
        return FS_ERR_CONFIG;
    const double U = p->N * p->W;
    const double row = p->D * p->dtype_bytes;                 // bytes of one row
    const double looked_up = p->B * p->L;                      // rows one GPU's batch asks for
    for (int i = 0; i < FS_COST_METRICS; ++i) out[i] = 0.0;
    out[FS_COST_ROWS_ACCESSED] = looked_up * p->D;             // the same in expectation under every strategy
    switch (strategy) {
        case FS_STRATEGY_RW:
            out[FS_COST_STATIC_MEMORY] = p->E / U * row;
            out[FS_COST_INPUT_DIST] = looked_up;
            out[FS_COST_DYNAMIC_MEMORY] = 2.0 * looked_up * row;
            out[FS_COST_DYNAMIC_COMM] = looked_up * row / p->a2a_global;
            break;
        case FS_STRATEGY_CW:
            out[FS_COST_STATIC_MEMORY] = p->E * (p->D / U) * p->dtype_bytes;
            out[FS_COST_INPUT_DIST] = U * looked_up;
            out[FS_COST_DYNAMIC_MEMORY] = 2.0 * looked_up * row;
            out[FS_COST_DYNAMIC_COMM] = looked_up * row / p->a2a_global;
            break;
        case FS_STRATEGY_DP:
            out[FS_COST_STATIC_MEMORY] = p->dp_multiplier * p->E * row;
            out[FS_COST_DYNAMIC_MEMORY] = looked_up * row;
            out[FS_COST_STATIC_COMM] = p->E * row / p->ar_global;
            break;
        case FS_STRATEGY_FLEX:
            out[FS_COST_STATIC_MEMORY] = p->dp_multiplier * (p->E / p->W) * row;
            out[FS_COST_INPUT_DIST] = looked_up;
            out[FS_COST_DYNAMIC_MEMORY] = 2.0 * looked_up * row;
            out[FS_COST_DYNAMIC_COMM] = looked_up * row / p->a2a_intra;
            out[FS_COST_STATIC_COMM] = (p->E / p->W) * row / p->ar_cross;
            break;
        default:
            return FS_ERR_CONFIG;
    }
    return FS_OK;
}

extern "C" fs_status fs_tier_traffic(const int64_t* tier_counts, int32_t D, int32_t dtype_bytes, double* out)
{
    if (!tier_counts || !out) return FS_ERR_NULL;
    if (D < 1 || dtype_bytes < 1 || tier_counts[0] < 0 || tier_counts[1] < 0 || tier_counts[2] < 0) return FS_ERR_SIZE;
    const double row = (double)D * dtype_bytes;
    const double n = (double)tier_counts[0] + (double)tier_counts[1] + (double)tier_counts[2];
    out[0] = n * row;
    out[1] = (double)tier_counts[2] * row;
    out[2] = (double)tier_counts[1] * row;
    out[3] = n > 0 ? ((double)tier_counts[0] + (double)tier_counts[1]) / n : 0.0;
    return FS_OK;
}
