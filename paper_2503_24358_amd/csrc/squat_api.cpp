// Version, status strings and the launch-shape query of libsquat.
#include "squat_internal.h"

extern "C" int squat_version(void) { return 100; /* 0.1.0 */ }

extern "C" const char* squat_strerror(int status) {
    switch (status) {
        case SQUAT_OK: return "ok";
        case SQUAT_E_NULLPTR: return "a required pointer is NULL";
        case SQUAT_E_BADSHAPE: return "unsupported shape, size or stride";
        case SQUAT_E_BADDTYPE: return "unsupported dtype";
        case SQUAT_E_ALIGN: return "pointer or stride not aligned as required";
        case SQUAT_E_WORKSPACE: return "workspace missing or too small";
        case SQUAT_E_HIP: return "HIP runtime error at launch";
        case SQUAT_E_BADVALUE: return "lambda must be >= 0 (or +inf)";
    }
    return "unknown status";
}

extern "C" int squat_quantize_keys_plan(squat_dtype k_dt, int64_t n_batch, int n_heads, int64_t n_tokens,
                                        int has_update, int64_t update_stride_batch, int bits, int group, int g,
                                        int per_channel, squat_quantize_plan* out) {
    if (!out) return SQUAT_E_NULLPTR;
    if (bits != 2 && bits != 4) return SQUAT_E_BADSHAPE;
    squat::QuantPlan plan;
    int rc;
    if (per_channel) {
        if (group != squat::kTileTokens) return SQUAT_E_BADSHAPE;
        rc = squat::plan_quantize_pc(k_dt, n_batch, n_heads, n_tokens, has_update != 0, update_stride_batch, g, plan);
    } else {
        rc = squat::plan_quantize(k_dt, n_batch, n_heads, n_tokens, has_update != 0, update_stride_batch, group, g, plan);
    }
    if (rc) return rc;
    out->problems = plan.n_prob;
    out->workgroups_per_problem = plan.wgs_per_prob;
    out->wavefronts_per_workgroup = plan.waves;
    out->tiles_per_problem = plan.units_per_prob;
    return SQUAT_OK;
}
