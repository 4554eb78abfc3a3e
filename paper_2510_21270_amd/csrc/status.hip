// Status strings, problem validation and workspace sizing of the C ABI.
#include "pbs_host.h"

namespace pbs {
size_t ws_key_scores(const pbs_problem *p);
size_t ws_block_mask(const pbs_problem *p);
size_t ws_attn_fwd(const pbs_problem *p);
size_t ws_query_permute(const pbs_problem *p);
}  // namespace pbs

extern "C" const char *pbs_status_string(pbs_status st)
{
    switch (st) {
    case PBS_OK: return "ok";
    case PBS_ERR_NULL: return "a required pointer is NULL";
    case PBS_ERR_SHAPE: return "inconsistent problem sizes or misaligned tensor";
    case PBS_ERR_UNSUPPORTED: return "problem outside the supported set";
    case PBS_ERR_WORKSPACE: return "workspace too small or misaligned";
    case PBS_ERR_HIP: return "kernel launch failed";
    }
    return "unknown status";
}

extern "C" pbs_status pbs_validate(const pbs_problem *p) { return pbs::validate(p); }

extern "C" size_t pbs_workspace_bytes(const pbs_problem *p, int stage)
{
    if (pbs::validate(p) != PBS_OK) return 0;
    switch (stage) {
    case PBS_STAGE_KEY_SCORES: return pbs::ws_key_scores(p);
    case PBS_STAGE_BLOCK_MASK: return pbs::ws_block_mask(p);
    case PBS_STAGE_ATTN_FWD: return pbs::ws_attn_fwd(p);
    case PBS_STAGE_QUERY_PERMUTE: return pbs::ws_query_permute(p);
    default: return 0;
    }
}

extern "C" size_t pbs_vt_bytes(const pbs_problem *p)
{
    if (pbs::validate(p) != PBS_OK) return 0;
    const pbs::Geo g = pbs::make_geo(p);
    const size_t half = (size_t)g.batch * g.h_kv * g.T * g.d * g.block * pbs::elem_size(p->dtype);
    return (p->flags & PBS_FLAG_TOKEN_ORDER_COPY) ? 2 * half : half;
}
