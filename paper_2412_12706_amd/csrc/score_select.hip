// placeholder until the scoring kernels land
#include "kvqp_internal.h"
namespace kvqp {
CompressPlan plan_compress(const kvqp_cfg& cfg) {
    CompressPlan p{};
    p.P = cfg.seq_len - cfg.window;
    p.n_kept = cfg.budget < p.P ? cfg.budget : p.P;
    p.off_idx = 0;
    p.total = (size_t)cfg.batch * cfg.n_kv_heads * (p.n_kept > 0 ? p.n_kept : 1) * 4;
    return p;
}
hipError_t launch_select(const kvqp_cfg&, const void*, const void*, int32_t*, void*, const CompressPlan&, hipStream_t) {
    return hipErrorNotSupported;
}
}  // namespace kvqp
