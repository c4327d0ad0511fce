// Attention forward placeholder until the kernel lands.
#include "mlt_common.h"
#include "mlt_internal.h"

namespace mlt {
MhaPlan plan_mha(const MhaArgs&) { return MhaPlan(); }
int run_mha(const MhaArgs&, const MhaPlan&, hipStream_t) { return MLT_ERR_UNSUPPORTED; }
}  // namespace mlt
