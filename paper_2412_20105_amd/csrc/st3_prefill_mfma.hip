// bf16 prefill attention on the MFMA units (placeholder until the tiled kernel lands).
#include "st3_common.h"

namespace st3 {
struct PrefillArgs;
st3_status launch_prefill_mfma(const PrefillArgs&, int, int, hipStream_t) { return ST3_ERR_UNSUPPORTED; }
}  // namespace st3
