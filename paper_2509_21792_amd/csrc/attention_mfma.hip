// placeholder until the MFMA kernel lands
#include "fg_common.h"
namespace fg {
bool attention_mfma_supported(const fg_kv_cache *, int, int) { return false; }
int64_t attention_mfma_ws_bytes(int, int, int, int, int, int) { return 0; }
int32_t launch_attention_mfma(const fg_kv_cache *, int, const fg_tree *, TreeDev, int, const void *, void *, int, void *, int64_t,
                              hipStream_t)
{
    return fail(FG_ERR_UNIMPLEMENTED, "MFMA attention not built");
}
}  // namespace fg
