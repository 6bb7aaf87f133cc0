#include "common.h"
namespace disco {
bool mfma_supported(int64_t, int64_t, int32_t, int) { return false; }
size_t mfma_stored_workspace_bytes(int64_t, int64_t, int32_t) { return 0; }
int mfma_stored_run(const Problem&) { return DISCO_ERR_UNSUPPORTED; }
}  // namespace disco
