#include "attend_mfma.h"

namespace esa {

bool attend_mfma_supported(int, int, int, int, int) { return false; }
bool attend_mfma_aligned(const void*, const void*, const void*, const void*, const void*, const void*, int64_t,
                         int64_t, int64_t, int64_t, int64_t) { return false; }
size_t attend_mfma_workspace_bytes(int, int, int, int, int) { return 256; }
int launch_attend_mfma(const void*, int, int, int, int, const void*, const void*, int64_t, int64_t, int64_t, int64_t,
                       const void*, const void*, int, float, void*, float*, int, int64_t, int64_t, int64_t, int64_t,
                       void*, size_t, hipStream_t) {
  ESA_FAIL(ESA_EUNSUPPORTED, "matrix-core attention not built");
}

}  // namespace esa
