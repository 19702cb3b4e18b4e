#include "gta_tuned.h"

namespace gta {

bool tuned_prefill_supported(const Dims &) { return false; }

int tuned_prefill(const Dims &, const gta_weights &, const void *, const int32_t *, int, int64_t, int,
                  const gta_cache *, const int32_t *, void *, const PrefillWs &, hipStream_t) {
  return GTA_ERR_UNSUPPORTED;
}
}  // namespace gta
