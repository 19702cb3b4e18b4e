// Tuned bf16 path for gfx950: MFMA GEMMs, MFMA prefill attention, streaming split-K decode.
#pragma once
#include "gta_internal.h"

namespace gta {

bool tuned_prefill_supported(const Dims &d);
bool tuned_decode_supported(const Dims &d);

int tuned_prefill(const Dims &d, const gta_weights &w, const void *x, const int32_t *cu, int batch,
                  int64_t total, int max_len, const gta_cache *cache, const int32_t *slots, void *out,
                  const PrefillWs &ws, hipStream_t st);
int tuned_decode(const Dims &d, const gta_weights &w, const void *x_new, int batch, const gta_cache &cache,
                 const int32_t *slots, void *out, const DecodeWs &ws, hipStream_t st);

}  // namespace gta
