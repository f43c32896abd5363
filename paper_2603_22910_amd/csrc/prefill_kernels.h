// Causal prefill attention over retained + materialised predicted heads (MFMA).
// Placeholder: reports "not supported" so the streaming path runs.
#pragma once
#include "common.h"
namespace echokv {
template <typename T> inline bool prefill_mfma_supported(int) { return false; }
template <typename T>
inline int launch_prefill_mfma(int, int, int, int, float, bool, const T*, const T*, const T*,
                               const T*, const T*, int, int, void*, float*, hipStream_t) { return 6; }
}  // namespace echokv
