// Fused reconstruct-then-attend decode kernel (bf16 MFMA).  Placeholder until
// the MFMA path lands: reports "not supported" so the unfused path runs.
#pragma once
#include "common.h"
namespace echokv {
template <typename T> inline bool fused_decode_supported(int, int) { return false; }
template <typename T>
inline int launch_fused_decode(int, int, int, int, float, const T*, const T*, const T*, const T*,
                               const T*, const T*, const T*, float*, float*, SeqMeta&, int*,
                               hipStream_t) { return 6; }
template <typename T> inline bool recon_mfma_supported() { return false; }
template <typename T>
inline int launch_recon_mfma(int, int, const T*, const T*, const T*, const T*, const T*, const T*,
                             T*, T*, int64_t, int, SeqMeta&, hipStream_t) { return 6; }
}  // namespace echokv
