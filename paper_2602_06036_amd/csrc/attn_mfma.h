// MFMA block attention for bf16 caches (see attn.h for the split / merge contract).
#pragma once
#include "attn.h"

// Returns true when it launched a kernel for this configuration; false -> caller uses the generic kernel.
template <typename T>
inline bool attn_mfma_launch(hipStream_t, const T*, const T*, SeqGeom, AttnArgs, int, float*, float2*) {
  return false;
}
