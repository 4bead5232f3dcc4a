// Block-table row compaction shared by the eviction kernels (Alg. 3 "Update the KV Cache Block Table").
#pragma once

#include "pe_device.h"

namespace pe {

// Delete logical entry jstar of a table row that holds n entries: later entries shift left by one (order
// kept), the vacated tail entry becomes -1; an optional score row follows the same motion (tail := +inf).
// One wave, 64 entries per pass: each pass loads its 64 sources before it stores, and a pass only stores to
// positions that later passes do not read.  Returns the physical page that was removed.  bt may be null (only
// the score row moves; the return value is then -1).
__device__ __forceinline__ int compact_row(int32_t* bt, float* sc_mut, int jstar, int n, int lane) {
  const int freed = bt != nullptr ? bt[jstar] : -1;
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_s_waitcnt(0);  // the evicted entry has been read before any store below is issued
  for (int base = (jstar / kWave) * kWave; base < n; base += kWave) {
    const int j = base + lane;
    const bool move = j >= jstar && j < n;
    int32_t v = -1;
    float sv = __builtin_inff();
    if (move && j + 1 < n) {
      if (bt != nullptr) v = bt[j + 1];
      if (sc_mut != nullptr) sv = sc_mut[j + 1];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_s_waitcnt(0);  // all 64 sources are in registers before the stores are issued
    if (move) {
      if (bt != nullptr) bt[j] = v;
      if (sc_mut != nullptr) sc_mut[j] = sv;
    }
  }
  return freed;
}

}  // namespace pe
