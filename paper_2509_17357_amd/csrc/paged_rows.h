// Device helper shared by the paged scatter and gather kernels: which sequence does
// work-group g of the grid serve?
#pragma once

#include <hip/hip_runtime.h>

namespace cronus {

// Last s in [0, n_seqs) with first_group(s) <= g, first_group(s) = cu_tokens[s] / 16 + 2 s
// (non-decreasing; first_group(0) = 0).  64-ary search: every lane of the wavefront probes
// one candidate and a ballot counts the hits, so the answer takes ceil(log64 n_seqs)
// dependent loads instead of log2 n_seqs.  All lanes return the same value.
__device__ __forceinline__ int find_sequence(const int* __restrict__ cu_tokens, int n_seqs, int g) {
  const int lane = threadIdx.x & 63;
  int lo = 0, len = n_seqs;
  while (len > 1) {
    const int stride = (len + 63) >> 6;
    const int idx = lo + lane * stride;
    const bool hit = lane * stride < len && (cu_tokens[idx] >> 4) + 2 * idx <= g;
    const int hits = __builtin_popcountll(__builtin_amdgcn_ballot_w64(hit));  // >= 1: lane 0 probes lo
    const int end = lo + len;
    lo += (hits - 1) * stride;
    len = min(stride, end - lo);
  }
  return lo;
}

}  // namespace cronus
