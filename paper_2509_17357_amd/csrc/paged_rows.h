// Device helper shared by the paged scatter and gather kernels: which sequence does
// work-group g of the grid serve, and which rows does that sequence have in this call?
#pragma once

#include <hip/hip_runtime.h>

namespace cronus {

struct SeqRows {
  int seq;     // last s in [0, n_seqs) with first_group(s) <= g
  int row0;    // cu_tokens[s]
  int n_rows;  // cu_tokens[s + 1] - cu_tokens[s]
  int start;   // start_pos[s]
};

// first_group(s) = cu_tokens[s] / 16 + 2 s is non-decreasing and first_group(0) = 0.
// 63-ary search: every lane of the wavefront probes one candidate (the range's end
// included) and a ballot counts the hits, so the answer takes ceil(log63 n_seqs) dependent
// loads instead of log2 n_seqs; the last round probes consecutive entries, so cu_tokens[s],
// cu_tokens[s + 1] and start_pos[s] are picked from the lanes that already hold them
// instead of being loaded again.  All lanes return the same values.
__device__ __forceinline__ SeqRows find_sequence(const int* __restrict__ cu_tokens,
                                                 const int* __restrict__ start_pos, int n_seqs, int g) {
  const int lane = threadIdx.x & 63;
  int lo = 0, len = n_seqs;
  for (;;) {
    const int stride = (len + 62) / 63;
    const int off = lane * stride;
    const int idx = lo + off;
    const int cu = off <= len ? cu_tokens[idx] : 0;         // idx = lo + len is cu_tokens' entry after the range
    const int sp = (stride == 1 && off < len) ? start_pos[idx] : 0;
    const bool hit = off < len && (cu >> 4) + 2 * idx <= g;
    const int hits = __builtin_amdgcn_readfirstlane(
        (int)__builtin_popcountll(__builtin_amdgcn_ballot_w64(hit)));  // >= 1: lane 0 probes lo
    if (stride == 1) {
      SeqRows r;
      r.seq = lo + hits - 1;
      r.row0 = __builtin_amdgcn_readlane(cu, hits - 1);
      r.n_rows = __builtin_amdgcn_readlane(cu, hits) - r.row0;
      r.start = __builtin_amdgcn_readlane(sp, hits - 1);
      return r;
    }
    const int end = lo + len;
    lo += (hits - 1) * stride;
    len = min(stride, end - lo);
  }
}

}  // namespace cronus
