// Paged gather of K/V rows: the inverse of the paged scatter (Cronus section 4.2: the
// instance that ran the partial prefill hands the prefix over as one contiguous KV
// buffer).  Same cache layout and the same numbering of work-groups as the scatter:
//   K pool [num_blocks][Hkv][D/8][16][8]   chunk = 8 consecutive d of one token
//   V pool [num_blocks][Hkv][2][D][8]      chunk = 8 consecutive tokens of one d
// One work-group exports one (cache block, KV head).  K chunks are read as stored and
// written to their rows; V is read in whole chunks (coalesced) and turned back into rows
// through LDS.  Elements are moved as they are (bf16 values or e4m3 codes).
#include <hip/hip_runtime.h>

#include "cronus_internal.h"
#include "paged_rows.h"

namespace cronus {
namespace {

template <int ESZ> struct ChunkOf;
template <> struct ChunkOf<2> { typedef unsigned int type __attribute__((ext_vector_type(4))); };
template <> struct ChunkOf<1> { typedef unsigned int type __attribute__((ext_vector_type(2))); };

// Work-group g of grid.x serves the last sequence s with cu_tokens[s]/16 + 2 s <= g and
// the (g - that)-th cache block its rows touch; grid.x = n_tokens/16 + 2 n_seqs + 1.
template <int ESZ>
__global__ __launch_bounds__(256) void kv_gather_kernel(
    const unsigned char* __restrict__ k_pool, const unsigned char* __restrict__ v_pool,
    unsigned char* __restrict__ k_dst, unsigned char* __restrict__ v_dst, const int* __restrict__ cu_tokens,
    const int* __restrict__ start_pos, const int* __restrict__ block_tables, int max_blocks, int n_seqs,
    int n_kv_heads, int head_dim) {
  using Chunk = typename ChunkOf<ESZ>::type;
  constexpr int CB = 8 * ESZ;                       // bytes of a chunk
  __shared__ __align__(16) unsigned char vt[256][CB + 2 * ESZ];  // [kc * D + d][8 tokens], padded rows
  const int g = blockIdx.x, head = blockIdx.y;
  const int t = threadIdx.x;
  const int slot = t & 15, dc = t >> 4;
  const int n_dc = head_dim >> 3;

  const SeqRows sr = find_sequence(cu_tokens, start_pos, n_seqs, g);
  const int s = sr.seq, row0 = sr.row0, n_rows = sr.n_rows, start = sr.start;
  const int j = g - ((row0 >> 4) + 2 * s);
  const int bi = (start >> 4) + j;
  const int pos_lo = max(start, bi * 16), pos_hi = min(start + n_rows, bi * 16 + 16);
  if (n_rows <= 0 || pos_lo >= pos_hi) return;      // uniform over the work-group
  const int slot_lo = pos_lo & 15, slot_hi = slot_lo + (pos_hi - pos_lo);

  const long long blk = block_tables[(long long)s * max_blocks + bi];
  const long long head_base = (blk * n_kv_heads + head) * (long long)(16 * head_dim) * ESZ;  // bytes
  const bool mine = slot >= slot_lo && slot < slot_hi && dc < n_dc;
  const long long dst_off =
      (((long long)(row0 + (bi * 16 + slot - start)) * n_kv_heads + head) * head_dim + dc * 8) * ESZ;

  // ---- V: chunk t of the block = (kc, d), kc = t / D, d = t % D
  if (t < 2 * head_dim) {
    const Chunk c = *reinterpret_cast<const Chunk*>(v_pool + head_base + (long long)t * CB);
    unsigned char* row = vt[t];
#pragma unroll
    for (int w = 0; w < CB / 4; ++w) {
      // rows are 2-byte aligned only (padding), so store in halves
      *reinterpret_cast<unsigned short*>(row + 4 * w) = (unsigned short)(c[w] & 0xffffu);
      *reinterpret_cast<unsigned short*>(row + 4 * w + 2) = (unsigned short)(c[w] >> 16);
    }
  }
  // ---- K: chunk (dc, slot) as stored
  if (mine) {
    const Chunk c = *reinterpret_cast<const Chunk*>(k_pool + head_base + ((long long)dc * 16 + slot) * CB);
    *reinterpret_cast<Chunk*>(k_dst + dst_off) = c;
  }
  __syncthreads();
  if (mine) {
    const int kc = slot >> 3, e = slot & 7;
    unsigned char out[CB];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) {
      const unsigned char* src = vt[kc * head_dim + dc * 8 + jj] + e * ESZ;
#pragma unroll
      for (int b = 0; b < ESZ; ++b) out[jj * ESZ + b] = src[b];
    }
    Chunk c;
#pragma unroll
    for (int w = 0; w < CB / 4; ++w)
      c[w] = (unsigned)out[4 * w] | ((unsigned)out[4 * w + 1] << 8) | ((unsigned)out[4 * w + 2] << 16) |
             ((unsigned)out[4 * w + 3] << 24);
    *reinterpret_cast<Chunk*>(v_dst + dst_off) = c;
  }
}

}  // namespace

int launch_kv_gather(const cronus_kv_cache* cache, void* k_dst, void* v_dst, const int32_t* cu_tokens,
                     const int32_t* start_pos, const int32_t* block_tables, int32_t max_blocks_per_seq,
                     int32_t n_seqs, int32_t n_tokens, void* stream) {
  const long long groups = (long long)n_tokens / 16 + 2LL * n_seqs + 1;
  if (groups > 0x7fffffffLL || cache->num_kv_heads > 65535) return CRONUS_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  const dim3 grid((unsigned)groups, (unsigned)cache->num_kv_heads);
  auto kp = static_cast<const unsigned char*>(cache->k_cache);
  auto vp = static_cast<const unsigned char*>(cache->v_cache);
  auto kd = static_cast<unsigned char*>(k_dst);
  auto vd = static_cast<unsigned char*>(v_dst);
  if (cache->kv_dtype == CRONUS_KV_FP8_E4M3) {
    hipLaunchKernelGGL(kv_gather_kernel<1>, grid, dim3(256), 0, s, kp, vp, kd, vd, cu_tokens, start_pos,
                       block_tables, max_blocks_per_seq, n_seqs, cache->num_kv_heads, cache->head_dim);
  } else {
    hipLaunchKernelGGL(kv_gather_kernel<2>, grid, dim3(256), 0, s, kp, vp, kd, vd, cu_tokens, start_pos,
                       block_tables, max_blocks_per_seq, n_seqs, cache->num_kv_heads, cache->head_dim);
  }
  return hipGetLastError() == hipSuccess ? CRONUS_OK : CRONUS_ERR_HIP;
}

}  // namespace cronus
