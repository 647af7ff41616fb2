// Paged scatter of K/V rows (Cronus section 4.2: the transferred prefix is stored in
// the chunked prefill instance's cache instead of being computed; the same scatter
// appends each iteration's new tokens).  Block granularity N_size = 16 (Algorithm 1).
//
// Destination layout (include/cronus.h):
//   K pool [num_blocks][Hkv][D/8][16][8]   chunk = 8 consecutive d of one token
//   V pool [num_blocks][Hkv][2][D][8]      chunk = 8 consecutive tokens of one d
//
// One work-group fills one (cache block, KV head): thread (slot, dc) reads the 8-element
// chunk dc of the row that goes to `slot`.  K chunks are written as they are (16 slots of
// a chunk index are adjacent, so a wave writes 256-byte runs); V is transposed through
// LDS so that whole 8-token chunks are written, 2 KiB contiguous per half block.  Slots
// the call does not address keep their contents: a V chunk with fewer than 8 addressed
// slots is written element by element.
#include <hip/hip_runtime.h>

#include "cronus_internal.h"
#include "paged_rows.h"

namespace cronus {
namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float bf16_bits_to_float(unsigned int b) { return __uint_as_float(b << 16); }

// e4m3_rne(clamp(x / scale, -448, 448)); the division is one IEEE fp32 division.
__device__ __forceinline__ unsigned int quant_e4m3(float x, float scale) {
  float y = x / scale;
  y = fminf(fmaxf(y, -448.0f), 448.0f);
  return (unsigned int)__builtin_amdgcn_cvt_pk_fp8_f32(y, y, 0, false) & 0xffu;
}

// Work-group g of the grid's x dimension serves sequence s = the last one with
// first_group(s) <= g, where first_group(s) = cu_tokens[s] / 16 + 2 s, and within it the
// j-th cache block the rows touch, j = g - first_group(s).  A sequence with n rows
// touches at most n / 16 + 2 blocks, which is what this numbering reserves; work-groups
// past the last touched block have nothing to do.  Host side: grid.x = n_tokens/16 + 2 n_seqs + 1.
template <bool FP8>
__global__ __launch_bounds__(256) void kv_append_kernel(
    const unsigned short* __restrict__ k_src, const unsigned short* __restrict__ v_src,
    void* __restrict__ k_pool, void* __restrict__ v_pool, const float* __restrict__ k_scale,
    const float* __restrict__ v_scale, const int* __restrict__ cu_tokens,
    const int* __restrict__ start_pos, const int* __restrict__ block_tables, int max_blocks,
    int n_seqs, int n_kv_heads, int head_dim) {
  __shared__ unsigned short vt[256][8 + 2];  // [thread = dc*16 + slot][8 d values], padded rows
  const int g = blockIdx.x, head = blockIdx.y;
  const int t = threadIdx.x;
  const int slot = t & 15, dc = t >> 4;
  const int n_dc = head_dim >> 3;

  const SeqRows sr = find_sequence(cu_tokens, start_pos, n_seqs, g);
  const int s = sr.seq, row0 = sr.row0, n_rows = sr.n_rows, start = sr.start;
  const int j = g - ((row0 >> 4) + 2 * s);
  const int bi = (start >> 4) + j;                  // logical block of the sequence
  const int pos_lo = max(start, bi * 16), pos_hi = min(start + n_rows, bi * 16 + 16);  // [lo, hi)
  if (n_rows <= 0 || pos_lo >= pos_hi) return;      // uniform over the work-group
  const int slot_lo = pos_lo & 15, slot_hi = slot_lo + (pos_hi - pos_lo);

  const long long blk = block_tables[(long long)s * max_blocks + bi];
  const long long head_base = (blk * n_kv_heads + head) * (long long)(16 * head_dim);  // elements
  const bool mine = slot >= slot_lo && slot < slot_hi && dc < n_dc;
  u32x4 kk = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
  if (mine) {
    const long long src_off = ((long long)(row0 + (bi * 16 + slot - start)) * n_kv_heads + head) * head_dim + dc * 8;
    kk = *reinterpret_cast<const u32x4*>(k_src + src_off);
    vv = *reinterpret_cast<const u32x4*>(v_src + src_off);
  }
  // ---- K: chunk (dc, slot) of the block
  if (mine) {
    const long long k_off = head_base + ((long long)dc * 16 + slot) * 8;
    if constexpr (!FP8) {
      *reinterpret_cast<u32x4*>(static_cast<unsigned short*>(k_pool) + k_off) = kk;
    } else {
      const float ks = k_scale[head];
      unsigned int c[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const unsigned int w = kk[e >> 1];
        c[e] = quant_e4m3(bf16_bits_to_float((e & 1) ? (w >> 16) : (w & 0xffffu)), ks);
      }
      u32x2 packed;
      packed[0] = c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24);
      packed[1] = c[4] | (c[5] << 8) | (c[6] << 16) | (c[7] << 24);
      *reinterpret_cast<u32x2*>(static_cast<unsigned char*>(k_pool) + k_off) = packed;
    }
  }
  // ---- V: through LDS; thread (dc, kc, jj) then owns the chunk of d = 8 dc + jj, slots 8 kc .. 8 kc + 7
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const unsigned int w = vv[e >> 1];
    vt[t][e] = (unsigned short)((e & 1) ? (w >> 16) : (w & 0xffffu));
  }
  __syncthreads();
  const int kc = slot >> 3, jj = slot & 7;
  if (dc < n_dc) {
    const int c_lo = max(slot_lo, 8 * kc), c_hi = min(slot_hi, 8 * kc + 8);  // addressed slots of this chunk
    if (c_lo < c_hi) {
      unsigned int el[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) el[e] = vt[dc * 16 + 8 * kc + e][jj];
      const int d = dc * 8 + jj;
      const long long v_off = head_base + ((long long)kc * head_dim + d) * 8;
      if constexpr (!FP8) {
        unsigned short* vp = static_cast<unsigned short*>(v_pool) + v_off;
        if (c_hi - c_lo == 8) {
          u32x4 o;
#pragma unroll
          for (int x = 0; x < 4; ++x) o[x] = el[2 * x] | (el[2 * x + 1] << 16);
          *reinterpret_cast<u32x4*>(vp) = o;
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (8 * kc + e >= c_lo && 8 * kc + e < c_hi) vp[e] = (unsigned short)el[e];
        }
      } else {
        const float vs = v_scale[head];
        unsigned int c[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) c[e] = quant_e4m3(bf16_bits_to_float(el[e]), vs);
        unsigned char* vp = static_cast<unsigned char*>(v_pool) + v_off;
        if (c_hi - c_lo == 8) {
          u32x2 packed;
          packed[0] = c[0] | (c[1] << 8) | (c[2] << 16) | (c[3] << 24);
          packed[1] = c[4] | (c[5] << 8) | (c[6] << 16) | (c[7] << 24);
          *reinterpret_cast<u32x2*>(vp) = packed;
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e)
            if (8 * kc + e >= c_lo && 8 * kc + e < c_hi) vp[e] = (unsigned char)c[e];
        }
      }
    }
  }
}

}  // namespace

int launch_kv_append(const cronus_kv_cache* cache, const void* k_src, const void* v_src,
                     const int32_t* cu_tokens, const int32_t* start_pos, const int32_t* block_tables,
                     int32_t max_blocks_per_seq, int32_t n_seqs, int32_t n_tokens, void* stream) {
  const long long groups = (long long)n_tokens / 16 + 2LL * n_seqs + 1;
  if (groups > 0x7fffffffLL || cache->num_kv_heads > 65535) return CRONUS_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  auto ks = static_cast<const unsigned short*>(k_src);
  auto vs = static_cast<const unsigned short*>(v_src);
  const dim3 grid((unsigned)groups, (unsigned)cache->num_kv_heads);
  if (cache->kv_dtype == CRONUS_KV_FP8_E4M3) {
    hipLaunchKernelGGL(kv_append_kernel<true>, grid, dim3(256), 0, s, ks, vs, cache->k_cache, cache->v_cache,
                       cache->k_scale, cache->v_scale, cu_tokens, start_pos, block_tables, max_blocks_per_seq,
                       n_seqs, cache->num_kv_heads, cache->head_dim);
  } else {
    hipLaunchKernelGGL(kv_append_kernel<false>, grid, dim3(256), 0, s, ks, vs, cache->k_cache, cache->v_cache,
                       cache->k_scale, cache->v_scale, cu_tokens, start_pos, block_tables, max_blocks_per_seq,
                       n_seqs, cache->num_kv_heads, cache->head_dim);
  }
  return hipGetLastError() == hipSuccess ? CRONUS_OK : CRONUS_ERR_HIP;
}

}  // namespace cronus
