// Paged scatter of K/V rows (Cronus section 4.2: the transferred prefix is stored in
// the chunked prefill instance's cache instead of being computed; the same scatter
// appends each iteration's new tokens).  Block granularity N_size = 16 (Algorithm 1).
//
// Destination layout (include/cronus.h):
//   K pool [num_blocks][Hkv][D/8][16][8]   chunk = 8 consecutive d of one token
//   V pool [num_blocks][Hkv][2][D][8]      chunk = 8 consecutive tokens of one d
#include <hip/hip_runtime.h>

#include "cronus_internal.h"

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

// One thread moves one 8-element chunk (token, kv head, d/8) of K and of V.
template <bool FP8>
__global__ __launch_bounds__(256) void kv_append_kernel(
    const unsigned short* __restrict__ k_src, const unsigned short* __restrict__ v_src,
    void* __restrict__ k_pool, void* __restrict__ v_pool, const float* __restrict__ k_scale,
    const float* __restrict__ v_scale, const int* __restrict__ cu_tokens,
    const int* __restrict__ start_pos, const int* __restrict__ block_tables, int max_blocks,
    int n_seqs, int n_tokens, int n_kv_heads, int head_dim) {
  const int chunks_per_head = head_dim >> 3;
  const int chunks_per_tok = n_kv_heads * chunks_per_head;
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long tok_ll = idx / chunks_per_tok;
  if (tok_ll >= n_tokens) return;
  const int tok = (int)tok_ll;
  const int rem = (int)(idx - tok_ll * chunks_per_tok);
  const int g = rem / chunks_per_head;
  const int dc = rem - g * chunks_per_head;

  // sequence of this row: the last s with cu_tokens[s] <= tok (skips empty sequences)
  int lo = 0, hi = n_seqs;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (cu_tokens[mid] <= tok) lo = mid; else hi = mid;
  }
  const int pos = start_pos[lo] + (tok - cu_tokens[lo]);
  const long long blk = block_tables[(long long)lo * max_blocks + (pos >> 4)];
  const int slot = pos & 15;

  const long long src_off = ((long long)tok * n_kv_heads + g) * head_dim + dc * 8;
  const u32x4 kk = *reinterpret_cast<const u32x4*>(k_src + src_off);
  const u32x4 vv = *reinterpret_cast<const u32x4*>(v_src + src_off);

  const long long head_base = (blk * n_kv_heads + g) * (long long)(16 * head_dim);  // elements
  const long long k_off = head_base + ((long long)dc * 16 + slot) * 8;
  const long long v_off = head_base + ((long long)(slot >> 3) * head_dim + dc * 8) * 8 + (slot & 7);

  if constexpr (!FP8) {
    *reinterpret_cast<u32x4*>(static_cast<unsigned short*>(k_pool) + k_off) = kk;
    unsigned short* vp = static_cast<unsigned short*>(v_pool) + v_off;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const unsigned int w = vv[e >> 1];
      vp[e * 8] = (unsigned short)((e & 1) ? (w >> 16) : (w & 0xffffu));
    }
  } else {
    const float ks = k_scale[g], vs = v_scale[g];
    unsigned int kc[8], vc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const unsigned int kw = kk[e >> 1], vw = vv[e >> 1];
      kc[e] = quant_e4m3(bf16_bits_to_float((e & 1) ? (kw >> 16) : (kw & 0xffffu)), ks);
      vc[e] = quant_e4m3(bf16_bits_to_float((e & 1) ? (vw >> 16) : (vw & 0xffffu)), vs);
    }
    u32x2 packed;
    packed[0] = kc[0] | (kc[1] << 8) | (kc[2] << 16) | (kc[3] << 24);
    packed[1] = kc[4] | (kc[5] << 8) | (kc[6] << 16) | (kc[7] << 24);
    *reinterpret_cast<u32x2*>(static_cast<unsigned char*>(k_pool) + k_off) = packed;
    unsigned char* vp = static_cast<unsigned char*>(v_pool) + v_off;
#pragma unroll
    for (int e = 0; e < 8; ++e) vp[e * 8] = (unsigned char)vc[e];
  }
}

}  // namespace

int launch_kv_append(const cronus_kv_cache* cache, const void* k_src, const void* v_src,
                     const int32_t* cu_tokens, const int32_t* start_pos, const int32_t* block_tables,
                     int32_t max_blocks_per_seq, int32_t n_seqs, int32_t n_tokens, void* stream) {
  const long long chunks = (long long)n_tokens * cache->num_kv_heads * (cache->head_dim / 8);
  const long long grid = (chunks + 255) / 256;
  if (grid <= 0) return CRONUS_OK;
  if (grid > 0x7fffffffLL) return CRONUS_ERR_INVALID_ARG;
  hipStream_t s = static_cast<hipStream_t>(stream);
  auto ks = static_cast<const unsigned short*>(k_src);
  auto vs = static_cast<const unsigned short*>(v_src);
  if (cache->kv_dtype == CRONUS_KV_FP8_E4M3) {
    hipLaunchKernelGGL(kv_append_kernel<true>, dim3((unsigned)grid), dim3(256), 0, s, ks, vs, cache->k_cache,
                       cache->v_cache, cache->k_scale, cache->v_scale, cu_tokens, start_pos, block_tables,
                       max_blocks_per_seq, n_seqs, n_tokens, cache->num_kv_heads, cache->head_dim);
  } else {
    hipLaunchKernelGGL(kv_append_kernel<false>, dim3((unsigned)grid), dim3(256), 0, s, ks, vs, cache->k_cache,
                       cache->v_cache, cache->k_scale, cache->v_scale, cu_tokens, start_pos, block_tables,
                       max_blocks_per_seq, n_seqs, n_tokens, cache->num_kv_heads, cache->head_dim);
  }
  return hipGetLastError() == hipSuccess ? CRONUS_OK : CRONUS_ERR_HIP;
}

}  // namespace cronus
