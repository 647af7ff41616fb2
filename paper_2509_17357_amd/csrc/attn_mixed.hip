// Mixed-iteration attention for gfx950 (Cronus section 4.4: one iteration of the
// chunked prefill instance batches a continuation chunk with decodes; Eq. 3 names
// the two attention terms).  One launch runs every work item of the batch:
//   wide item   - a tile of 256 chunk rows (tokens x the q heads of one KV head) against
//                 keys 0 .. its causal limit, or against one span of them when the
//                 planner cut a long tile; K/V blocks are staged through LDS and
//                 shared by the 8 waves, each wave owning 32 rows.  For a bf16 cache
//                 the blocks arrive by global->LDS DMA through a ring of four 64-key
//                 tiles, three tiles ahead; the waves run freely between one s_barrier
//                 per tile, so the two waves of a SIMD fill each other's MFMA and VALU
//                 gaps.  An item may name a second, earlier tile of the same sequence and
//                 KV head, which the work-group computes afterwards (whole prompts with
//                 many tiles per CU: half as many work-group starts).
//                 For an fp8 cache a chunk of few tiles converts the codes on their way
//                 into LDS (through registers, two stages); a chunk of many tiles reads a
//                 bf16 copy of its sequence that kv_stage_kernel makes first, through the
//                 same DMA pipeline as a bf16 cache.
//   narrow item - at most 32 rows (a decode, or a short chunk) against a span of
//                 keys; the 8 waves split the span and stream K/V from the paged pools
//                 through private LDS (bf16: the chunk each lane needs, 16 bytes; fp8:
//                 whole blocks, from which the lanes pick their 8-byte chunks).
// Items that cover a span only leave (O, m, l) partial results, which the merge kernel
// combines.
//
// Both compute S^T = K Q^T and O^T = V^T P^T with v_mfma_f32_32x32x16_bf16, so a
// lane owns one query row (column of S^T): its softmax statistics are lane-local
// except for one exchange with lane^32.  The row order of the K operand is permuted
// (perm32) so that the accumulators a lane holds after S^T are, in order, exactly
// the 8-key chunks the P^T operand needs; the same permutation on the V^T operand
// rows makes each lane own 8 consecutive output dims.
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <cstring>
#include <type_traits>

#include "cronus_internal.h"

// Scratch of cronus_attn_mixed_static (the entry point for callers that cannot allocate): the
// plan image and the partial results of one call.  Each GPU that loads the library holds its
// own copy of this array at its own address until the process ends.  In host code the name
// is only a handle for hipGetSymbolAddress: static_scratch_resolve() below turns it into the
// device address, and every kernel argument is derived from that address, never from the name.
static __device__ __align__(256) unsigned char scratch[cronus::kStaticScratchBytes];

// Heads of the work queues of the main kernel, kQueueSets sets (one per call that can be in
// flight on a device: the plan buffers of the ring, and the static entry point's).  Zero when
// the library's code object is loaded; the last work-group of a launch to finish puts its set
// back to zero, so that no launch has to be preceded by a reset.
static __device__ __align__(256) int queue_sets[cronus::kQueueSets * cronus::kQueueSetInts];

namespace cronus {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr float kLazyLog2 = 8.0f;  // slack of the running reference of the online softmax, in bits
constexpr float kNeg = -1.0e30f;  // initial running maximum: finite, so that differences of maxima stay finite

struct AttnParams {
  const unsigned short* q;
  unsigned short* out;
  const unsigned char* k_pool;
  const unsigned char* v_pool;
  const float* k_scale;
  const float* v_scale;
  const int* block_tables;
  const WorkItem* items;
  const MergeItem* merges;
  float* partials;
  const StageSeq* stage_seqs;   // fp8 cache: sequences with a bf16 copy of their K/V in the workspace
  unsigned char* stage_k;       // the copy: [block][Hkv][16 x D bf16], chunk layout as in the cache
  unsigned char* stage_v;
  int n_stage_seqs;
  int max_blocks;
  int n_q_heads;
  int n_kv_heads;
  float scale_log2e;  // sm_scale * log2(e)
  int* q_heads;       // head of queue x at q_heads[x * kCounterStride], finished work-groups at
                      // q_heads[kQueues * kCounterStride]; all zero when the kernel starts and when it ends
  int q_base[kQueues];
  int q_len[kQueues];
};

// S^T row r of a 32-row MFMA tile holds key perm32(r) of the 32-key sub-tile
// (bits 2 and 3 swapped), see the file comment.
__device__ __forceinline__ int perm32(int r) { return (r & ~12) | ((r & 4) << 1) | ((r & 8) >> 1); }

// Combine a value with the one held by lane^32 (rows of 32 lanes swapped).
__device__ __forceinline__ float pair_max(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float pair_sum(float x) {
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ unsigned int pack_bf16(float a, float b) {
  f32x2 f = {a, b};
  return __builtin_bit_cast(unsigned int, __builtin_convertvector(f, bf16x2));
}

// 8 e4m3 codes -> 8 bf16 (exact).
__device__ __forceinline__ u32x4 fp8x8_to_bf16x8(u32x2 c) {
  u32x4 r;
  f32x2 f;
  f = __builtin_amdgcn_cvt_pk_f32_fp8(c[0], false); r[0] = pack_bf16(f[0], f[1]);
  f = __builtin_amdgcn_cvt_pk_f32_fp8(c[0], true);  r[1] = pack_bf16(f[0], f[1]);
  f = __builtin_amdgcn_cvt_pk_f32_fp8(c[1], false); r[2] = pack_bf16(f[0], f[1]);
  f = __builtin_amdgcn_cvt_pk_f32_fp8(c[1], true);  r[3] = pack_bf16(f[0], f[1]);
  return r;
}

// Zero the elements e of a V chunk (8 consecutive keys kv0+e) whose key is >= kv_len:
// slots past the sequence's length hold arbitrary bits and P = 0 there must give 0.
__device__ __forceinline__ u32x4 zero_tail(u32x4 v, int kv0, int kv_len) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    unsigned int m = 0;
    if (kv0 + 2 * w < kv_len) m |= 0x0000ffffu;
    if (kv0 + 2 * w + 1 < kv_len) m |= 0xffff0000u;
    v[w] &= m;
  }
  return v;
}

template <bool FP8> struct RawChunk { using type = u32x4; };
template <> struct RawChunk<true> { using type = u32x2; };

template <bool FP8>
__device__ __forceinline__ typename RawChunk<FP8>::type load_chunk(const unsigned char* p) {
  return *reinterpret_cast<const typename RawChunk<FP8>::type*>(p);
}
template <bool FP8>
__device__ __forceinline__ u32x4 to_bf16_chunk(typename RawChunk<FP8>::type c) {
  if constexpr (FP8) return fp8x8_to_bf16x8(c); else return c;
}

// Online softmax update of one 32(q) x 32(key) S^T tile held as 16 accumulators per
// lane.  key of accumulator i = sub_base + 16*(i/8) + 8*half + i%8.
// Returns the two P^T operands (keys 0-15 and 16-31 of the sub-tile).
// First part: causal mask, running reference m (rescales O and l when some row's maximum
// outgrew it by more than kLazyLog2 bits).  Second part: numerators, their row sum, and
// the bf16 P^T operands.
template <int NDB, bool FORCE = false>
__device__ __forceinline__ void softmax_max_part(f32x16& s, bool need_mask, int sub_base, int half, int limit,
                                                 float c, float& m, float& l, f32x16 (&o)[NDB]) {
  if (need_mask) {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      const int kv = sub_base + 16 * (i >> 3) + 8 * half + (i & 7);
      s[i] = kv > limit ? -__builtin_inff() : s[i];  // weight becomes exactly 0
    }
  }
  float mx = s[0];
#pragma unroll
  for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s[i]);
  mx = pair_max(mx);
  // The reference m of a row only has to bound its scores loosely: numerators up to
  // 2^kLazyLog2 keep their relative precision in bf16 and their sums stay far from the
  // fp32 range, so O and l are rescaled only when some row's maximum outgrew its
  // reference by more than that (wave-uniform branch; every row then takes its true maximum).
  if (FORCE || __builtin_amdgcn_ballot_w64((mx - m) * c > kLazyLog2) != 0) {
    const float m_new = fmaxf(m, mx);
    const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
    l *= alpha;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
    m = m_new;
  }
}
// Numerators 2^(c (s - m)) as bf16 P^T operands, and this lane's sum of them.  The sum
// adds the ROUNDED numerators (one dot product with (1, 1) per packed pair), so l
// normalises exactly the weights that multiply V.
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float softmax_exp_part(const f32x16& s, float c, float m, u32x4 (&p)[2]) {
  const float mc = m * c;
  const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3f803f80u);
  float sum = 0.f;
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * t + 2 * w], c, -mc));
      const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s[8 * t + 2 * w + 1], c, -mc));
      const f32x2 e = {e0, e1};
      const bf16x2_t pk = __builtin_convertvector(e, bf16x2_t);
      p[t][w] = __builtin_bit_cast(unsigned int, pk);
      sum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, sum, false);
    }
  return sum;
}
template <int NDB>
__device__ __forceinline__ void softmax_tile(f32x16& s, bool need_mask, int sub_base, int half, int limit,
                                             float c, float& m, float& l, f32x16 (&o)[NDB], u32x4 (&p)[2]) {
  softmax_max_part<NDB>(s, need_mask, sub_base, half, limit, c, m, l, o);
  l += softmax_exp_part(s, c, m, p);
}
// A lane's 16 numerators are each at most 2^kLazyLog2 when its reference is fresh enough.
constexpr float kTileSumLimit = 16.0f * 256.0f;
static_assert(kLazyLog2 == 8.0f, "kTileSumLimit = 16 * 2^kLazyLog2");

// Store one lane's share of a finished row: dims 32*db + 16*j + 8*half + 0..7.
template <int NDB>
__device__ __forceinline__ void store_row_bf16(unsigned short* row_ptr, const f32x16 (&o)[NDB], float mul, int half) {
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      u32x4 w;
#pragma unroll
      for (int x = 0; x < 4; ++x) w[x] = pack_bf16(o[db][8 * j + 2 * x] * mul, o[db][8 * j + 2 * x + 1] * mul);
      *reinterpret_cast<u32x4*>(row_ptr + 32 * db + 16 * j + 8 * half) = w;
    }
}

// Leave one lane's share of an unfinished row in a partial-result slot (O[32][D] fp32,
// then m[32] in log2 units, then l[32]): `row` is the row's index inside the slot, lt the
// row sum over both lanes of the row.
template <int NDB, int D>
__device__ __forceinline__ void store_partial_row(float* slot, int row, const f32x16 (&o)[NDB], float m_log2,
                                                  float lt, int half) {
  float* orow = slot + row * D;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      f32x4 lo4 = {o[db][8 * j], o[db][8 * j + 1], o[db][8 * j + 2], o[db][8 * j + 3]};
      f32x4 hi4 = {o[db][8 * j + 4], o[db][8 * j + 5], o[db][8 * j + 6], o[db][8 * j + 7]};
      float* dp = orow + 32 * db + 16 * j + 8 * half;
      *reinterpret_cast<f32x4*>(dp) = lo4;
      *reinterpret_cast<f32x4*>(dp + 4) = hi4;
    }
  if (half == 0) {
    slot[kNarrowRows * D + row] = m_log2;
    slot[kNarrowRows * D + kNarrowRows + row] = lt;
  }
}

// ---------------------------------------- wide (chunk) tile, staged through registers
// Used for the fp8 cache: codes are converted to bf16 once, on their way into LDS.
template <int D, bool FP8, int QT>
__device__ __forceinline__ void run_wide_staged(const AttnParams& p, const WorkItem& it, unsigned char* smem) {
  constexpr int NSTEP = D / 16, NDB = D / 32;
  constexpr int BLK_LDS = 16 * D * 2;           // bytes of one (block, head) as bf16
  constexpr int KT_BYTES = 4 * BLK_LDS;         // K (or V) tile: 64 keys
  constexpr int STAGE = 2 * KT_BYTES;
  constexpr int CH_PER_BLK = 2 * D;             // 8-element chunks per (block, head)
  constexpr int PER = 8 * D / kThreads;         // chunks of K (and of V) each thread stages
  constexpr int ESZ = FP8 ? 1 : 2;
  using Raw = typename RawChunk<FP8>::type;

  const int tid = threadIdx.x;
  const int lane = tid & 63, half = lane >> 5, c32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const SeqInfo si = {it.prefix_len, it.chunk_len, it.q_off, it.n_blocks};
  const int gi_n = it.n_heads;
  const int rows_valid = it.n_tok * gi_n;
  const int row_base = wave * 32 * QT;
  const bool wave_active = row_base < rows_valid;
  const int kv_len = si.prefix_len + si.chunk_len;
  const int pos0 = si.prefix_len + it.q_tok0;   // absolute position of the tile's first token
  const float c = p.scale_log2e * (FP8 ? p.k_scale[it.kv_head] : 1.0f);

  // causal limits of the rows this wave owns (rows past the tile repeat the last row)
  const int wave_min_limit = pos0 + min(row_base, rows_valid - 1) / gi_n;
  const int wave_max_limit = pos0 + min(row_base + 32 * QT - 1, rows_valid - 1) / gi_n;

  bf16x8 qreg[QT][NSTEP];
  int limit[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int r = min(row_base + qt * 32 + c32, rows_valid - 1);
    const int t = r / gi_n, gi = r - t * gi_n;
    limit[qt] = pos0 + t;
    const unsigned short* qp =
        p.q + ((long long)(si.q_off + it.q_tok0 + t) * p.n_q_heads + it.head0 + gi) * D + 8 * half;
#pragma unroll
    for (int s = 0; s < NSTEP; ++s) qreg[qt][s] = as_bf16x8(*reinterpret_cast<const u32x4*>(qp + 16 * s));
  }

  f32x16 o[QT][NDB];
  float m[QT], l[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    m[qt] = kNeg;
    l[qt] = 0.f;
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[qt][db][i] = 0.f;
  }

  const int* bt = p.block_tables + (long long)it.seq * p.max_blocks;
  const long long head_stride = (long long)16 * D * ESZ;  // bytes of one (block, head)
  const int n_tiles = (it.kv_end - it.kv_begin + kWideKvTile - 1) / kWideKvTile;

  Raw rk[PER], rv[PER];
  int bt_next[PER];  // physical blocks of the tile that will be fetched next (looked up one tile early)
  auto lookup_blocks = [&](int tile_base) {
#pragma unroll
    for (int n = 0; n < PER; ++n) {
      const int bidx = (tile_base >> 4) + (tid + kThreads * n) / CH_PER_BLK;
      bt_next[n] = bt[min(bidx, si.n_blocks - 1)];
    }
  };
  auto stage_load = [&](int tile_base) {
#pragma unroll
    for (int n = 0; n < PER; ++n) {
      const int id = tid + kThreads * n;
      const int off = id % CH_PER_BLK;
      const long long base = ((long long)bt_next[n] * p.n_kv_heads + it.kv_head) * head_stride + (long long)off * 8 * ESZ;
      rk[n] = load_chunk<FP8>(p.k_pool + base);
      rv[n] = load_chunk<FP8>(p.v_pool + base);
    }
  };
  auto stage_store = [&](int buf, int tile_base) {
    unsigned char* kb = smem + buf * STAGE;
    unsigned char* vb = kb + KT_BYTES;
    const bool tail = tile_base + kWideKvTile > kv_len;
#pragma unroll
    for (int n = 0; n < PER; ++n) {
      const int id = tid + kThreads * n;
      u32x4 kk = to_bf16_chunk<FP8>(rk[n]);
      u32x4 vv = to_bf16_chunk<FP8>(rv[n]);
      if (tail) {
        const int blk = id / CH_PER_BLK, off = id - blk * CH_PER_BLK;
        vv = zero_tail(vv, tile_base + 16 * blk + 8 * (off / D), kv_len);
      }
      *reinterpret_cast<u32x4*>(kb + id * 16) = kk;
      *reinterpret_cast<u32x4*>(vb + id * 16) = vv;
    }
  };

  const int pr = perm32(c32);
  // byte offset of this lane's K chunk (step 0) inside a 32-key sub-tile, and of its V chunk (db 0)
  const int k_lane_off = (pr >> 4) * BLK_LDS + (half * 16 + (pr & 15)) * 16;
  const int v_lane_off = (half * D + pr) * 16;

  lookup_blocks(it.kv_begin);
  stage_load(it.kv_begin);
  lookup_blocks(it.kv_begin + kWideKvTile);
  int buf = 0;
  for (int j = 0; j < n_tiles; ++j) {
    const int tile_base = it.kv_begin + j * kWideKvTile;
    stage_store(buf, tile_base);
    __syncthreads();
    if (j + 1 < n_tiles) {
      stage_load(tile_base + kWideKvTile);
      lookup_blocks(tile_base + 2 * kWideKvTile);
    }
    if (wave_active && tile_base <= wave_max_limit) {
      const unsigned char* kb = smem + buf * STAGE;
      const unsigned char* vb = kb + KT_BYTES;
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int sub_base = tile_base + 32 * u;
        if (sub_base > wave_max_limit) break;
        const bool need_mask = sub_base + 31 > wave_min_limit;
        f32x16 s[QT];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
#pragma unroll
          for (int i = 0; i < 16; ++i) s[qt][i] = 0.f;
        const unsigned char* ksub = kb + u * 2 * BLK_LDS + k_lane_off;
#pragma unroll
        for (int st = 0; st < NSTEP; ++st) {
          const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(ksub + st * 512));
#pragma unroll
          for (int qt = 0; qt < QT; ++qt)
            s[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qt][st], s[qt], 0, 0, 0);
        }
        u32x4 pp[QT][2];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
          softmax_tile<NDB>(s[qt], need_mask, sub_base, half, limit[qt], c, m[qt], l[qt], o[qt], pp[qt]);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const unsigned char* vsub = vb + (u * 2 + t) * BLK_LDS + v_lane_off;
#pragma unroll
          for (int db = 0; db < NDB; ++db) {
            const bf16x8 a = as_bf16x8(*reinterpret_cast<const u32x4*>(vsub + db * 512));
#pragma unroll
            for (int qt = 0; qt < QT; ++qt)
              o[qt][db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, as_bf16x8(pp[qt][t]), o[qt][db], 0, 0, 0);
          }
        }
      }
    }
    buf ^= 1;
  }

  // epilogue: normalise and store, or leave this span's partial result for the merge
  static_assert(QT == 1, "one partial slot per wavefront");
  const float vmul = FP8 ? p.v_scale[it.kv_head] : 1.0f;
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const int r = row_base + qt * 32 + c32;
    const float lt = pair_sum(l[qt]);
    if (r < rows_valid) {
      if (it.partial >= 0) {
        float* ps = p.partials + (long long)(it.partial + wave) * (kNarrowRows * (D + 2));
        store_partial_row<NDB, D>(ps, c32, o[qt], m[qt] * c, lt, half);
        continue;
      }
      const int t = r / gi_n, gi = r - t * gi_n;
      unsigned short* op = p.out + ((long long)(si.q_off + it.q_tok0 + t) * p.n_q_heads + it.head0 + gi) * D;
      store_row_bf16<NDB>(op, o[qt], vmul / lt, half);
    }
  }
}


// ------------------------------------- wide (chunk) tile, bf16 cache: DMA-fed pipeline
typedef __attribute__((address_space(3))) unsigned char lds_byte;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"i"(N) : "memory");
}

// Copy 1 KiB, global -> LDS, by one wave (lane i moves bytes [16 i, 16 i + 16)): g and dst
// are the wave's bases (no lane term).  Four 4-byte-per-lane instructions measured the same.
__device__ __forceinline__ void dma_1k(const unsigned char* g, lds_byte* dst, int lane) {
  __builtin_amdgcn_global_load_lds(g + lane * 16, dst, 16, 0, 0);
}

// LDS reads of data that arrived by global_load_lds are written as asm, so that the
// waits on those loads are the explicit vmcnt waits of the pipelines and nothing coarser
// (the compiler would wait for every DMA in flight before any LDS read).  The reads and
// the wait for them form ONE asm statement: its outputs are valid when it ends, so no
// register copy the compiler may insert afterwards can see a value that has not arrived.
template <int O0, int O1, int O2, int O3>
__device__ __forceinline__ void lds_read4(u32x4& x0, u32x4& x1, u32x4& x2, u32x4& x3, unsigned addr) {
  asm volatile(
      "ds_read_b128 %0, %4 offset:%5\n\tds_read_b128 %1, %4 offset:%6\n\t"
      "ds_read_b128 %2, %4 offset:%7\n\tds_read_b128 %3, %4 offset:%8\n\ts_waitcnt lgkmcnt(0)"
      : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3)
      : "v"(addr), "i"(O0), "i"(O1), "i"(O2), "i"(O3)
      : "memory");
}
template <int O0, int O1, int O2, int O3, int O4, int O5, int O6, int O7>
__device__ __forceinline__ void lds_read8(u32x4 (&x)[8], unsigned addr) {
  asm volatile(
      "ds_read_b128 %0, %8 offset:%9\n\tds_read_b128 %1, %8 offset:%10\n\t"
      "ds_read_b128 %2, %8 offset:%11\n\tds_read_b128 %3, %8 offset:%12\n\t"
      "ds_read_b128 %4, %8 offset:%13\n\tds_read_b128 %5, %8 offset:%14\n\t"
      "ds_read_b128 %6, %8 offset:%15\n\tds_read_b128 %7, %8 offset:%16\n\ts_waitcnt lgkmcnt(0)"
      : "=&v"(x[0]), "=&v"(x[1]), "=&v"(x[2]), "=&v"(x[3]), "=&v"(x[4]), "=&v"(x[5]), "=&v"(x[6]), "=&v"(x[7])
      : "v"(addr), "i"(O0), "i"(O1), "i"(O2), "i"(O3), "i"(O4), "i"(O5), "i"(O6), "i"(O7)
      : "memory");
}

// Split form for the steady-state loop: a read is issued (`lds_issue1`), independent work
// follows, and a wait lands it.  The waits name the destination registers as in-out
// operands, so every later use of them depends on the wait; N = LDS reads issued after
// these that may still be outstanding (LDS reads return in order).
template <int N>
__device__ __forceinline__ void lds_land(u32x4 (&x)[4]) {
  asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]) : "i"(N) : "memory");
}
template <int N>
__device__ __forceinline__ void lds_land(u32x4 (&x)[8]) {
  asm volatile("s_waitcnt lgkmcnt(%8)"
               : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7])
               : "i"(N)
               : "memory");
}

// One read, and the wait that lands one register: the steady-state loop issues one read
// in front of every MFMA instead of eight in a burst.
template <int OFF>
__device__ __forceinline__ void lds_issue1(u32x4& x, unsigned addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=&v"(x) : "v"(addr), "i"(OFF) : "memory");
}
template <int N>
__device__ __forceinline__ void lds_land1(u32x4& x) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "i"(N) : "memory");
}
template <int I, int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

// Schedule per wave (n = number of 32-key sub-tiles, S(u) = K(u) Q^T, P(u) = softmax
// numerators), software-pipelined by one sub-tile so that the MFMA pipe has the S(u+1)
// products to work on while the VALU computes the softmax of S(u):
//   S(0); for u = 0 .. n-1 { S(u+1) (MFMA) | read V(u) | P(u) = softmax(S(u)) (VALU) |
//                            read K(u+2) | O += V(u)^T P(u) (MFMA) }
// K/V tiles of 64 keys arrive by DMA into a ring of kStages LDS stages, each wave
// fetching 1/8 of a tile; one s_barrier per tile publishes a landed tile and frees the
// stage of the tile before last.  Between barriers the 8 waves run freely, so the two
// waves of a SIMD fill each other's VALU and MFMA gaps.
// COPY: the item's sequence belongs to an fp8 cache and its K/V is read from the bf16 copy
// that kv_stage_kernel made for this launch (blocks it.wide - 2 .. in logical order, no
// table); the scale of K enters the exponent constant, that of V the normalisation.
template <int D, bool COPY>
__device__ __forceinline__ void run_wide_dma(const AttnParams& p, const WorkItem& it, unsigned char* smem) {
  constexpr int NSTEP = D / 16, NDB = D / 32;
  constexpr int BLK_LDS = 16 * D * 2;     // bytes of one (block, head)
  constexpr int KT_BYTES = 4 * BLK_LDS;   // K (or V) tile: 64 keys
  constexpr int STAGE = 2 * KT_BYTES;
  constexpr int kStages = 4, kAhead = kStages - 1;
  constexpr int UPW = D / 64;             // 1-KiB units of K (and of V) each wave fetches per tile
  constexpr int UPB = BLK_LDS / 1024;     // units per block
  constexpr int NI = 2 * UPW;             // DMA instructions per wave per tile

  const int tid = threadIdx.x;
  const int lane = tid & 63, half = lane >> 5, c32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const SeqInfo si = {it.prefix_len, it.chunk_len, it.q_off, it.n_blocks};
  const int gi_n = it.n_heads;
  const int rows_valid = it.n_tok * gi_n;
  const int row_base = wave * 32;
  const bool wave_has_rows = row_base < rows_valid;
  // key positions are counted from the item's first key (a multiple of the tile size)
  const int kv_len = si.prefix_len + si.chunk_len - it.kv_begin;
  const int pos0 = si.prefix_len + it.q_tok0 - it.kv_begin;
  float c = p.scale_log2e, vmul = 1.0f;
  if constexpr (COPY) {
    c *= p.k_scale[it.kv_head];
    vmul = p.v_scale[it.kv_head];
  }
  const unsigned char* const k_src = COPY ? p.stage_k : p.k_pool;
  const unsigned char* const v_src = COPY ? p.stage_v : p.v_pool;
  const int wave_min_limit = pos0 + min(row_base, rows_valid - 1) / gi_n;
  const int wave_max_limit = wave_has_rows ? pos0 + min(row_base + 31, rows_valid - 1) / gi_n : -1;

  const int r = min(row_base + c32, rows_valid - 1);
  const int t_row = r / gi_n, gi_row = r - t_row * gi_n;
  const int limit = pos0 + t_row;
  // Q is requested first and waited for only after the first K/V tiles have been
  // requested too: one memory latency, not two, before the first product
  u32x4 qraw[NSTEP];
  {
    const unsigned short* qp =
        p.q + ((long long)(si.q_off + it.q_tok0 + t_row) * p.n_q_heads + it.head0 + gi_row) * D + 8 * half;
#pragma unroll
    for (int s = 0; s < NSTEP; ++s) qraw[s] = *reinterpret_cast<const u32x4*>(qp + 16 * s);
  }
  f32x16 o[NDB];
  float m = kNeg, l = 0.f;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;

  const int blk0 = it.kv_begin >> 4;
  const int* bt = p.block_tables + (long long)it.seq * p.max_blocks + blk0;
  const int copy_blk0 = it.wide - 2 + blk0;  // COPY: the copy's block of the span's first key
  const long long head_stride = (long long)BLK_LDS;
  const int n_sub = (it.kv_end - it.kv_begin + 31) >> 5;
  const int last_blk = si.n_blocks - 1 - blk0;
  const int pr = perm32(c32);

  // ---- DMA of tile j: this wave moves UPW units of K and of V, all inside one block
  const int blk_w = (wave * UPW) / UPB, part_w = (wave * UPW) % UPB;
  lds_byte* const lds0 = (lds_byte*)smem;
  int bt_reg = 0;  // lane i: physical block of this wave's share of tile (64*k + i)
  auto issue_tile = [&](int j) {
    if ((j & 63) == 0) {
      if constexpr (COPY) bt_reg = copy_blk0 + min(4 * (j + lane) + blk_w, last_blk);
      else bt_reg = bt[min(4 * (j + lane) + blk_w, last_blk)];
      asm volatile("" : "+v"(bt_reg));
    }
    const long long b = __builtin_amdgcn_readlane(bt_reg, j & 63);
    const long long goff = (b * p.n_kv_heads + it.kv_head) * head_stride + part_w * 1024;
    lds_byte* dst = lds0 + (j % kStages) * STAGE + blk_w * BLK_LDS + part_w * 1024;
#pragma unroll
    for (int x = 0; x < UPW; ++x) {
      dma_1k(k_src + goff + x * 1024, dst + x * 1024, lane);
      dma_1k(v_src + goff + x * 1024, dst + KT_BYTES + x * 1024, lane);
    }
  };
  // one of the NI instructions of tile j (q = 2 x + is_v), for spreading a tile's fetch
  // over the two sub-tile steps of a period
  auto issue_part = [&](int j, int q) {
    if (q == 0 && (j & 63) == 0) {
      if constexpr (COPY) bt_reg = copy_blk0 + min(4 * (j + lane) + blk_w, last_blk);
      else bt_reg = bt[min(4 * (j + lane) + blk_w, last_blk)];
      asm volatile("" : "+v"(bt_reg));
    }
    const long long b = __builtin_amdgcn_readlane(bt_reg, j & 63);
    const long long goff = (b * p.n_kv_heads + it.kv_head) * head_stride + part_w * 1024;
    lds_byte* dst = lds0 + (j % kStages) * STAGE + blk_w * BLK_LDS + part_w * 1024;
    const int x = q >> 1;
    if (q & 1) dma_1k(v_src + goff + x * 1024, dst + KT_BYTES + x * 1024, lane);
    else dma_1k(k_src + goff + x * 1024, dst + x * 1024, lane);
  };

  // ---- LDS operand reads (byte addresses)
  const unsigned lds_base = (unsigned)(unsigned long long)lds0;
  const unsigned k_lane = lds_base + (pr >> 4) * BLK_LDS + (half * 16 + (pr & 15)) * 16;
  const unsigned v_lane = lds_base + KT_BYTES + (half * D + pr) * 16;
  u32x4 ka[NSTEP], va[NSTEP];
  auto read_k = [&](int u) {
    const unsigned a = k_lane + ((u >> 1) % kStages) * STAGE + (u & 1) * 2 * BLK_LDS;
    if constexpr (NSTEP == 8) lds_read8<0, 512, 1024, 1536, 2048, 2560, 3072, 3584>(ka, a);
    else lds_read4<0, 512, 1024, 1536>(ka[0], ka[1], ka[2], ka[3], a);
  };
  auto read_v = [&](int u) {
    const unsigned a = v_lane + ((u >> 1) % kStages) * STAGE + (u & 1) * 2 * BLK_LDS;
    if constexpr (NSTEP == 8)
      lds_read8<0, 512, 1024, 1536, BLK_LDS, BLK_LDS + 512, BLK_LDS + 1024, BLK_LDS + 1536>(va, a);
    else lds_read4<0, 512, BLK_LDS, BLK_LDS + 512>(va[0], va[1], va[2], va[3], a);
  };
  auto active = [&](int u) { return 32 * u <= wave_max_limit; };

  u32x4 pp[2];
  bf16x8 qreg[NSTEP];
  auto qk = [&](f32x16& s) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
    for (int st = 0; st < NSTEP; ++st)
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ka[st]), qreg[st], s, 0, 0, 0);
  };

  // ---- prologue: first tiles in flight, tile 0 landed everywhere, S(0), K(1) on its way
#pragma unroll
  for (int j = 0; j < kAhead; ++j) issue_tile(j);
#pragma unroll
  for (int s = 0; s < NSTEP; ++s) {
    asm volatile("" : "+v"(qraw[s]));  // the wait for Q sits here, not inside the pipeline
    qreg[s] = as_bf16x8(qraw[s]);
  }
  wait_vmcnt<NI * (kAhead - 1)>();
  __builtin_amdgcn_s_barrier();
  f32x16 s_even, s_odd;  // S(u) of even / odd sub-tiles
  read_k(0);
  if (active(0)) qk(s_even);
  if (n_sub > 1) read_k(1);

  // one sub-tile: s_cur = S(u) is consumed, s_nxt receives S(u+1)
  auto step = [&](int u, f32x16& s_cur, f32x16& s_nxt, bool opens_tile) {
    const int sub_base = 32 * u;
    const bool act = active(u);
    if (u + 1 < n_sub && active(u + 1)) qk(s_nxt);    // S(u+1): MFMA work that overlaps the softmax below
    if (act) softmax_tile<NDB>(s_cur, sub_base + 31 > wave_min_limit, sub_base, half, limit, c, m, l, o, pp);
    read_v(u);
    if (u + 2 < n_sub) {
      if (opens_tile) {
        // K(u+2) opens tile u/2 + 1: this wave's share of it has landed (the tile after it
        // may still be in flight); the barrier publishes it and tells that every wave is
        // done reading tile u/2 - 1, whose stage the next fetch overwrites
        wait_vmcnt<NI>();
        __builtin_amdgcn_s_barrier();
        issue_tile((u >> 1) + kAhead);
      }
      read_k(u + 2);
    }
    if (act) {
      if (sub_base + 32 > kv_len) {  // slots past the sequence's length hold anything
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int db = 0; db < NDB; ++db)
            va[t * NDB + db] = zero_tail(va[t * NDB + db], sub_base + 16 * t + 8 * half, kv_len);
      }
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va[t * NDB + db]), as_bf16x8(pp[t]), o[db], 0, 0, 0);
    }
  };
  // Steady state: sub-tiles that this wave sees whole (no causal mask, no tail) and that
  // are followed by two more.  No conditionals besides the once-per-tile hand-over.  The
  // instruction order is fixed by hand (a scheduling barrier closes every MFMA slot; the
  // compiler's own interleaving hints left the S(u+1) chain in one clump): each of the
  // NSTEP slots of the first block holds one LDS read of V(u), the MFMA of the S(u+1)
  // chain and the numerators of S(u) that go with it; each slot of the second block one
  // LDS read of K(u+2) and one O product.  An operand is thus requested NSTEP MFMA slots
  // before its use, and LDS sees single reads, not bursts of eight per wave.
  auto tile_sync = [&](int jn) {
    wait_vmcnt<NI>();
    __builtin_amdgcn_s_barrier();
    issue_part(jn, 0);
    issue_part(jn, 1);
  };
  auto fast_step = [&](int u, f32x16& s_cur, f32x16& s_nxt, bool opens_tile) {
    const int jn = (u >> 1) + kAhead;
    const unsigned av = v_lane + ((u >> 1) % kStages) * STAGE + (u & 1) * 2 * BLK_LDS;
    const unsigned ak = k_lane + (((u + 2) >> 1) % kStages) * STAGE + (u & 1) * 2 * BLK_LDS;
    // On entry the NSTEP reads of K(u+1) are in flight or landed and nothing else is.
    // Every MFMA slot issues one read and lands the operand it uses, which was issued
    // NSTEP reads earlier: after the slot's own issue NSTEP + 1 reads can be outstanding,
    // and waiting for all but NSTEP of them lands exactly the oldest.
    // Optimistic numerators: against the reference as it is; the row maxima are looked at
    // only if some lane's sum shows that a score outgrew the reference (or it is the first
    // sub-tile, whose reference is kNeg and whose numerators overflow).
    float tile_sum = 0.f;
    {
      const float mc = m * c;
      const bf16x2_t ones = __builtin_bit_cast(bf16x2_t, 0x3f803f80u);
      constexpr int PPM = 8 / NSTEP;  // numerator pairs per MFMA
#pragma unroll
      for (int i = 0; i < 16; ++i) s_nxt[i] = 0.f;
      __builtin_amdgcn_sched_barrier(0);
      static_for<0, NSTEP>([&](auto I) {
        constexpr int st = decltype(I)::value;
        lds_issue1<(st / NDB) * BLK_LDS + (st % NDB) * 512>(va[st], av);
        lds_land1<NSTEP>(ka[st]);
        s_nxt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(ka[st]), qreg[st], s_nxt, 0, 0, 0);
#pragma unroll
        for (int x = 0; x < PPM; ++x) {
          const int pr = st * PPM + x;
          const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[2 * pr], c, -mc));
          const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[2 * pr + 1], c, -mc));
          const f32x2 e = {e0, e1};
          const bf16x2_t pk = __builtin_convertvector(e, bf16x2_t);
          pp[pr >> 2][pr & 3] = __builtin_bit_cast(unsigned int, pk);
          tile_sum = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, tile_sum, false);
        }
        __builtin_amdgcn_sched_barrier(0);
      });
    }
    if (__builtin_amdgcn_ballot_w64(!(tile_sum <= kTileSumLimit)) != 0) {
      softmax_max_part<NDB, true>(s_cur, false, 32 * u, half, limit, c, m, l, o);
      tile_sum = softmax_exp_part(s_cur, c, m, pp);
    }
    l += tile_sum;
    if (opens_tile) {
      tile_sync(jn);
    } else if constexpr (UPW > 1) {
      issue_part(jn, 2);
      issue_part(jn, 3);
    }
    __builtin_amdgcn_sched_barrier(0);
    static_for<0, NSTEP>([&](auto I) {
      constexpr int i = decltype(I)::value;
      lds_issue1<i * 512>(ka[i], ak);
      lds_land1<NSTEP>(va[i]);
      o[i % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(va[i]), as_bf16x8(pp[i / NDB]), o[i % NDB], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    });
  };
  // sub-tile u is "whole" for this wave when u + 1 is too: 32 (u + 1) + 31 <= wave_min_limit
  int n_fast = wave_has_rows ? min(n_sub - 2, (wave_min_limit + 1) / 32 - 1) : 0;
  n_fast = max(n_fast, 0) & ~1;
  int u = 0;
  for (; u < n_fast; u += 2) {
    fast_step(u, s_even, s_odd, true);
    fast_step(u + 1, s_odd, s_even, false);
  }
  lds_land<0>(ka);  // the steps below expect K(u+1) in registers
  for (; u < n_sub; u += 2) {
    step(u, s_even, s_odd, true);
    if (u + 1 < n_sub) step(u + 1, s_odd, s_even, false);
  }
  wait_vmcnt<0>();  // fetches past the item's last tile are still landing in LDS
  __builtin_amdgcn_s_barrier();

  const float lt = pair_sum(l);
  if (row_base + c32 < rows_valid) {
    if (it.partial >= 0) {
      float* ps = p.partials + (long long)(it.partial + wave) * (kNarrowRows * (D + 2));
      store_partial_row<NDB, D>(ps, c32, o, m * c, lt, half);
    } else {
      unsigned short* op = p.out + ((long long)(si.q_off + it.q_tok0 + t_row) * p.n_q_heads + it.head0 + gi_row) * D;
      store_row_bf16<NDB>(op, o, vmul / lt, half);
    }
  }
}

// --------------------------------------------------------- narrow (decode-like) item
// Operand chunks of 8 bytes picked out of a block image in LDS (fp8 codes).
template <int O0, int O1, int O2, int O3, int O4, int O5, int O6, int O7>
__device__ __forceinline__ void lds_read8_b64(u32x2 (&x)[8], unsigned addr) {
  asm volatile(
      "ds_read_b64 %0, %8 offset:%9\n\tds_read_b64 %1, %8 offset:%10\n\t"
      "ds_read_b64 %2, %8 offset:%11\n\tds_read_b64 %3, %8 offset:%12\n\t"
      "ds_read_b64 %4, %8 offset:%13\n\tds_read_b64 %5, %8 offset:%14\n\t"
      "ds_read_b64 %6, %8 offset:%15\n\tds_read_b64 %7, %8 offset:%16\n\ts_waitcnt lgkmcnt(0)"
      : "=&v"(x[0]), "=&v"(x[1]), "=&v"(x[2]), "=&v"(x[3]), "=&v"(x[4]), "=&v"(x[5]), "=&v"(x[6]), "=&v"(x[7])
      : "v"(addr), "i"(O0), "i"(O1), "i"(O2), "i"(O3), "i"(O4), "i"(O5), "i"(O6), "i"(O7)
      : "memory");
}
template <int O0, int O1, int O2, int O3>
__device__ __forceinline__ void lds_read4_b64(u32x2 (&x)[4], unsigned addr) {
  asm volatile(
      "ds_read_b64 %0, %4 offset:%5\n\tds_read_b64 %1, %4 offset:%6\n\t"
      "ds_read_b64 %2, %4 offset:%7\n\tds_read_b64 %3, %4 offset:%8\n\ts_waitcnt lgkmcnt(0)"
      : "=&v"(x[0]), "=&v"(x[1]), "=&v"(x[2]), "=&v"(x[3])
      : "v"(addr), "i"(O0), "i"(O1), "i"(O2), "i"(O3)
      : "memory");
}

// Read the NOPS 1-KiB operand planes of this lane (plane n at addr + 1024 n).
template <int NOPS>
__device__ __forceinline__ void lds_read_planes(u32x4 (&x)[NOPS], unsigned addr) {
  static_assert(NOPS == 4 || NOPS == 8, "D = 64 or 128");
  if constexpr (NOPS == 8) lds_read8<0, 1024, 2048, 3072, 4096, 5120, 6144, 7168>(x, addr);
  else lds_read4<0, 1024, 2048, 3072>(x[0], x[1], x[2], x[3], addr);
}

template <int D, bool FP8>
__device__ __forceinline__ void run_narrow(const AttnParams& p, const WorkItem& it, unsigned char* smem) {
  constexpr int NSTEP = D / 16, NDB = D / 32;
  constexpr int ESZ = FP8 ? 1 : 2;
  constexpr int NACC = NDB * 16;
  constexpr int WAVE_LDS = 2 * NSTEP * 1024 + (FP8 ? 512 : 0);  // per-wave LDS: K planes then V planes (= NACC * 256); fp8: two sets of block images
  using Raw = typename RawChunk<FP8>::type;

  const int tid = threadIdx.x;
  const int lane = tid & 63, half = lane >> 5, c32 = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const SeqInfo si = {it.prefix_len, it.chunk_len, it.q_off, it.n_blocks};
  const int gi_n = it.n_heads;
  const int rows_valid = it.n_tok * gi_n;  // <= 32
  const int kv_len = si.prefix_len + si.chunk_len;
  const int pos0 = si.prefix_len + it.q_tok0;
  const float c = p.scale_log2e * (FP8 ? p.k_scale[it.kv_head] : 1.0f);
  const int min_limit = pos0;

  const int r = min(c32, rows_valid - 1);
  const int t_row = r / gi_n, gi_row = r - t_row * gi_n;
  const int limit = pos0 + t_row;
  // Q is requested here and waited for after the first block-table entries and K/V
  // chunks have been requested as well (pin_q below): the latencies overlap, and the wait
  // is not left to the streaming loop, where it would be a wait for every load in flight
  bf16x8 qreg[NSTEP];
  u32x4 qraw[NSTEP];
  {
    const unsigned short* qp =
        p.q + ((long long)(si.q_off + it.q_tok0 + t_row) * p.n_q_heads + it.head0 + gi_row) * D + 8 * half;
#pragma unroll
    for (int s = 0; s < NSTEP; ++s) qraw[s] = *reinterpret_cast<const u32x4*>(qp + 16 * s);
  }
  auto pin_q = [&]() {
#pragma unroll
    for (int s = 0; s < NSTEP; ++s) {
      asm volatile("" : "+v"(qraw[s]));
      qreg[s] = as_bf16x8(qraw[s]);
    }
  };

  f32x16 o[NDB];
  float m = kNeg, l = 0.f;
#pragma unroll
  for (int db = 0; db < NDB; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;

  const int* bt = p.block_tables + (long long)it.seq * p.max_blocks;
  const long long head_stride = (long long)16 * D * ESZ;
  const int n_sub = (it.kv_end - it.kv_begin + 31) >> 5;
  const int last_blk = si.n_blocks - 1;
  const int pr = perm32(c32);
  const long long k_lane_off = (long long)(half * 16 + (pr & 15)) * 8 * ESZ;
  const long long v_lane_off = (long long)(half * D + pr) * 8 * ESZ;

  auto compute_s = [&](const u32x4 (&kop)[NSTEP], f32x16& s) {
#pragma unroll
    for (int i = 0; i < 16; ++i) s[i] = 0.f;
#pragma unroll
    for (int st = 0; st < NSTEP; ++st)
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kop[st]), qreg[st], s, 0, 0, 0);
  };
  auto softmax = [&](f32x16& s, u32x4 (&pp)[2], int u) {
    const int sub_base = it.kv_begin + 32 * u;
    softmax_tile<NDB>(s, sub_base + 31 > min_limit, sub_base, half, limit, c, m, l, o, pp);
  };
  auto compute_pv = [&](u32x4 (&vop)[NSTEP], const u32x4 (&pp)[2], int u) {
    const int sub_base = it.kv_begin + 32 * u;
    if (sub_base + 32 > kv_len) {  // last sub-tile of the sequence: slots past its length hold anything
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int db = 0; db < NDB; ++db)
          vop[t * NDB + db] = zero_tail(vop[t * NDB + db], sub_base + 16 * t + 8 * half, kv_len);
    }
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int db = 0; db < NDB; ++db)
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(vop[t * NDB + db]), as_bf16x8(pp[t]), o[db], 0, 0, 0);
  };

  if constexpr (!FP8) {
    // K/V chunks go global -> LDS by DMA, one 16-byte chunk per lane per instruction, into
    // this wave's private planes; each lane later reads back exactly the chunk it fetched,
    // so LDS only serves as storage for loads in flight (no registers are tied up).
    lds_byte* wl = (lds_byte*)smem + wave * WAVE_LDS;
    const unsigned rd_addr = (unsigned)(unsigned long long)wl + lane * 16;  // LDS byte address
    // Block-table entries of this wave's next 32 sub-tiles live in one register (two
    // lanes per sub-tile) and are picked with readlane: a table load inside the loop
    // would have to wait behind every DMA load in flight.
    int bt_reg = 0;
    auto load_table = [&](int j0) {
      const int uu = wave + kWaves * (j0 + (lane >> 1));
      bt_reg = bt[min(((it.kv_begin + 32 * uu) >> 4) + (lane & 1), last_blk)];
      asm volatile("" : "+v"(bt_reg));  // wait for it here, not at each use
    };
    auto issue_k = [&](int j) {
      const long long b0 = __builtin_amdgcn_readlane(bt_reg, 2 * (j & 31));
      const long long b1 = __builtin_amdgcn_readlane(bt_reg, 2 * (j & 31) + 1);
      const unsigned char* g =
          p.k_pool + (((pr >> 4) ? b1 : b0) * p.n_kv_heads + it.kv_head) * head_stride + k_lane_off;
#pragma unroll
      for (int st = 0; st < NSTEP; ++st) __builtin_amdgcn_global_load_lds(g + st * 512, wl + st * 1024, 16, 0, 0);
    };
    auto issue_v = [&](int j) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const long long b = __builtin_amdgcn_readlane(bt_reg, 2 * (j & 31) + t);
        const unsigned char* g = p.v_pool + (b * p.n_kv_heads + it.kv_head) * head_stride + v_lane_off;
#pragma unroll
        for (int db = 0; db < NDB; ++db)
          __builtin_amdgcn_global_load_lds(g + db * 512, wl + (NSTEP + t * NDB + db) * 1024, 16, 0, 0);
      }
    };
    const int n_iter = n_sub > wave ? (n_sub - wave + kWaves - 1) / kWaves : 0;  // sub-tiles wave, wave+4, ...
    if (n_iter > 0) {
      load_table(0);
      issue_k(0);
      issue_v(0);
    }
    pin_q();
    for (int j = 0; j < n_iter; ++j) {
      const int u = wave + kWaves * j;
      const bool has_next = j + 1 < n_iter;
      u32x4 kop[NSTEP], vop[NSTEP], pp[2];
      f32x16 s;
      wait_vmcnt<NSTEP>();  // K(j) landed; the V(j) loads issued after it may still fly
      lds_read_planes<NSTEP>(kop, rd_addr);
      compute_s(kop, s);
      if (has_next) {
        if (((j + 1) & 31) == 0) load_table(j + 1);
        issue_k(j + 1);  // the K planes are free again
      }
      softmax(s, pp, u);
      if (has_next) wait_vmcnt<NSTEP>(); else wait_vmcnt<0>();  // V(j) landed
      lds_read_planes<NSTEP>(vop, rd_addr + NSTEP * 1024);
      compute_pv(vop, pp, u);
      if (has_next) issue_v(j + 1);
    }
  } else {
    // fp8: the two blocks of a sub-tile are copied whole, 16 bytes per lane, into block
    // images in this wave's LDS (K: 2 x 16*D bytes, the second image 128 bytes further so
    // that the two halves of a read hit different banks; V: 2 x 16*D bytes); the operand
    // chunks are picked out of the images with 8-byte reads and converted.  Two sets: the
    // sub-tile after next is requested as soon as a set has been read.
    constexpr int BLKB = 16 * D;                 // bytes of one (block, head) of codes
    constexpr int NIB = BLKB / 1024;             // transfers per block
    constexpr int NIK = 2 * NIB;                 // transfers of K (and of V) per sub-tile
    constexpr int KSET = 2 * BLKB + 128, SET = KSET + 2 * BLKB;
    static_assert(2 * SET <= WAVE_LDS, "two sets per wave");
    lds_byte* wl = (lds_byte*)smem + wave * WAVE_LDS;
    const unsigned wl_addr = (unsigned)(unsigned long long)wl;
    const unsigned k_rd = wl_addr + (pr >> 4) * (BLKB + 128) + (half * 16 + (pr & 15)) * 8;
    const unsigned v_rd = wl_addr + KSET + (half * D + pr) * 8;
    int bt_reg = 0;
    auto load_table = [&](int j0) {
      const int uu = wave + kWaves * (j0 + (lane >> 1));
      bt_reg = bt[min(((it.kv_begin + 32 * uu) >> 4) + (lane & 1), last_blk)];
      asm volatile("" : "+v"(bt_reg));
    };
    auto issue = [&](int j) {
      if ((j & 31) == 0) load_table(j);
      lds_byte* set = wl + (j & 1) * SET;
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) {
        const long long b = __builtin_amdgcn_readlane(bt_reg, 2 * (j & 31) + blk);
        const unsigned char* g = p.k_pool + (b * p.n_kv_heads + it.kv_head) * BLKB + lane * 16;
#pragma unroll
        for (int i = 0; i < NIB; ++i)
          __builtin_amdgcn_global_load_lds(g + i * 1024, set + blk * (BLKB + 128) + i * 1024, 16, 0, 0);
      }
#pragma unroll
      for (int blk = 0; blk < 2; ++blk) {
        const long long b = __builtin_amdgcn_readlane(bt_reg, 2 * (j & 31) + blk);
        const unsigned char* g = p.v_pool + (b * p.n_kv_heads + it.kv_head) * BLKB + lane * 16;
#pragma unroll
        for (int i = 0; i < NIB; ++i)
          __builtin_amdgcn_global_load_lds(g + i * 1024, set + KSET + blk * BLKB + i * 1024, 16, 0, 0);
      }
    };
    auto read_k = [&](u32x4 (&x)[NSTEP], int j) {
      u32x2 r[NSTEP];
      const unsigned a = k_rd + (j & 1) * SET;
      if constexpr (NSTEP == 8) lds_read8_b64<0, 256, 512, 768, 1024, 1280, 1536, 1792>(r, a);
      else lds_read4_b64<0, 256, 512, 768>(r, a);
#pragma unroll
      for (int n = 0; n < NSTEP; ++n) x[n] = fp8x8_to_bf16x8(r[n]);
    };
    auto read_v = [&](u32x4 (&x)[NSTEP], int j) {
      u32x2 r[NSTEP];
      const unsigned a = v_rd + (j & 1) * SET;
      if constexpr (NSTEP == 8) lds_read8_b64<0, 256, 512, 768, BLKB, BLKB + 256, BLKB + 512, BLKB + 768>(r, a);
      else lds_read4_b64<0, 256, BLKB, BLKB + 256>(r, a);
#pragma unroll
      for (int n = 0; n < NSTEP; ++n) x[n] = fp8x8_to_bf16x8(r[n]);
    };
    const int n_iter = n_sub > wave ? (n_sub - wave + kWaves - 1) / kWaves : 0;
    if (n_iter > 0) issue(0);
    if (n_iter > 1) issue(1);
    pin_q();
    for (int j = 0; j < n_iter; ++j) {
      const int u = wave + kWaves * j;
      const bool more = j + 1 < n_iter;  // sub-tile j + 1 has been requested
      u32x4 kop[NSTEP], vop[NSTEP], pp[2];
      f32x16 s;
      if (more) wait_vmcnt<3 * NIK>(); else wait_vmcnt<NIK>();   // K(j) landed
      read_k(kop, j);
      compute_s(kop, s);
      softmax(s, pp, u);
      if (more) wait_vmcnt<2 * NIK>(); else wait_vmcnt<0>();     // V(j) landed
      read_v(vop, j);
      if (j + 2 < n_iter) issue(j + 2);                          // this set is free again
      compute_pv(vop, pp, u);
    }
  }

  // combine the waves (each covered different keys) pairwise, in log2(waves) rounds: a
  // wave that is a source of the coming round parks its accumulators in its own LDS
  // planes (its reads of them are complete), the wave kWaves/2, then /4, ... below it
  // folds them into its own
  float* xo = reinterpret_cast<float*>(smem + wave * WAVE_LDS) + lane;        // [NACC][64]
  float* xs = reinterpret_cast<float*>(smem + kWaves * WAVE_LDS) + lane;      // [kWaves][2][64]
  auto park = [&]() {
#pragma unroll
    for (int db = 0; db < NDB; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) xo[(db * 16 + i) * 64] = o[db][i];
    xs[(wave * 2) * 64] = m;
    xs[(wave * 2 + 1) * 64] = l;
  };
  if (wave >= kWaves / 2) park();
#pragma unroll 1
  for (int n = kWaves / 2; n >= 1; n >>= 1) {
    __syncthreads();
    if (wave < n) {
      const int w2 = wave + n;
      const float* w = reinterpret_cast<const float*>(smem + w2 * WAVE_LDS) + lane;
      const float mo = xs[(w2 * 2) * 64], lo = xs[(w2 * 2 + 1) * 64];
      const float mn = fmaxf(m, mo);
      const float a0 = __builtin_amdgcn_exp2f((m - mn) * c), a1 = __builtin_amdgcn_exp2f((mo - mn) * c);
#pragma unroll
      for (int db = 0; db < NDB; ++db)
#pragma unroll
        for (int i = 0; i < 16; ++i) o[db][i] = o[db][i] * a0 + w[(db * 16 + i) * 64] * a1;
      l = l * a0 + lo * a1;
      m = mn;
      if (2 * wave >= n) park();  // n/2 <= wave < n: a source of the next round
    }
  }
  if (wave == 0) {
    float lt = pair_sum(l);
    if (c32 < rows_valid) {
      if (it.partial < 0) {
        const float vmul = FP8 ? p.v_scale[it.kv_head] : 1.0f;
        unsigned short* op =
            p.out + ((long long)(si.q_off + it.q_tok0 + t_row) * p.n_q_heads + it.head0 + gi_row) * D;
        store_row_bf16<NDB>(op, o, vmul / lt, half);
      } else {
        float* ps = p.partials + (long long)it.partial * (kNarrowRows * (D + 2));
        store_partial_row<NDB, D>(ps, c32, o, m * c, lt, half);  // running maximum in log2 units
      }
    }
  }
}

template <int D, bool FP8>
constexpr int attn_lds_bytes() {
  constexpr int wide_lds = 4 * 2 * 4 * 16 * D * 2;  // stages x (K + V tile of 64 keys)
  constexpr int narrow_lds = kWaves * (2 * (D / 16) * 1024 + (FP8 ? 512 : 0)) + kWaves * 2 * 64 * 4;
  constexpr int lds = wide_lds > narrow_lds ? wide_lds : narrow_lds;
  static_assert(lds + 64 <= 160 * 1024, "LDS budget (the buffers and the 64-byte mailbox of the item loop)");
  return lds;
}

// Index of the next work item for a work-group that runs on XCD `xcc`, or -1 when every
// queue is empty: the own queue first, then the others in ring order (a queue's head only
// grows, so a queue found empty stays empty).
__device__ __forceinline__ int take_item(const AttnParams& p, int xcc) {
  for (int k = 0; k < kQueues; ++k) {
    const int y = (xcc + k) & (kQueues - 1);
    if (p.q_len[y] == 0) continue;
    const int idx = __hip_atomic_fetch_add(p.q_heads + y * kCounterStride, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (idx < p.q_len[y]) return p.q_base[y] + idx;
  }
  return -1;
}

// The work-groups of a launch stay resident, one per CU (the LDS they use allows no second
// one), and work through the queues: the hardware dispatcher hands out work-groups strictly
// in index order and stalls on the first XCD without a free CU, which couples the per-XCD
// orders of a plain one-item-per-work-group launch; a resident work-group asks for its next
// item when it is done with the last, whichever XCD's queue still has one.
template <int D, bool FP8>
__global__ __launch_bounds__(kThreads) void attn_mixed_kernel(AttnParams p) {
  extern __shared__ __align__(16) unsigned char smem[];
  static_assert(kQueues == 8, "XCC_ID is masked to three bits");
  // hardware register XCC_ID (id 20), bits 3:0: the XCD this work-group runs on
  const int xcc = __builtin_amdgcn_s_getreg(20 | (0 << 6) | ((4 - 1) << 11)) & (kQueues - 1);
  int* const mailbox = reinterpret_cast<int*>(smem + attn_lds_bytes<D, FP8>());  // 16 ints behind the kernels' buffers
  for (;;) {
    // wave 0 takes the next item and posts its record; lanes 0-15 fetch one dword each
    if (threadIdx.x < 64) {
      int idx = 0;
      if (threadIdx.x == 0) idx = take_item(p, xcc);
      idx = __builtin_amdgcn_readfirstlane(idx);
      if (threadIdx.x < 16) {
        int v = threadIdx.x == 9 ? -1 : 0;  // field 9 = WorkItem::wide; -1: nothing left
        if (idx >= 0) v = reinterpret_cast<const int*>(p.items + idx)[threadIdx.x];
        mailbox[threadIdx.x] = v;
      }
    }
    __syncthreads();
    WorkItem it;
    {
      int* f = reinterpret_cast<int*>(&it);
#pragma unroll
      for (int i = 0; i < 16; ++i) f[i] = __builtin_amdgcn_readfirstlane(mailbox[i]);
    }
    __syncthreads();  // the mailbox may be rewritten, and the item's LDS buffers reused, from here on
    if (it.wide < 0) break;
    if (it.n_tok <= 0 || it.n_heads <= 0) continue;
    if (it.wide) {
      if constexpr (FP8) {
        if (it.wide >= 2) run_wide_dma<D, true>(p, it, smem);
        else run_wide_staged<D, FP8, 1>(p, it, smem);
      } else {
        run_wide_dma<D, false>(p, it, smem);
      }
    } else {
      run_narrow<D, FP8>(p, it, smem);
    }
    __syncthreads();  // every wave is done with this item's LDS before the next one's fetches land
  }
  // No queue has an item left for this work-group.  The last work-group of the launch to get
  // here (every other one has taken its last ticket) zeroes the heads for the next launch.
  if (threadIdx.x == 0) {
    int* const done = p.q_heads + kQueues * kCounterStride;
    const unsigned finished = __hip_atomic_fetch_add(done, 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
    if (finished == gridDim.x - 1) {
#pragma unroll
      for (int x = 0; x < kQueues; ++x)
        __hip_atomic_store(p.q_heads + x * kCounterStride, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(done, 0, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
}

// fp8 cache: bf16 copy of the K/V blocks of the sequences listed in p.stage_seqs (exact:
// every e4m3 value is a bf16 value), one work-group per block of the copy, all KV heads.
constexpr int kStageThreads = 256;
template <int D>
__global__ __launch_bounds__(kStageThreads) void kv_stage_kernel(AttnParams p) {
  const int b = blockIdx.x;
  // the entry that holds block b: entries are sorted by blk0; lanes test 64 of them at a time
  const int lane = threadIdx.x & 63;
  int e = 0;
  for (int base = 0; base < p.n_stage_seqs; base += 64) {
    const int i = base + lane;
    const bool le = i < p.n_stage_seqs && p.stage_seqs[i].blk0 <= b;
    const int n = __builtin_popcountll(__builtin_amdgcn_ballot_w64(le));
    if (n == 0) break;
    e = base + n - 1;
    if (n < 64) break;
  }
  const StageSeq sq = p.stage_seqs[e];
  const int j = b - sq.blk0;
  if (j < 0 || j >= sq.n_blocks) return;
  const long long phys = p.block_tables[(long long)sq.seq * p.max_blocks + j];
  constexpr int SRC = 16 * D, DST = 32 * D;  // bytes of one (block, head): codes, bf16
  for (int h = 0; h < p.n_kv_heads; ++h) {
    const long long so = (phys * p.n_kv_heads + h) * SRC, dn = ((long long)b * p.n_kv_heads + h) * DST;
    for (int ch = threadIdx.x; ch < SRC / 8; ch += kStageThreads) {
      const u32x2 kc = *reinterpret_cast<const u32x2*>(p.k_pool + so + ch * 8);
      const u32x2 vc = *reinterpret_cast<const u32x2*>(p.v_pool + so + ch * 8);
      *reinterpret_cast<u32x4*>(p.stage_k + dn + ch * 16) = fp8x8_to_bf16x8(kc);
      *reinterpret_cast<u32x4*>(p.stage_v + dn + ch * 16) = fp8x8_to_bf16x8(vc);
    }
  }
}

// Combine the partial results of a row group that was split over key spans:
// out = sum_s O_s 2^(m_s - M) / sum_s l_s 2^(m_s - M), M = max_s m_s (m in log2 units).
// D/4 threads share a row (four dims each); a work-group of 256 threads covers 1024/D rows
// per pass and keeps all passes of the item's (at most 32) rows in flight at once, so the
// loads of a span for every row are issued together: the kernel is bound by memory
// latency (a row's spans are combined in span order, the sums depend on each other).
constexpr int kMergeThreads = 256;
template <int D, bool FP8>
__global__ __launch_bounds__(kMergeThreads) void attn_merge_kernel(AttnParams p) {
  constexpr int TPR = D / 4, RPP = kMergeThreads / TPR, NPASS = kNarrowRows / RPP;
  static_assert(NPASS * RPP == kNarrowRows, "a merge item has at most kNarrowRows rows");
  const MergeItem mi = p.merges[blockIdx.x];
  const int dq = threadIdx.x % TPR;
  const size_t slot = (size_t)kNarrowRows * (D + 2);
  const size_t step = slot * (size_t)mi.stride;
  const float vmul = FP8 ? p.v_scale[mi.kv_head] : 1.0f;
  const float* base = p.partials + (size_t)mi.first_partial * slot;
  // pass k covers rows k * RPP ..; a pass past the item's last row is skipped as a whole
  // (decodes have G rows), inside a pass the rows past the last repeat it (loaded, never stored)
  int row[NPASS];
#pragma unroll
  for (int k = 0; k < NPASS; ++k) row[k] = min((int)threadIdx.x / TPR + k * RPP, mi.n_rows - 1);
  float mt[NPASS];
#pragma unroll
  for (int k = 0; k < NPASS; ++k) mt[k] = kNeg * 4.f;
  for (int s = 0; s < mi.n_split; ++s) {
#pragma unroll
    for (int k = 0; k < NPASS; ++k)
      if (k * RPP < mi.n_rows) mt[k] = fmaxf(mt[k], base[s * step + kNarrowRows * D + row[k]]);
  }
  f32x4 acc[NPASS];
  float ls[NPASS];
#pragma unroll
  for (int k = 0; k < NPASS; ++k) {
    acc[k] = f32x4{0.f, 0.f, 0.f, 0.f};
    ls[k] = 0.f;
  }
  for (int s = 0; s < mi.n_split; ++s) {
    const float* ps = base + s * step;
    float ms[NPASS], lsp[NPASS];
    f32x4 o4[NPASS];
#pragma unroll
    for (int k = 0; k < NPASS; ++k) {
      if (k * RPP < mi.n_rows) {
        ms[k] = ps[kNarrowRows * D + row[k]];
        o4[k] = *reinterpret_cast<const f32x4*>(ps + row[k] * D + 4 * dq);
        lsp[k] = ps[kNarrowRows * D + kNarrowRows + row[k]];
      } else {
        ms[k] = 0.f;
        o4[k] = f32x4{0.f, 0.f, 0.f, 0.f};
        lsp[k] = 0.f;
      }
    }
#pragma unroll
    for (int k = 0; k < NPASS; ++k) {
      const float w = __builtin_amdgcn_exp2f(ms[k] - mt[k]);
      acc[k] += o4[k] * w;
      ls[k] += lsp[k] * w;
    }
  }
#pragma unroll
  for (int k = 0; k < NPASS; ++k) {
    const int r = (int)threadIdx.x / TPR + k * RPP;
    if (r >= mi.n_rows) continue;
    const int tr = mi.row0 + r;
    const int t = tr / mi.n_heads, gi = tr - t * mi.n_heads;
    unsigned short* op = p.out + ((long long)(mi.q_off + mi.q_tok0 + t) * p.n_q_heads + mi.head0 + gi) * D + 4 * dq;
    const float f = vmul / ls[k];
    u32x2 w2 = {pack_bf16(acc[k][0] * f, acc[k][1] * f), pack_bf16(acc[k][2] * f, acc[k][3] * f)};
    *reinterpret_cast<u32x2*>(op) = w2;
  }
}

template <int D, bool FP8>
int prepare_typed() {
  auto kern = attn_mixed_kernel<D, FP8>;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                             attn_lds_bytes<D, FP8>() + 64) == hipSuccess ? CRONUS_OK : CRONUS_ERR_HIP;
}

// Launches of one call, in order: the fp8 copy (if any sequence has one), the main kernel, the
// merge (if any item was split).  prepare_attn_kernels() must have run on this device.  The
// optional events of a.ev become start/stop events of these dispatches themselves, so their
// differences are kernel durations without the launch latency around them.
template <int D, bool FP8>
int launch_typed(const AttnLaunch& a, const AttnParams& p) {
  constexpr int lds = attn_lds_bytes<D, FP8>() + 64;
  hipStream_t s = static_cast<hipStream_t>(a.stream);
  const Plan& pl = *a.plan;
  auto ev = [&](int i) { return static_cast<hipEvent_t>(a.ev[i]); };
  const bool timed = a.ev[0] && a.ev[1];
  if constexpr (FP8) {
    if (pl.n_stage_blocks > 0) {
      if (timed && a.ev[2])
        hipExtLaunchKernelGGL((kv_stage_kernel<D>), dim3((unsigned)pl.n_stage_blocks), dim3(kStageThreads), 0, s, ev(2),
                              nullptr, 0, p);
      else
        hipLaunchKernelGGL((kv_stage_kernel<D>), dim3((unsigned)pl.n_stage_blocks), dim3(kStageThreads), 0, s, p);
      if (hipGetLastError() != hipSuccess) return CRONUS_ERR_HIP;
    }
  }
  if (pl.n_items > 0) {
    auto kern = attn_mixed_kernel<D, FP8>;
    if (timed)
      hipExtLaunchKernelGGL(kern, dim3((unsigned)pl.n_workgroups), dim3(kThreads), lds, s, ev(0), ev(1), 0, p);
    else
      hipLaunchKernelGGL(kern, dim3((unsigned)pl.n_workgroups), dim3(kThreads), lds, s, p);
    if (hipGetLastError() != hipSuccess) return CRONUS_ERR_HIP;
  }
  if (pl.n_merge > 0) {
    if (timed && a.ev[3])
      hipExtLaunchKernelGGL((attn_merge_kernel<D, FP8>), dim3((unsigned)pl.n_merge), dim3(kMergeThreads), 0, s, nullptr,
                            ev(3), 0, p);
    else
      hipLaunchKernelGGL((attn_merge_kernel<D, FP8>), dim3((unsigned)pl.n_merge), dim3(kMergeThreads), 0, s, p);
    if (hipGetLastError() != hipSuccess) return CRONUS_ERR_HIP;
  }
  return CRONUS_OK;
}

// Plan upload of the no-allocation variant: the bytes travel as kernel arguments (copied by
// the runtime at launch, so neither a pinned staging buffer nor a host-to-device copy is
// needed), one work-group stores them.
constexpr int kUploadVecs = 192;  // 3 KiB of payload per launch, inside the 4 KiB argument limit
struct UploadChunk {
  u32x4 v[kUploadVecs];
};
__global__ __launch_bounds__(256) void plan_upload_kernel(UploadChunk c, u32x4* dst, int n_vec) {
  const int i = threadIdx.x;
  if (i < n_vec) dst[i] = c.v[i];
}

}  // namespace

int static_scratch_resolve(void** device_ptr) {
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) {
    (void)hipGetLastError();
    return CRONUS_ERR_HIP;
  }
  *device_ptr = ptr;
  return CRONUS_OK;
}

int queue_sets_resolve(int** device_ptr) {
  void* ptr = nullptr;
  if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(queue_sets)) != hipSuccess || ptr == nullptr) {
    (void)hipGetLastError();
    return CRONUS_ERR_HIP;
  }
  *device_ptr = static_cast<int*>(ptr);
  return CRONUS_OK;
}

int static_scratch_upload(void* dst, const void* host_src, size_t bytes, void* stream) {
  // dst is 256-byte aligned and bytes a multiple of 16 (the plan image is padded to 256)
  const unsigned char* src = static_cast<const unsigned char*>(host_src);
  unsigned char* out = static_cast<unsigned char*>(dst);
  for (size_t off = 0; off < bytes; off += sizeof(UploadChunk)) {
    const size_t n = bytes - off < sizeof(UploadChunk) ? bytes - off : sizeof(UploadChunk);
    UploadChunk c;
    memcpy(&c, src + off, n);
    hipLaunchKernelGGL(plan_upload_kernel, dim3(1), dim3(256), 0, static_cast<hipStream_t>(stream), c,
                       reinterpret_cast<u32x4*>(out + off), (int)((n + 15) / 16));
    if (hipGetLastError() != hipSuccess) return CRONUS_ERR_HIP;
  }
  return CRONUS_OK;
}

int wide_rows_for(int /*head_dim*/, int /*kv_dtype*/) { return kWaves * 32; }

int prepare_attn_kernels() {
  if (int rc = prepare_typed<128, false>()) return rc;
  if (int rc = prepare_typed<128, true>()) return rc;
  if (int rc = prepare_typed<64, false>()) return rc;
  return prepare_typed<64, true>();
}

int launch_attn(const AttnLaunch& a) {
  const cronus_kv_cache& c = *a.cache;
  const Plan& pl = *a.plan;
  unsigned char* ws = static_cast<unsigned char*>(a.workspace);
  AttnParams p;
  p.q = static_cast<const unsigned short*>(a.q);
  p.out = static_cast<unsigned short*>(a.out);
  p.k_pool = static_cast<const unsigned char*>(c.k_cache);
  p.v_pool = static_cast<const unsigned char*>(c.v_cache);
  p.k_scale = c.k_scale;
  p.v_scale = c.v_scale;
  p.block_tables = a.block_tables;
  const unsigned char* image = static_cast<const unsigned char*>(a.plan_image);
  p.items = reinterpret_cast<const WorkItem*>(image + pl.off_items);
  p.merges = reinterpret_cast<const MergeItem*>(image + pl.off_merge);
  p.partials = reinterpret_cast<float*>(ws + pl.off_partials);
  p.q_heads = a.queue_set;
  for (int x = 0; x < kQueues; ++x) {
    p.q_base[x] = pl.q_base[x];
    p.q_len[x] = pl.q_len[x];
  }
  p.stage_seqs = reinterpret_cast<const StageSeq*>(image + pl.off_stage);
  p.stage_k = ws + pl.off_stage_k;
  p.stage_v = ws + pl.off_stage_v;
  p.n_stage_seqs = pl.n_stage_seqs;
  p.max_blocks = a.max_blocks_per_seq;
  p.n_q_heads = c.num_q_heads;
  p.n_kv_heads = c.num_kv_heads;
  p.scale_log2e = a.sm_scale * 1.4426950408889634f;
  const bool fp8 = c.kv_dtype == CRONUS_KV_FP8_E4M3;
  if (c.head_dim == 128) return fp8 ? launch_typed<128, true>(a, p) : launch_typed<128, false>(a, p);
  if (c.head_dim == 64) return fp8 ? launch_typed<64, true>(a, p) : launch_typed<64, false>(a, p);
  return CRONUS_ERR_UNSUPPORTED;
}

}  // namespace cronus
