// Device-side helpers shared by the kernels of libssd (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ssd {

constexpr int WAVE = 64;
constexpr int BLOCK = 256;            // threads per workgroup of every kernel here (4 waves)
constexpr int ATT_CHUNK = 64;         // keys per attention work item; chunk c covers positions [64c, 64c+64)

typedef uint16_t bf16_t;              // raw bf16 bits
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

__device__ __forceinline__ float bf16_to_f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
// Round to nearest even with the gfx950 conversion instruction (two values per instruction).
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
__device__ __forceinline__ uint32_t f2_to_bf16x2(float lo, float hi) {      // bits [15:0] = bf16(lo), [31:16] = bf16(hi)
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2_t{lo, hi}, bf16x2_t));
}
__device__ __forceinline__ bf16_t f_to_bf16(float f) { return (bf16_t)(f2_to_bf16x2(f, 0.f) & 0xFFFFu); }

// Storage types of activations / weights / KV: load as float, store from float.
struct F32 {
  typedef float T;
  static __device__ __forceinline__ float ld(const T* p) { return *p; }
  static __device__ __forceinline__ void st(T* p, float v) { *p = v; }
};
struct BF16 {
  typedef bf16_t T;
  static __device__ __forceinline__ float ld(const T* p) { return bf16_to_f(*p); }
  static __device__ __forceinline__ void st(T* p, float v) { *p = f_to_bf16(v); }
};

// Butterfly reductions over the 64 lanes of a wave: every lane ends with the same value, and the
// association order is fixed, so results do not depend on anything but the inputs.
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}
__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}

// Block-wide (256 threads) reductions through a 4-entry LDS array; all threads get the result.
__device__ __forceinline__ float block_sum(float v, float* s4) {
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) s4[threadIdx.x >> 6] = v;
  __syncthreads();
  return (s4[0] + s4[1]) + (s4[2] + s4[3]);
}
__device__ __forceinline__ float block_max(float v, float* s4) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) s4[threadIdx.x >> 6] = v;
  __syncthreads();
  return fmaxf(fmaxf(s4[0], s4[1]), fmaxf(s4[2], s4[3]));
}

// Philox-4x32-10 (Salmon et al., SC'11).  Counter (slot, seq, step_lo, step_hi), key (seed_lo, seed_hi).
// Returns output word 0; the uniform of a slot is its top 24 bits times 2^-24.
__device__ __forceinline__ uint32_t philox_word0(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                 uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
    const uint32_t hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c0;
}
__device__ __forceinline__ float philox_uniform(uint64_t seed, uint32_t seq, uint64_t step, uint32_t slot) {
  const uint32_t w = philox_word0(slot, seq, (uint32_t)step, (uint32_t)(step >> 32), (uint32_t)seed,
                                  (uint32_t)(seed >> 32));
  return (float)(w >> 8) * 5.9604644775390625e-08f;   // exact: 24-bit integer times 2^-24
}

// ---------------------------------------------------------------------------------------------------
// Device-resident state of a paged KV cache (all pointers into caller-provided device memory).
struct KvView {
  int32_t* len;        // [max_seqs] cached positions
  int32_t* n_pend;     // [max_seqs] pending tokens not yet in the cache (1, or 2 for a draft that owes x_K)
  int32_t* pend;       // [max_seqs][2]
  int32_t* owned;      // [max_seqs] blocks owned
  int32_t* table;      // [max_seqs][mbps] block ids
  int32_t* free_stack; // [n_blocks]
  int32_t* ctl;        // [0] free_top  [1] state error bits (KV_ERR_*)  [2] arrival counter of the accept kernel
                       // [3] number of the next forward launch on this cache (the tag of its hand-over words)
                       // [4],[5] cycle counter of a captured cycle (low, high word of the random counter's step)
  uint32_t* err;       // sticky error word of the persistent forward kernels: DEV_ERR_* bits
  int32_t* mirror;     // host-mapped copy: [max_seqs][2] = (len, n_pend), then [2*max_seqs] = ctl[1], [2*max_seqs+1] = *err
  void* pool;
  int n_blocks, bt, mbps, max_seqs, pcap;
  int n_layers, nkv, hd;
};

constexpr int KV_ERR_POOL = 1;        // the device allocator ran out of blocks
constexpr int KV_ERR_ROLLBACK = 4;    // a rollback asked for more positions than the sequence holds (refused)
constexpr uint32_t DEV_ERR_TIMEOUT = 1u;   // a bounded wait inside a persistent forward gave up
constexpr uint32_t DEV_ERR_TAGS = 2u;      // the launch counter reached its limit: the tagged workspace must be cleared
// Launch numbers tag the hand-over words of the barrier-free forward; the MLP partials carry launch * 128 + layer in
// 32 bits, so launch numbers stay below 2^25.  The host clears the workspace and restarts the numbering before that;
// a forward that still finds the limit reached does nothing and raises DEV_ERR_TAGS.
constexpr uint32_t TAG_LIMIT = (1u << 25) - 1u;

// Element offset of (layer, which(0=K,1=V), block, kv head, token in block, 0) in the pool.  Keys are stored
// [token][dim]; values [dim][token], so for values only tok == 0 (the head's base) is meaningful here.
__device__ __forceinline__ size_t kv_offset(const KvView& kv, int layer, int which, int blk, int head, int tok) {
  return ((((size_t)(layer * 2 + which) * kv.n_blocks + blk) * kv.nkv + head) * kv.bt + tok) * (size_t)kv.hd;
}

// All-reduce over the 16 lanes of a DPP row (lanes 16k .. 16k+15) with data-parallel primitives instead of LDS
// shuffles: pairs, quads (quad_perm), half rows (row_half_mirror), rows (row_mirror).  Every step combines a lane's
// value with the value of a lane of the complementary group, so all 16 lanes end with bit-identical results.
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float row16_sum(float v) {
  v += dpp_f<0xB1>(v);       // quad_perm [1,0,3,2]
  v += dpp_f<0x4E>(v);       // quad_perm [2,3,0,1]
  v += dpp_f<0x141>(v);      // row_half_mirror
  v += dpp_f<0x140>(v);      // row_mirror
  return v;
}
__device__ __forceinline__ float row16_max(float v) {
  v = fmaxf(v, dpp_f<0xB1>(v));
  v = fmaxf(v, dpp_f<0x4E>(v));
  v = fmaxf(v, dpp_f<0x141>(v));
  v = fmaxf(v, dpp_f<0x140>(v));
  return v;
}

// --------------------------------------------------------------------------------------- bf16 / MFMA
// Activations are kept in fp32 and fed to the matrix core as a sum of two bf16 values, x = hi + lo with
// hi = the upper 16 bits of x and lo = bf16(x - hi): two MFMAs per weight fragment instead of one, which
// the weight-streaming regime does not notice, and activation rounding (2^-17 instead of 2^-9 relative)
// stops being the largest error of the bf16 path.  Weights are bf16 as stored.
struct SplitA {
  bf16x8 hi, lo;
};
__device__ __forceinline__ SplitA split_bf16(const u32x4 a, const u32x4 b) {
  const uint32_t x[8] = {a[0], a[1], a[2], a[3], b[0], b[1], b[2], b[3]};
  uint32_t h[4], l[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t u0 = x[2 * i], u1 = x[2 * i + 1];
    const uint32_t h0 = u0 & 0xFFFF0000u, h1 = u1 & 0xFFFF0000u;
    const float r0 = __uint_as_float(u0) - __uint_as_float(h0);       // exact
    const float r1 = __uint_as_float(u1) - __uint_as_float(h1);
    h[i] = (h0 >> 16) | h1;
    l[i] = f2_to_bf16x2(r0, r1);
  }
  SplitA s;
  s.hi = __builtin_bit_cast(bf16x8, u32x4{h[0], h[1], h[2], h[3]});
  s.lo = __builtin_bit_cast(bf16x8, u32x4{l[0], l[1], l[2], l[3]});
  return s;
}

// "Split rows": GEMM operand rows [M][K] kept as the matrix core takes them, for the kernels that serve many rows
// (gemm_rows.h).  Value x of (row, k) is stored as hi = upper 16 bits of x and lo = bf16(x - hi); the fragment of row
// tile mt = row / 16 and k-tile kt = k / 32 is 64 lanes x 8 bf16 with lane = row % 16 + 16 * ((k % 32) / 8), element k % 8:
// 1 KB of hi followed by 1 KB of lo, fragments ordered [mt][kt].  A wave loads a fragment with one contiguous 16-byte
// load per lane.  Index (in bf16 elements) of the hi value; the lo value is 512 elements further.
__device__ __forceinline__ size_t split_index(int row, int k, int KT) {
  return ((size_t)((row >> 4) * KT + (k >> 5)) * 2) * 512 + (size_t)(((row & 15) + 16 * ((k & 31) >> 3)) * 8 + (k & 7));
}
__device__ __forceinline__ void st_split_value(bf16_t* base, int KT, int row, int k, float x) {
  const uint32_t u = __float_as_uint(x), h = u & 0xFFFF0000u;
  const size_t i = split_index(row, k, KT);
  base[i] = (bf16_t)(h >> 16);
  base[i + 512] = f_to_bf16(x - __uint_as_float(h));
}

__device__ __forceinline__ int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Make `seq` own the blocks that cover `tokens` positions (one thread).
__device__ inline void kv_reserve(const KvView& kv, int seq, int tokens) {
  const int need = ceil_div(tokens, kv.bt);
  int own = kv.owned[seq];
  int top = kv.ctl[0];
  while (own < need) {
    if (top <= 0 || own >= kv.mbps) { kv.ctl[1] = 1; break; }
    kv.table[seq * kv.mbps + own] = kv.free_stack[--top];
    ++own;
  }
  kv.owned[seq] = own;
  kv.ctl[0] = top;
}

// Truncate `seq` to new_len positions, returning whole blocks past it, highest table index first (one thread).
__device__ inline void kv_truncate(const KvView& kv, int seq, int new_len) {
  const int keep = ceil_div(new_len, kv.bt);
  int own = kv.owned[seq];
  int top = kv.ctl[0];
  while (own > keep) {
    --own;
    kv.free_stack[top++] = kv.table[seq * kv.mbps + own];
    kv.table[seq * kv.mbps + own] = -1;
  }
  kv.owned[seq] = own;
  kv.ctl[0] = top;
  kv.len[seq] = new_len;
}

__device__ inline void kv_publish_flags(const KvView& kv) {
  kv.mirror[2 * kv.max_seqs] = kv.ctl[1];
  kv.mirror[2 * kv.max_seqs + 1] = (int32_t)*kv.err;
}
__device__ inline void kv_publish(const KvView& kv, int seq) {
  kv.mirror[2 * seq] = kv.len[seq];
  kv.mirror[2 * seq + 1] = kv.n_pend[seq];
  kv_publish_flags(kv);
}
// After a forward: the next launch on this cache gets the next number (one thread, the kernel that follows the forward).
__device__ inline void kv_bump_launch(const KvView& kv) {
  const uint32_t t = (uint32_t)kv.ctl[3] + 1u;
  kv.ctl[3] = (int32_t)t;
}

// Rows of one forward: row m belongs to sequence seq0 + m / R at offset j = m % R.
struct Rows {
  int32_t* pos;      // [M] position of the row
  int32_t* active;   // [M] 1 if the row's key/value is to be written
  int M, R, seq0;
};

}  // namespace ssd
