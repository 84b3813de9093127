// The decoder forward of one verification (Eq. 4) as one persistent kernel WITHOUT grid barriers between phases.
//
// Phases per layer: QKV (+bias, rotary, cache append) -> attention (parts of 256 keys, then the merge of the parts)
// -> output projection (+residual) -> MLP (gate/up + SwiGLU + down projection fused inside a workgroup) -> sum of the
// MLP partials (+residual).  Weights are packed as matrix-core fragments; a unit of 4 waves takes an item.
//
// Dependent phases are ordered by the data itself: everything a workgroup hands to another workgroup is an 8-byte
// word {payload, tag}, stored with one agent-scope 64-bit store, where tag is the number of this launch.  A consumer
// loads the words it needs with agent-scope 64-bit loads and repeats the loads whose tag is not yet this launch's.
// An aligned 8-byte store is observed whole, so a matching tag proves the payload; no store has to be acknowledged
// before a flag is raised, no counter is shared, and a dependency costs one store plus one load instead of the
// chain of memory round trips of a barrier.  Every word is written exactly once per launch (each layer and phase
// has its own buffers; the MLP partials alternate between two buffers and carry the layer in their tag), and
// launches on one cache workspace are ordered by the stream, so a tag cannot be matched by an older value.
//
// Payloads: a GEMM operand value x is hi | lo << 16 with hi = upper 16 bits of x and lo = bf16(x - hi) (the two
// bf16 whose sum the matrix core consumes); residual rows, sums of squares and partial results are fp32 bits; new
// keys / values are bf16 bits.
//
// A workgroup stages the operand rows it needs in LDS once (all its threads poll in parallel, SB words in flight
// each: the kernel is instantiated for SB = 2, 4, 10, 12 and the host picks the smallest that holds the launch's rows
// in one flight) and feeds the matrix cores from LDS.  The weights of an item are requested at the entry of its phase, into
// registers, before that wait: workgroups arrive at a phase before its operands do, so the wait hides the HBM latency.
// The phases with few items (QKV, attention, output projection) run on workgroups of their own, beyond those that
// take the MLP items, so that no workgroup is late for the MLP, the phase every workgroup waits for.
// Polling costs fabric bandwidth that the producers' stores need: a wave whose first flight fails first watches a
// single word of the PRECEDING phase's operands with long sleeps, and polls in earnest only from then on.
//
// Attention never reads this launch's new keys from the cache pool: the QKV phase stores them in the pool for
// later launches and, tagged, in a side buffer; a wave whose 64-key chunk reaches the new positions patches its
// key / value fragments from that buffer at the same fragment slots the pool would have supplied, so a row's bits
// do not depend on how many rows are verified together.
//
// There is no grid barrier: phase 0 (row bookkeeping, embedding, block reservation) hands over like every other phase.
// All waits are bounded; a timeout raises the error word and every workgroup leaves; the kernel that follows the
// forward then commits nothing and copies the word to the host-mapped mirror, where the next call on the cache finds it.
//
// The launch number is not a kernel argument: it is read from the cache's control words, and the kernel that follows
// every forward on the stream advances it, so a captured graph of launches can be replayed.
#pragma once
#include "persistent.h"

namespace ssd {

typedef unsigned long long u64;
constexpr int DF_B = 12;                  // tagged words a thread keeps in flight while it stages attention operands (and the
                                          // largest choice for the GEMM operands, see SB below)
constexpr int DF_AW = 21504;              // LDS words of the operand staging area (84 KB)
constexpr int DF_ATT_ROWS = 256;          // query rows of a sequence (rows x heads of a group): at most 16 tiles of 16
constexpr int DF_NPF = 5;                 // attention parts merged per flight
constexpr long DF_SPIN_LIMIT = 1L << 18;
// LDS words: staging | sums of squares | unit reduction buffers, overlaid by the attention buffers of the two units
constexpr int DF_SQ_WORDS = 1024;
constexpr int DF_RED_WORDS = 2 * 2048;
constexpr int DF_ATT_UNIT = 4096 + 512 + 512 + 4096 + 4096 + 128;      // Q | new K | new V | P | merge O | merge m,l
constexpr int DF_LDS_WORDS = (DF_AW + DF_SQ_WORDS + DF_RED_WORDS) > 2 * DF_ATT_UNIT ? (DF_AW + DF_SQ_WORDS + DF_RED_WORDS)
                                                                                  : 2 * DF_ATT_UNIT;

// Which single word a wave watches after a failed first flight (see df_wait_hint): the phases with many consumers (QKV,
// MLP) watch a word of their OWN operands, the others a word of the preceding phase's operands.
constexpr int DF_HINT_SLEEP = 2;

struct DArgs {
  int n_layers, d, nq, nkv, ffn, vocab, n_embed;
  float eps, scale;
  const bf16_t* embed;
  const float* final_norm;
  const void* head;
  const float2* rope;
  PLayer layer0;
  size_t layer_stride;
  KvView kv;
  Rows rows;
  int pcap, n_seqs, tok_stride, with_head;
  const int32_t* tokens;
  u64* tw;                // base of the tagged workspace; the members below point into it
  u64* h;                 // [2L+1][PR][d]      fp32: residual stream entering layer l at 2l, after attention at 2l+1
  u64* hg;                // [2L+1][PR][d]      operand: h times the gain of the RMSNorm that consumes it
  u64* sq;                // [2L+1][PR][d/32]   fp32: sums of squares of h over 32 columns
  u64* q;                 // [L][PR][nq*64]     operand: rotated queries
  u64* kvn;               // [L][PR][2][nkv*64] bf16: this launch's keys (rotated) and values
  u64* attn;              // [L][PR][nq*64]     operand: attention output
  u64* att_p;             // [L][PR][nq][NP][16][6] fp32: per part and 4-dim chunk: 4 weighted values, max, sum
  u64* part2;             // [2][ffn/32][PR][d] fp32: down-projection partials of one 32-column slice of the SwiGLU output each,
                          // tagged with launch and layer (buffer = layer parity)
  size_t st_part2;
  u64* rowblk;            // [16] per row: the pool block that takes the row's new key and value (-1: none), from the reservation
  float* logits;
  size_t st_h, st_sq, st_q, st_kvn, st_att_p;   // strides in words
  int NP, n_parts;
  int g_mlp;              // workgroups [0, g_mlp) take the MLP items; the phases with few items start on the workgroups after them
  int small_stride;       // 2: a small-phase item has a workgroup to itself; 1: two items per workgroup
  uint32_t* bar;          // [64] error flag (sticky until the host reads it); [0], [32] belong to the kernel with grid barriers
  unsigned long long* trace;
};

__device__ __forceinline__ u64 ld_word(const u64* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, AG); }
__device__ __forceinline__ void st_word(u64* p, uint32_t payload, uint32_t tag) {
  __hip_atomic_store(p, (u64)payload | ((u64)tag << 32), __ATOMIC_RELAXED, AG);
}
__device__ __forceinline__ void st_wordf(u64* p, float x, uint32_t tag) { st_word(p, __float_as_uint(x), tag); }
__device__ __forceinline__ uint32_t split_payload(float x) {
  const uint32_t u = __float_as_uint(x), h = u & 0xFFFF0000u;
  return (h >> 16) | ((uint32_t)f_to_bf16(x - __uint_as_float(h)) << 16);
}

// A workgroup that arrives at a phase long before its operands would poll them the whole time, and the polls of all
// such workgroups load the fabric that the producers' stores travel through.  After a first failed flight a wave
// therefore watches one word of the operands of the PRECEDING phase (one hand-over earlier) with a single
// address and long sleeps, and resumes the full polling when that word is there.  Purely a hint: bounded, and
// nothing depends on what it saw.
__device__ __forceinline__ void df_wait_hint(const u64* word, uint32_t tag, uint32_t* err) {
  for (int i = 0; i < (1 << 14); ++i) {
    if ((uint32_t)(ld_word(word) >> 32) == tag) return;
    if ((i & 63) == 63 && __hip_atomic_load(err, __ATOMIC_RELAXED, AG) != 0) return;
    __builtin_amdgcn_s_sleep(DF_HINT_SLEEP);
  }
}

// Loads the words base[off[i]] (off == ~0: none) until every tag is this launch's.  False on a timeout.
template <int N>
__device__ __forceinline__ bool poll_words(const u64* base, const uint32_t (&off)[N], uint32_t tag, uint32_t (&out)[N],
                                           uint32_t* err, const u64* hint = nullptr, uint32_t hint_tag = 0u) {
  u64 v[N];
#pragma unroll
  for (int i = 0; i < N; ++i) v[i] = off[i] != 0xFFFFFFFFu ? ld_word(base + off[i]) : ((u64)tag << 32);
  long spins = 0;
  bool ok = true;
  for (;;) {
    bool all = true;
#pragma unroll
    for (int i = 0; i < N; ++i) all = all && ((uint32_t)(v[i] >> 32) == tag);
    if (all) break;
    if (spins == 0 && hint) df_wait_hint(hint, hint_tag, err);
    if (++spins > DF_SPIN_LIMIT || ((spins & 63) == 0 && __hip_atomic_load(err, __ATOMIC_RELAXED, AG) != 0)) {
      __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, AG);
      ok = false;
      break;
    }
    __builtin_amdgcn_s_sleep(1);
#pragma unroll
    for (int i = 0; i < N; ++i)
      if ((uint32_t)(v[i] >> 32) != tag) v[i] = ld_word(base + off[i]);
  }
#pragma unroll
  for (int i = 0; i < N; ++i) out[i] = (uint32_t)v[i];
  return ok;
}

// The 6 words of up to DF_NPF consecutive attention parts (96 words apart) of one 4-dim chunk.
__device__ __forceinline__ bool poll_parts(const u64* base, uint32_t off0, int nparts, uint32_t tag, uint32_t (&out)[DF_NPF * 6],
                                           uint32_t* err) {
  u64 v[DF_NPF * 6];
#pragma unroll
  for (int i = 0; i < DF_NPF * 6; ++i) v[i] = (i / 6 < nparts) ? ld_word(base + off0 + (i / 6) * 96 + i % 6) : ((u64)tag << 32);
  long spins = 0;
  bool ok = true;
  for (;;) {
    bool all = true;
#pragma unroll
    for (int i = 0; i < DF_NPF * 6; ++i) all = all && ((uint32_t)(v[i] >> 32) == tag);
    if (all) break;
    if (++spins > DF_SPIN_LIMIT || ((spins & 63) == 0 && __hip_atomic_load(err, __ATOMIC_RELAXED, AG) != 0)) {
      __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, AG);
      ok = false;
      break;
    }
    __builtin_amdgcn_s_sleep(1);
#pragma unroll
    for (int i = 0; i < DF_NPF * 6; ++i)
      if ((uint32_t)(v[i] >> 32) != tag) v[i] = ld_word(base + off0 + (i / 6) * 96 + i % 6);
  }
#pragma unroll
  for (int i = 0; i < DF_NPF * 6; ++i) out[i] = (uint32_t)v[i];
  return ok;
}

// ------------------------------------------------------------------------------------------------ GEMM phases
struct DPhase {
  const u64* A;           // operand rows [PR][K]
  const u64* sq;          // [PR][K/32] sums of squares of the un-gained rows (nullptr: no RMSNorm)
  const void* W0;
  const void* W1;
  int N, K, gs, items;    // gs: k-splits, always 1 here (the field the shared k-range helper reads)
  int shift, stride;      // item i of round 0 runs on unit (shift + stride * i) % units
  const u64* hint;        // a word of the preceding phase's operands (see df_wait_hint), or null
  uint32_t hint_tag;
  int layer;
  const float* bias;
  const u64* h_in;        // PE_RESID: residual input and outputs
  u64* h_out;
  u64* hg_out;
  u64* sq_out;
  const float* gain_next;
  u64* out;               // PE_QKV: q
  u64* kvn;               // PE_QKV: side buffer of the new keys / values
  float* logits;          // PE_LOGITS
};

// Operand words of rows [0, M) (K words each, the rows contiguous) -> As[row * (K + 4) + k], and the rows' sums of
// squares [M][KT] -> sqs.  Thread gt of gn; the whole group polls in parallel.  Two more words per thread (x0, x1:
// offsets, or ~0) ride in the first flight and come back in xo0, xo1.  Word offsets are recomputed for a repeated
// load instead of being kept in registers; with whole rows a word's offset is its index, and only the padded LDS
// address needs the row (every slot of a flight costs its instructions whether it holds a word or not).
template <int SB>
__device__ __forceinline__ bool stage_operand(const DArgs& a, const u64* A, int K, const u64* sq, int KT,
                                              uint32_t* As, float* sqs, int gt, int gn, uint32_t x0, uint32_t x1,
                                              uint32_t& xo0, uint32_t& xo1, const u64* hint, uint32_t hint_tag,
                                              const uint32_t tag) {
  const int M = a.rows.M, kn = K, nA = M * kn, total = nA + (sq ? M * KT : 0);
  const uint32_t a_off = (uint32_t)(A - a.tw), s_off = sq ? (uint32_t)(sq - a.tw) : 0u;
  const float rkn = 1.0f / (float)kn;
  uint32_t* err = a.bar + 64;
  bool ok = true;
  for (int base = 0; base < total || base == 0; base += gn * SB) {
    int g2 = gt;
    auto off_of = [&](int u) -> uint32_t {
      if (u >= SB) return base == 0 ? (u == SB ? x0 : x1) : 0xFFFFFFFFu;
      const int idx = base + u * gn + g2;
      if (idx < nA) return a_off + (uint32_t)idx;
      return idx < total ? s_off + (uint32_t)(idx - nA) : 0xFFFFFFFFu;
    };
    u64 v[SB + 2];
#pragma unroll
    for (int u = 0; u < SB + 2; ++u) {
      const uint32_t o = off_of(u);
      v[u] = o != 0xFFFFFFFFu ? ld_word(a.tw + o) : ((u64)tag << 32);
    }
    long spins = 0;
    for (;;) {
      bool all = true;
#pragma unroll
      for (int u = 0; u < SB + 2; ++u) all = all && ((uint32_t)(v[u] >> 32) == tag);
      if (all) break;
      if (spins == 0 && hint) df_wait_hint(hint, hint_tag, err);       // far too early: wait cheaply for the phase before
      if (++spins > DF_SPIN_LIMIT || ((spins & 63) == 0 && __hip_atomic_load(err, __ATOMIC_RELAXED, AG) != 0)) {
        __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, AG);
        ok = false;
        break;
      }
      __builtin_amdgcn_s_sleep(1);
      asm volatile("" : "+v"(g2));                       // keeps the offsets out of registers across the wait
#pragma unroll
      for (int u = 0; u < SB + 2; ++u)
        if ((uint32_t)(v[u] >> 32) != tag) v[u] = ld_word(a.tw + off_of(u));
    }
#pragma unroll
    for (int u = 0; u < SB; ++u) {
      const int idx = base + u * gn + gt;
      if (idx < nA) {
        const int row = (int)(((float)idx + 0.5f) * rkn);
        As[idx + 4 * row] = (uint32_t)v[u];
      } else if (idx < total) {
        sqs[idx - nA] = __uint_as_float((uint32_t)v[u]);
      }
    }
    if (base == 0) { xo0 = (uint32_t)v[SB]; xo1 = (uint32_t)v[SB + 1]; }
  }
  return ok;
}

// hi / lo fragments (8 consecutive k each) of a lane from 8 staged payload words
__device__ __forceinline__ void frag_from_lds(const uint32_t* p, u32x4& hi, u32x4& lo) {
  const u32x4 w0 = *(const u32x4*)p, w1 = *(const u32x4*)(p + 4);
  hi = u32x4{__builtin_amdgcn_perm(w0[1], w0[0], 0x05040100u), __builtin_amdgcn_perm(w0[3], w0[2], 0x05040100u),
             __builtin_amdgcn_perm(w1[1], w1[0], 0x05040100u), __builtin_amdgcn_perm(w1[3], w1[2], 0x05040100u)};
  lo = u32x4{__builtin_amdgcn_perm(w0[1], w0[0], 0x07060302u), __builtin_amdgcn_perm(w0[3], w0[2], 0x07060302u),
             __builtin_amdgcn_perm(w1[1], w1[0], 0x07060302u), __builtin_amdgcn_perm(w1[3], w1[2], 0x07060302u)};
}

// Clock samples per workgroup and phase, only in builds with -DSSD_TRACE (see ssd_trace_barriers).
#ifdef SSD_TRACE
#define DF_STAMP(slot) do { if (a.trace && threadIdx.x == 0) a.trace[(size_t)blockIdx.x * 512 + (slot)] = wall_clock64(); } while (0)
#else
#define DF_STAMP(slot) do { } while (0)
#endif

// Item of round 0 that `unit` takes when items start at unit `shift` and take every `stride`-th unit (stride 2: one
// item per workgroup, its other unit idles, so the item's waves have their SIMDs to themselves); a huge number where none.
__device__ __forceinline__ int df_item_of_unit(int unit, int shift, int NU, int stride = 1) {
  int i = unit - shift;
  if (i < 0) i += NU;
  if (stride == 2) return (i & 1) ? 0x3FFFFFFF : (i >> 1);
  return i;
}

// One GEMM phase (QKV, output projection, head); the caller skips it for a workgroup none of whose units has an
// item.  The weight fragments of the unit's item are requested at entry, into registers, before the wait for the
// operands: units arrive well before their operands do, so the weights' HBM latency is hidden by that wait.
// Returns true if the workgroup has to leave (timeout somewhere in the grid).
template <int EPI, int SB>
__device__ __forceinline__ bool df_gemm_phase(const DArgs& a, const uint32_t tag, const DPhase& ph, uint32_t* lds,
                                              const int* srow, int* sdead, int slot) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int usel = wave >> 2, uw = wave & 3, ut = tid & 255;
  const int unit = blockIdx.x * 2 + usel, NU = gridDim.x * 2;
  const int uitem = df_item_of_unit(unit, ph.shift, NU, ph.stride);
  uint32_t* As = lds;
  float* sqs = (float*)(lds + DF_AW);
  float (*red)[2][256] = (float (*)[2][256])((float*)(lds + DF_AW + DF_SQ_WORDS) + usel * 2048);
  const int M = a.rows.M;
  const int KT = ph.K >> 5, ntiles = (ph.N + 15) >> 4;
  const int arow = lane & 15, g = lane >> 4;
  const int row = ut >> 4, col = ut & 15;
  const int rounds = (ph.items + NU - 1) / NU;
  for (int rd = 0; rd < rounds; ++rd) {
    const int item = rd * NU + uitem;
    int t0, t1, split, kb = 0, ke = 0;
    const bool valid = gemm_item<EPI>(ph, item, t0, t1, split);
    if (valid) wave_krange(ph, 0, uw, kb, ke);
    const bool has1 = t1 < ntiles;
    const bool live = valid && row < M;
    const int n0 = t0 * 16 + col, n1 = t1 * 16 + col;
    const u32x4* w0 = (const u32x4*)ph.W0 + (size_t)t0 * KT * 64 + lane;
    const u32x4* w1 = (const u32x4*)ph.W1 + (size_t)(has1 ? t1 : t0) * KT * 64 + lane;
    WPre wl;
    if (valid) {
#pragma unroll
      for (int u = 0; u < PF_K; ++u) {
        const int kt = (kb + u < ke) ? kb + u : kb;
        wl.b0[u] = __builtin_nontemporal_load(w0 + (size_t)kt * 64);
        wl.b1[u] = __builtin_nontemporal_load(w1 + (size_t)kt * 64);
      }
    }
    // ---- operands (both units of the workgroup consume the same rows); the unit that finishes residual rows takes
    //      its residual inputs in the same flight
    uint32_t hx0 = 0xFFFFFFFFu, hx1 = 0xFFFFFFFFu, hv0 = 0u, hv1 = 0u;
    if (EPI == PE_RESID && live) {
      const uint32_t h_off = (uint32_t)(ph.h_in - a.tw) + (uint32_t)(row * ph.N);
      hx0 = h_off + n0;
      hx1 = h_off + n1;
    }
    bool ok = true;
    if (rd == 0) ok = stage_operand<SB>(a, ph.A, ph.K, ph.sq, KT, As, sqs, tid, PBLOCK, hx0, hx1, hv0, hv1, ph.hint, ph.hint_tag, tag);
    if (!ok) *sdead = 1;
    __syncthreads();
    if (*sdead) return true;
    // ---- epilogue operands that do not depend on the product
    float bias0 = 0.f, bias1 = 0.f, gn0 = 0.f, gn1 = 0.f;
    float2 cs = float2{1.f, 0.f};
    int pos = 0, active = 0, rblk = -1;
    if (EPI == PE_QKV && live) {
      if (ph.bias) { bias0 = ph.bias[n0]; bias1 = ph.bias[n0 + 32]; }
      pos = srow[row]; active = srow[16 + row]; rblk = srow[32 + row];
      cs = a.rope[(size_t)pos * 32 + (n0 & 63)];
    }
    if (EPI == PE_RESID && live) { gn0 = ph.gain_next[n0]; gn1 = ph.gain_next[n1]; }
    if (rd == 0) DF_STAMP(slot);
    // ---- products
    f32x4 acc0 = f32x4{0, 0, 0, 0}, acc1 = f32x4{0, 0, 0, 0};
    const uint32_t* arow_p = As + arow * (ph.K + 4) + g * 8;
    if (valid) {
      // all operand fragments first (their LDS latencies overlap), then the products
      u32x4 fh[PF_K], fl[PF_K];
#pragma unroll
      for (int u = 0; u < PF_K; ++u) {
        fh[u] = u32x4{0u, 0u, 0u, 0u};
        fl[u] = fh[u];
        if (kb + u < ke && arow < M) frag_from_lds(arow_p + (kb + u) * 32, fh[u], fl[u]);
      }
#pragma unroll
      for (int u = 0; u < PF_K; ++u)
        if (kb + u < ke) mfma_pair(fh[u], fl[u], wl.b0[u], wl.b1[u], acc0, acc1);
      for (int kt = kb + PF_K; kt < ke; ++kt) {                       // waves with more than PF_K k-tiles
        u32x4 xh = u32x4{0u, 0u, 0u, 0u}, xl = xh;
        if (arow < M) frag_from_lds(arow_p + kt * 32, xh, xl);
        mfma_pair(xh, xl, __builtin_nontemporal_load(w0 + (size_t)kt * 64), __builtin_nontemporal_load(w1 + (size_t)kt * 64),
                  acc0, acc1);
      }
    }
    const int obase = (g * 4) * 16 + (lane & 15);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      red[uw][0][obase + r * 16] = acc0[r];
      red[uw][1][obase + r * 16] = acc1[r];
    }
    float sq = 0.f;
    if (ph.sq && row < M)
      for (int p = col; p < KT; p += 16) sq += sqs[row * KT + p];
    __syncthreads();
    float v0 = (red[0][0][ut] + red[1][0][ut]) + (red[2][0][ut] + red[3][0][ut]);
    float v1 = (red[0][1][ut] + red[1][1][ut]) + (red[2][1][ut] + red[3][1][ut]);
    if (ph.sq) {
      sq = row16_sum(sq);
      const float inv = 1.0f / sqrtf(sq / (float)ph.K + a.eps);
      v0 *= inv;
      v1 *= inv;
    }
    if (EPI == PE_QKV) {
      if (live) {
        const int head = n0 >> 6, dd = n0 & 63;                      // dd < 32
        v0 += bias0; v1 += bias1;
        if (head < a.nq + a.nkv) {
          const float r0 = v0 * cs.x - v1 * cs.y, r1 = v1 * cs.x + v0 * cs.y;
          v0 = r0; v1 = r1;
        }
        if (head < a.nq) {
          u64* qo = ph.out + (size_t)row * (a.nq * 64) + head * 64 + dd;
          st_word(qo, split_payload(v0), tag);
          st_word(qo + 32, split_payload(v1), tag);
        } else {
          const int which = head < a.nq + a.nkv ? 0 : 1;
          const int kvh = head - a.nq - which * a.nkv;
          const bf16_t b0 = f_to_bf16(v0), b1 = f_to_bf16(v1);
          u64* ko = ph.kvn + ((size_t)row * 2 + which) * (a.nkv * 64) + kvh * 64 + dd;
          st_word(ko, b0, tag);
          st_word(ko + 32, b1, tag);
          if (active && rblk >= 0) {
            bf16_t* base = (bf16_t*)a.kv.pool + kv_offset(a.kv, ph.layer, which, rblk, kvh, 0);
            const int tok = pos & 15;
            if (which == 0) { st_ag(base + tok * 64 + dd, b0); st_ag(base + tok * 64 + dd + 32, b1); }
            else { st_ag(base + dd * 16 + tok, b0); st_ag(base + (dd + 32) * 16 + tok, b1); }
          }
        }
      }
    } else if (EPI == PE_LOGITS) {
      if (live) {
        if (n0 < ph.N) ph.logits[(size_t)row * ph.N + n0] = v0;
        if (has1 && n1 < ph.N) ph.logits[(size_t)row * ph.N + n1] = v1;
      }
    } else {  // PE_RESID: N == d (a multiple of 32): residual, and the operand / statistics of the next RMSNorm
      if (valid) {
        const int pair = t0 >> 1;
        float q2 = 0.f;
        if (row < M) {
          v0 += __uint_as_float(hv0);
          v1 += __uint_as_float(hv1);
          st_wordf(ph.h_out + (size_t)row * ph.N + n0, v0, tag);
          st_wordf(ph.h_out + (size_t)row * ph.N + n1, v1, tag);
          st_word(ph.hg_out + (size_t)row * ph.N + n0, split_payload(v0 * gn0), tag);
          st_word(ph.hg_out + (size_t)row * ph.N + n1, split_payload(v1 * gn1), tag);
          q2 = v0 * v0 + v1 * v1;
        }
        q2 = row16_sum(q2);
        if (col == 0 && row < M) st_wordf(ph.sq_out + (size_t)row * (ph.N >> 5) + pair, q2, tag);
      }
    }
    if (rd == 0) DF_STAMP(slot + 1);
    __syncthreads();
  }
  return false;
}

// ------------------------------------------------------------------------------------------------ fused MLP
// Gate/up + SwiGLU + down projection inside one workgroup: its two units produce 32 consecutive columns of the
// SwiGLU output, which is exactly one k-tile of the down projection; the workgroup multiplies it with that k-tile of
// every output tile (8 waves x DF_DN tiles) and publishes a partial of the whole row.  The SwiGLU output never
// leaves the workgroup, and one dependency per layer disappears; the price is ffn/32 partials per output.
constexpr int DF_DN = 7;                  // down-projection output tiles a wave keeps prefetched
struct WDown { u32x4 b[DF_DN]; };

__device__ __forceinline__ uint32_t df_tag2(const uint32_t tag, int layer) { return tag * 128u + (uint32_t)layer; }

// Fragments (n-tile wave + 8 i, k-tile kt2) of the down projection for i < DF_DN; exactly DF_DN loads.
__device__ __forceinline__ void df_prefetch_down(const DArgs& a, const void* wdown, int kt2, WDown& wd) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int ntiles = a.d >> 4, KTd = a.ffn >> 5;
#pragma unroll
  for (int i = 0; i < DF_DN; ++i) {
    const int nt = (wave + 8 * i < ntiles) ? wave + 8 * i : wave;
    wd.b[i] = __builtin_nontemporal_load((const u32x4*)wdown + ((size_t)nt * KTd + kt2) * 64 + lane);
  }
}

template <int SB>
__device__ __forceinline__ bool df_mlp_phase(const DArgs& a, const uint32_t tag, const DPhase& ph, const void* wdown, u64* part2, uint32_t tag2,
                                             uint32_t* lds, uint32_t* sact, int* sdead, int slot) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int usel = wave >> 2, uw = wave & 3, ut = tid & 255;
  const int unit = blockIdx.x * 2 + usel, NU = a.g_mlp * 2;
  uint32_t* As = lds;
  float* sqs = (float*)(lds + DF_AW);
  float (*red)[2][256] = (float (*)[2][256])((float*)(lds + DF_AW + DF_SQ_WORDS) + usel * 2048);
  const int M = a.rows.M, PR = (int)(a.st_h / a.d);
  const int KT = ph.K >> 5, ntiles_d = a.d >> 4, KTd = a.ffn >> 5;
  const int arow = lane & 15, g = lane >> 4, c16 = lane & 15;
  const int row = ut >> 4, col = ut & 15;
  const int rounds = (ph.items + NU - 1) / NU;
  for (int rd = 0; rd < rounds; ++rd) {
    const int item = rd * NU + unit;
    const bool valid = item < ph.items;
    const int kt2 = item >> 1;                          // the workgroup's k-tile of the down projection
    int kb = 0, ke = 0;
    if (valid) wave_krange(ph, 0, uw, kb, ke);
    const bool live = valid && row < M;
    const int n0 = item * 16 + col;
    // the weights of the unit's item and the workgroup's down-projection tiles: requested at entry, they arrive
    // while the workgroup waits for its operands
    WPre pre;
    WDown wd;
    if (valid) {
      const u32x4* w0 = (const u32x4*)ph.W0 + (size_t)item * KT * 64 + lane;
      const u32x4* w1 = (const u32x4*)ph.W1 + (size_t)item * KT * 64 + lane;
#pragma unroll
      for (int u = 0; u < PF_K; ++u) {
        const int kt = (kb + u < ke) ? kb + u : kb;
        pre.b0[u] = __builtin_nontemporal_load(w0 + (size_t)kt * 64);
        pre.b1[u] = __builtin_nontemporal_load(w1 + (size_t)kt * 64);
      }
    }
    if ((rd * NU + blockIdx.x * 2) < ph.items) df_prefetch_down(a, wdown, kt2, wd);
    uint32_t dummy0, dummy1;
    bool ok = true;
    if (rd == 0) ok = stage_operand<SB>(a, ph.A, ph.K, ph.sq, KT, As, sqs, tid, PBLOCK, 0xFFFFFFFFu, 0xFFFFFFFFu, dummy0, dummy1, ph.hint, ph.hint_tag, tag);
    if (!ok) *sdead = 1;
    __syncthreads();
    if (*sdead) return true;
    if (rd == 0) DF_STAMP(slot);
    f32x4 acc0 = f32x4{0, 0, 0, 0}, acc1 = f32x4{0, 0, 0, 0};
    const uint32_t* arow_p = As + arow * (ph.K + 4) + g * 8;
    if (valid) {
      const u32x4* w0 = (const u32x4*)ph.W0 + (size_t)item * KT * 64 + lane;
      const u32x4* w1 = (const u32x4*)ph.W1 + (size_t)item * KT * 64 + lane;
      // all operand fragments first (their LDS latencies overlap), then the products
      u32x4 fh[PF_K], fl[PF_K];
#pragma unroll
      for (int u = 0; u < PF_K; ++u) {
        fh[u] = u32x4{0u, 0u, 0u, 0u};
        fl[u] = fh[u];
        if (kb + u < ke && arow < M) frag_from_lds(arow_p + (kb + u) * 32, fh[u], fl[u]);
      }
#pragma unroll
      for (int u = 0; u < PF_K; ++u)
        if (kb + u < ke) mfma_pair(fh[u], fl[u], pre.b0[u], pre.b1[u], acc0, acc1);
      for (int kt = kb + PF_K; kt < ke; ++kt) {
        u32x4 xh = u32x4{0u, 0u, 0u, 0u}, xl = xh;
        if (arow < M) frag_from_lds(arow_p + kt * 32, xh, xl);
        mfma_pair(xh, xl, __builtin_nontemporal_load(w0 + (size_t)kt * 64), __builtin_nontemporal_load(w1 + (size_t)kt * 64),
                  acc0, acc1);
      }
    }
    const int obase = (g * 4) * 16 + (lane & 15);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      red[uw][0][obase + r * 16] = acc0[r];
      red[uw][1][obase + r * 16] = acc1[r];
    }
    float sq = 0.f;
    if (row < M)
      for (int p = col; p < KT; p += 16) sq += sqs[row * KT + p];
    __syncthreads();
    float v0 = (red[0][0][ut] + red[1][0][ut]) + (red[2][0][ut] + red[3][0][ut]);
    float v1 = (red[0][1][ut] + red[1][1][ut]) + (red[2][1][ut] + red[3][1][ut]);
    sq = row16_sum(sq);
    const float inv = 1.0f / sqrtf(sq / (float)ph.K + a.eps);
    v0 *= inv;
    v1 *= inv;
    const float actv = (live && n0 < ph.N) ? v0 / (1.0f + expf(-v0)) * v1 : 0.f;
    sact[row * 36 + usel * 16 + col] = split_payload(actv);          // [16 rows][32 columns of the workgroup's k-tile]
    __syncthreads();
    // ---- down projection of the workgroup's 32 columns: wave takes output tiles wave, wave + 8, ...
    if ((rd * NU + blockIdx.x * 2) < ph.items) {
      u32x4 xh = u32x4{0u, 0u, 0u, 0u}, xl = xh;
      if (arow < M) frag_from_lds(sact + arow * 36 + g * 8, xh, xl);
      const bf16x8 ah = __builtin_bit_cast(bf16x8, xh), al = __builtin_bit_cast(bf16x8, xl);
      u64* po = part2 + ((size_t)kt2 * PR) * a.d;
#pragma unroll
      for (int i = 0; i < DF_DN; ++i) {
        const int nt = wave + 8 * i;
        if (nt < ntiles_d) {
          const bf16x8 bv = __builtin_bit_cast(bf16x8, wd.b[i]);
          f32x4 acc = f32x4{0, 0, 0, 0};
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, bv, acc, 0, 0, 0);
          acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bv, acc, 0, 0, 0);
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (4 * g + r < M) st_wordf(po + (size_t)(4 * g + r) * a.d + nt * 16 + c16, acc[r], tag2);
        }
      }
      for (int nt = wave + 8 * DF_DN; nt < ntiles_d; nt += 8) {      // wider models: the remaining tiles, not prefetched
        const bf16x8 bv = __builtin_bit_cast(bf16x8, __builtin_nontemporal_load((const u32x4*)wdown + ((size_t)nt * KTd + kt2) * 64 + lane));
        f32x4 acc = f32x4{0, 0, 0, 0};
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, bv, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bv, acc, 0, 0, 0);
#pragma unroll
        for (int r = 0; r < 4; ++r)
          if (4 * g + r < M) st_wordf(po + (size_t)(4 * g + r) * a.d + nt * 16 + c16, acc[r], tag2);
      }
    }
    if (rd == 0) DF_STAMP(slot + 1);
    __syncthreads();
  }
  return false;
}

// Sum of the ffn/32 down-projection partials in ascending order, residual, and the operand / statistics of the next
// RMSNorm.  Task = (row, 32 output columns) on a whole workgroup; thread (column c, group g of 16) sums the partials of
// its group, the groups meet in LDS in ascending order.  (With a task per 4-wave unit and 8 groups a thread had 19
// words in flight and two tasks polled through one CU: 30 us more per five-row forward.)
constexpr int DF_RG = 16;                 // groups of partials per task: 512 threads = 32 columns x 16 groups
constexpr int DF_RW = 10;                 // partials a thread keeps in flight
__device__ __forceinline__ bool df_reduce_phase(const DArgs& a, const uint32_t tag, int layer, const u64* part2, uint32_t tag2, const u64* h_in,
                                                u64* h_out, u64* hg_out, u64* sq_out, const float* gain_next, int shift,
                                                uint32_t* lds, int* sdead, int slot) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int NW = gridDim.x;
  const int M = a.rows.M, d = a.d, np = d >> 5, nW = a.ffn >> 5, PR = (int)(a.st_h / a.d);
  const int tasks = M * np, rounds = (tasks + NW - 1) / NW;
  const int witem = df_item_of_unit(blockIdx.x, shift >> 1, NW);     // a task has the whole workgroup
  float* rs = (float*)(lds + DF_AW + DF_SQ_WORDS);                     // [16 groups][32]
  const int c = tid & 31, grp = tid >> 5;
  const int per = (nW + DF_RG - 1) / DF_RG;
  uint32_t* err = a.bar + 64;
  bool bad = false;
  for (int rd = 0; rd < rounds; ++rd) {
    const int task = rd * NW + witem;
    const bool valid = task < tasks;
    const int m = valid ? task / np : 0, p = valid ? task - m * np : 0;
    const int w0 = grp * per, cnt = valid ? max(0, min(per, nW - w0)) : 0;
    const u64* src = part2 + ((size_t)w0 * PR + m) * d + 32 * p + c;
    const size_t wstride = (size_t)PR * d;
    float sum = 0.f;
    u64 hw = (u64)tag << 32;
    const bool want_h = valid && grp == 0;
    for (int b0 = 0; b0 < cnt || (b0 == 0 && want_h); b0 += DF_RW) {
      u64 v[DF_RW];
#pragma unroll
      for (int i = 0; i < DF_RW; ++i) v[i] = (b0 + i < cnt) ? ld_word(src + (size_t)(b0 + i) * wstride) : ((u64)tag2 << 32);
      if (b0 == 0 && want_h) hw = ld_word(h_in + (size_t)m * d + 32 * p + c);
      long spins = 0;
      for (;;) {
        bool all = (uint32_t)(hw >> 32) == tag;
#pragma unroll
        for (int i = 0; i < DF_RW; ++i) all = all && ((uint32_t)(v[i] >> 32) == tag2);
        if (all) break;
        // a workgroup that comes here from its own MLP item is not early: no hint for it
        if (spins == 0 && (int)blockIdx.x >= a.g_mlp) df_wait_hint(a.hg + (size_t)(2 * layer + 1) * a.st_h, tag, err);
        if (++spins > DF_SPIN_LIMIT || ((spins & 63) == 0 && __hip_atomic_load(err, __ATOMIC_RELAXED, AG) != 0)) {
          __hip_atomic_store(err, 1u, __ATOMIC_RELAXED, AG);
          bad = true;
          break;
        }
        __builtin_amdgcn_s_sleep(1);
#pragma unroll
        for (int i = 0; i < DF_RW; ++i)
          if ((uint32_t)(v[i] >> 32) != tag2) v[i] = ld_word(src + (size_t)(b0 + i) * wstride);
        if ((uint32_t)(hw >> 32) != tag) hw = ld_word(h_in + (size_t)m * d + 32 * p + c);
      }
#pragma unroll
      for (int i = 0; i < DF_RW; ++i)
        if (b0 + i < cnt) sum += __uint_as_float((uint32_t)v[i]);
    }
    rs[grp * 32 + c] = sum;
    if (bad) *sdead = 1;
    __syncthreads();
    if (*sdead) return true;
    if (rd == 0) DF_STAMP(slot);
    if (valid && tid < 32) {
      float v = rs[c];
#pragma unroll
      for (int gq = 1; gq < DF_RG; ++gq) v += rs[gq * 32 + c];
      v += __uint_as_float((uint32_t)hw);
      const size_t o = (size_t)m * d + 32 * p + c;
      st_wordf(h_out + o, v, tag);
      st_word(hg_out + o, split_payload(v * gain_next[32 * p + c]), tag);
      float q2 = v * v;
#pragma unroll
      for (int off = 16; off > 0; off >>= 1) q2 += __shfl_xor(q2, off, 32);
      if (c == 0) st_wordf(sq_out + (size_t)m * np + p, q2, tag);
    }
    if (rd == 0) DF_STAMP(slot + 1);
    __syncthreads();
  }
  return false;
}

// ------------------------------------------------------------------------------------------------ phase 0
// Rows and embedding.  Item = row.
__device__ __forceinline__ void df_embed_phase(const DArgs& a, const uint32_t tag) {
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), usel = wave >> 2, ut = tid & 255;
  const int unit = blockIdx.x * 2 + usel, NU = gridDim.x * 2;
  const int M = a.rows.M, R = a.rows.R, d = a.d;
  for (int m = unit; m < M; m += NU) {
    const int brel = m / R, j = m - brel * R;
    const int seq = a.rows.seq0 + brel;
    // every candidate is requested at once: which of them is the row's token follows from the pending count
    const int npend = a.pcap ? ld_state(a.kv.n_pend + seq) : 0;
    const int len = ld_state(a.kv.len + seq);
    const int p0 = a.pcap ? ld_state(a.kv.pend + seq * 2) : 0;
    const int p1 = a.pcap > 1 ? ld_state(a.kv.pend + seq * 2 + 1) : 0;
    const int tx = j >= a.pcap ? ld_state(a.tokens + (size_t)brel * a.tok_stride + (j - a.pcap)) : 0;
    const int off = a.pcap - npend;
    int tok, pos, active;
    if (j < off) { tok = p0; pos = len; active = 0; }
    else {
      pos = len + (j - off); active = 1;
      tok = j < a.pcap ? ((j - off) ? p1 : p0) : tx;
    }
    tok = min(max(tok, 0), a.n_embed - 1);
    if (ut == 0) { st_ag(a.rows.pos + m, pos); st_ag(a.rows.active + m, active); }
    const bf16_t* src = a.embed + (size_t)tok * d;
    const float* gain = a.layer0.ln1;
    for (int p = ut >> 5; p < (d >> 5); p += 8) {
      const int c = p * 32 + (ut & 31);
      const float v = bf16_to_f(src[c]);
      st_wordf(a.h + (size_t)m * d + c, v, tag);
      st_word(a.hg + (size_t)m * d + c, split_payload(v * gain[c]), tag);
      float sq = v * v;
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) sq += __shfl_xor(sq, o, WAVE);
      if ((ut & 31) == 0) st_wordf(a.sq + (size_t)m * (d >> 5) + p, sq, tag);
    }
  }
}

// Block reservation for the rows of this launch: lane b of the first wave of workgroup 0 takes sequence b (at most
// 16 sequences).  Two memory round trips for all of them: the state words, then the ids (free-stack entries for new
// blocks, table entries for blocks already owned).  Sequences take from the free stack in ascending order, top first,
// as a serial walk over the sequences would.  Nothing waits for the table itself: the block that holds a row's new
// key goes out as a tagged word per row (the workgroups with QKV items, whose epilogue appends the keys and values,
// wait for it once), and attention never reads a position of this launch from the pool.  The launch therefore has no
// grid barrier.
__device__ __forceinline__ bool df_tag_ok(uint32_t tag) { return tag != 0u && tag < TAG_LIMIT; }

__device__ __forceinline__ void df_reserve_blocks(const DArgs& a, const int tag_v) {
  if (blockIdx.x != 0 || threadIdx.x >= 64) return;
  const int b = threadIdx.x, R = a.rows.R;
  const bool on = b < a.n_seqs;
  const int s = a.rows.seq0 + (on ? b : 0);
  const int top = ld_state(a.kv.ctl);
  const int np_s = a.pcap ? ld_state(a.kv.n_pend + s) : 0;
  const int len_s = ld_state(a.kv.len + s);
  const int own = ld_state(a.kv.owned + s);
  const int off = a.pcap ? a.pcap - np_s : 0;
  const int need = ceil_div(len_s + R - off, a.kv.bt);
  const uint32_t tag = (uint32_t)__builtin_amdgcn_readfirstlane(tag_v);
  if (!df_tag_ok(tag)) return;                                     // a refused launch changes nothing
  const int want = on ? max(0, need - own) : 0, room = max(0, a.kv.mbps - own);
  const int take = min(want, room);
  int before = take;                                               // blocks that lower sequences take: exclusive prefix sum
#pragma unroll
  for (int o = 1; o < 16; o <<= 1) {
    const int v = __shfl_up(before, o, WAVE);
    if (b >= o) before += v;
  }
  const int total = __shfl(before, 15, WAVE);
  before -= take;
  const int got = max(0, min(take, top - before));
  // ids of the (at most two) blocks that hold the positions of this launch's rows
  const int bi0 = len_s >> 4;
  int id[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int bi = bi0 + i;
    id[i] = -1;
    if (on && bi < own) id[i] = ld_state(a.kv.table + s * a.kv.mbps + bi);
    else if (on && bi - own < got) id[i] = ld_state(a.kv.free_stack + (top - before - 1 - (bi - own)));
  }
  if (on) {
    for (int i = 0; i < got; ++i) {
      const int bi = own + i;
      const int v = bi == bi0 ? id[0] : bi == bi0 + 1 ? id[1] : ld_state(a.kv.free_stack + (top - before - 1 - i));
      st_ag(a.kv.table + s * a.kv.mbps + bi, v);
    }
    a.kv.owned[s] = own + got;
    if (got < want) a.kv.ctl[1] = 1;
    for (int j = 0; j < R; ++j) {
      const int pos = j < off ? len_s : len_s + (j - off);
      const int bi = pos >> 4;
      const int v = bi == bi0 ? id[0] : bi == bi0 + 1 ? id[1] : -1;
      st_word(a.rowblk + b * R + j, (uint32_t)v, tag);
    }
  }
  if (b == 0) a.kv.ctl[0] = max(0, top - total);
}

// ------------------------------------------------------------------------------------------------ attention
// Item = (sequence, kv head, part of 256 keys, tile of 16 query rows); the query rows of a sequence are its R rows
// times the G query heads of the group, row index qr = j * G + head-in-group.  Wave w of the unit takes keys
// [256 part + 64 w, +64).  Scores are kept in the base-2 domain (scale * log2 e folded in), so that the
// exponentials are single instructions.
struct DAttItem {
  int valid, b, kvh, part, rt, seq, len, nact, off, pos_last, nparts_b;
  int koff[4], voff[2];
};

// Everything here is requested at once (one memory round trip, not six): the cached length and the pending count do
// not change during the launch, and the block ids of positions below the cached length do not either.  A block all of
// whose positions are at or beyond the cached length may be reserved concurrently by this launch: whatever id is read
// for it is only checked to be inside the pool, since each of its positions is either a row of this launch (taken from
// the tagged side buffer, never from the pool) or masked.
__device__ __forceinline__ DAttItem df_att_item(const DArgs& a, int item, int ntile, int uw, int lane) {
  DAttItem it;
  it.valid = item < a.n_seqs * a.nkv * a.n_parts * ntile;
  it.b = 0; it.kvh = 0; it.part = 0; it.rt = 0;
  if (it.valid) {
    it.rt = item % ntile;
    int t = item / ntile;
    it.b = t % a.n_seqs;
    t /= a.n_seqs;
    it.kvh = t % a.nkv;
    it.part = t / a.nkv;
  }
  it.seq = a.rows.seq0 + it.b;
  const int kbase = it.part * ATT_PART + uw * 64;
  // (only by the waves that have an item: a few hundred workgroups asking for the same words queue up at one channel)
  int len_v = 0, npend_v = 0;
  int braw[4] = {-1, -1, -1, -1};
  if (it.valid) {
    len_v = ld_state(a.kv.len + it.seq);
    npend_v = a.pcap ? ld_state(a.kv.n_pend + it.seq) : 0;
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int bi = (kbase >> 4) + t;
      if (bi < a.kv.mbps) braw[t] = ld_state(a.kv.table + it.seq * a.kv.mbps + bi);
    }
  }
  it.len = __builtin_amdgcn_readfirstlane(len_v);
  const int npend = __builtin_amdgcn_readfirstlane(npend_v);
  it.off = a.pcap - npend;
  it.nact = a.rows.R - it.off;
  it.pos_last = it.len + it.nact - 1;
  it.valid = it.valid && it.part * ATT_PART <= it.pos_last;
  it.nparts_b = it.pos_last / ATT_PART + 1;
  const int g = lane >> 4, c16 = lane & 15;
  // The four block ids go through a shared array indexed by the thread id.  As a private array the compiler moves them
  // to LDS on its own and indexes by a flat thread id that it derives from the dispatch packet: a read of host memory
  // by every workgroup, 4-15 us at each launch.  (Measured: forms that keep the ids in registers run the layer loop
  // 4 % slower at identical instruction counts; this form is the one that is fast in both parts.)
  __shared__ int blk_all[PBLOCK * 4];
  int* blk = blk_all + threadIdx.x * 4;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int bi = (kbase >> 4) + t;
    const int b = (it.valid && bi * 16 <= it.pos_last) ? __builtin_amdgcn_readfirstlane(braw[t]) : -1;
    blk[t] = (b < 0 || b >= a.kv.n_blocks) ? 0 : b;            // masked keys may read any block
    it.koff[t] = ((blk[t] * a.nkv + it.kvh) * 16 + c16) * 64 + g * 8;
  }
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int vblk = (g >> 1) ? blk[2 * ks + 1] : blk[2 * ks];
    it.voff[ks] = (vblk * a.nkv + it.kvh) * 1024 + c16 * 16 + (g & 1) * 8;
  }
  return it;
}

// The 16 fragment loads of a wave's chunk from the pool.  Positions at or beyond the sequence's cached length hold
// whatever an earlier launch left there; they are patched or masked later, never used.
__device__ __forceinline__ void df_load_kv(const DArgs& a, int layer, const DAttItem& it, KVPre& kv) {
  const size_t plane = (size_t)a.kv.n_blocks * a.kv.nkv * 1024;
  const bf16_t* kp = (const bf16_t*)a.kv.pool + (size_t)(2 * layer) * plane;
  const bf16_t* vp = kp + plane;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    kv.kf[t][0] = *(const u32x4*)(kp + it.koff[t]);
    kv.kf[t][1] = *(const u32x4*)(kp + it.koff[t] + 32);
  }
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) kv.vf[ks][dt] = *(const u32x4*)(vp + it.voff[ks] + dt * 256);
}

__device__ __forceinline__ float df_exp2(float x) { return __builtin_amdgcn_exp2f(x); }     // x <= 0 here, or -inf


__device__ __forceinline__ bool df_attn_phase(const DArgs& a, const uint32_t tag, int layer, const DAttItem& it, uint32_t* lds,
                                              const int* srow, int* sdead, int slot) {
  // The pool fragments are requested first: the queries of this layer are not there yet in any case.
  KVPre kvp;
  df_load_kv(a, layer, it, kvp);
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int usel = wave >> 2, uw = wave & 3, ut = tid & 255;
  uint32_t* ub = lds + usel * DF_ATT_UNIT;
  uint32_t* Qs = ub;                                   // [16 rows][64] operand words
  bf16_t* Kn = (bf16_t*)(ub + 4096);                   // [16][64] new keys
  bf16_t* Vn = (bf16_t*)(ub + 4096 + 512);             // [16][64] new values
  float* Pw = (float*)(ub + 4096 + 1024) + uw * 1024;  // [16][64] per wave
  float* MO = (float*)(ub + 4096 + 1024 + 4096);       // [4][16][64]
  float* ML = (float*)(ub + 4096 + 1024 + 8192);       // [4][16][2]
  const int R = a.rows.R, G = a.nq / a.nkv, nqd = a.nq * 64, RG = R * G;
  const int g = lane >> 4, c16 = lane & 15;
  const int kbase = it.part * ATT_PART + uw * 64;
  const int r0 = 16 * it.rt, nrt = min(16, RG - r0);                         // first query row and rows of this tile
  const bool wlive = it.valid && kbase <= it.pos_last;
  const bool unew = it.valid && it.part * ATT_PART + ATT_PART > it.len;      // the part reaches this launch's positions
  const u64* q = a.q + (size_t)layer * a.st_q;
  const u64* kvn = a.kvn + (size_t)layer * a.st_kvn;
  u64* attn = a.attn + (size_t)layer * a.st_q;
  u64* att_p = a.att_p + (size_t)layer * a.st_att_p;
  const int* rowpos = srow + it.b * R;                 // positions of the sequence's rows
  const float sc2 = a.scale * 1.44269504088896340736f;
  int qpos[4];                                         // positions of the 4 query rows this lane holds scores of
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int qr = r0 + 4 * g + r;
    qpos[r] = qr < RG ? rowpos[qr / G] : -1;
  }
  bool bad = false;
  // ---- one flight per thread: the queries of the tile's rows and this launch's keys / values of the kv head
  if (it.valid) {
    const int nQ = nrt * 64, total = nQ + (unew ? it.nact * 128 : 0);       // <= 1024 + 2048 words
    const uint32_t q_off = (uint32_t)(q - a.tw), n_off = (uint32_t)(kvn - a.tw);
    uint32_t off[DF_B], out[DF_B];
#pragma unroll
    for (int u = 0; u < DF_B; ++u) {
      const int idx = u * 256 + ut;
      off[u] = 0xFFFFFFFFu;
      if (idx < nQ) {
        const int r = r0 + (idx >> 6), dd = idx & 63, j = r / G, gq = r - j * G;
        off[u] = q_off + (uint32_t)((it.b * R + j) * nqd + (it.kvh * G + gq) * 64 + dd);
      } else if (idx < total) {
        const int i2 = idx - nQ, jn = i2 >> 7, which = (i2 >> 6) & 1, dd = i2 & 63;
        off[u] = n_off + (uint32_t)((((it.b * R + it.off + jn) * 2 + which) * a.nkv + it.kvh) * 64 + dd);
      }
    }
    bad = !poll_words<DF_B>(a.tw, off, tag, out, a.bar + 64, a.hg + (size_t)(2 * layer) * a.st_h, tag);
#pragma unroll
    for (int u = 0; u < DF_B; ++u) {
      const int idx = u * 256 + ut;
      if (idx < nQ) Qs[idx] = out[u];
      else if (idx < total) {
        const int i2 = idx - nQ, jn = i2 >> 7, which = (i2 >> 6) & 1, dd = i2 & 63;
        (which ? Vn : Kn)[jn * 64 + dd] = (bf16_t)out[u];
      }
    }
    for (int idx = nQ + ut; idx < 1024; idx += 256) Qs[idx] = 0u;           // padding rows of the tile
  }
  if (bad) *sdead = 1;
  __syncthreads();
  if (*sdead) return true;
  DF_STAMP(slot);
  // ---- fragments of positions written by this launch come from the side buffer, at the pool's fragment slots
  if (wlive && kbase + 64 > it.len) {
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int jn = kbase + 16 * t + c16 - it.len;
      if ((unsigned)jn < (unsigned)it.nact) {
        kvp.kf[t][0] = *(const u32x4*)(Kn + jn * 64 + g * 8);
        kvp.kf[t][1] = *(const u32x4*)(Kn + jn * 64 + 32 + g * 8);
      }
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const int dim = 16 * dt + c16;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          uint32_t x = kvp.vf[ks][dt][w];
          const int j0 = kbase + 32 * ks + 8 * g + 2 * w - it.len, j1 = j0 + 1;
          if ((unsigned)j0 < (unsigned)it.nact) x = (x & 0xFFFF0000u) | (uint32_t)Vn[j0 * 64 + dim];
          if ((unsigned)j1 < (unsigned)it.nact) x = (x & 0x0000FFFFu) | ((uint32_t)Vn[j1 * 64 + dim] << 16);
          kvp.vf[ks][dt][w] = x;
        }
      }
  }
  float mrow[4], lrow[4];
  f32x4 oacc[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) { mrow[r] = -INFINITY; lrow[r] = 0.f; oacc[r] = f32x4{0, 0, 0, 0}; }
  if (wlive) {
    u32x4 qh[2], ql[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) frag_from_lds(Qs + c16 * 64 + ks * 32 + g * 8, qh[ks], ql[ks]);
    f32x4 s[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const bf16x8 k0 = __builtin_bit_cast(bf16x8, kvp.kf[t][0]), k1 = __builtin_bit_cast(bf16x8, kvp.kf[t][1]);
      f32x4 z = f32x4{0, 0, 0, 0};
      z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ql[0]), k0, z, 0, 0, 0);
      z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ql[1]), k1, z, 0, 0, 0);
      z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qh[0]), k0, z, 0, 0, 0);
      z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qh[1]), k1, z, 0, 0, 0);
      s[t] = z;
    }
    // element (reg r, tile t) = (query row r0 + 4g + r, key kbase + 16t + c16)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int pos = qpos[r];
      float mx = -INFINITY;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const bool ok = kbase + 16 * t + c16 <= pos;
        s[t][r] = ok ? s[t][r] * sc2 : -INFINITY;
        mx = fmaxf(mx, s[t][r]);
      }
      mx = row16_max(mx);
      float sum = 0.f;
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const float p = (s[t][r] == -INFINITY) ? 0.f : df_exp2(s[t][r] - mx);
        Pw[(4 * g + r) * 64 + 16 * t + c16] = p;
        sum += p;
      }
      sum = row16_sum(sum);
      mrow[r] = mx;
      lrow[r] = sum;
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const u32x4* pp = (const u32x4*)(Pw + c16 * 64 + ks * 32 + g * 8);
      const SplitA pf = split_bf16(pp[0], pp[1]);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        const bf16x8 vv = __builtin_bit_cast(bf16x8, kvp.vf[ks][dt]);
        oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf.lo, vv, oacc[dt], 0, 0, 0);
        oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf.hi, vv, oacc[dt], 0, 0, 0);
      }
    }
  }
  // ---- merge the unit's four chunks (ascending key order) and publish the part
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int row = 4 * g + r;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) MO[(uw * 16 + row) * 64 + 16 * dt + c16] = oacc[dt][r];
    if (c16 == 0) { ML[(uw * 16 + row) * 2] = mrow[r]; ML[(uw * 16 + row) * 2 + 1] = lrow[r]; }
  }
  __syncthreads();
  {
    const int row = ut >> 4, ch = ut & 15, d0 = ch * 4, qr = r0 + row;
    if (it.valid && qr < RG) {
      const int j = qr / G, gq = qr - j * G, m = it.b * R + j, head = it.kvh * G + gq;
      const int np_row = rowpos[j] / ATT_PART + 1;
      if (it.part < np_row) {
        float mx = -INFINITY;
        for (int w = 0; w < 4; ++w) mx = fmaxf(mx, ML[(w * 16 + row) * 2]);
        float l = 0.f, o[4] = {0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < 4; ++w) {
          const float mw = ML[(w * 16 + row) * 2];
          if (mw == -INFINITY) continue;
          const float e = df_exp2(mw - mx);
          l = fmaf(ML[(w * 16 + row) * 2 + 1], e, l);
#pragma unroll
          for (int i = 0; i < 4; ++i) o[i] = fmaf(MO[(w * 16 + row) * 64 + d0 + i], e, o[i]);
        }
        if (np_row == 1) {                                  // a single part: this is the result
#pragma unroll
          for (int i = 0; i < 4; ++i) st_word(attn + (size_t)m * nqd + head * 64 + d0 + i, split_payload(o[i] / l), tag);
        } else {
          u64* pp = att_p + ((((size_t)m * a.nq + head) * a.NP + it.part) * 16 + ch) * 6;
#pragma unroll
          for (int i = 0; i < 4; ++i) st_wordf(pp + i, o[i], tag);
          st_wordf(pp + 4, mx, tag);
          st_wordf(pp + 5, l, tag);
        }
      }
    }
  }
  // ---- merge of the parts: of the tile's rows, the unit of part p finishes those with row index = p mod P
  if (it.valid && it.nparts_b > 1) {
    const int P = it.nparts_b;
    const int ri = ut >> 4, ch = ut & 15, d0 = ch * 4;
    const int first = ((it.part - r0) % P + P) % P;                          // first row of the tile this unit finishes
    const int qr = r0 + first + ri * P;
    if (first + ri * P < nrt) {
      const int j = qr / G, gq = qr - j * G, m = it.b * R + j, head = it.kvh * G + gq;
      const int np_row = rowpos[j] / ATT_PART + 1;
      if (np_row > 1) {
        const uint32_t p_off = (uint32_t)(att_p - a.tw) + (uint32_t)(((m * a.nq + head) * a.NP) * 96 + ch * 6);
        float mx = -INFINITY, l = 0.f, o[4] = {0.f, 0.f, 0.f, 0.f};
        for (int p0 = 0; p0 < np_row; p0 += DF_NPF) {
          uint32_t out[DF_NPF * 6];
          bad = !poll_parts(a.tw, p_off + (uint32_t)(p0 * 96), np_row - p0, tag, out, a.bar + 64) || bad;
          float gm = mx;
#pragma unroll
          for (int p = 0; p < DF_NPF; ++p)
            if (p0 + p < np_row) gm = fmaxf(gm, __uint_as_float(out[p * 6 + 4]));
          if (p0 > 0) {                                      // more than DF_NPF parts: rescale what is already summed
            const float e = df_exp2(mx - gm);
            l *= e;
#pragma unroll
            for (int i = 0; i < 4; ++i) o[i] *= e;
          }
          mx = gm;
#pragma unroll
          for (int p = 0; p < DF_NPF; ++p)
            if (p0 + p < np_row) {
              const float e = df_exp2(__uint_as_float(out[p * 6 + 4]) - mx);
              l = fmaf(__uint_as_float(out[p * 6 + 5]), e, l);
#pragma unroll
              for (int i = 0; i < 4; ++i) o[i] = fmaf(__uint_as_float(out[p * 6 + i]), e, o[i]);
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) st_word(attn + (size_t)m * nqd + head * 64 + d0 + i, split_payload(o[i] / l), tag);
      }
    }
  }
  DF_STAMP(slot + 1);
  if (bad) *sdead = 1;
  __syncthreads();
  return *sdead != 0;
}

// ------------------------------------------------------------------------------------------------ attention, short prefixes
// Up to DF_WHOLE_CHUNKS chunks of 64 keys (the host decides from its bound of the cached lengths, the same for a
// verification and an autoregressive step from one state): item = (sequence, kv head, row tile) on a workgroup of its
// own, no parts.  Wave w walks chunks w, w + 8, w + 16 with a running (max, sum, weighted values) per row, the eight
// waves meet once in LDS, and the result goes out as operand words: no partial leaves the workgroup, which takes the
// parts' hand-over (store, find, merge) out of every layer.
constexpr int DF_WHOLE_CHUNKS = 24;
struct DAttWhole {
  int valid, b, kvh, rt, seq, len, nact, off, pos_last, nch;
};

__device__ __forceinline__ DAttWhole df_att_whole_item(const DArgs& a, int item, int ntile, int* sblk) {
  DAttWhole it;
  it.valid = item < a.n_seqs * a.nkv * ntile;
  it.b = 0; it.kvh = 0; it.rt = 0;
  if (it.valid) {
    it.rt = item % ntile;
    const int t = item / ntile;
    it.b = t % a.n_seqs;
    it.kvh = t / a.n_seqs;
  }
  it.seq = a.rows.seq0 + it.b;
  // one round trip for all of it (see df_att_item)
  const int len_v = it.valid ? ld_state(a.kv.len + it.seq) : 0;
  const int npend_v = (it.valid && a.pcap) ? ld_state(a.kv.n_pend + it.seq) : 0;
  const int i = threadIdx.x;
  int bid = -1;
  if (i < DF_WHOLE_CHUNKS * 4 && it.valid && i < a.kv.mbps) bid = ld_state(a.kv.table + it.seq * a.kv.mbps + i);
  it.len = __builtin_amdgcn_readfirstlane(len_v);
  const int npend = __builtin_amdgcn_readfirstlane(npend_v);
  it.off = a.pcap - npend;
  it.nact = a.rows.R - it.off;
  it.pos_last = it.len + it.nact - 1;
  it.nch = min(DF_WHOLE_CHUNKS, it.pos_last / 64 + 1);
  // block ids of the sequence's positions (masked positions may read any block)
  if (i < DF_WHOLE_CHUNKS * 4) sblk[i] = (bid < 0 || bid >= a.kv.n_blocks || i * 16 > it.pos_last) ? 0 : bid;
  return it;
}

__device__ __forceinline__ void df_load_kv_chunk(const DArgs& a, int layer, int kvh, int chunk, const int* sblk, int lane, KVPre& kv) {
  const size_t plane = (size_t)a.kv.n_blocks * a.kv.nkv * 1024;
  const bf16_t* kp = (const bf16_t*)a.kv.pool + (size_t)(2 * layer) * plane;
  const bf16_t* vp = kp + plane;
  const int g = lane >> 4, c16 = lane & 15;
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int koff = ((sblk[chunk * 4 + t] * a.kv.nkv + kvh) * 16 + c16) * 64 + g * 8;
    kv.kf[t][0] = *(const u32x4*)(kp + koff);
    kv.kf[t][1] = *(const u32x4*)(kp + koff + 32);
  }
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int vblk = sblk[chunk * 4 + 2 * ks + (g >> 1)];
    const int voff = (vblk * a.kv.nkv + kvh) * 1024 + c16 * 16 + (g & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) kv.vf[ks][dt] = *(const u32x4*)(vp + voff + dt * 256);
  }
}

__device__ __forceinline__ bool df_attn_whole(const DArgs& a, const uint32_t tag, int layer, const DAttWhole& it, uint32_t* lds, const int* sblk,
                                              const int* srow, int* sdead, int slot) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c16 = lane & 15;
  // the first two chunks of the wave are requested before anything else: the queries are not there yet in any case
  KVPre kvp[2];
  const bool live0 = it.valid && wave < it.nch, live1 = it.valid && wave + 8 < it.nch, live2 = it.valid && wave + 16 < it.nch;
  if (live0) df_load_kv_chunk(a, layer, it.kvh, wave, sblk, lane, kvp[0]);
  if (live1) df_load_kv_chunk(a, layer, it.kvh, wave + 8, sblk, lane, kvp[1]);
  uint32_t* Qs = lds;                                  // [16 rows][64] operand words
  bf16_t* Kn = (bf16_t*)(lds + 1024);                  // [16][64] new keys
  bf16_t* Vn = (bf16_t*)(lds + 1536);                  // [16][64] new values
  float* Pw = (float*)(lds + 2048) + wave * 1024;      // [16][64] per wave
  float* MO = (float*)(lds + 2048 + 8192);             // [8 waves][16][64]
  float* ML = (float*)(lds + 2048 + 16384);            // [8 waves][16][2]
  const int R = a.rows.R, G = a.nq / a.nkv, nqd = a.nq * 64, RG = R * G;
  const int r0 = 16 * it.rt, nrt = min(16, RG - r0);
  const u64* q = a.q + (size_t)layer * a.st_q;
  const u64* kvn = a.kvn + (size_t)layer * a.st_kvn;
  u64* attn = a.attn + (size_t)layer * a.st_q;
  const int* rowpos = srow + it.b * R;
  const float sc2 = a.scale * 1.44269504088896340736f;
  int qpos[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int qr = r0 + 4 * g + r;
    qpos[r] = qr < RG ? rowpos[qr / G] : -1;
  }
  bool bad = false;
  // ---- one flight per thread: the queries of the tile's rows and this launch's keys / values of the kv head
  if (it.valid) {
    constexpr int NB = 6;                               // 6 x 512 threads >= 1024 + 2048 words
    const int nQ = nrt * 64, total = nQ + it.nact * 128;
    const uint32_t q_off = (uint32_t)(q - a.tw), n_off = (uint32_t)(kvn - a.tw);
    uint32_t off[NB], out[NB];
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int idx = u * PBLOCK + tid;
      off[u] = 0xFFFFFFFFu;
      if (idx < nQ) {
        const int r = r0 + (idx >> 6), dd = idx & 63, j = r / G, gq = r - j * G;
        off[u] = q_off + (uint32_t)((it.b * R + j) * nqd + (it.kvh * G + gq) * 64 + dd);
      } else if (idx < total) {
        const int i2 = idx - nQ, jn = i2 >> 7, which = (i2 >> 6) & 1, dd = i2 & 63;
        off[u] = n_off + (uint32_t)((((it.b * R + it.off + jn) * 2 + which) * a.nkv + it.kvh) * 64 + dd);
      }
    }
    bad = !poll_words<NB>(a.tw, off, tag, out, a.bar + 64, a.hg + (size_t)(2 * layer) * a.st_h, tag);
#pragma unroll
    for (int u = 0; u < NB; ++u) {
      const int idx = u * PBLOCK + tid;
      if (idx < nQ) Qs[idx] = out[u];
      else if (idx < total) {
        const int i2 = idx - nQ, jn = i2 >> 7, which = (i2 >> 6) & 1, dd = i2 & 63;
        (which ? Vn : Kn)[jn * 64 + dd] = (bf16_t)out[u];
      }
    }
    for (int idx = nQ + tid; idx < 1024; idx += PBLOCK) Qs[idx] = 0u;       // padding rows of the tile
  }
  if (bad) *sdead = 1;
  __syncthreads();
  if (*sdead) return true;
  DF_STAMP(slot);
  float mrow[4], lrow[4];
  f32x4 oacc[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) { mrow[r] = -INFINITY; lrow[r] = 0.f; oacc[r] = f32x4{0, 0, 0, 0}; }
  if (live0) {
    u32x4 qh[2], ql[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) frag_from_lds(Qs + c16 * 64 + ks * 32 + g * 8, qh[ks], ql[ks]);
#pragma unroll
    for (int j = 0; j < 3; ++j) {
      const bool livej = j == 0 ? live0 : (j == 1 ? live1 : live2);
      if (livej) {
        KVPre& kc = kvp[j & 1];
        const int kbase = 64 * (wave + 8 * j);
        // fragments of positions written by this launch come from the side buffer, at the pool's fragment slots
        if (kbase + 64 > it.len) {
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const int jn = kbase + 16 * t + c16 - it.len;
            if ((unsigned)jn < (unsigned)it.nact) {
              kc.kf[t][0] = *(const u32x4*)(Kn + jn * 64 + g * 8);
              kc.kf[t][1] = *(const u32x4*)(Kn + jn * 64 + 32 + g * 8);
            }
          }
#pragma unroll
          for (int ks = 0; ks < 2; ++ks)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
              const int dim = 16 * dt + c16;
#pragma unroll
              for (int w = 0; w < 4; ++w) {
                uint32_t x = kc.vf[ks][dt][w];
                const int j0 = kbase + 32 * ks + 8 * g + 2 * w - it.len, j1 = j0 + 1;
                if ((unsigned)j0 < (unsigned)it.nact) x = (x & 0xFFFF0000u) | (uint32_t)Vn[j0 * 64 + dim];
                if ((unsigned)j1 < (unsigned)it.nact) x = (x & 0x0000FFFFu) | ((uint32_t)Vn[j1 * 64 + dim] << 16);
                kc.vf[ks][dt][w] = x;
              }
            }
        }
        f32x4 s[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const bf16x8 k0 = __builtin_bit_cast(bf16x8, kc.kf[t][0]), k1 = __builtin_bit_cast(bf16x8, kc.kf[t][1]);
          f32x4 z = f32x4{0, 0, 0, 0};
          z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ql[0]), k0, z, 0, 0, 0);
          z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ql[1]), k1, z, 0, 0, 0);
          z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qh[0]), k0, z, 0, 0, 0);
          z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qh[1]), k1, z, 0, 0, 0);
          s[t] = z;
        }
        // element (reg r, tile t) = (query row r0 + 4g + r, key kbase + 16t + c16)
        float alpha[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int pos = qpos[r];
          float mx = -INFINITY;
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const bool ok = kbase + 16 * t + c16 <= pos;
            s[t][r] = ok ? s[t][r] * sc2 : -INFINITY;
            mx = fmaxf(mx, s[t][r]);
          }
          const float mnew = fmaxf(mrow[r], row16_max(mx));
          alpha[r] = (mrow[r] == -INFINITY) ? 0.f : df_exp2(mrow[r] - mnew);
          float sum = 0.f;
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const float p = (s[t][r] == -INFINITY) ? 0.f : df_exp2(s[t][r] - mnew);
            Pw[(4 * g + r) * 64 + 16 * t + c16] = p;
            sum += p;
          }
          mrow[r] = mnew;
          lrow[r] = fmaf(lrow[r], alpha[r], row16_sum(sum));
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
          for (int r = 0; r < 4; ++r) oacc[dt][r] *= alpha[r];
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
          const u32x4* pp = (const u32x4*)(Pw + c16 * 64 + ks * 32 + g * 8);
          const SplitA pf = split_bf16(pp[0], pp[1]);
#pragma unroll
          for (int dt = 0; dt < 4; ++dt) {
            const bf16x8 vv = __builtin_bit_cast(bf16x8, kc.vf[ks][dt]);
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf.lo, vv, oacc[dt], 0, 0, 0);
            oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf.hi, vv, oacc[dt], 0, 0, 0);
          }
        }
        __builtin_amdgcn_wave_barrier();               // P is rewritten by the next chunk
        if (j == 0 && live2) df_load_kv_chunk(a, layer, it.kvh, wave + 16, sblk, lane, kvp[0]);   // its fragments are free now
      }
    }
  }
  // ---- the eight waves meet (fixed order: wave 0 .. 7) and the tile's rows go out as operand words
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int row = 4 * g + r;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) MO[(wave * 16 + row) * 64 + 16 * dt + c16] = oacc[dt][r];
    if (c16 == 0) { ML[(wave * 16 + row) * 2] = mrow[r]; ML[(wave * 16 + row) * 2 + 1] = lrow[r]; }
  }
  __syncthreads();
  if (tid < 256) {
    const int row = tid >> 4, ch = tid & 15, d0 = ch * 4, qr = r0 + row;
    if (it.valid && qr < RG) {
      const int j = qr / G, gq = qr - j * G, m = it.b * R + j, head = it.kvh * G + gq;
      float mx = -INFINITY;
#pragma unroll
      for (int w = 0; w < 8; ++w) mx = fmaxf(mx, ML[(w * 16 + row) * 2]);
      float l = 0.f, o[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int w = 0; w < 8; ++w) {
        const float mw = ML[(w * 16 + row) * 2];
        const float e = (mw == -INFINITY) ? 0.f : df_exp2(mw - mx);
        l = fmaf(ML[(w * 16 + row) * 2 + 1], e, l);
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = fmaf(MO[(w * 16 + row) * 64 + d0 + i], e, o[i]);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) st_word(attn + (size_t)m * nqd + head * 64 + d0 + i, split_payload(o[i] / l), tag);
    }
  }
  DF_STAMP(slot + 1);
  __syncthreads();
  return false;
}

// ------------------------------------------------------------------------------------------------ the kernel
// The launch's arguments, read again from the kernel-argument segment through a pointer the compiler cannot see
// through.  The arguments are some 130 dwords; held in scalar registers across the layer loop they do not fit, and
// the compiler parks them in vector-register lanes (a readlane per use).  Every phase asks for the arguments anew,
// so only what that phase uses is live, and the loads hit the scalar cache.
__device__ __forceinline__ const DArgs& df_args() {
  auto p = __builtin_amdgcn_kernarg_segment_ptr();
  asm volatile("" : "+s"(p));
  return *(const DArgs*)p;
}

// WHOLE: attention of short prefixes without parts (df_attn_whole).  SB: tagged words a thread keeps in flight while
// it stages GEMM operands -- every slot costs instructions whether it is used or not, and a second flight costs a
// round trip, so the host picks the smallest SB whose single flight (512 threads x SB) holds the launch's rows.
template <bool WHOLE, int SB>
__global__ void __launch_bounds__(PBLOCK) k_forward_dataflow(DArgs) {
  const DArgs& a = df_args();
  __shared__ __attribute__((aligned(16))) uint32_t lds[DF_LDS_WORDS];
  __shared__ int srow[3 * 16];
  __shared__ uint32_t sact[16 * 36];
  __shared__ int sdead;
  if (threadIdx.x == 0) sdead = 0;
  // this launch's number (the kernel that follows a forward on the stream advances the word; nothing in this launch
  // does).  Requested first, looked at after the other start-up loads have been requested.
  const int tag_v = ld_state(a.kv.ctl + 3);
  uint32_t tag = 0u;
  const int nqkv = (a.nq + 2 * a.nkv) * 64, nqd = a.nq * 64, L = a.n_layers, np = a.d >> 5;
  const int NU = gridDim.x * 2;
  // items of every phase kind, and the unit that takes item 0 (the kinds with few items go to different workgroups)
  const int n_qkv = (a.nq + 2 * a.nkv) * 2, ntile = (a.rows.R * (a.nq / a.nkv) + 15) >> 4,
            n_att = a.n_seqs * a.nkv * (WHOLE ? 1 : a.n_parts) * ntile, n_o = np, n_gu = a.ffn >> 4,
            n_lg = (((a.vocab + 15) >> 4) + 1) >> 1;
  const int st = a.small_stride;
  const int st_lg = 2 * n_lg <= NU ? 2 : 1;               // the head's items: a workgroup each where there are enough (a CU's intake bounds an item's weight stream)
  const int s_qkv = (2 * a.g_mlp) % NU, s_att = (s_qkv + st * n_qkv) % NU, s_o = (s_att + st * n_att) % NU,
            s_red = (s_o + st * n_o) % NU;
  auto make_qkv = [&](const DArgs& a, int l) {
    const PLayer Y = layer_ptrs(a, l);
    DPhase x = DPhase{};
    x.layer = l; x.A = a.hg + (size_t)(2 * l) * a.st_h; x.sq = a.sq + (size_t)(2 * l) * a.st_sq;
    x.W0 = Y.wqkv; x.W1 = Y.wqkv; x.N = nqkv; x.K = a.d; x.gs = 1; x.items = n_qkv; x.shift = s_qkv; x.stride = st;
    x.bias = Y.bqkv; x.out = a.q + (size_t)l * a.st_q; x.kvn = a.kvn + (size_t)l * a.st_kvn;
    x.hint = x.A + (size_t)(a.rows.M - 1) * a.d + (a.d - 32); x.hint_tag = tag;   // a word of the last sum task
    return x;
  };
  auto make_o = [&](const DArgs& a, int l) {
    const PLayer Y = layer_ptrs(a, l);
    DPhase x = DPhase{};
    x.layer = l;
    x.A = a.attn + (size_t)l * a.st_q;
    x.W0 = Y.wo; x.W1 = Y.wo; x.N = a.d; x.K = nqd; x.gs = 1; x.items = n_o; x.shift = s_o; x.stride = st;
    const size_t hi = (size_t)(2 * l);
    x.h_in = a.h + hi * a.st_h; x.h_out = a.h + (hi + 1) * a.st_h; x.hg_out = a.hg + (hi + 1) * a.st_h;
    x.sq_out = a.sq + (hi + 1) * a.st_sq;
    x.gain_next = Y.ln2;
    x.hint = a.q + (size_t)l * a.st_q; x.hint_tag = tag;
    return x;
  };
  auto make_swiglu = [&](const DArgs& a, int l) {
    const PLayer Y = layer_ptrs(a, l);
    DPhase x = DPhase{};
    x.layer = l; x.A = a.hg + (size_t)(2 * l + 1) * a.st_h; x.sq = a.sq + (size_t)(2 * l + 1) * a.st_sq;
    x.W0 = Y.wgate; x.W1 = Y.wup; x.N = a.ffn; x.K = a.d; x.gs = 1; x.items = n_gu; x.shift = 0; x.stride = 1;
    x.hint = a.hg + (size_t)(2 * l + 1) * a.st_h; x.hint_tag = tag;
    return x;
  };
  auto make_head = [&](const DArgs& a) {
    DPhase x = DPhase{};
    x.A = a.hg + (size_t)(2 * L) * a.st_h; x.sq = a.sq + (size_t)(2 * L) * a.st_sq;
    x.W0 = a.head; x.W1 = a.head; x.N = a.vocab; x.K = a.d; x.gs = 1; x.items = n_lg; x.shift = 0; x.stride = st_lg; x.logits = a.logits;
    return x;
  };
  // which phase kinds this wave's unit / this workgroup has a round-0 item in
  const int wave_k = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int unit = blockIdx.x * 2 + (wave_k >> 2);
  auto has = [&](int u, int shift, int items, int stride = 1) { return df_item_of_unit(u, shift, NU, stride) < items; };
  const int n_red = a.rows.M * np;
  const int u0 = blockIdx.x * 2, u1 = u0 + 1;
  const bool g_q = has(u0, s_qkv, n_qkv, st) || has(u1, s_qkv, n_qkv, st) || st * n_qkv > NU,
             g_a = has(u0, s_att, n_att, st) || has(u1, s_att, n_att, st),
             g_o = has(u0, s_o, n_o, st) || has(u1, s_o, n_o, st), g_g = (int)blockIdx.x < a.g_mlp,
             g_r = df_item_of_unit((int)blockIdx.x, s_red >> 1, (int)gridDim.x) < n_red || n_red > (int)gridDim.x, g_l = has(u0, 0, n_lg, st_lg) || has(u1, 0, n_lg, st_lg) || st_lg * n_lg > NU;

  DF_STAMP(1);
  df_reserve_blocks(a, tag_v);
  // What the launch needs of the cache state (none of it changes during the launch): the waves' attention items, and
  // per row its position and whether it is active.
  __shared__ int sblk[DF_WHOLE_CHUNKS * 4];
  DAttItem ait = DAttItem{};
  DAttWhole aw = DAttWhole{};
  if (WHOLE) aw = df_att_whole_item(a, df_item_of_unit(u0, s_att, NU, st), ntile, sblk);     // the item has the workgroup (stride 2)
  else ait = df_att_item(a, df_item_of_unit(unit, s_att, NU, st), ntile, wave_k & 3, threadIdx.x & 63);
  if ((g_q || g_a) && threadIdx.x < a.rows.M) {           // the QKV epilogue and the attention masks use them
    const int m = threadIdx.x, brel = m / a.rows.R, j = m - brel * a.rows.R, seq = a.rows.seq0 + brel;
    const int len = ld_state(a.kv.len + seq);
    const int npend = a.pcap ? ld_state(a.kv.n_pend + seq) : 0;
    const int off = a.pcap - npend;
    srow[m] = j < off ? len : len + (j - off);
    srow[16 + m] = j < off ? 0 : 1;
  }
  tag = (uint32_t)__builtin_amdgcn_readfirstlane(tag_v);
  if (!df_tag_ok(tag)) {                                   // numbering exhausted: do nothing; the host must clear the workspace
    if (blockIdx.x == 0 && threadIdx.x == 0) __hip_atomic_fetch_or(a.bar + 64, DEV_ERR_TAGS, __ATOMIC_RELAXED, AG);
    return;
  }
  df_embed_phase(a, tag);
  if (g_q && threadIdx.x < a.rows.M) {                    // the QKV epilogue appends keys and values: block of each row's position
    u64 w = ld_word(a.rowblk + threadIdx.x);
    for (long spins = 0; (uint32_t)(w >> 32) != tag; w = ld_word(a.rowblk + threadIdx.x)) {
      if (++spins > DF_SPIN_LIMIT || ((spins & 63) == 0 && __hip_atomic_load(a.bar + 64, __ATOMIC_RELAXED, AG) != 0)) {
        __hip_atomic_store(a.bar + 64, 1u, __ATOMIC_RELAXED, AG);
        w = 0xFFFFFFFFull;                                 // no block: the row is not appended, every later wait sees the flag
        break;
      }
      __builtin_amdgcn_s_sleep(1);
    }
    srow[32 + threadIdx.x] = (int)(uint32_t)w;
  }
  __syncthreads();
  DF_STAMP(0);
  for (int l = 0; l < L; ++l) {
    const int s0 = 2 + l * 10;
    if (g_q) {
      const DArgs& a = df_args();
      const DPhase cur = make_qkv(a, l);
      if (df_gemm_phase<PE_QKV, SB>(a, tag, cur, lds, srow, &sdead, s0)) return;
    }
    if (g_a) {
      const DArgs& a = df_args();
      if (WHOLE ? df_attn_whole(a, tag, l, aw, lds, sblk, srow, &sdead, s0 + 2) : df_attn_phase(a, tag, l, ait, lds, srow, &sdead, s0 + 2)) return;
    }
    if (g_o) {
      const DArgs& a = df_args();
      const DPhase cur = make_o(a, l);
      if (df_gemm_phase<PE_RESID, SB>(a, tag, cur, lds, srow, &sdead, s0 + 4)) return;
    }
    if (g_g) {
      const DArgs& a = df_args();
      const DPhase cur = make_swiglu(a, l);
      u64* p2 = a.part2 + (size_t)(l & 1) * a.st_part2;
      if (df_mlp_phase<SB>(a, tag, cur, layer_ptrs(a, l).wdown, p2, df_tag2(tag, l), lds, sact, &sdead, s0 + 6)) return;
    }
    if (g_r) {
      const DArgs& a = df_args();
      const size_t hi = (size_t)(2 * l + 1);
      const float* gain_next = l + 1 < L ? layer_ptrs(a, l + 1).ln1 : a.final_norm;
      if (df_reduce_phase(a, tag, l, a.part2 + (size_t)(l & 1) * a.st_part2, df_tag2(tag, l), a.h + hi * a.st_h, a.h + (hi + 1) * a.st_h,
                          a.hg + (hi + 1) * a.st_h, a.sq + (hi + 1) * a.st_sq, gain_next, s_red, lds, &sdead, s0 + 8)) return;
    }
  }
  if (a.with_head && g_l) {
    const DArgs& a = df_args();
    const DPhase cur = make_head(a);
    df_gemm_phase<PE_LOGITS, SB>(a, tag, cur, lds, srow, &sdead, 2 + L * 10);
  }
}

}  // namespace ssd
