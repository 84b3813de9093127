// The whole decoder forward of one verification (Eq. 4) as ONE persistent kernel.
//
// Why: at batch 1 every operator of a layer is a few microseconds of weight streaming, and a dependent kernel
// launch costs about as much as the operator itself.  Here a fixed set of workgroups stays resident, walks
// the layers phase by phase and meets at a grid barrier between dependent phases (5 per layer):
//     A  RMSNorm (folded into the GEMM) + QKV GEMM + bias + rotary + cache append
//     B  attention over the paged cache on the matrix cores, split into 256-key parts; the last part of a
//        (row, kv head) to finish merges the parts
//     C  output projection, k-split; the last split of a column tile to finish adds the residual
//     D  RMSNorm + gate/up GEMM + SwiGLU
//     E  down projection, k-split; the last split adds the residual
// While a workgroup waits at a barrier, the weight fragments of its next item are already in flight: weight
// addresses do not depend on data, so they are requested before the barrier and consumed after it.
//
// Data that crosses workgroups inside the kernel (residual stream, GEMM operand rows, split partials, new cache
// rows, row bookkeeping) obeys one rule: every address is written at most once per launch, with agent-scope
// (sc1, write-through) stores, before a barrier or ticket that orders it ahead of its readers, and is read with
// ordinary loads.  Each layer and phase therefore has its own buffers.  A reader's L2 cannot hold a stale copy
// (it has never seen the address in this launch, and L2 is invalidated between launches), the first reader on
// an XCD pulls the line from memory and the other workgroups of that XCD hit it in L2, and no cache
// write-back / invalidate is needed at a barrier.  Reductions across splits are done by whichever workgroup
// arrives last (a ticket counter), always in ascending split order, so results are deterministic and do not
// depend on the number of rows verified together.
//
// GEMM operand rows are produced once and consumed by hundreds of workgroups, so the producer stores them in the
// form the matrix core takes: each fp32 value x as two bf16, hi = upper 16 bits of x and lo = bf16(x - hi), laid
// out so that a lane's fragment (8 consecutive k of hi, then of lo) is 32 contiguous bytes.
//
// Unit of work: a workgroup has 8 waves = 2 units of 4 waves; unit u of NU = 2*gridDim.x takes items u, u+NU, ...
// Every unit runs the same number of rounds per phase so that __syncthreads() stays uniform.
// Supported: bf16 storage, head_dim 64, 16-token blocks, M <= 16 rows, <= 16 query heads per kv head.
#pragma once
#include "common.h"
#include "gemm.h"

namespace ssd {

constexpr int PBLOCK = 512;          // threads per workgroup of the persistent kernel
constexpr int ATT_PART = 256;        // keys per attention item (4 waves x 64)
constexpr int P_MAX_SPLITS = 8;
constexpr int PF_K = 7;               // k-tiles of weights a wave prefetches across a barrier (2 loads each)
#define AG __HIP_MEMORY_SCOPE_AGENT

// Loads of state that kernels modify (lengths, pending tokens, rows, block table, draft tokens).  The compiler keeps
// uniform plain loads in the scalar cache, which assumes memory that no kernel writes; an agent-scope load is
// always a vector load past the caches, and the value is then made wave-uniform by the caller where needed.
__device__ __forceinline__ int ld_state(const int32_t* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, AG); }
__device__ __forceinline__ void st_ag(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, AG); }
__device__ __forceinline__ void st_ag(int32_t* p, int v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, AG); }
__device__ __forceinline__ void st_ag(bf16_t* p, bf16_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, AG); }

// Operand rows [M][K] in split form: element (row, k) has hi at ((row*K/8 + k/8)*2)*8 + k%8 and lo 8 entries later.
__device__ __forceinline__ void st_split(bf16_t* base, int K, int row, int k, float x) {
  const uint32_t u = __float_as_uint(x), h = u & 0xFFFF0000u;
  bf16_t* p = base + ((size_t)row * (K >> 3) + (k >> 3)) * 16 + (k & 7);
  st_ag(p, (bf16_t)(h >> 16));
  st_ag(p + 8, f_to_bf16(x - __uint_as_float(h)));
}
// Fragment of lane (row, g) for k-tile kt: hi in [0], lo in [1].
__device__ __forceinline__ const u32x4* frag_ptr(const bf16_t* base, int K, int row, int kt, int g) {
  return (const u32x4*)(base + ((size_t)row * (K >> 3) + kt * 4 + g) * 16);
}

struct PLayer {
  const void *wqkv, *wo, *wgate, *wup, *wdown;
  const float *ln1, *ln2, *bqkv;
};

struct PArgs {
  int n_layers, d, nq, nkv, ffn, vocab, n_embed;
  float eps, scale;
  const bf16_t* embed;
  const float* final_norm;
  const void* head;
  const float2* rope;
  PLayer layer0;          // pointers of layer 0; layer l is layer_stride bytes further for every member
  size_t layer_stride;
  KvView kv;
  Rows rows;
  int pcap, n_seqs, tok_stride, with_head;
  const int32_t* tokens;
  // write-once buffers, one instance per layer (strides in elements)
  float* h;               // [2L+1][Mmax][d] residual stream entering layer l at 2l, after its attention block at 2l+1
  bf16_t* hg;             // [2L+1] split operand rows: h times the gain of the RMSNorm that consumes it
  float* sumsq;           // [2L+1][Mmax][d/32] sums of squares of h over each 32-column group
  bf16_t* q;              // [L] split operand rows [Mmax][nq*64]
  bf16_t* attn;           // [L] split operand rows [Mmax][nq*64]
  bf16_t* act;            // [L] split operand rows [Mmax][ffn]
  float* part;            // [2L][splits][Mmax][d]: k-split partials of the output (2l) and down (2l+1) projections
  float* att_o;           // [L][Mmax][nq][NP][64]
  float* att_ml;          // [L][Mmax][nq][NP][2]
  float* logits;
  size_t st_h, st_hg, st_sq, st_q, st_act, st_part, st_att_o, st_att_ml;
  int NP;                 // part capacity of att_o / att_ml per (row, head)
  int n_parts;            // parts launched this call (upper bound from the host's length bound)
  int32_t* tickets;       // [max(d/32, Mmax*nkv)] zero between uses
  uint32_t* bar;          // [0] arrivals, [32] epoch flag, [64] error flag
  uint32_t epoch_base;
  int gs_o, gs_d;
  size_t part_stride;     // floats between the partials of consecutive splits
  unsigned long long* trace;   // optional [gridDim.x][512] clock samples (arrive / leave per barrier), or null
};

template <typename AR>
__device__ __forceinline__ PLayer layer_ptrs(const AR& a, int l) {
  const size_t o = (size_t)l * a.layer_stride;
  PLayer y;
  y.wqkv = (const char*)a.layer0.wqkv + o; y.wo = (const char*)a.layer0.wo + o; y.wgate = (const char*)a.layer0.wgate + o;
  y.wup = (const char*)a.layer0.wup + o; y.wdown = (const char*)a.layer0.wdown + o;
  y.ln1 = (const float*)((const char*)a.layer0.ln1 + o); y.ln2 = (const float*)((const char*)a.layer0.ln2 + o);
  y.bqkv = a.layer0.bqkv ? (const float*)((const char*)a.layer0.bqkv + o) : nullptr;
  return y;
}

// ------------------------------------------------------------------------------------------------ barrier
// Arrive on a counter; the last arrival clears it and publishes the epoch on a separate line; the others poll
// that line (polling the counter itself is slower: the polls contend with the arrivals).  The wait is bounded:
// on a timeout the error flag is raised and every workgroup skips the rest.
// With PF > 0, `prefetch` issues exactly PF vector loads per wave (weights of the wave's next item; repeats where
// it has fewer).  Waves 1..7 issue them after their stores and wait only for what is older (vmcnt(PF):
// vector memory operations of a wave complete in issue order), so the loads stay in flight across the barrier.
// Wave 0 runs the barrier itself and issues its prefetch between its arrival and its first poll.
template <int PF, typename F>
__device__ __forceinline__ bool grid_barrier(const PArgs& a, uint32_t epoch, int* sdead, F&& prefetch) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (PF && wave != 0) {
    __builtin_amdgcn_sched_barrier(0);
    prefetch();
    __builtin_amdgcn_sched_barrier(0);
    // vmcnt(PF): everything issued before the PF prefetch loads has completed (expcnt / lgkmcnt unconstrained)
    __builtin_amdgcn_s_waitcnt(0x0F70 | (PF & 15) | ((PF >> 4) << 14));
  } else {
    __builtin_amdgcn_s_waitcnt(0);        // this thread's agent-scope stores have completed
  }
  __syncthreads();
  if (wave == 0) {
    const uint32_t slot = 2 * (epoch - a.epoch_base - 1);
    const uint32_t G = gridDim.x;
    int dead = *sdead;
    bool last = false;
    if (threadIdx.x == 0) {
#ifdef SSD_TRACE
      if (a.trace) a.trace[(size_t)blockIdx.x * 512 + slot] = wall_clock64();
#endif
      if (!dead) last = __hip_atomic_fetch_add(a.bar, 1u, __ATOMIC_RELAXED, AG) == G - 1;
    }
    __builtin_amdgcn_sched_barrier(0);
    if (PF) prefetch();
    __builtin_amdgcn_sched_barrier(0);
    if (threadIdx.x == 0) {
      if (!dead) {
        if (last) {
          __hip_atomic_store(a.bar, 0u, __ATOMIC_RELAXED, AG);
          __builtin_amdgcn_s_waitcnt(0);
          __hip_atomic_store(a.bar + 32, epoch, __ATOMIC_RELAXED, AG);
        } else {
          long spins = 0;
          while ((int32_t)(__hip_atomic_load(a.bar + 32, __ATOMIC_RELAXED, AG) - epoch) < 0) {
            if (++spins > (1L << 21) || __hip_atomic_load(a.bar + 64, __ATOMIC_RELAXED, AG) != 0) {
              __hip_atomic_store(a.bar + 64, 1u, __ATOMIC_RELAXED, AG);
              dead = 1;
              break;
            }
            __builtin_amdgcn_s_sleep(1);
          }
        }
        *sdead = dead;
      }
#ifdef SSD_TRACE
      if (a.trace) a.trace[(size_t)blockIdx.x * 512 + slot + 1] = wall_clock64();
#endif
    }
  }
  __syncthreads();
  return *sdead != 0;
}

// ------------------------------------------------------------------------------------------------ GEMM phases
enum { PE_QKV = 0, PE_RESID = 1, PE_SWIGLU = 2, PE_LOGITS = 3 };

struct GemmPhase {
  const bf16_t* A;        // split operand rows [M][K], written earlier in this launch (for a normed GEMM: h * gain)
  const float* sumsq;     // [M][K/32] sums of squares of the un-gained rows (nullptr: no RMSNorm)
  const void* W0;
  const void* W1;
  int N, K, gs, items;
  int layer;
  const float* bias;
  const float* h_in;      // PE_RESID: residual input
  float* h_out;           // PE_RESID: residual output, and the derived operand / statistics of the next norm
  bf16_t* hg_out;
  float* sumsq_out;
  const float* gain_next;
  float* part;            // PE_RESID: this phase's split partials
  void* out;              // PE_QKV: q (split rows); PE_SWIGLU: act (split rows); PE_LOGITS: logits (fp32)
};


struct WPre {             // weight fragments of a wave's first PF_K k-tiles of its first item in a phase
  u32x4 b0[PF_K], b1[PF_K];
};

template <int EPI, typename PH>
__device__ __forceinline__ bool gemm_item(const PH& ph, int item, int& t0, int& t1, int& split) {
  t0 = 0; t1 = 0; split = 0;
  if (item >= ph.items) return false;
  if (EPI == PE_QKV) {
    const int head = item >> 1, i = item & 1;                        // head_dim 64: two tile pairs per head
    t0 = head * 4 + i; t1 = t0 + 2;
  } else if (EPI == PE_SWIGLU) {
    t0 = item; t1 = item;
  } else {
    const int npairs = (((ph.N + 15) >> 4) + 1) >> 1;
    split = item / npairs;
    const int p = item - split * npairs;
    t0 = 2 * p; t1 = 2 * p + 1;
  }
  return true;
}

// k-tiles [kb, ke) of wave uw (0..3) of the unit that owns global split `split`
template <typename PH>
__device__ __forceinline__ void wave_krange(const PH& ph, int split, int uw, int& kb, int& ke) {
  const int KT = ph.K >> 5;
  const int per_s = KT / ph.gs, rem_s = KT - per_s * ph.gs;
  const int wg_b = split * per_s + min(split, rem_s), wg_n = per_s + (split < rem_s ? 1 : 0);
  const int per_w = wg_n >> 2, rem_w = wg_n & 3;
  kb = wg_b + uw * per_w + min(uw, rem_w);
  ke = kb + per_w + (uw < rem_w ? 1 : 0);
}

// Exactly 2*PF_K loads: the wave's first PF_K k-tiles of its round-0 item, or the first tile again where it has fewer.
template <int EPI, typename PH>
__device__ __forceinline__ void prefetch_weights(const PH& ph, WPre& pre) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: scalar registers
  const int unit = blockIdx.x * 2 + (wave >> 2);
  int t0, t1, split, kb = 0, ke = 0;
  const bool valid = gemm_item<EPI>(ph, unit, t0, t1, split);
  if (valid) wave_krange(ph, split, wave & 3, kb, ke);
  const int KT = ph.K >> 5, ntiles = (ph.N + 15) >> 4;
  const u32x4* w0 = (const u32x4*)ph.W0 + (size_t)t0 * KT * 64 + lane;
  const u32x4* w1 = (const u32x4*)ph.W1 + (size_t)(t1 < ntiles ? t1 : t0) * KT * 64 + lane;
#pragma unroll
  for (int u = 0; u < PF_K; ++u) {
    const int kt = (kb + u < ke) ? kb + u : 0;
    pre.b0[u] = __builtin_nontemporal_load(w0 + (size_t)kt * 64);
    pre.b1[u] = __builtin_nontemporal_load(w1 + (size_t)kt * 64);
  }
}

__device__ __forceinline__ void mfma_pair(const u32x4 hi, const u32x4 lo, const u32x4 b0, const u32x4 b1, f32x4& acc0,
                                          f32x4& acc1) {
  const bf16x8 ah = __builtin_bit_cast(bf16x8, hi), al = __builtin_bit_cast(bf16x8, lo);
  const bf16x8 bv0 = __builtin_bit_cast(bf16x8, b0), bv1 = __builtin_bit_cast(bf16x8, b1);
  acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, bv0, acc0, 0, 0, 0);
  acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, bv1, acc1, 0, 0, 0);
  acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bv0, acc0, 0, 0, 0);
  acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bv1, acc1, 0, 0, 0);
}

// RMSNorm: the producer of a residual row also stores row * gain (the GEMM operand) and the row's sums of squares
// per 32 columns; the consumer scales its outputs by 1/rms in the epilogue ((x*g).W / rms(x) == norm(x).W).
template <int EPI>
__device__ __forceinline__ void gemm_phase(const PArgs& a, const GemmPhase& ph, const WPre& pre, float* lds, int* sflag) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));      // recompute per-thread indices per phase instead of keeping them live throughout
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: scalar registers
  const int usel = wave >> 2, uw = wave & 3, ut = tid & 255;
  const int unit = blockIdx.x * 2 + usel, NU = gridDim.x * 2;
  float (*red)[2][256] = (float (*)[2][256])(lds + usel * 2048);      // [4][2][256] per unit
  const int M = a.rows.M;
  const int KT = ph.K >> 5, ntiles = (ph.N + 15) >> 4;
  const int arow = lane & 15, g = lane >> 4;
  const int row = ut >> 4, col = ut & 15;                             // epilogue element of this thread
  const int rounds = (ph.items + NU - 1) / NU;
  for (int rd = 0; rd < rounds; ++rd) {
    const int item = rd * NU + unit;
    int t0, t1, split, kb = 0, ke = 0;
    const bool valid = gemm_item<EPI>(ph, item, t0, t1, split);
    if (valid) wave_krange(ph, split, uw, kb, ke);
    const bool has1 = t1 < ntiles;
    const bool live = valid && row < M;
    const int n0 = t0 * 16 + col, n1 = t1 * 16 + col;
    f32x4 acc0 = f32x4{0, 0, 0, 0}, acc1 = f32x4{0, 0, 0, 0};
    // operand fragments of the first PF_K k-tiles, all in flight at once
    u32x4 xh[PF_K], xl[PF_K];
#pragma unroll
    for (int u = 0; u < PF_K; ++u) {
      xh[u] = u32x4{0u, 0u, 0u, 0u};
      xl[u] = u32x4{0u, 0u, 0u, 0u};
      if (kb + u < ke && arow < M) {
        const u32x4* ap = frag_ptr(ph.A, ph.K, arow, kb + u, g);
        xh[u] = ap[0];
        xl[u] = ap[1];
      }
    }
    // epilogue operands that do not depend on the product
    float sq = 0.f, bias0 = 0.f, bias1 = 0.f, hi0 = 0.f, hi1 = 0.f, gn0 = 0.f, gn1 = 0.f;
    int pos = 0, active = 0;
    if (ph.sumsq && row < M)
      for (int p = col; p < KT; p += 16) sq += ph.sumsq[(size_t)row * KT + p];
    if (EPI == PE_QKV && live) {
      if (ph.bias) { bias0 = ph.bias[n0]; bias1 = ph.bias[n0 + 32]; }
      pos = a.rows.pos[row];
      active = a.rows.active[row];
    }
    if (EPI == PE_RESID && live) {
      hi0 = ph.h_in[(size_t)row * ph.N + n0]; hi1 = ph.h_in[(size_t)row * ph.N + n1];
      gn0 = ph.gain_next[n0]; gn1 = ph.gain_next[n1];
    }
    if (rd == 0) {
#pragma unroll
      for (int u = 0; u < PF_K; ++u)
        if (kb + u < ke) mfma_pair(xh[u], xl[u], pre.b0[u], pre.b1[u], acc0, acc1);
    }
    if (valid) {
      const u32x4* w0 = (const u32x4*)ph.W0 + (size_t)t0 * KT * 64 + lane;
      const u32x4* w1 = (const u32x4*)ph.W1 + (size_t)(has1 ? t1 : t0) * KT * 64 + lane;
      if (rd != 0) {
#pragma unroll
        for (int u = 0; u < PF_K; ++u)
          if (kb + u < ke)
            mfma_pair(xh[u], xl[u], __builtin_nontemporal_load(w0 + (size_t)(kb + u) * 64),
                      __builtin_nontemporal_load(w1 + (size_t)(kb + u) * 64), acc0, acc1);
      }
      for (int kt = kb + PF_K; kt < ke; ++kt) {                       // waves with more than PF_K k-tiles
        u32x4 yh = u32x4{0u, 0u, 0u, 0u}, yl = yh;
        if (arow < M) {
          const u32x4* ap = frag_ptr(ph.A, ph.K, arow, kt, g);
          yh = ap[0];
          yl = ap[1];
        }
        mfma_pair(yh, yl, __builtin_nontemporal_load(w0 + (size_t)kt * 64), __builtin_nontemporal_load(w1 + (size_t)kt * 64),
                  acc0, acc1);
      }
    }
    const int obase = (g * 4) * 16 + (lane & 15);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      red[uw][0][obase + r * 16] = acc0[r];
      red[uw][1][obase + r * 16] = acc1[r];
    }
    __syncthreads();
    float v0 = (red[0][0][ut] + red[1][0][ut]) + (red[2][0][ut] + red[3][0][ut]);
    float v1 = (red[0][1][ut] + red[1][1][ut]) + (red[2][1][ut] + red[3][1][ut]);
    if (ph.sumsq) {
#pragma unroll
      for (int o = 8; o > 0; o >>= 1) sq += __shfl_xor(sq, o, WAVE);  // over the 16 lanes of the row
      const float inv = 1.0f / sqrtf(sq / (float)ph.K + a.eps);
      v0 *= inv;
      v1 *= inv;
    }
    if (EPI == PE_QKV) {
      if (live) {
        const int head = n0 >> 6, dd = n0 & 63;                      // dd < 32
        v0 += bias0; v1 += bias1;
        if (head < a.nq + a.nkv) {
          const float2 cs = a.rope[(size_t)pos * 32 + dd];
          const float r0 = v0 * cs.x - v1 * cs.y, r1 = v1 * cs.x + v0 * cs.y;
          v0 = r0; v1 = r1;
        }
        if (head < a.nq) {
          st_split((bf16_t*)ph.out, a.nq * 64, row, head * 64 + dd, v0);
          st_split((bf16_t*)ph.out, a.nq * 64, row, head * 64 + dd + 32, v1);
        } else if (active) {
          const int which = head < a.nq + a.nkv ? 0 : 1;
          const int kvh = head - a.nq - which * a.nkv;
          const int seq = a.rows.seq0 + row / a.rows.R;
          const int blk = a.kv.table[seq * a.kv.mbps + (pos >> 4)];
          if (blk >= 0) {
            bf16_t* base = (bf16_t*)a.kv.pool + kv_offset(a.kv, ph.layer, which, blk, kvh, 0);
            const int tok = pos & 15;
            if (which == 0) { st_ag(base + tok * 64 + dd, f_to_bf16(v0)); st_ag(base + tok * 64 + dd + 32, f_to_bf16(v1)); }
            else { st_ag(base + dd * 16 + tok, f_to_bf16(v0)); st_ag(base + (dd + 32) * 16 + tok, f_to_bf16(v1)); }
          }
        }
      }
      __syncthreads();
    } else if (EPI == PE_SWIGLU) {
      if (live && n0 < ph.N) st_split((bf16_t*)ph.out, ph.N, row, n0, v0 / (1.0f + expf(-v0)) * v1);
      __syncthreads();
    } else if (EPI == PE_LOGITS) {
      if (live) {
        float* lg = (float*)ph.out;
        if (n0 < ph.N) lg[(size_t)row * ph.N + n0] = v0;
        if (has1 && n1 < ph.N) lg[(size_t)row * ph.N + n1] = v1;
      }
      __syncthreads();
    } else {  // PE_RESID: N == d (a multiple of 32), k-split partials, last split adds the residual
      const int pair = t0 >> 1;
      if (ph.gs > 1) {
        if (live) {
          float* o = ph.part + (size_t)split * a.part_stride + (size_t)row * ph.N;
          st_ag(o + n0, v0);
          st_ag(o + n1, v1);
        }
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
        if (ut == 0) {
          int last = 0;
          if (valid) {
            last = (__hip_atomic_fetch_add(a.tickets + pair, 1, __ATOMIC_RELAXED, AG) == ph.gs - 1);
            if (last) __hip_atomic_store(a.tickets + pair, 0, __ATOMIC_RELAXED, AG);
          }
          sflag[usel] = last;
        }
        __syncthreads();
        if (sflag[usel] && row < M) {
          float p0[P_MAX_SPLITS], p1[P_MAX_SPLITS];
#pragma unroll
          for (int s = 0; s < P_MAX_SPLITS; ++s) {
            p0[s] = 0.f; p1[s] = 0.f;
            if (s < ph.gs) {
              const float* o = ph.part + (size_t)s * a.part_stride + (size_t)row * ph.N;
              p0[s] = o[n0];
              p1[s] = o[n1];
            }
          }
          v0 = 0.f; v1 = 0.f;
#pragma unroll
          for (int s = 0; s < P_MAX_SPLITS; ++s) { v0 += p0[s]; v1 += p1[s]; }      // ascending split order
        }
      } else {
        if (ut == 0) sflag[usel] = valid;
        __syncthreads();
      }
      if (sflag[usel]) {
        float q2 = 0.f;
        if (row < M) {
          v0 += hi0; v1 += hi1;
          st_ag(ph.h_out + (size_t)row * ph.N + n0, v0);
          st_ag(ph.h_out + (size_t)row * ph.N + n1, v1);
          st_split(ph.hg_out, ph.N, row, n0, v0 * gn0);
          st_split(ph.hg_out, ph.N, row, n1, v1 * gn1);
          q2 = v0 * v0 + v1 * v1;
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) q2 += __shfl_xor(q2, o, WAVE);            // over the 16 columns of the row
        if (col == 0 && row < M) st_ag(ph.sumsq_out + (size_t)row * (ph.N >> 5) + pair, q2);
      }
      __syncthreads();
    }
  }
}

// ------------------------------------------------------------------------------------------------ phase 0
// Rows, embedding, block reservation.  Item = row.
__device__ __forceinline__ void embed_phase(const PArgs& a) {
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), usel = wave >> 2, ut = tid & 255;
  const int unit = blockIdx.x * 2 + usel, NU = gridDim.x * 2;
  const int M = a.rows.M, R = a.rows.R, d = a.d;
  for (int m = unit; m < M; m += NU) {
    const int brel = m / R, j = m - brel * R;
    const int seq = a.rows.seq0 + brel;
    const int npend = a.pcap ? ld_state(a.kv.n_pend + seq) : 0;
    const int off = a.pcap - npend;
    const int len = ld_state(a.kv.len + seq);
    int tok, pos, active;
    if (j < off) { tok = ld_state(a.kv.pend + seq * 2); pos = len; active = 0; }
    else {
      pos = len + (j - off); active = 1;
      tok = j < a.pcap ? ld_state(a.kv.pend + seq * 2 + (j - off)) : ld_state(a.tokens + (size_t)brel * a.tok_stride + (j - a.pcap));
    }
    tok = min(max(tok, 0), a.n_embed - 1);
    if (ut == 0) { st_ag(a.rows.pos + m, pos); st_ag(a.rows.active + m, active); }
    const bf16_t* src = a.embed + (size_t)tok * d;
    const float* gain = a.layer0.ln1;
    // the 32-lane halves of the unit's waves take the 32-column groups p = ut/32, ut/32 + 8, ...
    for (int p = ut >> 5; p < (d >> 5); p += 8) {
      const int c = p * 32 + (ut & 31);
      const float v = bf16_to_f(src[c]);
      st_ag(a.h + (size_t)m * d + c, v);
      st_split(a.hg, d, m, c, v * gain[c]);
      float sq = v * v;
#pragma unroll
      for (int o = 16; o > 0; o >>= 1) sq += __shfl_xor(sq, o, WAVE);
      if ((ut & 31) == 0) st_ag(a.sumsq + (size_t)m * (d >> 5) + p, sq);
    }
  }
  if (blockIdx.x == 0 && tid == 0) {
    int top = ld_state(a.kv.ctl);
    for (int b = 0; b < a.n_seqs; ++b) {
      const int s = a.rows.seq0 + b;
      const int o = a.pcap ? a.pcap - ld_state(a.kv.n_pend + s) : 0;
      const int need = ceil_div(ld_state(a.kv.len + s) + a.rows.R - o, a.kv.bt);
      int own = ld_state(a.kv.owned + s);
      while (own < need) {
        if (top <= 0 || own >= a.kv.mbps) { a.kv.ctl[1] = 1; break; }
        st_ag(a.kv.table + s * a.kv.mbps + own, ld_state(a.kv.free_stack + --top));
        ++own;
      }
      a.kv.owned[s] = own;
    }
    a.kv.ctl[0] = top;
  }
}

// ------------------------------------------------------------------------------------------------ attention
// What a wave needs to address its chunk of its unit's round-0 attention item.  Positions and block ids do not
// depend on the layer, so this is computed once per launch (after phase 0) and kept in registers.
struct AttItem {
  int valid, m, kvh, part, pos, seq, old;     // old: every key of the wave's chunk was cached before this launch
  int koff[4];                                // per lane: element offset of its K fragment of key tile t in a layer's K plane
  int voff[2];                                // per lane: element offset of its V fragment (dim tile 0) of k-step ks in a V plane
};

__device__ __forceinline__ AttItem att_item(const PArgs& a, int item, int uw, int lane) {
  AttItem it;
  const int M = a.rows.M;
  it.valid = item < a.n_parts * a.nkv * M;
  it.m = 0; it.kvh = 0; it.part = 0; it.pos = 0; it.seq = a.rows.seq0; it.old = 0;
  if (it.valid) {
    it.m = item % M;
    const int t = item / M;
    it.kvh = t % a.nkv;
    it.part = t / a.nkv;
    it.pos = __builtin_amdgcn_readfirstlane(ld_state(a.rows.pos + it.m));
    it.seq = a.rows.seq0 + it.m / a.rows.R;
    it.valid = it.part * ATT_PART <= it.pos;
  }
  const int kbase = it.part * ATT_PART + uw * 64;
  const int g = lane >> 4, c16 = lane & 15;
  int blk[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int bi = (kbase >> 4) + t;
    const int b = (it.valid && bi < a.kv.mbps && bi * 16 <= it.pos)
                      ? __builtin_amdgcn_readfirstlane(ld_state(a.kv.table + it.seq * a.kv.mbps + bi)) : -1;
    blk[t] = b < 0 ? 0 : b;                                    // masked keys may read any valid block
    it.koff[t] = ((blk[t] * a.nkv + it.kvh) * 16 + c16) * 64 + g * 8;
  }
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int vblk = (g >> 1) ? blk[2 * ks + 1] : blk[2 * ks];   // keys 32ks + 8g.. live in block 2ks + g/2
    it.voff[ks] = (vblk * a.nkv + it.kvh) * 1024 + c16 * 16 + (g & 1) * 8;
  }
  it.old = it.valid && (kbase + 64 <= __builtin_amdgcn_readfirstlane(ld_state(a.kv.len + it.seq)));
  return it;
}

struct KVPre {            // K fragments [key tile][k-step] and V fragments [k-step][dim tile] of a wave's chunk
  u32x4 kf[4][2], vf[2][4];
};

// Exactly 16 loads, issued before the barrier that completes this layer's cache append.  Only a chunk that was
// entirely cached before the launch may be touched here: reading a line that another workgroup is still
// appending to would leave a stale copy in this XCD's L2 for the real read after the barrier.  Other waves load
// 16 pieces of the (never written) head matrix to keep the barrier's load count.
__device__ __forceinline__ void load_kv(const PArgs& a, int layer, const AttItem& it, int lane, KVPre& kv);
__device__ __forceinline__ void prefetch_kv(const PArgs& a, int layer, const AttItem& it, int lane, KVPre& kv) {
  if (it.old) {
    load_kv(a, layer, it, lane, kv);
  } else {
    const u32x4* w = (const u32x4*)a.head + lane;
#pragma unroll
    for (int t = 0; t < 4; ++t) { kv.kf[t][0] = w[(2 * t) * 64]; kv.kf[t][1] = w[(2 * t + 1) * 64]; }
#pragma unroll
    for (int t = 0; t < 8; ++t) kv.vf[t >> 2][t & 3] = w[(8 + t) * 64];
  }
}

// The 16 fragment loads of a wave's chunk: a scalar plane base per layer plus the lane offsets of the item.
__device__ __forceinline__ void load_kv(const PArgs& a, int layer, const AttItem& it, int lane, KVPre& kv) {
  const size_t plane = (size_t)a.kv.n_blocks * a.kv.nkv * 1024;            // elements of one layer's K (or V) plane
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

// ------------------------------------------------------------------------------------------------ attention phase
// Item = (part of 256 keys, kv head, row m).  The G query heads of the row that share the kv head are the
// 16-row tile (padded); wave w of the unit takes keys [256 part + 64 w, +64).  S = Q K^T and O = P V run on the
// matrix cores with K fragments read straight from the cache rows and V fragments from the token-minor V layout.
__device__ __forceinline__ void attn_phase(const PArgs& a, int layer, const AttItem& it0, KVPre& kvp, float* lds, int* sflag) {
  int tid = threadIdx.x;
  asm volatile("" : "+v"(tid));
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);     // wave-uniform: scalar registers
  const int usel = wave >> 2, uw = wave & 3, ut = tid & 255;
  const int unit = blockIdx.x * 2 + usel, NU = gridDim.x * 2;
  // LDS per unit: P [4 waves][16][64] fp32 (16 KB) | merge O [4][16][64] (16 KB) | m,l [4][16][2]
  float* Pw = lds + usel * (4096 + 4096 + 128) + uw * 1024;
  float* MO = lds + usel * (4096 + 4096 + 128) + 4096;
  float* ML = lds + usel * (4096 + 4096 + 128) + 8192;
  const int M = a.rows.M, G = a.nq / a.nkv, nqd = a.nq * 64;
  const int items = a.n_parts * a.nkv * M;
  const int rounds = (items + NU - 1) / NU;
  const int g = lane >> 4, c16 = lane & 15;
  const bf16_t* q = a.q + (size_t)layer * a.st_q;
  float* att_o = a.att_o + (size_t)layer * a.st_att_o;
  float* att_ml = a.att_ml + (size_t)layer * a.st_att_ml;
  bf16_t* attn = a.attn + (size_t)layer * a.st_q;
  for (int rd = 0; rd < rounds; ++rd) {
    const AttItem it = rd == 0 ? it0 : att_item(a, rd * NU + unit, uw, lane);
    const bool valid = it.valid;
    const int part = it.part, kvh = it.kvh, m = it.m, pos = it.pos;
    const int kbase = part * ATT_PART + uw * 64;             // first key of this wave's chunk
    const bool wlive = valid && kbase <= pos;
    float mrow[4], lrow[4];
    f32x4 oacc[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) { mrow[r] = -INFINITY; lrow[r] = 0.f; oacc[r] = f32x4{0, 0, 0, 0}; }
    if (wlive) {
      // Q fragments (row c16 = query head kvh*G + c16, dims 8g.. and 32+8g..)
      u32x4 qh[2], ql[2];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        qh[ks] = u32x4{0u, 0u, 0u, 0u};
        ql[ks] = qh[ks];
        if (c16 < G) {
          const u32x4* qp = frag_ptr(q, nqd, m, (kvh * G + c16) * 2 + ks, g);
          qh[ks] = qp[0];
          ql[ks] = qp[1];
        }
      }
      if (rd != 0 || !it.old) load_kv(a, layer, it, lane, kvp);     // not prefetched (or holds rows of this launch)
      auto& kf = kvp.kf;
      auto& vf = kvp.vf;
      f32x4 s[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const bf16x8 k0 = __builtin_bit_cast(bf16x8, kf[t][0]), k1 = __builtin_bit_cast(bf16x8, kf[t][1]);
        f32x4 z = f32x4{0, 0, 0, 0};
        z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ql[0]), k0, z, 0, 0, 0);
        z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ql[1]), k1, z, 0, 0, 0);
        z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qh[0]), k0, z, 0, 0, 0);
        z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, qh[1]), k1, z, 0, 0, 0);
        s[t] = z;
      }
      // element (reg r, tile t) = (query row 4g + r, key kbase + 16t + c16)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const bool ok = kbase + 16 * t + c16 <= pos;
          s[t][r] = ok ? s[t][r] * a.scale : -INFINITY;
          mx = fmaxf(mx, s[t][r]);
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, WAVE));
        float sum = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float p = (s[t][r] == -INFINITY) ? 0.f : expf(s[t][r] - mx);
          Pw[(4 * g + r) * 64 + 16 * t + c16] = p;
          sum += p;
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o, WAVE);
        mrow[r] = mx;
        lrow[r] = sum;
      }
      __builtin_amdgcn_wave_barrier();
      // O = P V: P fragment row c16, keys 32ks + 8g..; V fragment dim 16dt + c16, same keys (token-minor layout)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const u32x4* pp = (const u32x4*)(Pw + c16 * 64 + ks * 32 + g * 8);
        const SplitA pf = split_bf16(pp[0], pp[1]);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          const bf16x8 vv = __builtin_bit_cast(bf16x8, vf[ks][dt]);
          oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf.lo, vv, oacc[dt], 0, 0, 0);
          oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf.hi, vv, oacc[dt], 0, 0, 0);
        }
      }
    }
    // merge the unit's four chunks (ascending key order) and publish the part
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = 4 * g + r;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) MO[(uw * 16 + row) * 64 + 16 * dt + c16] = oacc[dt][r];
      if (c16 == 0) { ML[(uw * 16 + row) * 2] = mrow[r]; ML[(uw * 16 + row) * 2 + 1] = lrow[r]; }
    }
    __syncthreads();
    const int nparts_row = (pos / ATT_PART) + 1;
    {
      const int row = ut >> 4, d0 = (ut & 15) * 4;
      if (valid && row < G) {
        float mx = -INFINITY;
        for (int w = 0; w < 4; ++w) mx = fmaxf(mx, ML[(w * 16 + row) * 2]);
        float l = 0.f, o[4] = {0.f, 0.f, 0.f, 0.f};
        for (int w = 0; w < 4; ++w) {
          const float mw = ML[(w * 16 + row) * 2];
          if (mw == -INFINITY) continue;
          const float e = expf(mw - mx);
          l = fmaf(ML[(w * 16 + row) * 2 + 1], e, l);
#pragma unroll
          for (int i = 0; i < 4; ++i) o[i] = fmaf(MO[(w * 16 + row) * 64 + d0 + i], e, o[i]);
        }
        if (nparts_row == 1) {                              // a single part: this is the result
#pragma unroll
          for (int i = 0; i < 4; ++i) st_split(attn, nqd, m, (kvh * G + row) * 64 + d0 + i, o[i] / l);
        } else {
          const size_t pidx = ((size_t)m * a.nq + kvh * G + row) * a.NP + part;
#pragma unroll
          for (int i = 0; i < 4; ++i) st_ag(att_o + pidx * 64 + d0 + i, o[i]);
          if ((ut & 15) == 0) { st_ag(att_ml + pidx * 2, mx); st_ag(att_ml + pidx * 2 + 1, l); }
        }
      }
    }
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (ut == 0) {
      int last = 0;
      if (valid && nparts_row > 1) {
        int32_t* tk = a.tickets + m * a.nkv + kvh;
        last = (__hip_atomic_fetch_add(tk, 1, __ATOMIC_RELAXED, AG) == nparts_row - 1);
        if (last) __hip_atomic_store(tk, 0, __ATOMIC_RELAXED, AG);
      }
      sflag[usel] = last;
    }
    __syncthreads();
    if (sflag[usel]) {
      const int row = ut >> 4, d0 = (ut & 15) * 4;
      if (row < G) {
        const size_t base = ((size_t)m * a.nq + kvh * G + row) * a.NP;
        float mx = -INFINITY;
        for (int p = 0; p < nparts_row; ++p) mx = fmaxf(mx, att_ml[(base + p) * 2]);
        float l = 0.f, o[4] = {0.f, 0.f, 0.f, 0.f};
        for (int p = 0; p < nparts_row; ++p) {
          const float e = expf(att_ml[(base + p) * 2] - mx);
          l = fmaf(att_ml[(base + p) * 2 + 1], e, l);
          const float4 op = *(const float4*)(att_o + (base + p) * 64 + d0);
          o[0] = fmaf(op.x, e, o[0]); o[1] = fmaf(op.y, e, o[1]); o[2] = fmaf(op.z, e, o[2]); o[3] = fmaf(op.w, e, o[3]);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) st_split(attn, nqd, m, (kvh * G + row) * 64 + d0 + i, o[i] / l);
      }
    }
    __syncthreads();
  }
}

// ------------------------------------------------------------------------------------------------ the kernel
__global__ void __launch_bounds__(PBLOCK) k_forward_persistent(PArgs a) {
  __shared__ __attribute__((aligned(16))) float lds[2 * (4096 + 4096 + 128)];
  __shared__ int sflag[2];
  __shared__ int sdead;
  if (threadIdx.x == 0) sdead = 0;
  __syncthreads();
  uint32_t epoch = a.epoch_base;
  const int nqkv = (a.nq + 2 * a.nkv) * 64, nqd = a.nq * 64, L = a.n_layers, np = a.d >> 5;
  WPre pre;
  GemmPhase nx;                                            // the next GEMM phase (its weights are prefetched at the barrier)
  auto set_qkv = [&](int l) {
    const PLayer Y = layer_ptrs(a, l);
    nx = GemmPhase{};
    nx.layer = l; nx.A = a.hg + (size_t)(2 * l) * a.st_hg; nx.sumsq = a.sumsq + (size_t)(2 * l) * a.st_sq;
    nx.W0 = Y.wqkv; nx.W1 = Y.wqkv; nx.N = nqkv; nx.K = a.d; nx.gs = 1; nx.items = (a.nq + 2 * a.nkv) * 2;
    nx.bias = Y.bqkv; nx.out = a.q + (size_t)l * a.st_q;
  };
  auto set_resid = [&](int l, int second) {                // second = 0: output projection, 1: down projection
    const PLayer Y = layer_ptrs(a, l);
    nx = GemmPhase{};
    nx.layer = l;
    nx.A = second ? a.act + (size_t)l * a.st_act : a.attn + (size_t)l * a.st_q;
    nx.W0 = second ? Y.wdown : Y.wo; nx.W1 = nx.W0; nx.N = a.d; nx.K = second ? a.ffn : nqd;
    nx.gs = second ? a.gs_d : a.gs_o; nx.items = np * nx.gs;
    const size_t hi = (size_t)(2 * l + second);
    nx.h_in = a.h + hi * a.st_h; nx.h_out = a.h + (hi + 1) * a.st_h; nx.hg_out = a.hg + (hi + 1) * a.st_hg;
    nx.sumsq_out = a.sumsq + (hi + 1) * a.st_sq;
    nx.gain_next = second ? (l + 1 < L ? layer_ptrs(a, l + 1).ln1 : a.final_norm) : Y.ln2;
    nx.part = a.part + hi * a.st_part;
  };
  auto set_swiglu = [&](int l) {
    const PLayer Y = layer_ptrs(a, l);
    nx = GemmPhase{};
    nx.layer = l; nx.A = a.hg + (size_t)(2 * l + 1) * a.st_hg; nx.sumsq = a.sumsq + (size_t)(2 * l + 1) * a.st_sq;
    nx.W0 = Y.wgate; nx.W1 = Y.wup; nx.N = a.ffn; nx.K = a.d; nx.gs = 1; nx.items = a.ffn >> 4;
    nx.out = a.act + (size_t)l * a.st_act;
  };
  auto set_head = [&]() {
    nx = GemmPhase{};
    nx.A = a.hg + (size_t)(2 * L) * a.st_hg; nx.sumsq = a.sumsq + (size_t)(2 * L) * a.st_sq;
    nx.W0 = a.head; nx.W1 = a.head; nx.N = a.vocab; nx.K = a.d; nx.gs = 1;
    nx.items = (((a.vocab + 15) >> 4) + 1) >> 1; nx.out = a.logits;
  };
  auto nothing = []() {};

  embed_phase(a);
  set_qkv(0);
  if (grid_barrier<2 * PF_K>(a, ++epoch, &sdead, [&]() { prefetch_weights<PE_QKV>(nx, pre); })) return;
  // every wave's round-0 attention item: rows and block table are final after phase 0
  const int wave_k = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const AttItem ait = att_item(a, blockIdx.x * 2 + (wave_k >> 2), wave_k & 3, threadIdx.x & 63);
  KVPre kvp;
  for (int l = 0; l < L; ++l) {
    gemm_phase<PE_QKV>(a, nx, pre, lds, sflag);
    if (grid_barrier<16>(a, ++epoch, &sdead, [&]() { prefetch_kv(a, l, ait, threadIdx.x & 63, kvp); })) return;
    attn_phase(a, l, ait, kvp, lds, sflag);
    set_resid(l, 0);
    if (grid_barrier<2 * PF_K>(a, ++epoch, &sdead, [&]() { prefetch_weights<PE_RESID>(nx, pre); })) return;
    gemm_phase<PE_RESID>(a, nx, pre, lds, sflag);
    set_swiglu(l);
    if (grid_barrier<2 * PF_K>(a, ++epoch, &sdead, [&]() { prefetch_weights<PE_SWIGLU>(nx, pre); })) return;
    gemm_phase<PE_SWIGLU>(a, nx, pre, lds, sflag);
    set_resid(l, 1);
    if (grid_barrier<2 * PF_K>(a, ++epoch, &sdead, [&]() { prefetch_weights<PE_RESID>(nx, pre); })) return;
    gemm_phase<PE_RESID>(a, nx, pre, lds, sflag);
    if (l + 1 < L) {
      set_qkv(l + 1);
      if (grid_barrier<2 * PF_K>(a, ++epoch, &sdead, [&]() { prefetch_weights<PE_QKV>(nx, pre); })) return;
    } else {
      if (!a.with_head) return;
      set_head();
      if (grid_barrier<2 * PF_K>(a, ++epoch, &sdead, [&]() { prefetch_weights<PE_LOGITS>(nx, pre); })) return;
    }
  }
  gemm_phase<PE_LOGITS>(a, nx, pre, lds, sflag);
}

}  // namespace ssd
