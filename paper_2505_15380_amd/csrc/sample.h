// Row kernels around the vocabulary: embedding gather + row bookkeeping, residual add + RMSNorm,
// warp + softmax, and the acceptance / resampling / commit kernel (Eq. 5-6, Alg. 1).
#pragma once
#include "common.h"

namespace ssd {

// ------------------------------------------------------------------------------------------ rows + embed
struct EmbedArgs {
  KvView kv;
  Rows rows;
  int pcap;                 // pending slots at the head of each sequence's rows (0 for a prefill chunk)
  int n_seqs;
  const int32_t* tokens;    // explicit tokens [n_seqs][tok_stride] for rows j >= pcap
  int tok_stride;
  const void* embed;        // [n_embed][d]
  int n_embed, d;
  float* h;                 // [M][d]
};

// One workgroup per row: resolve the row's token and position, copy its embedding into the residual stream.
// Workgroup 0 also reserves the cache blocks the forward will write (sequences in ascending order).
template <typename WT>
__global__ void __launch_bounds__(BLOCK) k_embed(EmbedArgs e) {
  const int m = blockIdx.x;
  const int brel = m / e.rows.R, j = m - brel * e.rows.R;
  const int seq = e.rows.seq0 + brel;
  const int npend = e.pcap ? e.kv.n_pend[seq] : 0;
  const int off = e.pcap - npend;                          // leading rows that carry nothing
  const int len = e.kv.len[seq];
  int tok, pos, active;
  if (j < off) { tok = e.kv.pend[seq * 2]; pos = len; active = 0; }
  else {
    pos = len + (j - off); active = 1;
    tok = j < e.pcap ? e.kv.pend[seq * 2 + (j - off)] : e.tokens[(size_t)brel * e.tok_stride + (j - e.pcap)];
  }
  tok = min(max(tok, 0), e.n_embed - 1);
  if (threadIdx.x == 0) { e.rows.pos[m] = pos; e.rows.active[m] = active; }
  const typename WT::T* src = (const typename WT::T*)e.embed + (size_t)tok * e.d;
  for (int i = threadIdx.x; i < e.d; i += BLOCK) e.h[(size_t)m * e.d + i] = WT::ld(src + i);
  if (m == 0 && threadIdx.x == 0) {
    for (int b = 0; b < e.n_seqs; ++b) {
      const int s = e.rows.seq0 + b;
      const int o = e.pcap ? e.pcap - e.kv.n_pend[s] : 0;
      kv_reserve(e.kv, s, e.kv.len[s] + e.rows.R - o);
    }
  }
}

// h[m] += sum of the k-split partials of the previous GEMM (ascending split order); xn[m] = RMSNorm(h[m]) * gain.
template <typename AT>
__global__ void __launch_bounds__(BLOCK) k_add_norm(float* h, const float* part, int n_part, size_t part_stride,
                                                    const float* gain, float eps, void* xn, int d) {
  __shared__ float s4[4];
  const int m = blockIdx.x;
  float* hr = h + (size_t)m * d;
  float ss = 0.f;
  for (int i = threadIdx.x; i < d; i += BLOCK) {
    float v = hr[i];
    const float* pp = part + (size_t)m * d + i;
    for (int s0 = 0; s0 < n_part; s0 += 4) {              // four loads in flight; the sum stays in ascending split order
      float x[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) x[u] = s0 + u < n_part ? pp[(size_t)(s0 + u) * part_stride] : 0.f;
#pragma unroll
      for (int u = 0; u < 4; ++u)
        if (s0 + u < n_part) v += x[u];
    }
    hr[i] = v;
    ss = fmaf(v, v, ss);
  }
  const float tot = block_sum(ss, s4);
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
  typename AT::T* xr = (typename AT::T*)xn + (size_t)m * d;
  for (int i = threadIdx.x; i < d; i += BLOCK) AT::st(xr + i, hr[i] * inv * gain[i]);
}

// The same for the kernels that serve many rows: the normalised row goes out as split rows (see common.h), eight
// consecutive columns per thread (d <= 4096).
__global__ void __launch_bounds__(BLOCK) k_add_norm_split(float* h, const float* part, int n_part, size_t part_stride,
                                                          const float* gain, float eps, bf16_t* xs, int d) {
  __shared__ float s4[4];
  const int m = blockIdx.x, KT = d >> 5, nslot = d >> 3;
  float* hr = h + (size_t)m * d;
  float v[2][8];
  float ss = 0.f;
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int sl = threadIdx.x + q * BLOCK;
    if (sl < nslot) {
      const float4 x0 = *(const float4*)(hr + sl * 8), x1 = *(const float4*)(hr + sl * 8 + 4);
      v[q][0] = x0.x; v[q][1] = x0.y; v[q][2] = x0.z; v[q][3] = x0.w; v[q][4] = x1.x; v[q][5] = x1.y; v[q][6] = x1.z; v[q][7] = x1.w;
      const float* pp = part + (size_t)m * d + sl * 8;
      for (int s0 = 0; s0 < n_part; ++s0) {                 // ascending split order, as k_add_norm
        const float4 p0 = *(const float4*)(pp + (size_t)s0 * part_stride), p1 = *(const float4*)(pp + (size_t)s0 * part_stride + 4);
        v[q][0] += p0.x; v[q][1] += p0.y; v[q][2] += p0.z; v[q][3] += p0.w; v[q][4] += p1.x; v[q][5] += p1.y; v[q][6] += p1.z; v[q][7] += p1.w;
      }
      *(float4*)(hr + sl * 8) = make_float4(v[q][0], v[q][1], v[q][2], v[q][3]);
      *(float4*)(hr + sl * 8 + 4) = make_float4(v[q][4], v[q][5], v[q][6], v[q][7]);
#pragma unroll
      for (int i = 0; i < 8; ++i) ss = fmaf(v[q][i], v[q][i], ss);
    }
  }
  const float tot = block_sum(ss, s4);
  const float inv = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
  for (int q = 0; q < 2; ++q) {
    const int sl = threadIdx.x + q * BLOCK;
    if (sl < nslot) {
      uint32_t y[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) y[i] = __float_as_uint(v[q][i] * inv * gain[sl * 8 + i]);
      const SplitA sp = split_bf16(u32x4{y[0], y[1], y[2], y[3]}, u32x4{y[4], y[5], y[6], y[7]});
      u32x4* o = (u32x4*)(xs + split_index(m, sl * 8, KT));
      o[0] = __builtin_bit_cast(u32x4, sp.hi);
      o[64] = __builtin_bit_cast(u32x4, sp.lo);            // 512 bf16 further
    }
  }
}

// ------------------------------------------------------------------------------------------ warp + softmax
__device__ __forceinline__ uint32_t order_key(float f) {      // larger float <-> larger key
  const uint32_t u = __float_as_uint(f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

struct WarpArgs {
  const float* logits;   // [rows][ld]
  int ld, V;
  float temperature;
  int top_k, greedy;
  float* probs;          // [rows][V] or strided
  size_t probs_stride;
};

constexpr int SBLOCK = 1024;          // threads of the two sampler kernels (16 waves): short unrolled loops, small code
constexpr int SPER = 16;              // elements per thread at most: vocab <= 16384.  The kernels are instantiated for 8 and 16
                                      // (the loops over a thread's elements are unrolled to that count, so a small vocabulary pays for 8)

// Reductions over the 16 waves of a sampler workgroup through 16 LDS entries; all threads get the result.
__device__ __forceinline__ float sblock_max(float v, float* s16) {
  v = wave_max(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) s16[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = s16[0];
#pragma unroll
  for (int i = 1; i < 16; ++i) r = fmaxf(r, s16[i]);
  return r;
}
__device__ __forceinline__ float sblock_sum(float v, float* s16) {      // fixed order: waves ascending
  v = wave_sum(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) s16[threadIdx.x >> 6] = v;
  __syncthreads();
  float r = s16[0];
#pragma unroll
  for (int i = 1; i < 16; ++i) r += s16[i];
  return r;
}

// One workgroup per row.  Top-k keeps exactly k entries: everything above the k-th largest value, and of the
// entries equal to it the ones with the lowest indices.
template <int SP>
__device__ __forceinline__ void warp_softmax_row(const WarpArgs w, const int row, float* lds_probs = nullptr) {
  __shared__ float s16[16];
  __shared__ int i16[16];
  __shared__ int hist[256];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_krem, sh_idxmax;
  const int tid = threadIdx.x;
  const float* x = w.logits + (size_t)row * w.ld;
  float* p = w.probs + (size_t)row * w.probs_stride;
  const int V = w.V;
  // the row is read once into registers (all loads in flight together)
  float xv[SP];
#pragma unroll
  for (int e = 0; e < SP; ++e) {
    const int i = tid + e * SBLOCK;
    xv[e] = i < V ? x[i] : -INFINITY;
  }

  if (w.greedy) {                                            // one-hot at the arg-max, lowest index on ties
    float best = -INFINITY; int bi = 0x7fffffff;
#pragma unroll
    for (int e = 0; e < SP; ++e) { if (xv[e] > best) { best = xv[e]; bi = tid + e * SBLOCK; } }
    const float mx = sblock_max(best, s16);
    int cand = (best == mx) ? bi : 0x7fffffff;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) cand = min(cand, __shfl_xor(cand, o, WAVE));
    if ((tid & 63) == 0) i16[tid >> 6] = cand;
    __syncthreads();
    int arg = i16[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) arg = min(arg, i16[i]);
#pragma unroll
    for (int e = 0; e < SP; ++e) {
      const int i = tid + e * SBLOCK;
      if (i < V) {
        p[i] = (i == arg) ? 1.0f : 0.0f;
        if (lds_probs) lds_probs[i] = (i == arg) ? 1.0f : 0.0f;
      }
    }
    return;
  }

  // threshold key of the top-k set (radix select, 8 bits per pass, most significant first)
  uint32_t kth = 0;          // keep keys > kth, and keys == kth with index <= idxmax
  int idxmax = 0x7fffffff;
  const bool use_k = w.top_k > 0 && w.top_k < V;
  if (use_k) {
    if (tid == 0) { sh_prefix = 0; sh_krem = w.top_k; }
    for (int pass = 0; pass < 4; ++pass) {
      const int shift = 24 - 8 * pass;
      if (tid < 256) hist[tid] = 0;
      __syncthreads();
      const uint32_t prefix = sh_prefix;
      const uint32_t himask = pass ? (0xFFFFFFFFu << (shift + 8)) : 0u;
#pragma unroll
      for (int e = 0; e < SP; ++e) {
        if (tid + e * SBLOCK < V) {
          const uint32_t k = order_key(xv[e]);
          if ((k & himask) == prefix) atomicAdd(&hist[(k >> shift) & 255], 1);
        }
      }
      __syncthreads();
      if (tid == 0) {
        int krem = sh_krem, dsel = 0;
        for (int dgt = 255; dgt >= 0; --dgt) {
          if (hist[dgt] >= krem) { dsel = dgt; break; }
          krem -= hist[dgt];
        }
        sh_krem = krem;
        sh_prefix = prefix | ((uint32_t)dsel << shift);
      }
      __syncthreads();
    }
    kth = sh_prefix;
    const int need_eq = sh_krem;                             // entries equal to kth that survive (>= 1)
    int eq = 0;
#pragma unroll
    for (int e = 0; e < SP; ++e) eq += (tid + e * SBLOCK < V && order_key(xv[e]) == kth);
    eq = wave_sum_i(eq);
    if ((tid & 63) == 0) i16[tid >> 6] = eq;
    __syncthreads();
    int n_eq = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) n_eq += i16[i];
    if (n_eq > need_eq) {                                    // a tie straddles the cut: rare, resolved serially
      if (tid == 0) {
        int seen = 0, im = V - 1;
        for (int i = 0; i < V; ++i)
          if (order_key(x[i]) == kth && ++seen == need_eq) { im = i; break; }
        sh_idxmax = im;
      }
      __syncthreads();
      idxmax = sh_idxmax;
    }
  }
  const float T = w.temperature;
  float z[SP];
  float mx = -INFINITY;
#pragma unroll
  for (int e = 0; e < SP; ++e) {
    const int i = tid + e * SBLOCK;
    z[e] = -INFINITY;
    if (i < V) {
      const uint32_t k = order_key(xv[e]);
      const bool keep = !use_k || k > kth || (k == kth && i <= idxmax);
      if (keep) z[e] = xv[e] / T;
    }
    mx = fmaxf(mx, z[e]);
  }
  mx = sblock_max(mx, s16);
  float sum = 0.f;
#pragma unroll
  for (int e = 0; e < SP; ++e) {
    z[e] = (z[e] == -INFINITY) ? 0.f : expf(z[e] - mx);
    sum += z[e];
  }
  sum = sblock_sum(sum, s16);
#pragma unroll
  for (int e = 0; e < SP; ++e) {
    const int i = tid + e * SBLOCK;
    if (i < V) {
      const float q = z[e] / sum;
      p[i] = q;
      if (lds_probs) lds_probs[i] = q;                        // k_warp_accept: the draw reads the row from LDS
    }
  }
}

template <int SP>
__global__ void __launch_bounds__(SBLOCK) k_warp_softmax(WarpArgs w) { warp_softmax_row<SP>(w, blockIdx.x); }

// ------------------------------------------------------------------------------ acceptance + resampling
struct AcceptArgs {
  const float* pt;       // [B][K+1][V]
  size_t pt_seq_stride;  // elements between sequences
  const float* pd;       // [B][K][V]
  const int32_t* x;      // [B][K]
  const float* uniforms; // [B][K+1] or NULL -> Philox(seed, seq, step, slot)
  uint64_t seed, step;
  const int32_t* step_dev;  // when set: two words (low, high) of a device-resident cycle counter that is added to `step`, so
                         // that a captured graph of a cycle draws fresh uniforms at every replay
  int bump_step;         // the committing thread advances that counter (the last sampling kernel of a cycle without drafts)
  int bump_launch;       // this kernel follows a forward on a.kv: the committing thread advances the cache's launch number
  int slot_base;         // r_i uses slot slot_base + i - 1, the emitted token slot_base + K
  int B, K, V;
  float beta;
  int32_t* n_acc;        // [B] (may be NULL)
  int32_t* next_tok;     // [B*tok_stride]
  int tok_stride;
  int32_t* flags;        // [B] or NULL
  int32_t* ticket;       // arrival counter of the workgroups of a multi-sequence commit: zero before the launch, zero after it
  // commit (kv.len == NULL: decisions only)
  KvView kv;
  int seq0;
};

// Fixed-point weight of the canonical sampler: floor(w * 2^40) for a non-negative float w < 2^23, exactly (the
// product is a shift of the 24-bit significand; subnormals are below 2^-40 and give 0).
__device__ __forceinline__ unsigned long long fix40(float w) {
  const uint32_t u = __float_as_uint(w);
  const int ex = (int)((u >> 23) & 255u);
  if (ex == 0 || (u >> 31)) return 0ull;
  const unsigned long long mant = (unsigned long long)((u & 0x7FFFFFu) | 0x800000u);
  const int sh = ex - 127 + 17;                              // value = mant * 2^(ex - 150); times 2^40
  return sh >= 0 ? (mant << sh) : (sh > -24 ? (mant >> (-sh)) : 0ull);
}

// Exclusive prefix sum of one 64-bit value per thread over the 1024 threads of a sampler workgroup (integer: exact
// in any order).  w16: 16 entries of LDS.
__device__ __forceinline__ unsigned long long sblock_excl_scan_u64(unsigned long long v, unsigned long long* w16,
                                                                   unsigned long long* total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  unsigned long long inc = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const unsigned long long t = __shfl_up(inc, o, WAVE);
    if (lane >= o) inc += t;
  }
  __syncthreads();
  if (lane == 63) w16[wave] = inc;
  __syncthreads();
  unsigned long long base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    if (i < wave) base += w16[i];
    tot += w16[i];
  }
  *total = tot;
  return base + inc - v;
}

// One workgroup per sequence.
//  1. lanes i < K: threshold min(1, pt_i(x_i)/pd_i(x_i)) + beta in fp32 (division only when pd > pt, so never by
//     zero), accept iff r_i < threshold; n = number of leading accepts via a wave ballot.
//  2. emitted token: inverse CDF over w_j = max(0, pt_{n+1}(j) - pd_{n+1}(j)) (n < K) or pt_{K+1}(j) (n == K), with the
//     weights in 2^40 fixed point so that the total and the prefix sums are integers (no dependence on the
//     summation tree): smallest j whose inclusive prefix exceeds floor(total * u).
//  3. the last workgroup to finish commits every sequence in ascending order: len += pending + n, pending =
//     emitted token, blocks past the new length go back to the free stack.
template <int SP>
__device__ __forceinline__ void accept_seq(const AcceptArgs a, const int b, const float* lds_row0 = nullptr) {
  __shared__ unsigned long long w16[16];
  __shared__ int sh_n, sh_tok, sh_last;
  __shared__ float sh_u;
  const int tid = threadIdx.x;
  const int K = a.K, V = a.V;
  const float* pt = a.pt + (size_t)b * a.pt_seq_stride;
  const float* pd = a.pd + (size_t)b * K * V;
  const uint32_t seq = (uint32_t)(a.seq0 + b);
  uint64_t step = a.step;
  if (a.step_dev) step += (uint64_t)(uint32_t)a.step_dev[0] | ((uint64_t)(uint32_t)a.step_dev[1] << 32);
  // a single sequence commits without waiting for anyone: its cache state is requested now (nothing but this kernel's
  // own commit changes it), so that the commit at the end is stores only
  const bool solo = a.kv.len != nullptr && a.B == 1;
  int st_len = 0, st_npend = 0, st_owned = 0, st_top = 0, st_err = 0, st_launch = 0;
  uint32_t st_dev_err = 0;
  if (solo && tid == 0) {
    st_len = a.kv.len[seq]; st_npend = a.kv.n_pend[seq]; st_owned = a.kv.owned[seq];
    st_top = a.kv.ctl[0]; st_err = a.kv.ctl[1]; st_launch = a.kv.ctl[3]; st_dev_err = *a.kv.err;
  }

  if (tid < WAVE) {
    bool acc = false;
    if (tid < K) {
      const int xi = min(max(a.x[b * K + tid], 0), V - 1);
      const float ptx = pt[(size_t)tid * V + xi], pdx = pd[(size_t)tid * V + xi];
      const float r = a.uniforms ? a.uniforms[b * (K + 1) + tid] : philox_uniform(a.seed, seq, step, a.slot_base + tid);
      float thr;
      if (pdx > ptx) thr = __fadd_rn(__fdiv_rn(ptx, pdx), a.beta);
      else thr = __fadd_rn(1.0f, a.beta);
      acc = r < thr;
    }
    const unsigned long long rej = ~__ballot(acc);          // lanes >= K vote "reject"
    if (tid == 0) sh_n = min(__ffsll((long long)rej) - 1, K);
  }
  if (tid == WAVE)                                         // the uniform of the draw: one thread of the second wave
    sh_u = a.uniforms ? a.uniforms[b * (K + 1) + K] : philox_uniform(a.seed, seq, step, a.slot_base + K);
  __syncthreads();
  const int n = sh_n;
  const float u = sh_u;
  const float* prow = (lds_row0 && n == 0) ? lds_row0 : pt + (size_t)n * V;
  const float* drow = pd + (size_t)n * V;                   // only read when n < K
  const int per = (V + SBLOCK - 1) / SBLOCK;                // contiguous span of indices per thread (<= SP)
  const int j0 = tid * per;
  int fallback = 0;
  bool residual = n < K;
  unsigned long long total, excl, mine;
  float wgt[SP];
  for (;;) {
    // the thread's span of weights, all loads in flight together
#pragma unroll
    for (int e = 0; e < SP; ++e) {
      const int j = j0 + e;
      wgt[e] = 0.f;
      if (e < per && j < V) wgt[e] = residual ? fmaxf(__fsub_rn(prow[j], drow[j]), 0.f) : prow[j];
    }
    mine = 0;
#pragma unroll
    for (int e = 0; e < SP; ++e) mine += fix40(wgt[e]);
    excl = sblock_excl_scan_u64(mine, w16, &total);          // sum of the spans before this thread's, and of all
    if (total == 0 && residual) { residual = false; fallback = 1; continue; }
    break;
  }
  if (total == 0) {
    if (tid == 0) sh_tok = 0;
  } else {
    const unsigned long long Ru = (unsigned long long)(u * 16777216.0f);
    const unsigned long long tgt = (__umul64hi(total, Ru) << 40) | ((total * Ru) >> 24);   // floor(total*Ru / 2^24)
    if (excl <= tgt && tgt < excl + mine) {
      unsigned long long c = excl;
      int tok = min(j0 + per, V) - 1;
      bool found = false;
#pragma unroll
      for (int e = 0; e < SP; ++e) {
        c += fix40(wgt[e]);
        if (!found && c > tgt) { tok = j0 + e; found = true; }
      }
      sh_tok = tok;
    }
  }
  __syncthreads();
  if (tid == 0) {
    if (a.n_acc) a.n_acc[b] = n;
    a.next_tok[(size_t)b * a.tok_stride] = sh_tok;
    if (a.flags) a.flags[b] = fallback;
  }
  if (a.kv.len == nullptr) return;
  if (solo) {                                              // kv_truncate + kv_publish on the values read at the start
    if (tid == 0) {
      if (a.bump_launch) a.kv.ctl[3] = st_launch + 1;
      if (a.bump_step && a.step_dev) {
        const uint64_t nx = step - a.step + 1;
        ((int32_t*)a.step_dev)[0] = (int32_t)(uint32_t)nx;
        ((int32_t*)a.step_dev)[1] = (int32_t)(uint32_t)(nx >> 32);
      }
      a.kv.mirror[2 * a.kv.max_seqs] = st_err;
      a.kv.mirror[2 * a.kv.max_seqs + 1] = (int32_t)st_dev_err;
      if (st_dev_err) return;                              // the forward did not finish: its logits mean nothing, commit nothing
      const int new_len = st_len + st_npend + n;
      const int keep = ceil_div(new_len, a.kv.bt);
      int own = st_owned, top = st_top;
      while (own > keep) {
        --own;
        a.kv.free_stack[top++] = a.kv.table[seq * a.kv.mbps + own];
        a.kv.table[seq * a.kv.mbps + own] = -1;
      }
      a.kv.owned[seq] = own;
      a.kv.ctl[0] = top;
      a.kv.len[seq] = new_len;
      a.kv.pend[seq * 2] = sh_tok;
      a.kv.n_pend[seq] = 1;
      a.kv.mirror[2 * seq] = new_len;
      a.kv.mirror[2 * seq + 1] = 1;
    }
    return;
  }
  // ---- commit by the last workgroup to arrive
  if (tid == 0) {
    __threadfence();
    const int arrived = atomicAdd(a.ticket, 1);
    sh_last = (arrived == a.B - 1);
  }
  __syncthreads();
  if (!sh_last || tid != 0) return;
  __threadfence();
  *a.ticket = 0;
  if (a.bump_launch) kv_bump_launch(a.kv);
  if (a.bump_step && a.step_dev) {
    const uint64_t nx = step - a.step + 1;
    ((int32_t*)a.step_dev)[0] = (int32_t)(uint32_t)nx;
    ((int32_t*)a.step_dev)[1] = (int32_t)(uint32_t)(nx >> 32);
  }
  if (*a.kv.err) { kv_publish_flags(a.kv); return; }        // the forward did not finish: commit nothing
  for (int s = 0; s < a.B; ++s) {
    const int sq = a.seq0 + s;
    const int nn = a.n_acc ? ((volatile int32_t*)a.n_acc)[s] : 0;
    const int tok = ((volatile int32_t*)a.next_tok)[(size_t)s * a.tok_stride];
    kv_truncate(a.kv, sq, a.kv.len[sq] + a.kv.n_pend[sq] + nn);
    a.kv.pend[sq * 2] = tok;
    a.kv.n_pend[sq] = 1;
    kv_publish(a.kv, sq);
  }
}

template <int SP>
__global__ void __launch_bounds__(SBLOCK) k_accept(AcceptArgs a) { accept_seq<SP>(a, blockIdx.x); }

// One row per sequence (a draft step, an autoregressive step): the row's distribution and the token drawn from it in
// one launch.  The probabilities go to memory (the caller wants the row) and, for the draw, through LDS (the halves
// assign elements to threads differently); the arithmetic is that of the two kernels above, bit for bit.
template <int SP>
__global__ void __launch_bounds__(SBLOCK) k_warp_accept(WarpArgs w, AcceptArgs a) {
  constexpr bool STAGE = SP <= 8;                           // 32 KB of LDS; the larger instantiation re-reads the row from memory
  __shared__ float row_probs[STAGE ? SP * SBLOCK : 1];
  float* lds_row = (STAGE && a.K == 0) ? row_probs : nullptr;   // K == 0: the row of the draw is the row just computed
  warp_softmax_row<SP>(w, blockIdx.x, lds_row);
  __threadfence_block();
  __syncthreads();
  accept_seq<SP>(a, blockIdx.x, lds_row);
}

// ------------------------------------------------------------------------------------------ small state kernels
// Truncate one sequence and (optionally) set its pending token from a value or from device memory.  new_len >= 0 is a
// rollback: a target beyond the cached length is refused (the state stays, KV_ERR_ROLLBACK is raised).  add_len is
// the commit of a prefill chunk.  after_forward: the kernel follows a forward on this cache (advances its launch number;
// commits nothing if that forward did not finish).
__global__ void k_kv_set(KvView kv, int seq, int new_len, int add_len, int set_pending, int pending_value,
                         const int32_t* pending_ptr, int after_forward) {
  if (threadIdx.x || blockIdx.x) return;
  if (after_forward) kv_bump_launch(kv);
  if (*kv.err) { kv_publish_flags(kv); return; }
  if (new_len > kv.len[seq]) { kv.ctl[1] |= KV_ERR_ROLLBACK; kv_publish_flags(kv); return; }
  const int target = new_len >= 0 ? new_len : kv.len[seq] + add_len;
  kv_truncate(kv, seq, target);
  if (set_pending) {
    kv.pend[seq * 2] = pending_ptr ? *pending_ptr : pending_value;
    kv.n_pend[seq] = 1;
  }
  kv_publish(kv, seq);
}

// Draft cache after a verification of K drafts (see ssd_kv_follow).
__global__ void k_kv_follow(KvView kv, int n_seqs, int K, const int32_t* n_acc, const int32_t* next_tok,
                            const int32_t* x, int32_t* step_dev) {
  if (threadIdx.x || blockIdx.x) return;
  if (step_dev) {                                          // last kernel of a captured cycle: the next replay is the next step
    const uint64_t nx = ((uint64_t)(uint32_t)step_dev[0] | ((uint64_t)(uint32_t)step_dev[1] << 32)) + 1;
    step_dev[0] = (int32_t)(uint32_t)nx;
    step_dev[1] = (int32_t)(uint32_t)(nx >> 32);
  }
  if (*kv.err) { kv_publish_flags(kv); return; }
  for (int s = 0; s < n_seqs; ++s) {
    const int n = n_acc[s];
    if (n < K) {
      kv_truncate(kv, s, kv.len[s] - (K - 1 - n));
      kv.pend[s * 2] = next_tok[s];
      kv.n_pend[s] = 1;
    } else {
      kv.pend[s * 2] = x[s * K + K - 1];
      kv.pend[s * 2 + 1] = next_tok[s];
      kv.n_pend[s] = 2;
    }
    kv_publish(kv, s);
  }
}

__global__ void k_kv_init(KvView kv) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < kv.n_blocks) kv.free_stack[i] = kv.n_blocks - 1 - i;       // lowest id on top
  if (i < kv.max_seqs) {
    kv.len[i] = 0; kv.n_pend[i] = 0; kv.pend[2 * i] = 0; kv.pend[2 * i + 1] = 0; kv.owned[i] = 0;
    kv.mirror[2 * i] = 0; kv.mirror[2 * i + 1] = 0;
  }
  if (i < kv.max_seqs * kv.mbps) kv.table[i] = -1;
  if (i == 0) {
    kv.ctl[0] = kv.n_blocks; kv.ctl[1] = 0; kv.ctl[2] = 0; kv.ctl[3] = 1; kv.ctl[4] = 0; kv.ctl[5] = 0;
    kv.mirror[2 * kv.max_seqs] = 0; kv.mirror[2 * kv.max_seqs + 1] = 0;
  }
}

// Clears the sticky error state (the caller has re-zeroed the barrier words and the tagged workspace on the same stream)
// and restarts the launch numbering; sequence state is left as it is.
__global__ void k_kv_clear_error(KvView kv) {
  if (threadIdx.x || blockIdx.x) return;
  kv.ctl[1] = 0; kv.ctl[2] = 0; kv.ctl[3] = 1;
  *kv.err = 0u;
  kv_publish_flags(kv);
}

// Clears n 32-bit words (a kernel, not a memset: callers may be capturing the stream).
__global__ void k_zero_words(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Test hook: raise device error bits / set the launch number (see ssd_kv_test_hook).
__global__ void k_kv_poke(KvView kv, uint32_t err_bits, int launch_no) {
  if (threadIdx.x || blockIdx.x) return;
  if (err_bits) *kv.err = *kv.err | err_bits;
  if (launch_no > 0) kv.ctl[3] = launch_no;
}

// Rotary table: (cos, sin)(pos * base^(-2i/hd)) evaluated in fp64, rounded once to fp32.
__global__ void k_rope_table(float2* tab, int max_pos, int half, double base) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= max_pos * half) return;
  const int pos = i / half, f = i - pos * half;
  const double ang = (double)pos * pow(base, -(double)f / (double)half);
  tab[i] = make_float2((float)cos(ang), (float)sin(ang));
}

}  // namespace ssd
