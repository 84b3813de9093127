// Skinny GEMMs of the decoder: Y[M,N] = X[M,Kd] . W[N,Kd]^T with M = rows of one forward (<= 512).
// Up to a few tens of rows the work is weight streaming: every weight byte is read once, coalesced, and the
// contraction runs on MFMA 16x16x32 bf16 tiles (rows padded to 16; padded rows cost nothing that matters).
//
// Work decomposition, identical for both storage types:
//   a workgroup (4 waves) owns two 16-column tiles (t0 from W0, t1 from W1) and one global k-split;
//   its waves split the k range between them, partial tiles are summed through LDS in a fixed order,
//   and one thread per (row, col) applies the epilogue.  Nothing is accumulated with atomics, so every output
//   element has one summation order that does not depend on M: a row computed alone (autoregressive step)
//   and the same row computed among K+1 (verification) give the same bits.
//
// bf16 weights are pre-packed so that a wave reads one tile (16 out-features x 32 in-features) as 64
// consecutive 16-byte pieces: piece l of tile (nt, kt) = W[nt*16 + l%16][kt*32 + 8*(l/16) .. +7], tiles ordered
// [nt][kt].  That is exactly the B-operand fragment of the MFMA, so a weight goes from HBM to the matrix
// core through one dwordx4 load and nothing else.
#pragma once
#include "common.h"

namespace ssd {

enum { EPI_PARTIAL = 0, EPI_QKV = 1, EPI_SWIGLU = 2 };

struct GemmArgs {
  const void* A;     // activations [M][lda]
  int lda;
  const void* W0;    // weight matrix of tile slot 0 (packed bf16, or canonical fp32 [N][K])
  const void* W1;    // weight matrix of tile slot 1
  int M, N, K;       // N = out features of one matrix (unpadded)
  int gs;            // global k-splits
  // EPI_PARTIAL: out[s][m][n]
  float* out;
  size_t out_split_stride;
  int ldo;
  // EPI_QKV: bias, rotary table, destination of q and of the cache rows
  const float* bias;
  const float2* rope;   // [pos][hd/2] (cos, sin)
  Rows rows;
  float* q;             // [M][nq*hd]
  KvView kv;
  int layer, nq;
  // EPI_SWIGLU
  void* act;            // [M][N]
  int act_split_kt;     // > 0: act is written as split rows (common.h) with this many k-tiles per row (N / 32)
};

// ------------------------------------------------------------------------------------------ epilogues
template <int EPI, typename AT, typename KVT>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs& g, int t0, int t1, int split, int row, int col,
                                              float v0, float v1) {
  if (row >= g.M) return;
  if (EPI == EPI_PARTIAL) {
    float* o = g.out + (size_t)split * g.out_split_stride + (size_t)row * g.ldo;
    const int n0 = t0 * 16 + col, n1 = t1 * 16 + col;
    if (n0 < g.N) o[n0] = v0;
    if (n1 < g.N) o[n1] = v1;
  } else if (EPI == EPI_SWIGLU) {
    const int n = t0 * 16 + col;
    if (n < g.N) {
      const float s = v0 / (1.0f + expf(-v0));
      if (g.act_split_kt > 0) st_split_value((bf16_t*)g.act, g.act_split_kt, row, n, s * v1);
      else AT::st((typename AT::T*)g.act + (size_t)row * g.N + n, s * v1);
    }
  } else {  // EPI_QKV: the two tiles hold dims d and d + hd/2 of one head
    const int hd = g.kv.hd, half = hd >> 1;
    const int n0 = t0 * 16 + col;
    const int head = n0 / hd, d = n0 - head * hd;
    if (g.bias) { v0 += g.bias[n0]; v1 += g.bias[n0 + half]; }
    const int nq = g.nq, nkv = g.kv.nkv;
    const int pos = g.rows.pos[row];
    if (head < nq + nkv) {
      const float2 cs = g.rope[(size_t)pos * half + d];
      const float r0 = v0 * cs.x - v1 * cs.y;
      const float r1 = v1 * cs.x + v0 * cs.y;
      v0 = r0; v1 = r1;
    }
    if (head < nq) {
      float* qo = g.q + (size_t)row * nq * hd + head * hd + d;
      qo[0] = v0; qo[half] = v1;
    } else if (g.rows.active[row]) {
      const int which = head < nq + nkv ? 0 : 1;
      const int kvh = head - nq - which * nkv;
      const int seq = g.rows.seq0 + row / g.rows.R;
      const int blk = g.kv.table[seq * g.kv.mbps + pos / g.kv.bt];
      if (blk >= 0) {
        typename KVT::T* base = (typename KVT::T*)g.kv.pool + kv_offset(g.kv, g.layer, which, blk, kvh, 0);
        const int tok = pos % g.kv.bt;
        if (which == 0) {                                   // keys: [token][dim]
          KVT::st(base + tok * hd + d, v0);
          KVT::st(base + tok * hd + d + half, v1);
        } else {                                            // values: [dim][token] (token-minor)
          KVT::st(base + d * g.kv.bt + tok, v0);
          KVT::st(base + (d + half) * g.kv.bt + tok, v1);
        }
      }
    }
  }
}

template <int EPI>
__device__ __forceinline__ bool gemm_tiles(const GemmArgs& g, int item, int hd, int& t0, int& t1, int& split) {
  const int ntiles = (g.N + 15) >> 4;
  if (EPI == EPI_PARTIAL) {
    const int npairs = (ntiles + 1) >> 1;
    split = item / npairs;
    const int p = item - split * npairs;
    t0 = 2 * p; t1 = 2 * p + 1;
  } else if (EPI == EPI_SWIGLU) {
    split = 0; t0 = item; t1 = item;
  } else {
    const int per_head = hd >> 5;              // pairs of tiles per head
    const int head = item / per_head, i = item - head * per_head;
    split = 0; t0 = head * (hd >> 4) + i; t1 = t0 + per_head;
  }
  return t0 < ntiles;
}

// Sum the four waves' partial tiles (fixed order) and run the epilogue: thread tid owns (row tid/16, col tid%16).
template <int EPI, typename AT, typename KVT>
__device__ __forceinline__ void gemm_reduce_tile(const GemmArgs& g, float (*red)[2][256], int t0, int t1, int split,
                                                 int mt) {
  const int tid = threadIdx.x;
  const float v0 = (red[0][0][tid] + red[1][0][tid]) + (red[2][0][tid] + red[3][0][tid]);
  const float v1 = (red[0][1][tid] + red[1][1][tid]) + (red[2][1][tid] + red[3][1][tid]);
  gemm_epilogue<EPI, AT, KVT>(g, t0, t1, split, mt * 16 + (tid >> 4), tid & 15, v0, v1);
}

// grid.x = work items (tile pairs x global splits); grid.y = groups of MT 16-row tiles of M (a workgroup reads its
// weights once for its MT row tiles; more groups = more workgroups for the same weights).  A is fp32 [M][lda].
template <int MT, int EPI, typename KVT>
__global__ void __launch_bounds__(BLOCK) k_gemm_bf16(GemmArgs g) {
  __shared__ float red[4][2][256];
  int t0, t1, split;
  if (!gemm_tiles<EPI>(g, blockIdx.x, g.kv.hd, t0, t1, split)) return;
  const int ntiles = (g.N + 15) >> 4;
  const bool has1 = (EPI != EPI_PARTIAL) || (t1 < ntiles);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int KT = g.K >> 5;
  const int mt0 = blockIdx.y * MT;
  // k-tiles of this workgroup, then of this wave (contiguous ranges, earlier ranges get the remainder)
  const int per_s = KT / g.gs, rem_s = KT - per_s * g.gs;
  const int wg_b = split * per_s + min(split, rem_s), wg_n = per_s + (split < rem_s ? 1 : 0);
  const int per_w = wg_n >> 2, rem_w = wg_n & 3;
  const int kb = wg_b + wave * per_w + min(wave, rem_w), ke = kb + per_w + (wave < rem_w ? 1 : 0);

  const u32x4* w0 = (const u32x4*)g.W0 + (size_t)t0 * KT * 64 + lane;
  const u32x4* w1 = (const u32x4*)g.W1 + (size_t)(has1 ? t1 : t0) * KT * 64 + lane;
  const float* A = (const float*)g.A;
  const int arow = lane & 15, akoff = (lane >> 4) * 8;

  f32x4 acc[MT][2];
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) { acc[mt][0] = f32x4{0, 0, 0, 0}; acc[mt][1] = f32x4{0, 0, 0, 0}; }

  constexpr int U = 4;
  int kt = kb;
  for (; kt + U <= ke; kt += U) {
    u32x4 b0[U], b1[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      b0[u] = __builtin_nontemporal_load(w0 + (size_t)(kt + u) * 64);
      b1[u] = __builtin_nontemporal_load(w1 + (size_t)(kt + u) * 64);
    }
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int row = (mt0 + mt) * 16 + arow;
      u32x4 a[U][2];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        a[u][0] = u32x4{0u, 0u, 0u, 0u};
        a[u][1] = u32x4{0u, 0u, 0u, 0u};
        if (row < g.M) {
          const u32x4* ap = (const u32x4*)(A + (size_t)row * g.lda + (kt + u) * 32 + akoff);
          a[u][0] = ap[0];
          a[u][1] = ap[1];
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const SplitA av = split_bf16(a[u][0], a[u][1]);
        const bf16x8 bv0 = __builtin_bit_cast(bf16x8, b0[u]), bv1 = __builtin_bit_cast(bf16x8, b1[u]);
        acc[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.lo, bv0, acc[mt][0], 0, 0, 0);
        acc[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.lo, bv1, acc[mt][1], 0, 0, 0);
        acc[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.hi, bv0, acc[mt][0], 0, 0, 0);
        acc[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.hi, bv1, acc[mt][1], 0, 0, 0);
      }
    }
  }
  for (; kt < ke; ++kt) {
    const bf16x8 bv0 = __builtin_bit_cast(bf16x8, __builtin_nontemporal_load(w0 + (size_t)kt * 64));
    const bf16x8 bv1 = __builtin_bit_cast(bf16x8, __builtin_nontemporal_load(w1 + (size_t)kt * 64));
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      const int row = (mt0 + mt) * 16 + arow;
      u32x4 a0 = u32x4{0u, 0u, 0u, 0u}, a1 = u32x4{0u, 0u, 0u, 0u};
      if (row < g.M) {
        const u32x4* ap = (const u32x4*)(A + (size_t)row * g.lda + kt * 32 + akoff);
        a0 = ap[0];
        a1 = ap[1];
      }
      const SplitA av = split_bf16(a0, a1);
      acc[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.lo, bv0, acc[mt][0], 0, 0, 0);
      acc[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.lo, bv1, acc[mt][1], 0, 0, 0);
      acc[mt][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.hi, bv0, acc[mt][0], 0, 0, 0);
      acc[mt][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av.hi, bv1, acc[mt][1], 0, 0, 0);
    }
  }
  // accumulator register r of lane l is element (row 4*(l/16)+r, col l%16) of the 16x16 tile
  const int obase = ((lane >> 4) * 4) * 16 + (lane & 15);
#pragma unroll
  for (int mt = 0; mt < MT; ++mt) {
    if ((mt0 + mt) * 16 < g.M) {
      __syncthreads();
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        red[wave][0][obase + r * 16] = acc[mt][0][r];
        red[wave][1][obase + r * 16] = acc[mt][1][r];
      }
      __syncthreads();
      gemm_reduce_tile<EPI, F32, KVT>(g, red, t0, has1 ? t1 : ntiles, split, mt0 + mt);
    }
  }
}

// -------------------------------------------------------------------------------------- many rows
// With several row tiles the decomposition above re-reads the activations once per pair of column tiles, and that
// traffic, not the weights, sets the time of the wide operators.  Here a workgroup of 8 waves takes MTW row tiles
// x 8 column-tile pairs (x one k-slice for the operators whose output is k-split partials): the rows' activations
// are split into hi + lo bf16 once per workgroup and parked in LDS in A-fragment order, a chunk of KC k-tiles at a
// time (MTW * KC * 2 KB), and every wave runs its own pair over the whole k range of the workgroup against them,
// so nothing is reduced across waves.  Weight fragments are prefetched U k-tiles ahead, across chunk boundaries,
// so they travel while the next chunk is staged.  Accumulation order of an element: k ascending, lo before hi.
constexpr int WIDE_WAVES = 8;              // waves per workgroup of the shape for about a hundred rows
constexpr int WIDE_LDS_BYTES = 128 * 1024;
constexpr int WIDE_MAX_MTW = 8;
constexpr int WIDE_SG = 4;                 // activation fragments a thread stages per chunk

struct WideArgs {
  int KC;            // k-tiles per staged chunk (multiple of 4, MTW * KC <= WIDE_SG * waves, two buffers of MTW * KC * 2 KB)
  int slice_kt;      // k-tiles per workgroup (multiple of 4; the whole k range for the SwiGLU epilogue)
  int n_slices, n_rowg, n_colg;
};

// W waves per workgroup, NPW column-tile pairs per wave; (8, 1) is the shape described above and the one that is
// launched (some tens of rows up to 255; from 256 rows on the kernels of gemm_rows.h take over).
template <int MTW, int EPI, int W, int NPW>
__global__ void __launch_bounds__(W * 64, W == 4 ? 2 : 1) k_gemm_wide(GemmArgs g, WideArgs wa) {
  extern __shared__ u32x4 afrag[];                        // two buffers of [(mt * KC + kt in chunk) * 2 + {hi, lo}][lane]
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int KT = g.K >> 5, KC = wa.KC;
  // Workgroups are dealt to the 8 XCDs round-robin by their index; the row groups of one (column group, slice) take
  // indices that differ by 8, so they run on one XCD, close in time, and all but the first find the weights in its L2.
  const int ntiles = (g.N + 15) >> 4;
  const int xk = blockIdx.x >> 3;
  const int per_col = wa.n_rowg * wa.n_slices;
  const int colg = (xk / per_col) * 8 + (blockIdx.x & 7);
  const int rem = xk % per_col;
  const int mt0 = (rem % wa.n_rowg) * MTW, slice = rem / wa.n_rowg;
  if (colg >= wa.n_colg) return;
  const int kb = slice * wa.slice_kt, ke = min(KT, kb + wa.slice_kt);
  constexpr int NT = 2 * NPW;                             // column tiles of a wave: slot 2q from W0, slot 2q + 1 from W1
  int tl[NT];
  const u32x4* wp[NT];
#pragma unroll
  for (int q = 0; q < NPW; ++q) {
    const int pair = (colg * W + wave) * NPW + q;
    tl[2 * q] = EPI == EPI_SWIGLU ? pair : 2 * pair;
    tl[2 * q + 1] = EPI == EPI_SWIGLU ? pair : 2 * pair + 1;
    wp[2 * q] = (const u32x4*)g.W0 + (size_t)(tl[2 * q] < ntiles ? tl[2 * q] : 0) * KT * 64 + lane;
    wp[2 * q + 1] = (const u32x4*)g.W1 + (size_t)(tl[2 * q + 1] < ntiles ? tl[2 * q + 1] : 0) * KT * 64 + lane;
  }
  constexpr int U = 4;                                    // k-tiles of weights in flight per wave and tile (KC % 4 == 0)
  u32x4 bw[NT][U];
#pragma unroll
  for (int t = 0; t < NT; ++t)
#pragma unroll
    for (int u = 0; u < U; ++u) {
      bw[t][u] = u32x4{0u, 0u, 0u, 0u};
      if (kb + u < ke) bw[t][u] = wp[t][(size_t)(kb + u) * 64];
    }
  const float* A = (const float*)g.A;
  f32x4 acc[MTW][NT];
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[mt][t] = f32x4{0, 0, 0, 0};
  // The rows' activations go through LDS a chunk of KC k-tiles at a time, two buffers: the loads of chunk c + 1 are
  // in flight (in registers) while chunk c is contracted, and are split and written to the other buffer afterwards.
  // A thread holds WIDE_SG fragments (16 floats each: KC * MTW <= WIDE_SG * W); one barrier per chunk.
  u32x4 x0[WIDE_SG], x1[WIDE_SG];
  auto load_chunk = [&](int kt0) {
    const int n = min(KC, ke - kt0), total = MTW * n * 64;
#pragma unroll
    for (int u = 0; u < WIDE_SG; ++u) {
      const int i = tid + u * W * 64;
      const int l = i & 63, f = i >> 6;                   // f = k-tile in chunk * MTW + mt (division by a constant)
      const int kk = f / MTW, mt = f - kk * MTW;
      const int row = (mt0 + mt) * 16 + (l & 15);
      x0[u] = u32x4{0u, 0u, 0u, 0u};
      x1[u] = x0[u];
      if (i < total && row < g.M) {
        const u32x4* ap = (const u32x4*)(A + (size_t)row * g.lda + (kt0 + kk) * 32 + (l >> 4) * 8);
        x0[u] = ap[0];
        x1[u] = ap[1];
      }
    }
  };
  auto store_chunk = [&](int kt0, u32x4* buf) {
    const int n = min(KC, ke - kt0), total = MTW * n * 64;
#pragma unroll
    for (int u = 0; u < WIDE_SG; ++u) {
      const int i = tid + u * W * 64;
      if (i < total) {
        const int l = i & 63, f = i >> 6;
        const int kk = f / MTW, mt = f - kk * MTW;
        const SplitA sp = split_bf16(x0[u], x1[u]);
        buf[((mt * KC + kk) * 2) * 64 + l] = __builtin_bit_cast(u32x4, sp.hi);
        buf[((mt * KC + kk) * 2 + 1) * 64 + l] = __builtin_bit_cast(u32x4, sp.lo);
      }
    }
  };
  const int buf_words = MTW * KC * 2 * 64;                // u32x4 elements of one buffer
  load_chunk(kb);
  int cidx = 0;
  for (int c0 = kb; c0 < ke; c0 += KC, ++cidx) {
    u32x4* buf = afrag + (cidx & 1) * buf_words;
    store_chunk(c0, buf);
    __syncthreads();
    if (c0 + KC < ke) load_chunk(c0 + KC);
    const int cend = min(ke, c0 + KC);
    for (int kt0 = c0; kt0 < cend; kt0 += U) {
      // slot u holds k-tile kt0 + u and is refilled with k-tile kt0 + U + u as soon as its MFMAs are issued: U - 1
      // k-tiles of weights stay in flight behind the one being contracted
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (kt0 + u < cend) {
#pragma unroll
          for (int mt = 0; mt < MTW; ++mt) {
            const int f = mt * KC + (kt0 + u - c0);
            const bf16x8 hi = __builtin_bit_cast(bf16x8, buf[(f * 2) * 64 + lane]);
            const bf16x8 lo = __builtin_bit_cast(bf16x8, buf[(f * 2 + 1) * 64 + lane]);
#pragma unroll
            for (int t = 0; t < NT; ++t)
              acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo, __builtin_bit_cast(bf16x8, bw[t][u]), acc[mt][t], 0, 0, 0);
#pragma unroll
            for (int t = 0; t < NT; ++t)
              acc[mt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi, __builtin_bit_cast(bf16x8, bw[t][u]), acc[mt][t], 0, 0, 0);
          }
        }
        if (kt0 + U + u < ke) {
#pragma unroll
          for (int t = 0; t < NT; ++t) bw[t][u] = wp[t][(size_t)(kt0 + U + u) * 64];
        }
      }
    }
  }
  // accumulator register r of lane l is element (row 4*(l/16)+r, col l%16) of the 16x16 tile
#pragma unroll
  for (int q = 0; q < NPW; ++q)
#pragma unroll
  for (int mt = 0; mt < MTW; ++mt)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int n0 = tl[2 * q] * 16 + (lane & 15), n1 = tl[2 * q + 1] * 16 + (lane & 15);
      const int row = (mt0 + mt) * 16 + (lane >> 4) * 4 + r;
      if (row < g.M) {
        const float v0 = acc[mt][2 * q][r], v1 = acc[mt][2 * q + 1][r];
        if (EPI == EPI_SWIGLU) {
          if (n0 < g.N) {
            const float sg = v0 / (1.0f + expf(-v0));
            ((float*)g.act)[(size_t)row * g.N + n0] = sg * v1;
          }
        } else {
          float* o = g.out + (size_t)slice * g.out_split_stride + (size_t)row * g.ldo;
          if (n0 < g.N) o[n0] = v0;
          if (n1 < g.N) o[n1] = v1;
        }
      }
    }
}

// -------------------------------------------------------------------------------------- fp32 / VALU
// Same decomposition for the fp32 parity configuration; weights canonical [N][K] fp32, K % 32 == 0.
template <int EPI, typename KVT>
__global__ void __launch_bounds__(BLOCK) k_gemm_f32(GemmArgs g) {
  __shared__ float red[4][2][256];
  int t0, t1, split;
  if (!gemm_tiles<EPI>(g, blockIdx.x, g.kv.hd, t0, t1, split)) return;
  const int ntiles = (g.N + 15) >> 4;
  const bool has1 = (EPI != EPI_PARTIAL) || (t1 < ntiles);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int KT = g.K >> 5;
  const int per_s = KT / g.gs, rem_s = KT - per_s * g.gs;
  const int wg_b = split * per_s + min(split, rem_s), wg_n = per_s + (split < rem_s ? 1 : 0);
  const int per_w = wg_n >> 2, rem_w = wg_n & 3;
  const int kb = wg_b + wave * per_w + min(wave, rem_w), ke = kb + per_w + (wave < rem_w ? 1 : 0);
  const int col = lane & 15, kg = lane >> 4;
  const int n0 = min(t0 * 16 + col, g.N - 1), n1 = min((has1 ? t1 : t0) * 16 + col, g.N - 1);
  const float* w0 = (const float*)g.W0 + (size_t)n0 * g.K;
  const float* w1 = (const float*)g.W1 + (size_t)n1 * g.K;
  const float* A = (const float*)g.A;
  const int MTn = (g.M + 15) >> 4;
  for (int mt = 0; mt < MTn; ++mt) {
    float a0[16], a1[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) { a0[r] = 0.f; a1[r] = 0.f; }
    const int rows = min(16, g.M - mt * 16);
    for (int k = kb * 32 + kg; k < ke * 32; k += 4) {
      const float x0 = w0[k], x1 = w1[k];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (r < rows) {
          const float a = A[(size_t)(mt * 16 + r) * g.lda + k];
          a0[r] = fmaf(a, x0, a0[r]);
          a1[r] = fmaf(a, x1, a1[r]);
        }
      }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float s0 = a0[r], s1 = a1[r];
      s0 += __shfl_xor(s0, 16, WAVE); s0 += __shfl_xor(s0, 32, WAVE);
      s1 += __shfl_xor(s1, 16, WAVE); s1 += __shfl_xor(s1, 32, WAVE);
      if (kg == 0) { red[wave][0][r * 16 + col] = s0; red[wave][1][r * 16 + col] = s1; }
    }
    __syncthreads();
    gemm_reduce_tile<EPI, F32, KVT>(g, red, t0, has1 ? t1 : ntiles, split, mt);
  }
}

// Repack a canonical bf16 matrix [N][K] into MFMA B-fragment tiles (see the top of this file).
// One thread per 16-byte piece; rows >= N are zero.
__global__ void k_pack_bf16(const bf16_t* __restrict__ w, uint4* __restrict__ out, int N, int K, int ntiles) {
  const int KT = K >> 5;
  const size_t total = (size_t)ntiles * KT * 64;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    const int l = (int)(i & 63);
    const size_t tile = i >> 6;
    const int kt = (int)(tile % KT), nt = (int)(tile / KT);
    const int n = nt * 16 + (l & 15), k = kt * 32 + (l >> 4) * 8;
    uint4 v = uint4{0, 0, 0, 0};
    if (n < N) v = *(const uint4*)(w + (size_t)n * K + k);
    out[i] = v;
  }
}

}  // namespace ssd
