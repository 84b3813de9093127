// GEMMs of the decoder for some hundreds of rows (prefill chunks, very large batches):
// Y[M,N] = X[M,Kd] . W[N,Kd]^T on MFMA 16x16x32 bf16 tiles.
//
// With a few rows the projections are weight streaming and a workgroup may re-read the activations per column tile
// (gemm.h); with about a hundred rows the kernel that shares the rows through LDS serves (k_gemm_wide).  From a few
// hundred rows on, what sets the time is how many bytes a CU takes in (measured: 40-45 GB/s per CU whatever the depth of
// prefetch), so a workgroup has to own as large a tile of the output as its registers hold: a workgroup of WM x WN waves
// owns (WM*TM*16) rows x (WN*TN) weight tiles (x one k-slice where the output is k-split partials), and a wave owns
// TM row tiles x TN weight tiles of it over the workgroup's whole k range:
//   - the activations arrive as split rows (common.h): hi and lo bf16 in A-fragment order, written that way by whatever
//     produced them, so that a fragment is one contiguous kilobyte.  (Fragments gathered from row-major fp32 rows touch
//     sixteen cache lines per load instruction, and the address path, not the data, then sets the kernel's time.)
//   - a wave loads its row tiles' activation fragments itself; the WM waves that share weight tiles each load a
//     1/WM share of them (8-byte pieces, so that any TN divides evenly) and pass them round through LDS (two buffers,
//     one barrier per k-tile).  Loads are requested U k-tiles ahead;
//   - an activation fragment feeds 2*TN matrix-core instructions (lo, hi), a weight fragment 2*TM per wave;
//   - an output element is accumulated over k ascending, lo before hi, by one wave: nothing is reduced across waves.
// Workgroup index -> (XCD, column block, row block, slice) such that what an XCD's workgroups read overlaps as much as
// possible (see the index map in the kernel): every XCD has its own L2.
#pragma once
#include "gemm.h"

namespace ssd {

struct RowsPlan {
  int n_colb, n_rowb, n_slices, slice_kt;     // slice_kt: k-tiles per workgroup
};

template <int EPI, int TM, int TN, int WM, int WN, int U, int MINB>
__global__ void __launch_bounds__(WM * WN * 64, MINB) k_gemm_rows(GemmArgs g, RowsPlan p) {
  constexpr int RT = WM * TM;                  // row tiles of the workgroup
  constexpr int TS = TN * 2 / WM;              // 8-byte pieces of weight fragments a lane fetches per k-tile (a fragment: 128)
  static_assert((TN * 2) % WM == 0, "the waves of a column group share its weight fragments evenly");
  __shared__ u32x4 bsh[2][WN][TN][64];         // weight fragments of one k-tile per column group, two buffers
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave % WM, wn = wave / WM;
  const int KT = g.K >> 5, ntiles = (g.N + 15) >> 4;
  // blockIdx.x & 7 is the XCD a workgroup lands on.  Without k-slices an XCD takes whole column blocks (all their row blocks
  // find the weights in its L2); with k-slices it takes whole slices (their workgroups share both operands' k range).
  const int xk = blockIdx.x >> 3, xcd = blockIdx.x & 7;
  int colb, rowb, slice;
  if (p.n_slices > 1) {
    const int per = p.n_colb * p.n_rowb, rem = xk % per;
    slice = (xk / per) * 8 + xcd;
    colb = rem % p.n_colb; rowb = rem / p.n_colb;
    if (slice >= p.n_slices) return;                      // (the whole workgroup)
  } else {
    colb = (xk / p.n_rowb) * 8 + xcd;
    rowb = xk % p.n_rowb; slice = 0;
    if (colb >= p.n_colb) return;
  }
  const int row0 = (rowb * RT + wm * TM) * 16;            // first row of this wave
  const int kb = slice * p.slice_kt, ke = min(KT, kb + p.slice_kt), nk = ke - kb;
  // The workgroup walks its k-tiles in rotated order, starting at a k-tile that depends on its column block: workgroups
  // that start together would otherwise all read fragment k of tiles that lie a fixed stride (KT KB) apart.  (The same
  // order for all its waves: the column groups of a row group then ask for the same activation fragments at the same time.)
  const int rot = (int)(((unsigned)colb * 5u + (unsigned)slice * 3u) % (unsigned)nk);
  auto kt_of = [&](int kk) { const int t = kk + rot; return kb + (t >= nk ? t - nk : t); };
  // weight tiles of this wave's column group: slot j < TN.  SwiGLU: the first half from the gate matrix, the second half
  // the same rows of the up matrix; otherwise TN consecutive tiles of one matrix.
  const int cb = colb * WN + wn;
  int tl[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) tl[j] = EPI == EPI_SWIGLU ? cb * (TN / 2) + (j % (TN / 2)) : cb * TN + j;
  // share of this wave: piece (q * WM + wm) * 64 + lane of the TN * 128 pieces of a k-tile, i.e. half (q*WM + wm) & 1 of
  // the fragment of slot (q*WM + wm) / 2
  const uint2* wp[TS];
#pragma unroll
  for (int q = 0; q < TS; ++q) {
    const int j = (q * WM + wm) >> 1, half = (q * WM + wm) & 1;
    const int t = EPI == EPI_SWIGLU ? cb * (TN / 2) + (j % (TN / 2)) : cb * TN + j;
    const void* w = (EPI == EPI_SWIGLU && j >= TN / 2) ? g.W1 : g.W0;
    wp[q] = (const uint2*)w + (size_t)(t < ntiles ? t : 0) * KT * 128 + half * 64 + lane;
  }
  // activation fragments of row tile i, k-tile kt: hi at ((mt * KT + kt) * 2) * 64 + lane, lo 64 pieces further.  A row
  // tile wholly beyond M is not there: its slots re-read the last valid tile and its outputs are dropped.
  const u32x4* ap[TM];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int mt = min((row0 >> 4) + i, (g.M - 1) >> 4);
    ap[i] = (const u32x4*)g.A + (size_t)mt * KT * 128 + lane;
  }
  uint2 bm[U][TS];
  u32x4 a0[U][TM], a1[U][TM];
  auto request = [&](int u, int kt) {                      // slot u <- k-tile kt
#pragma unroll
    for (int q = 0; q < TS; ++q) bm[u][q] = wp[q][(size_t)kt * 128];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      a0[u][i] = ap[i][(size_t)kt * 128];
      a1[u][i] = ap[i][(size_t)kt * 128 + 64];
    }
  };
  // QKV epilogue: what an element's stores depend on (position, cache block, rotary factors) is requested here, ahead of
  // the k loop, so that the epilogue does not wait out three dependent round trips
  int pos[TM][4], blk[TM][4];
  bool on[TM][4];
  float2 cs[TM][4][TN / 2];
  if (EPI == EPI_QKV) {
    const int half = g.kv.hd >> 1;                           // (TN tiles are one head: head_dim == 16 * TN)
    const bool rot_head = cb < g.nq + g.kv.nkv;              // (WN == 1: the column group is one head)
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int row = row0 + i * 16 + (lane >> 4) * 4 + r;
        on[i][r] = row < g.M;
        pos[i][r] = on[i][r] ? g.rows.pos[row] : 0;
        const int active = on[i][r] ? g.rows.active[row] : 0;
        const int seq = g.rows.seq0 + (on[i][r] ? row : 0) / g.rows.R;
        blk[i][r] = active ? g.kv.table[seq * g.kv.mbps + pos[i][r] / g.kv.bt] : -1;
#pragma unroll
        for (int j = 0; j < TN / 2; ++j) {
          const int d = j * 16 + (lane & 15);
          cs[i][r][j] = rot_head ? g.rope[(size_t)pos[i][r] * half + d] : make_float2(1.f, 0.f);
        }
      }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) request(u, kt_of(min(u, nk - 1)));
  f32x4 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) acc[i][j] = f32x4{0, 0, 0, 0};
  // One k-tile: pass this wave's share of the weight fragments round, then contract.  A buffer is rewritten two k-tiles
  // later, after a barrier that every wave reaches only when it has read the buffer.
  auto step = [&](int u, int par) {
#pragma unroll
    for (int q = 0; q < TS; ++q) ((uint2*)bsh[par][wn])[(q * WM + wm) * 64 + lane] = bm[u][q];
    __syncthreads();
    u32x4 bw[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j) bw[j] = bsh[par][wn][j][lane];
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const bf16x8 hi = __builtin_bit_cast(bf16x8, a0[u][i]), lo = __builtin_bit_cast(bf16x8, a1[u][i]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(lo, __builtin_bit_cast(bf16x8, bw[j]), acc[i][j], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(hi, __builtin_bit_cast(bf16x8, bw[j]), acc[i][j], 0, 0, 0);
    }
  };
  // Whole groups of U k-tiles in a loop body without branches (slot u: use, then request the k-tile U ahead; past the end
  // the last k-tile is requested again and never used), so that the wait before a slot's use counts only the loads issued
  // after that slot's: U - 1 k-tiles stay in flight.  The scheduler is kept from moving the requests (left to itself it
  // collects them at the end of the body, and the next iteration then waits out a whole round trip).  U is even, so
  // slot parity is buffer parity.  Then the remaining k-tiles.
  static_assert(U % 2 == 0, "slot parity selects the LDS buffer");
  const int kfull = (nk / U) * U;
  for (int k0 = 0; k0 < kfull; k0 += U) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      step(u, u & 1);
      __builtin_amdgcn_sched_barrier(0);
      request(u, kt_of(min(k0 + u + U, nk - 1)));
      __builtin_amdgcn_sched_barrier(0);
    }
  }
#pragma unroll
  for (int u = 0; u < U - 1; ++u)
    if (kfull + u < nk) step(u, u & 1);                    // (uniform over the workgroup)
  if (row0 >= g.M) return;
  // accumulator register r of lane l is element (row 4*(l/16)+r, col l%16) of the 16x16 tile
  const int col = lane & 15;
  if (EPI == EPI_QKV) {
    // bias, rotary embedding, queries out, keys / values into the paged cache (as gemm_epilogue<EPI_QKV>); tiles j and
    // j + TN/2 of the head hold dims d and d + head_dim/2
    const int hd = g.kv.hd, half = hd >> 1, nq = g.nq, nkv = g.kv.nkv, head = cb;
    if (tl[0] >= ntiles) return;
#pragma unroll
    for (int j = 0; j < TN / 2; ++j) {
      const int d = j * 16 + col, n0 = head * hd + d;
      const float b0 = g.bias ? g.bias[n0] : 0.f, b1 = g.bias ? g.bias[n0 + half] : 0.f;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          if (!on[i][r]) continue;
          const int row = row0 + i * 16 + (lane >> 4) * 4 + r;
          float v0 = acc[i][j][r] + b0, v1 = acc[i][j + TN / 2][r] + b1;
          if (head < nq + nkv) {
            const float2 c = cs[i][r][j];
            const float r0 = v0 * c.x - v1 * c.y, r1 = v1 * c.x + v0 * c.y;
            v0 = r0; v1 = r1;
          }
          if (head < nq) {
            float* qo = g.q + (size_t)row * nq * hd + head * hd + d;
            qo[0] = v0; qo[half] = v1;
          } else if (blk[i][r] >= 0) {
            const int which = head < nq + nkv ? 0 : 1, kvh = head - nq - which * nkv;
            bf16_t* base = (bf16_t*)g.kv.pool + kv_offset(g.kv, g.layer, which, blk[i][r], kvh, 0);
            const int tok = pos[i][r] % g.kv.bt;
            if (which == 0) { base[tok * hd + d] = f_to_bf16(v0); base[tok * hd + d + half] = f_to_bf16(v1); }
            else { base[d * g.kv.bt + tok] = f_to_bf16(v0); base[(d + half) * g.kv.bt + tok] = f_to_bf16(v1); }
          }
        }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = row0 + i * 16 + (lane >> 4) * 4 + r;
      if (row >= g.M) continue;
      if (EPI == EPI_SWIGLU) {
#pragma unroll
        for (int j = 0; j < TN / 2; ++j)
          if (tl[j] < ntiles) gemm_epilogue<EPI_SWIGLU, F32, BF16>(g, tl[j], tl[j], 0, row, col, acc[i][j][r], acc[i][j + TN / 2][r]);
      } else {
#pragma unroll
        for (int j = 0; j < TN; ++j)
          if (tl[j] < ntiles) gemm_epilogue<EPI_PARTIAL, F32, BF16>(g, tl[j], 0x7FFFFFF, slice, row, col, acc[i][j][r], 0.f);
      }
    }
}

}  // namespace ssd
