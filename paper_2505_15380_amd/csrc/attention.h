// Multi-query decode attention over the paged cache (Eq. 4: the K+1 rows of a verification attend to the
// whole prefix and causally to each other).
//
// Work item = (chunk of 64 key positions, kv head, sequence).  The workgroup stages the chunk's keys and
// values in LDS once and serves every query row that shares them: R rows of the sequence x the G query
// heads of the group.  Each query row gets a partial (max, sum, weighted values) per chunk; k_attn_combine
// merges the chunks in ascending order.  Chunks are cut at absolute positions, so the partials a row
// combines - and therefore its bits - do not depend on how many rows are verified together.
#pragma once
#include "common.h"

namespace ssd {

struct AttnArgs {
  const float* q;       // [M][nq*hd] rotated queries
  KvView kv;
  Rows rows;
  int layer, nq;
  float scale;
  float* o_part;        // [M][nq][NC][hd]
  float* ml_part;       // [M][nq][NC][2]
  int NC;               // chunk capacity of the partial buffers
  void* out;            // [M][nq*hd] (combine)
  int split_kt;         // > 0: `out` is written as split rows (common.h) with this many k-tiles per row (nq*hd / 32)
  int nparts, tiles_per_wg;   // k_attn_part_mfma: grid.x = nparts x groups of tiles_per_wg row tiles (a multiple of 4)
};

template <int HD, typename KVT>
__global__ void __launch_bounds__(BLOCK) k_attn_chunk(AttnArgs a) {
  __shared__ float Ks[ATT_CHUNK][HD + 1];
  __shared__ float Vs[ATT_CHUNK][HD];
  __shared__ float Qs[4][HD];
  __shared__ float Ps[4][ATT_CHUNK];
  const int chunk = blockIdx.x, kvh = blockIdx.y, brel = blockIdx.z;
  const int seq = a.rows.seq0 + brel;
  const int R = a.rows.R, G = a.nq / a.kv.nkv;
  const int m_first = brel * R, m_last = m_first + R - 1;
  const int cstart = chunk * ATT_CHUNK;
  const int pos_max = a.rows.pos[m_last];
  if (cstart > pos_max) return;                          // no row of this sequence reaches the chunk
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

  // stage keys / values of positions cstart .. cstart+63 (zero where beyond pos_max or unmapped)
  typedef typename KVT::T kv_t;
  const kv_t* pool = (const kv_t*)a.kv.pool;
  for (int i = tid; i < ATT_CHUNK * HD; i += BLOCK) {
    const int c = i / HD, d = i - c * HD;
    const int p = cstart + c;
    float kx = 0.f, vx = 0.f;
    if (p <= pos_max) {
      const int blk = a.kv.table[seq * a.kv.mbps + p / a.kv.bt];
      if (blk >= 0) {
        kx = KVT::ld(pool + kv_offset(a.kv, a.layer, 0, blk, kvh, p % a.kv.bt) + d);
        vx = KVT::ld(pool + kv_offset(a.kv, a.layer, 1, blk, kvh, 0) + d * a.kv.bt + p % a.kv.bt);
      }
    }
    Ks[c][d] = kx;
    Vs[c][d] = vx;
  }
  __syncthreads();

  const int nrows = R * G;
  for (int r = wave; r < nrows; r += 4) {
    const int j = r / G, gq = r - j * G;
    const int m = m_first + j, hq = kvh * G + gq;
    const int pos = a.rows.pos[m];
    const float* qrow = a.q + (size_t)m * a.nq * HD + hq * HD;
    for (int d = lane; d < HD; d += WAVE) Qs[wave][d] = qrow[d];
    __builtin_amdgcn_wave_barrier();
    // score of key `lane`
    float s = 0.f;
#pragma unroll 8
    for (int d = 0; d < HD; ++d) s = fmaf(Qs[wave][d], Ks[lane][d], s);
    const bool valid = (cstart + lane) <= pos;
    s = valid ? s * a.scale : -INFINITY;
    const float mx = wave_max(s);
    const size_t pidx = ((size_t)m * a.nq + hq) * a.NC + chunk;
    float* op = a.o_part + pidx * HD;
    if (mx == -INFINITY) {                               // the row sees nothing of this chunk
      if (lane == 0) { a.ml_part[pidx * 2] = -INFINITY; a.ml_part[pidx * 2 + 1] = 0.f; }
      for (int d = lane; d < HD; d += WAVE) op[d] = 0.f;
      __builtin_amdgcn_wave_barrier();
      continue;
    }
    const float p = valid ? expf(s - mx) : 0.f;
    const float l = wave_sum(p);
    Ps[wave][lane] = p;
    __builtin_amdgcn_wave_barrier();
    for (int d = lane; d < HD; d += WAVE) {
      float o = 0.f;
#pragma unroll 8
      for (int c = 0; c < ATT_CHUNK; ++c) o = fmaf(Ps[wave][c], Vs[c][d], o);
      op[d] = o;
    }
    if (lane == 0) { a.ml_part[pidx * 2] = mx; a.ml_part[pidx * 2 + 1] = l; }
    __builtin_amdgcn_wave_barrier();
  }
}

// One wave per (row, query head): merge the row's chunk partials in ascending chunk order.
template <int HD, typename AT>
__global__ void __launch_bounds__(WAVE) k_attn_combine(AttnArgs a) {
  const int m = blockIdx.x / a.nq, hq = blockIdx.x - m * a.nq;
  const int lane = threadIdx.x;
  const int nc = a.rows.pos[m] / ATT_CHUNK + 1;
  const size_t base = ((size_t)m * a.nq + hq) * a.NC;
  float mx = -INFINITY;
  for (int c = 0; c < nc; ++c) mx = fmaxf(mx, a.ml_part[(base + c) * 2]);
  float l = 0.f;
  float o[(HD + WAVE - 1) / WAVE];
#pragma unroll
  for (int i = 0; i < (HD + WAVE - 1) / WAVE; ++i) o[i] = 0.f;
  for (int c = 0; c < nc; ++c) {
    const float mc = a.ml_part[(base + c) * 2];
    if (mc == -INFINITY) continue;
    const float w = expf(mc - mx);
    l = fmaf(a.ml_part[(base + c) * 2 + 1], w, l);
#pragma unroll
    for (int i = 0; i < (HD + WAVE - 1) / WAVE; ++i) {
      const int d = lane + i * WAVE;
      if (d < HD) o[i] = fmaf(a.o_part[(base + c) * HD + d], w, o[i]);
    }
  }
  typename AT::T* out = (typename AT::T*)a.out + (size_t)m * a.nq * HD + hq * HD;
#pragma unroll
  for (int i = 0; i < (HD + WAVE - 1) / WAVE; ++i) {
    const int d = lane + i * WAVE;
    if (d < HD) {
      if (a.split_kt > 0) st_split_value((bf16_t*)a.out, a.split_kt, m, hq * HD + d, o[i] / l);
      else AT::st(out + d, o[i] / l);
    }
  }
}

// ------------------------------------------------------------------------------------------------ matrix-core variant
// The same operation for bf16 caches with 16-token blocks and head_dim 64 or 128, for launches with many rows
// (batched verification).  Work item = (part of 256 key positions, kv head, sequence).  The query rows that share
// the keys - R rows of the sequence x the G query heads of the group - form tiles of 16; wave w of the workgroup
// takes tiles w, w+4, .. and walks the part's four 64-key chunks in ascending order with a running (max, sum,
// weighted values) per row, so no partial ever crosses waves.  Keys and values are read once, as MFMA operand
// fragments straight from the cache (a K fragment is 8 consecutive dims of one cached key row, a V fragment 8
// consecutive tokens of one dim of the token-minor value layout): wave w loads the fragments of chunk w and parks
// them in LDS in fragment order, so the whole part is in flight at once and every wave then reads any chunk with
// conflict-free 16-byte LDS reads.  S = Q K^T with the queries as hi + lo bf16, a masked softmax in the base-2
// domain, O = P V with P split the same way.  The result is one partial per (row, head, part);
// k_attn_combine_parts merges the parts in ascending order.  Parts and chunks are cut at absolute positions, so a
// row's bits do not depend on which other rows share the launch.
constexpr int ATT_PART_KEYS = 256;

template <int HD>
struct KVFrag {
  u32x4 kf[4][HD / 32], vf[2][HD / 16];
};

// Fragments of keys [kbase, kbase + 64) of (seq, kvh); masked keys may read any valid block.
template <int HD>
__device__ __forceinline__ void attn_load_chunk(const AttnArgs& a, const bf16_t* kp, const bf16_t* vp, int seq, int kvh,
                                                int kbase, int pos_max, int g, int c16, KVFrag<HD>& f) {
  const int nkv = a.kv.nkv;
  int blk[4];
#pragma unroll
  for (int t = 0; t < 4; ++t) {
    const int bi = (kbase >> 4) + t;
    const int b = (bi < a.kv.mbps && bi * 16 <= pos_max) ? a.kv.table[seq * a.kv.mbps + bi] : -1;
    blk[t] = b < 0 ? 0 : b;
    const bf16_t* kr = kp + ((size_t)(blk[t] * nkv + kvh) * 16 + c16) * HD + g * 8;
#pragma unroll
    for (int ks = 0; ks < HD / 32; ++ks) f.kf[t][ks] = *(const u32x4*)(kr + 32 * ks);
  }
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    const int b0 = blk[2 * ks], b1 = blk[2 * ks + 1];
    const int vblk = (g >> 1) ? b1 : b0;                              // keys 32ks + 8g.. live in block 2ks + g/2
    const bf16_t* vr = vp + ((size_t)(vblk * nkv + kvh) * HD + c16) * 16 + (g & 1) * 8;
#pragma unroll
    for (int dt = 0; dt < HD / 16; ++dt) f.vf[ks][dt] = *(const u32x4*)(vr + dt * 256);
  }
}

template <int HD>
__global__ void __launch_bounds__(BLOCK) k_attn_part_mfma(AttnArgs a) {
  constexpr int KS = HD / 32, DT = HD / 16, NF = 4 * KS + 2 * DT;     // fragments of a chunk: 16 (HD 64) or 32 (HD 128)
  // A wave's P tile, 16 rows x 64 keys: row r keeps key column c at c ^ 4 (r & 7), so that the 16-byte reads of eight
  // consecutive rows fall into distinct banks (unswizzled they all hit the same four)
  __shared__ __attribute__((aligned(16))) float Pw[4][16 * 64];
  __shared__ u32x4 KV[4][NF][64];                        // the part's fragments, [chunk][fragment][lane]
  const int part = blockIdx.x % a.nparts, tgroup = blockIdx.x / a.nparts, kvh = blockIdx.y, brel = blockIdx.z;
  const int seq = a.rows.seq0 + brel;
  const int R = a.rows.R, nkv = a.kv.nkv, G = a.nq / nkv, RG = R * G;
  const int m_first = brel * R;
  const int ntiles = (RG + 15) >> 4;
  const int rt_begin = tgroup * a.tiles_per_wg, rt_end = min(ntiles, rt_begin + a.tiles_per_wg);
  // rows are in ascending position order: the last row of this workgroup's tiles sees the most keys
  const int pos_max = a.rows.pos[m_first + (min(16 * rt_end, RG) - 1) / G];
  const int pbase = part * ATT_PART_KEYS;
  if (pbase > pos_max) return;                           // no row of these tiles reaches the part
  const int tid = threadIdx.x, lane = tid & 63, uw = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int g = lane >> 4, c16 = lane & 15;
  const int nch = min(4, ((pos_max - pbase) >> 6) + 1);  // chunks of the part that some row reaches
  // wave w brings chunk w into LDS: every fragment load of the part is in flight at once
  if (uw < nch) {
    const size_t plane = (size_t)a.kv.n_blocks * nkv * 16 * HD;
    const bf16_t* kp = (const bf16_t*)a.kv.pool + (size_t)(2 * a.layer) * plane;
    KVFrag<HD> f;
    attn_load_chunk<HD>(a, kp, kp + plane, seq, kvh, pbase + 64 * uw, pos_max, g, c16, f);
#pragma unroll
    for (int t = 0; t < 4; ++t)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) KV[uw][t * KS + ks][lane] = f.kf[t][ks];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) KV[uw][4 * KS + ks * DT + dt][lane] = f.vf[ks][dt];
  }
  const float scale2 = a.scale * 1.4426950408889634f;
  float* P = Pw[uw];
  // Q fragments of the wave's first tile travel while the keys do
  auto load_q = [&](int rt, u32x4 (&x)[KS][2]) {
    const int qr = 16 * rt + c16;                        // A-operand row c16 = (row j of the sequence, query head gq)
    const bool qok = qr < RG;
    const int j = qok ? qr / G : 0, gq = qok ? qr - j * G : 0;
    const u32x4* qp = (const u32x4*)(a.q + ((size_t)(m_first + j) * a.nq + kvh * G + gq) * HD + g * 8);
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      x[ks][0] = u32x4{0u, 0u, 0u, 0u};
      x[ks][1] = x[ks][0];
      if (qok) { x[ks][0] = qp[8 * ks]; x[ks][1] = qp[8 * ks + 1]; }
    }
  };
  auto load_pos = [&](int rt, int (&pos)[4]) {           // of accumulator rows 4g + r; -1: not a row
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int qr = 16 * rt + 4 * g + r;
      pos[r] = qr < RG ? a.rows.pos[m_first + qr / G] : -1;
    }
  };
  // position of the last row of tile rt (rows ascend in position: what the tile reaches)
  auto tile_reach = [&](int rt) { return a.rows.pos[m_first + (min(16 * rt + 16, RG) - 1) / G]; };
  u32x4 qraw[KS][2], qnext[KS][2];
  int pos[4], pnext[4], reach = -1, reach_next = -1;
  if (rt_begin + uw < rt_end) { load_q(rt_begin + uw, qraw); load_pos(rt_begin + uw, pos); reach = tile_reach(rt_begin + uw); }
  __syncthreads();
  for (int rt = rt_begin + uw; rt < rt_end; rt += 4) {
    if (rt != rt_begin + uw) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) { qraw[ks][0] = qnext[ks][0]; qraw[ks][1] = qnext[ks][1]; }
#pragma unroll
      for (int r = 0; r < 4; ++r) pos[r] = pnext[r];
      reach = reach_next;
    }
    // the wave's next tile travels while this one is worked on
    if (rt + 4 < rt_end) { load_q(rt + 4, qnext); load_pos(rt + 4, pnext); reach_next = tile_reach(rt + 4); }
    __builtin_amdgcn_sched_barrier(0);
    // causal skip: a tile whose last row does not reach the part has nothing here
    if (reach < pbase) continue;
    SplitA qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = split_bf16(qraw[ks][0], qraw[ks][1]);
    float mrow[4], lrow[4];
    f32x4 oacc[DT];
#pragma unroll
    for (int r = 0; r < 4; ++r) { mrow[r] = -INFINITY; lrow[r] = 0.f; }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) oacc[dt] = f32x4{0, 0, 0, 0};
    for (int c = 0; c < nch; ++c) {
      const int kbase = pbase + 64 * c;
      f32x4 s[4];
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        bf16x8 kf[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kf[ks] = __builtin_bit_cast(bf16x8, KV[c][t * KS + ks][lane]);
        f32x4 z = f32x4{0, 0, 0, 0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[ks].lo, kf[ks], z, 0, 0, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) z = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[ks].hi, kf[ks], z, 0, 0, 0);
        s[t] = z;
      }
      // element (reg r, tile t) = (tile row 4g + r, key kbase + 16t + c16)
      float alpha[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const bool ok = kbase + 16 * t + c16 <= pos[r];
          s[t][r] = ok ? s[t][r] * scale2 : -INFINITY;
          mx = fmaxf(mx, s[t][r]);
        }
        const float mnew = fmaxf(mrow[r], row16_max(mx));
        alpha[r] = (mrow[r] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mrow[r] - mnew);
        float sum = 0.f;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
          const float p = (s[t][r] == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(s[t][r] - mnew);
          P[(4 * g + r) * 64 + ((16 * t + c16) ^ (((4 * g + r) & 7) << 2))] = p;
          sum += p;
        }
        mrow[r] = mnew;
        lrow[r] = fmaf(lrow[r], alpha[r], row16_sum(sum));
      }
      __builtin_amdgcn_wave_barrier();
      // O = alpha O + P V: P fragment row c16, keys 32ks + 8g..; V fragment dim 16dt + c16, same keys
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 4; ++r) oacc[dt][r] *= alpha[r];
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const int pc = ks * 32 + g * 8, sw = (c16 & 7) << 2;
        const SplitA pf = split_bf16(*(const u32x4*)(P + c16 * 64 + (pc ^ sw)), *(const u32x4*)(P + c16 * 64 + ((pc + 4) ^ sw)));
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
          const bf16x8 vv = __builtin_bit_cast(bf16x8, KV[c][4 * KS + ks * DT + dt][lane]);
          oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf.lo, vv, oacc[dt], 0, 0, 0);
          oacc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(pf.hi, vv, oacc[dt], 0, 0, 0);
        }
      }
      __builtin_amdgcn_wave_barrier();                   // P is rewritten by the next chunk
    }
    // the part's partial of every row that reaches the part (the combine reads no others)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int qr = 16 * rt + 4 * g + r;
      if (pbase <= pos[r]) {
        const int j = qr / G, gq = qr - j * G;
        const size_t pidx = ((size_t)(m_first + j) * a.nq + kvh * G + gq) * a.NC + part;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) a.o_part[pidx * HD + 16 * dt + c16] = oacc[dt][r];
        if (c16 == 0) { a.ml_part[pidx * 2] = mrow[r]; a.ml_part[pidx * 2 + 1] = lrow[r]; }
      }
    }
  }
}

// One wave per (row, query head): merge the row's part partials (base-2 maxima) in ascending part order.
template <int HD, typename AT>
__global__ void __launch_bounds__(WAVE) k_attn_combine_parts(AttnArgs a) {
  const int m = blockIdx.x / a.nq, hq = blockIdx.x - m * a.nq;
  const int lane = threadIdx.x;
  const int np = a.rows.pos[m] / ATT_PART_KEYS + 1;
  const size_t base = ((size_t)m * a.nq + hq) * a.NC;
  float mx = -INFINITY;
  for (int p = 0; p < np; ++p) mx = fmaxf(mx, a.ml_part[(base + p) * 2]);
  float l = 0.f, o[HD / 64];
#pragma unroll
  for (int i = 0; i < HD / 64; ++i) o[i] = 0.f;
#pragma unroll 4
  for (int p = 0; p < np; ++p) {
    const float mc = a.ml_part[(base + p) * 2];
    const float w = (mc == -INFINITY) ? 0.f : __builtin_amdgcn_exp2f(mc - mx);
    l = fmaf(a.ml_part[(base + p) * 2 + 1], w, l);
#pragma unroll
    for (int i = 0; i < HD / 64; ++i) o[i] = fmaf(a.o_part[(base + p) * HD + lane + i * WAVE], w, o[i]);
  }
  if (a.split_kt > 0) {
#pragma unroll
    for (int i = 0; i < HD / 64; ++i) st_split_value((bf16_t*)a.out, a.split_kt, m, hq * HD + lane + i * WAVE, o[i] / l);
    return;
  }
  typename AT::T* out = (typename AT::T*)a.out + (size_t)m * a.nq * HD + hq * HD;
#pragma unroll
  for (int i = 0; i < HD / 64; ++i) AT::st(out + lane + i * WAVE, o[i] / l);
}

}  // namespace ssd
