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
    if (d < HD) AT::st(out + d, o[i] / l);
  }
}

}  // namespace ssd
