// Pass 1 kernels: calibration (range and sums per tile) over stream tiles and LDS-staged row
// tiles, and the lane-to-row mapping that all row kernels share.
#pragma once
#include "qv2_dev_common.h"

namespace {

// ---------------------------------------------------------------------------
// pass 1 (calibration stage, Sec. 5; x_min / x_max of Eq. 2): stream tiles
// ---------------------------------------------------------------------------
// partial record of the calibration pass: with the pair comparison it also carries sum (x - qrun)^2
template <bool PAIR, bool COS = false> struct StatRec { typedef StatPartial type; };
template <> struct StatRec<true, false> { typedef StatPairPartial type; };
template <> struct StatRec<true, true> { typedef StatPairCosPartial type; };
__device__ __forceinline__ void set_pair_energy(StatPartial&, double, double) {}
__device__ __forceinline__ void set_pair_energy(StatPairPartial& o, double sd2, double) { o.sd2 = sd2; }
__device__ __forceinline__ void set_pair_energy(StatPairCosPartial& o, double sd2, double sxq) { o.sd2 = sd2; o.sxq = sxq; }

struct StatAcc {
  f4 mn4 = {INFINITY, INFINITY, INFINITY, INFINITY};
  f4 mx4 = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  Acc4 s, s2, d2, xq;
  __device__ __forceinline__ void take(const f4& r) {
    mn4.x = fminf(mn4.x, r.x); mn4.y = fminf(mn4.y, r.y);
    mn4.z = fminf(mn4.z, r.z); mn4.w = fminf(mn4.w, r.w);
    mx4.x = fmaxf(mx4.x, r.x); mx4.y = fmaxf(mx4.y, r.y);
    mx4.z = fmaxf(mx4.z, r.z); mx4.w = fmaxf(mx4.w, r.w);
    s.add(r); s2.add_sq(r.x, r.y, r.z, r.w);
  }
};

// vector body of a calibration tile; WITHB: a second stream (qrun) is compared in the same visit
// (BAL: its vectors are 16-byte aligned like x's; otherwise only 4-byte aligned)
template <int BLOCK, int V, bool WITHB, bool COS, bool BAL>
__device__ __forceinline__ void stats_body(gf4_ptr v4, gf_ptr b, int nvec, StatAcc& a) {
  const int tid = threadIdx.x;
  int base = 0;
  for (; base + V * BLOCK <= nvec; base += V * BLOCK) {          // uniform: whole batches
    f4 r[V], g[V];
#pragma unroll
    for (int u = 0; u < V; ++u) {
      r[u] = ld4(v4 + base + u * BLOCK + tid);
      if (WITHB) g[u] = ld4b<BAL>(b, base + u * BLOCK + tid);
    }
#pragma unroll
    for (int u = 0; u < V; ++u) {
      a.take(r[u]);
      if (WITHB) a.d2.add_sq(r[u].x - g[u].x, r[u].y - g[u].y, r[u].z - g[u].z, r[u].w - g[u].w);
      if (WITHB && COS) a.xq.add_prod(r[u], g[u]);
    }
  }
  if (base < nvec) {
    // the last, partial batch: its loads go out together like a whole batch's; a lane whose
    // vector lies past the end reads the last vector instead and leaves it out
    f4 r[V], g[V];
#pragma unroll
    for (int u = 0; u < V; ++u) {
      const int i = base + u * BLOCK + tid, j = i < nvec ? i : nvec - 1;
      r[u] = ld4(v4 + j);
      if (WITHB) g[u] = ld4b<BAL>(b, j);
    }
#pragma unroll
    for (int u = 0; u < V; ++u) {
      if (base + u * BLOCK + tid >= nvec) continue;
      a.take(r[u]);
      if (WITHB) a.d2.add_sq(r[u].x - g[u].x, r[u].y - g[u].y, r[u].z - g[u].z, r[u].w - g[u].w);
      if (WITHB && COS) a.xq.add_prod(r[u], g[u]);
    }
  }
}

// PAIR: tiles whose tensor has a quantized-run partner also yield sum (x - qrun)^2 (Algorithm 2's
// D[i] against Q[i]) from the same visit: 8 B read per element, nothing but the partial written.
// COS: also sum x * qrun, the cross term of cos(x, qrun) (Sec. 6.1 Eq. 8).
template <int BLOCK, int V, bool PAIR, bool COS>
__global__ __launch_bounds__(BLOCK) void k_stats_stream(const StreamView tiles,
                                                        typename StatRec<PAIR, COS>::type* __restrict__ parts) {
  // XCD-aware tile order (see xcd_blocked) for the sweep that also reads qrun: -2 %.  The sweep
  // over x alone is 1 % faster in table order.
  int bt = blockIdx.x;
  if (PAIR) bt = xcd_blocked(bt, static_cast<int>(gridDim.x), kXcdBlockRead);
  const TileRef tl = decode_tile(tiles, bt);
  const gf_ptr p = (gf_ptr)tl.x;
  const gf_ptr b = (gf_ptr)tl.q;
  const int len = tl.len, tid = threadIdx.x;
  const int head = head_elems(tl.x, len);
  const int body = len - head, nvec = body >> 2, tail = body & 3;
  const bool has_b = PAIR && tl.q != nullptr;
  // qrun at a different offset inside 16 bytes than x: its vectors are loaded from 4-byte
  // aligned addresses (the vectors start where x's alignment puts them)
  const bool b_al = ((reinterpret_cast<uintptr_t>(tl.x) ^ reinterpret_cast<uintptr_t>(tl.q)) & 15u) == 0;

  float mn = INFINITY, mx = -INFINITY;
  double sx = 0.0, sx2 = 0.0, sd2 = 0.0, sxq = 0.0;
  for (int k = 0; k < 2; ++k) {
    const bool on = k == 0 ? tid < head : tid < tail;
    if (!on) continue;
    const int idx = k == 0 ? tid : head + (nvec << 2) + tid;
    const float v = p[idx];
    mn = fminf(mn, v); mx = fmaxf(mx, v);
    sx += v; sx2 += static_cast<double>(v) * v;
    if (has_b) {
      const float qv = b[idx], d = v - qv;
      sd2 += static_cast<double>(d) * d;
      if (COS) sxq = fma(static_cast<double>(v), static_cast<double>(qv), sxq);
    }
  }
  const gf4_ptr v4 = (gf4_ptr)(tl.x + head);
  StatAcc a;
  if (PAIR && has_b) {
    if (b_al) stats_body<BLOCK, (V > 1 ? V / 2 : 1), true, COS, true>(v4, b + head, nvec, a);
    else stats_body<BLOCK, (V > 1 ? V / 2 : 1), true, COS, false>(v4, b + head, nvec, a);
  } else {
    stats_body<BLOCK, V, false, false, true>(v4, b, nvec, a);
  }
  sx += a.s.total(); sx2 += a.s2.total(); sd2 += a.d2.total(); sxq += a.xq.total();
  mn = fminf(fminf(mn, a.mn4.x), fminf(fminf(a.mn4.y, a.mn4.z), a.mn4.w));
  mx = fmaxf(fmaxf(mx, a.mx4.x), fmaxf(fmaxf(a.mx4.y, a.mx4.z), a.mx4.w));

  block_minmax<BLOCK>(mn, mx);
  if (COS) {
    double v[4] = {sx, sx2, sd2, sxq};
    block_sum<BLOCK, 4>(v);
    sx = v[0]; sx2 = v[1]; sd2 = v[2]; sxq = v[3];
  } else {
    block_sum3<BLOCK>(sx, sx2, sd2);
  }
  if (tid == 0) {
    typename StatRec<PAIR, COS>::type o;
    o.mn = mn; o.mx = mx; o.sx = sx; o.sx2 = sx2;
    set_pair_energy(o, sd2, sxq);
    st_record<true>(&parts[tl.part0], o);
  }
}

// Copies a row-group tile into LDS with 16-byte transfers.  Element e of the
// tile lands at xs[e + shift]; returns shift (0..3).
template <int BLOCK>
__device__ __forceinline__ int stage_tile(const float* x, int len, float* xs) {
  const int tid = threadIdx.x;
  const gf_ptr p = (gf_ptr)x;
  const int head = head_elems(x, len);
  const int shift = (4 - head) & 3;
  const int body = len - head, nvec = body >> 2, tail = body & 3;
  if (tid < head) xs[shift + tid] = p[tid];
  const gf4_ptr v4 = (gf4_ptr)(x + head);
  f4* d4 = reinterpret_cast<f4*>(xs + shift + head);
  constexpr int kPer = (kRowGroupCap / 4 + BLOCK - 1) / BLOCK;   // all loads of a lane go out before its LDS stores
  f4 r[kPer];
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int i = tid + u * BLOCK;
    if (i < nvec) r[u] = ld4(v4 + i);
  }
#pragma unroll
  for (int u = 0; u < kPer; ++u) {
    const int i = tid + u * BLOCK;
    if (i < nvec) d4[i] = r[u];
  }
  if (tid < tail) xs[shift + head + (nvec << 2) + tid] = p[head + (nvec << 2) + tid];
  return shift;
}

// Lanes per row of a row-group tile: the power of two >= inner, at most a wavefront.
__device__ __forceinline__ int row_width(int inner) {
  int w = 1;
  while (w < inner && w < kWave) w <<= 1;
  return w;
}

// How the lanes of a workgroup of W wavefronts share the rows of a row-group tile.
//  plain: w lanes of one wavefront per row, 64 / w rows per wavefront at a time, the
//         wavefronts take rounds of rows;
//  split: a tile of at most W / 2 (long) rows gives every row `wpr` whole wavefronts, whose
//         partial results are joined through LDS in wavefront order; one round.
// `rounds` is the same for every thread, so the loop over rounds may hold barriers.
struct RowMap {
  int w;        // lanes of a wavefront that share a row (width of the shuffle reductions)
  int stride;   // lanes that share a row in all
  int gl;       // index of this lane among them
  int row0;     // row of this lane in round 0
  int step;     // rows per round
  int rounds;
  int wpr;      // wavefronts per row (1 = plain)
  int part;     // index of this wavefront among the wpr of its row
};

template <int W>
__device__ __forceinline__ RowMap row_map(int rows, int inner) {
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  RowMap m;
  if (rows * 2 <= W) {
    int wpr = W;
    while (wpr * rows > W) wpr >>= 1;
    m.w = kWave; m.stride = kWave * wpr; m.wpr = wpr; m.part = wave % wpr;
    m.gl = m.part * kWave + lane; m.row0 = wave / wpr; m.step = W / wpr; m.rounds = 1;
  } else {
    const int w = row_width(inner), gpw = kWave / w;
    m.w = w; m.stride = w; m.wpr = 1; m.part = 0;
    m.gl = lane & (w - 1); m.row0 = wave * gpw + (lane >> __builtin_ctz(w)); m.step = W * gpw;
    m.rounds = (rows + m.step - 1) / m.step;
  }
  return m;
}

// Range and sums of one row over the lanes that share it; the results are valid in all of
// them.  N sums; RANGE = false skips mn / mx.  sf / sd: LDS exchange areas of the split
// form, [2][W] and [N][W].  Every butterfly step moves all values before it combines them,
// so the steps of the different values overlap instead of forming one long dependent chain.
template <int W, int N, bool RANGE>
__device__ __forceinline__ void row_join(const RowMap& m, float& mn, float& mx, double (&v)[N],
                                         float (*sf)[W], double (*sd)[W]) {
  for (int o = m.w >> 1; o > 0; o >>= 1) {
    float a = 0.0f, b = 0.0f;
    double t[N];
    if (RANGE) { a = __shfl_xor(mn, o); b = __shfl_xor(mx, o); }
#pragma unroll
    for (int k = 0; k < N; ++k) t[k] = __shfl_xor(v[k], o);
    if (RANGE) { mn = fminf(mn, a); mx = fmaxf(mx, b); }
#pragma unroll
    for (int k = 0; k < N; ++k) v[k] += t[k];
  }
  if (m.wpr == 1) return;                           // uniform over the workgroup
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  if (lane == 0) {
    if (RANGE) { sf[0][wave] = mn; sf[1][wave] = mx; }
#pragma unroll
    for (int k = 0; k < N; ++k) sd[k][wave] = v[k];
  }
  __syncthreads();
  const int w0 = wave - m.part;
  if (RANGE) { mn = sf[0][w0]; mx = sf[1][w0]; }
#pragma unroll
  for (int k = 0; k < N; ++k) v[k] = sd[k][w0];
  for (int i = 1; i < m.wpr; ++i) {
    if (RANGE) { mn = fminf(mn, sf[0][w0 + i]); mx = fmaxf(mx, sf[1][w0 + i]); }
#pragma unroll
    for (int k = 0; k < N; ++k) v[k] += sd[k][w0 + i];
  }
}

// pass 1, row-group tiles: many short segments (output channels) per workgroup
template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_stats_rows(const Tile* __restrict__ tiles,
                                                      StatPartial* __restrict__ parts) {
  constexpr int W = BLOCK / kWave;
  __shared__ __attribute__((aligned(16))) float xs[kRowGroupCap + 4];
  __shared__ float sf[2][W];
  __shared__ double sd[2][W];
  const Tile tl = tiles[blockIdx.x];
  const int shift = stage_tile<BLOCK>(tl.x, tl.len, xs);
  __syncthreads();

  const int inner = tl.inner;
  const RowMap m = row_map<W>(tl.rows, inner);
  for (int round = 0; round < m.rounds; ++round) {
    const int r = m.row0 + round * m.step;
    const bool live = r < tl.rows;
    float mn = INFINITY, mx = -INFINITY;
    double v[2] = {0.0, 0.0};                                  // sum x, sum x^2
    if (live) {
      const float* row = xs + shift + r * inner;
      auto take = [&](float x) {
        mn = fminf(mn, x); mx = fmaxf(mx, x);
        v[0] += x; v[1] = fma(static_cast<double>(x), static_cast<double>(x), v[1]);
      };
      int j = m.gl;
      for (; j + 3 * m.stride < inner; j += 4 * m.stride) {      // four LDS reads in flight
        const float x0 = row[j], x1 = row[j + m.stride], x2 = row[j + 2 * m.stride], x3 = row[j + 3 * m.stride];
        take(x0); take(x1); take(x2); take(x3);
      }
      for (; j < inner; j += m.stride) take(row[j]);
    }
    row_join<W, 2, true>(m, mn, mx, v, sf, sd);
    if (live && m.gl == 0) {
      StatPartial o;
      o.mn = mn; o.mx = mx; o.sx = v[0]; o.sx2 = v[1];
      parts[tl.part0 + r] = o;
    }
  }
}

// Scale and zero-point from a segment's range (Eq. 2 with N = 256; Eq. 4 with b = 8).
__device__ __forceinline__ void make_params(float mn, float mx, int scheme, qv2_qparams& o) {
  o.min = mn + 0.0f;                               // -0.0 -> +0.0
  o.max = mx + 0.0f;
  o._pad = 0;
  float s, lo = 0.0f;
  if (scheme == QV2_ASYM_TENSOR) {
    lo = fminf(mn, 0.0f);
    const float hi = fmaxf(mx, 0.0f);
    s = (hi - lo) / 255.0f;
  } else {
    s = fmaxf(fabsf(mn), fabsf(mx)) / 127.0f;
  }
  if (!(s >= FLT_MIN)) { o.scale = 1.0f; o.inv_scale = 1.0f; o.zp = 0; return; }
  const float inv = 1.0f / s;
  o.scale = s; o.inv_scale = inv; o.zp = 0;
  if (scheme == QV2_ASYM_TENSOR) {
    const float prod = lo * inv;
    const float z = rintf(-128.0f - prod);
    o.zp = static_cast<int>(fminf(fmaxf(z, -128.0f), 127.0f));
  }
}

}  // namespace
