// Pass 2 kernels: quantize, dequantize and error energies (Eq. 1, 3, 5; Eq. 6-7), optionally
// with the comparison against the quantized run, over stream tiles and LDS-staged row tiles;
// and the register form of the row kernels, which serves passes 1 and 2 and both in one read.
#pragma once
#include "qv2_dev_fold.h"

namespace {

// ---------------------------------------------------------------------------
// pass 2 (Eq. 1, 3, 5 and the energies of Eq. 6-7), optionally with pass 3
// (Algorithm 2's D[i] vs Q[i]) in the same sweep: stream tiles.
// Per element 4 B read + 1 B code written (+ 4 B of qrun read when PAIR).
// ---------------------------------------------------------------------------
// STORE: 0 no code buffer, 1 packed dwords, 2 single bytes (misaligned code buffer)
template <int BLOCK, int V, int STORE, bool PAIR, bool COS, bool X2, bool BAL>
__device__ __forceinline__ void quant_body(gf4_ptr v4, gf_ptr b, gu32_ptr cw, gi8_ptr cb, int nvec,
                                           const QP& q, Acc4& ae2, Acc4& ax2, Acc4& ad2, Acc4& axh,
                                           Acc4& axq) {
  const int tid = threadIdx.x;
  auto put = [&](int i, uint32_t pk) {
    if (STORE == 1) {
      st_codes(cw + i, pk);
    } else if (STORE == 2) {
      gi8_ptr d = cb + (i << 2);
      d[0] = static_cast<int8_t>(pk); d[1] = static_cast<int8_t>(pk >> 8);
      d[2] = static_cast<int8_t>(pk >> 16); d[3] = static_cast<int8_t>(pk >> 24);
    }
  };
  int base = 0;
  for (; base + V * BLOCK <= nvec; base += V * BLOCK) {          // uniform: whole batches
    f4 r[V], g[V];
#pragma unroll
    for (int u = 0; u < V; ++u) {
      r[u] = ld4(v4 + base + u * BLOCK + tid);
      if (PAIR) g[u] = ld4b<BAL>(b, base + u * BLOCK + tid);
    }
#pragma unroll
    for (int u = 0; u < V; ++u) {
      put(base + u * BLOCK + tid, quant4<COS, X2>(r[u], q, ae2, ax2, axh));
      if (PAIR) ad2.add_sq(r[u].x - g[u].x, r[u].y - g[u].y, r[u].z - g[u].z, r[u].w - g[u].w);
      if (PAIR && COS) axq.add_prod(r[u], g[u]);
    }
  }
  // (what is left of a tile after its whole batches: one vector per lane and turn.  Loading it as
  // one masked batch, as the read-only sweeps do, made this kernel 4 % slower on tiles that are
  // exactly one batch long, which is nearly all of them.)
  for (int i = base + tid; i < nvec; i += BLOCK) {
    const f4 r = ld4(v4 + i);
    put(i, quant4<COS, X2>(r, q, ae2, ax2, axh));
    if (PAIR) {
      const f4 g = ld4b<BAL>(b, i);
      ad2.add_sq(r.x - g.x, r.y - g.y, r.z - g.z, r.w - g.w);
      if (COS) axq.add_prod(r, g);
    }
  }
}

#ifndef QV2_QUANT_WAVES_PER_EU
#define QV2_QUANT_WAVES_PER_EU 1    // occupancy floor asked of the register allocator
#endif
#ifndef QV2_QUANT_PLAIN_WAVES_PER_EU
#define QV2_QUANT_PLAIN_WAVES_PER_EU 8
#endif
// partial record of a quantize pass: 3 energies, plus the 2 cross terms when COS
template <bool COS> struct ErrRec { typedef ErrPartial3 type; };
template <> struct ErrRec<true> { typedef ErrPartial5 type; };
// ... of its stream tiles: the same, except that the sweep which takes the error energy only
// (no partner, no cross terms, sum x^2 kept from the first sweep) leaves just that one double
template <bool PAIR, bool COS, bool X2> struct StreamRec { typedef typename ErrRec<COS>::type type; };
template <> struct StreamRec<false, false, false> { typedef ErrPartial1 type; };
__device__ __forceinline__ void set_cross(ErrPartial1&, double, double) {}
__device__ __forceinline__ void set_cross(ErrPartial3&, double, double) {}
__device__ __forceinline__ void set_energies(ErrPartial1& o, double, double se2, double) { o.se2 = se2; }
__device__ __forceinline__ void set_energies(ErrPartial3& o, double sx2, double se2, double sd2) {
  o.sx2 = sx2; o.se2 = se2; o.sd2 = sd2;
}
__device__ __forceinline__ void set_energies(ErrPartial5& o, double sx2, double se2, double sd2) {
  o.sx2 = sx2; o.se2 = se2; o.sd2 = sd2;
}
__device__ __forceinline__ void set_cross(ErrPartial5& o, double sxh, double sxq) { o.sxh = sxh; o.sxq = sxq; }

// RO: tiles of tensors without a code buffer (no store is compiled in; long tiles).
template <int BLOCK, int V, bool PAIR, bool COS, bool X2 = true, bool RO = false>
__global__ __launch_bounds__(BLOCK, (PAIR ? QV2_QUANT_WAVES_PER_EU : QV2_QUANT_PLAIN_WAVES_PER_EU)) void k_quant_stream(
    const StreamView tiles, const qv2_qparams* __restrict__ params,
    typename StreamRec<PAIR, COS, X2>::type* __restrict__ parts) {
  // XCD-aware tile order (see xcd_blocked): blocks of 2 MB of x per XCD.  The sweeps with one
  // read stream gain 1-1.5 % (6 % without codes); with qrun as a second read stream they do not.
  int bt = blockIdx.x;
  if (!PAIR) bt = xcd_blocked(bt, static_cast<int>(gridDim.x), RO ? kXcdBlockRead : kXcdBlockQuant);
  const TileRef tl = decode_tile<(!PAIR && !COS && !X2 && !RO)>(tiles, bt);
  const QP q = load_qp(params, tl.seg0);
  const gf_ptr p = (gf_ptr)tl.x;
  const gf_ptr b = (gf_ptr)tl.q;
  const gi8_ptr c = (gi8_ptr)tl.c;
  const bool has_c = !RO && tl.c != nullptr;
  const bool has_b = PAIR && tl.q != nullptr;
  const int len = tl.len, tid = threadIdx.x;
  double sx2 = 0.0, se2 = 0.0, sd2 = 0.0, sxh = 0.0, sxq = 0.0;

  // qrun at a different offset inside 16 bytes than x: its vectors are loaded from 4-byte
  // aligned addresses (the vectors start where x's alignment puts them)
  const bool b_al = ((reinterpret_cast<uintptr_t>(tl.x) ^ reinterpret_cast<uintptr_t>(tl.q)) & 15u) == 0;
  const int head = head_elems(tl.x, len);
  const int body = len - head, nvec = body >> 2, tail = body & 3;
  for (int k = 0; k < 2; ++k) {
    const bool on = k == 0 ? tid < head : tid < tail;
    if (!on) continue;
    const int idx = k == 0 ? tid : head + (nvec << 2) + tid;
    const float v = p[idx];
    float e, h;
    const float code = quant1(v, q, e, h);
    if (has_c) c[idx] = static_cast<int8_t>(static_cast<int>(code));
    if (X2) sx2 += static_cast<double>(v) * v;
    se2 += static_cast<double>(e) * e;
    if (COS) sxh = fma(static_cast<double>(v), static_cast<double>(h), sxh);
    if (has_b) {
      const float qv = b[idx], d = v - qv;
      sd2 += static_cast<double>(d) * d;
      if (COS) sxq = fma(static_cast<double>(v), static_cast<double>(qv), sxq);
    }
  }
  const gf4_ptr v4 = (gf4_ptr)(tl.x + head);
  const gf_ptr bh = b + head;
  const gi8_ptr cb = c + head;
  const gu32_ptr cw = (gu32_ptr)(tl.c + head);
  const bool cw_ok = has_c && ((reinterpret_cast<uintptr_t>(tl.c + head) & 3u) == 0);
  Acc4 ae2, ax2, ad2, axh, axq;
  if (has_b && b_al) {
    if (cw_ok) quant_body<BLOCK, V, 1, PAIR, COS, X2, true>(v4, bh, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
    else if (has_c) quant_body<BLOCK, V, 2, PAIR, COS, X2, true>(v4, bh, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
    else quant_body<BLOCK, V, 0, PAIR, COS, X2, true>(v4, bh, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
  } else if (has_b) {
    if (cw_ok) quant_body<BLOCK, V, 1, PAIR, COS, X2, false>(v4, bh, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
    else if (has_c) quant_body<BLOCK, V, 2, PAIR, COS, X2, false>(v4, bh, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
    else quant_body<BLOCK, V, 0, PAIR, COS, X2, false>(v4, bh, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
  } else {
    if (cw_ok) quant_body<BLOCK, V, 1, false, COS, X2, true>(v4, bh, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
    else if (has_c) quant_body<BLOCK, V, 2, false, COS, X2, true>(v4, bh, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
    else quant_body<BLOCK, V, 0, false, COS, X2, true>(v4, bh, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
  }
  se2 += ae2.total(); sx2 += ax2.total(); sd2 += ad2.total();
  typename StreamRec<PAIR, COS, X2>::type o;
  if (COS) {
    double v[5] = {sx2, se2, sd2, sxh + axh.total(), sxq + axq.total()};
    block_sum<BLOCK, 5>(v);
    set_energies(o, v[0], v[1], v[2]);
    set_cross(o, v[3], v[4]);
  } else if (!X2 && !PAIR) {
    double v[1] = {se2};                            // the only energy this form takes
    block_sum<BLOCK, 1>(v);
    set_energies(o, 0.0, v[0], 0.0);
  } else {
    block_sum3<BLOCK>(sx2, se2, sd2);
    set_energies(o, sx2, se2, sd2);
  }
  if (tid == 0) st_record<RO>(&parts[tl.part0], o);
}

// pass 2 (+3), row-group tiles.  CALIB: pass 1 in the same visit - the tile sits in LDS, so
// every row's range, parameters, codes and energies come from ONE read of it from HBM; the
// rows' parameter and sum records are written here (same arithmetic and order as the
// separate kernels and their folds, hence the same bits) instead of by the folds.
template <int BLOCK, bool PAIR, bool COS, bool CALIB>
__global__ __launch_bounds__(BLOCK) void k_quant_rows(const Tile* __restrict__ tiles,
                                                      const Segment* __restrict__ segs,
                                                      const qv2_qparams* __restrict__ params,
                                                      qv2_qparams* __restrict__ params_out,
                                                      qv2_sums* __restrict__ sums_out,
                                                      typename ErrRec<COS>::type* __restrict__ parts) {
  constexpr int W = BLOCK / kWave;
  __shared__ __attribute__((aligned(16))) float xs[kRowGroupCap + 4];
  __shared__ __attribute__((aligned(16))) int8_t cs[kRowGroupCap + 8];
  __shared__ float sf[2][W];                        // exchange areas of the split row form
  __shared__ double sd1[1][W], sd2[COS ? 5 : 3][W];
  const Tile tl = tiles[blockIdx.x];
  const int shift = stage_tile<BLOCK>(tl.x, tl.len, xs);
  const gf_ptr b = (gf_ptr)tl.q;
  const bool has_b = PAIR && tl.q != nullptr;
  const int ca = static_cast<int>(reinterpret_cast<uintptr_t>(tl.c) & 3u);   // code e sits at cs[e + ca]
  const int scheme = CALIB ? segs[tl.seg0].scheme : 0;      // one tensor, one scheme per tile
  __syncthreads();

  const int inner = tl.inner;
  const RowMap m = row_map<W>(tl.rows, inner);
  for (int round = 0; round < m.rounds; ++round) {
    const int r = m.row0 + round * m.step;
    const bool live = r < tl.rows;
    const float* row = xs + shift + r * inner;
    qv2_qparams qp;
    double sx = 0.0;
    QP q{1.0f, 1.0f, 0.0f};
    if (CALIB) {
      float mn = INFINITY, mx = -INFINITY;
      double v[1] = {0.0};
      if (live) {
        auto take = [&](float x) { mn = fminf(mn, x); mx = fmaxf(mx, x); v[0] += x; };
        int j = m.gl;
        for (; j + 3 * m.stride < inner; j += 4 * m.stride) {    // four LDS reads in flight
          const float x0 = row[j], x1 = row[j + m.stride], x2 = row[j + 2 * m.stride], x3 = row[j + 3 * m.stride];
          take(x0); take(x1); take(x2); take(x3);
        }
        for (; j < inner; j += m.stride) take(row[j]);
      }
      row_join<W, 1, true>(m, mn, mx, v, sf, sd1);
      sx = v[0];
      make_params(mn, mx, scheme, qp);
      q = QP{qp.scale, qp.inv_scale, static_cast<float>(qp.zp)};
    } else if (live) {
      q = load_qp(params, tl.seg0 + r);
    }
    constexpr int NE = COS ? 5 : 3;
    double e[NE] = {};                                         // x^2, e^2, d^2 (, x*xhat, x*qrun)
    if (live) {
      int8_t* crow = cs + ca + r * inner;
      const gf_ptr brow = b + r * inner;
      auto take = [&](int j, float x, float qv) {
        float err, h;
        const float code = quant1(x, q, err, h);
        crow[j] = static_cast<int8_t>(static_cast<int>(code));
        e[0] = fma(static_cast<double>(x), static_cast<double>(x), e[0]);
        e[1] = fma(static_cast<double>(err), static_cast<double>(err), e[1]);
        if (COS) e[NE - 2] = fma(static_cast<double>(x), static_cast<double>(h), e[NE - 2]);
        if (has_b) {
          const double d = static_cast<double>(x - qv);
          e[2] = fma(d, d, e[2]);
          if (COS) e[NE - 1] = fma(static_cast<double>(x), static_cast<double>(qv), e[NE - 1]);
        }
      };
      int j = m.gl;
      for (; j + 3 * m.stride < inner; j += 4 * m.stride) {      // four reads in flight per stream
        const int j1 = j + m.stride, j2 = j + 2 * m.stride, j3 = j + 3 * m.stride;
        const float x0 = row[j], x1 = row[j1], x2 = row[j2], x3 = row[j3];
        float q0 = 0.0f, q1 = 0.0f, q2 = 0.0f, q3 = 0.0f;
        if (has_b) { q0 = brow[j]; q1 = brow[j1]; q2 = brow[j2]; q3 = brow[j3]; }
        take(j, x0, q0); take(j1, x1, q1); take(j2, x2, q2); take(j3, x3, q3);
      }
      for (; j < inner; j += m.stride) take(j, row[j], has_b ? brow[j] : 0.0f);
    }
    float u0 = 0.0f, u1 = 0.0f;
    row_join<W, NE, false>(m, u0, u1, e, sf, sd2);
    if (live && m.gl == 0) {
      typename ErrRec<COS>::type o;
      o.sx2 = e[0]; o.se2 = e[1]; o.sd2 = e[2];
      set_cross(o, COS ? e[NE - 2] : 0.0, COS ? e[NE - 1] : 0.0);
      parts[tl.part0 + r] = o;
      if (CALIB) {
        params_out[tl.seg0 + r] = qp;
        qv2_sums u;
        u.sum_x = sx; u.sum_x2 = e[0]; u.sum_e2 = e[1]; u.n = inner;
        sums_out[tl.seg0 + r] = u;
      }
    }
  }
  if (!tl.c) return;
  __syncthreads();
  // copy the codes out as whole dwords where the destination allows it
  const int total = tl.len + ca;
  const gi8_ptr base = (gi8_ptr)(tl.c - ca);
  for (int k = threadIdx.x; (k << 2) < total; k += BLOCK) {
    const int b0 = k << 2;
    if (b0 >= ca && b0 + 4 <= total) {
      *(gu32_ptr)(base + b0) = *reinterpret_cast<const uint32_t*>(cs + b0);
    } else {
      const int lo = b0 > ca ? b0 : ca, hi = b0 + 4 < total ? b0 + 4 : total;
      for (int bb = lo; bb < hi; ++bb) base[bb] = cs[bb];
    }
  }
}

// Row-group tiles, register form: rows of whole 16-byte vectors on 16-byte boundaries.  tl.lanes
// lanes share a row (a power of two, 16 .. BLOCK), each holds at most kRowRegVecs vectors of it
// in registers; a workgroup takes BLOCK / lanes rows, all at once.  Nothing is staged in LDS
// (only the partial results of rows that span several wavefronts cross it), loads and code stores
// are coalesced 16-byte / 4-byte accesses, and the arithmetic is the 4-wide form of the stream
// kernels.
//  ROLE 0: pass 1 (range, sum x, sum x^2 -> one StatPartial per row)
//  ROLE 1: pass 2 (+3) with given parameters
//  ROLE 2: both from the one copy in registers: the row is read from HBM once; writes the rows'
//          parameter and sum records itself.
template <int BLOCK, int ROLE, bool PAIR, bool COS>
__global__ __launch_bounds__(BLOCK) void k_rows_reg(const Tile* __restrict__ tiles,
                                                    const qv2_qparams* __restrict__ params,
                                                    qv2_qparams* __restrict__ params_out,
                                                    qv2_sums* __restrict__ sums_out,
                                                    void* __restrict__ parts_any) {
  constexpr int W = BLOCK / kWave;
  constexpr int K = kRowRegVecs;
  constexpr int NE = COS ? 5 : 3;
  __shared__ float sf[2][W];
  __shared__ double sd1[2][W], sd2[NE][W];
  const Tile tl = tiles[blockIdx.x];
  const int inner = tl.inner, nvec = inner >> 2, G = tl.lanes;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  RowMap m;
  m.step = 0; m.rounds = 1; m.stride = G;
  if (G >= kWave) {
    m.w = kWave; m.wpr = G >> 6; m.part = wave % m.wpr;
    m.gl = m.part * kWave + lane; m.row0 = wave / m.wpr;
  } else {
    m.w = G; m.wpr = 1; m.part = 0;
    m.gl = lane & (G - 1); m.row0 = wave * (kWave / G) + lane / G;
  }
  const int r = m.row0;
  const bool live = r < tl.rows;
  const size_t row_off = static_cast<size_t>(live ? r : 0) * inner;
  const gf4_ptr v4 = (gf4_ptr)(tl.x + row_off);
  const gf4_ptr b4 = (gf4_ptr)(tl.q + row_off);
  const bool has_b = PAIR && ROLE != 0 && tl.q != nullptr;

  // all loads go out back to back: a lane whose vector lies past the row's end (or whose row
  // is past the tile's end) reads the row's (or row 0's) last vector instead and ignores it
  f4 xv[K], gv[K];
  bool on[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const int i = m.gl + k * G;
    on[k] = live && i < nvec;
    xv[k] = ld4(v4 + (i < nvec ? i : nvec - 1));
  }
  if (has_b) {                                   // uniform over the workgroup
#pragma unroll
    for (int k = 0; k < K; ++k) {
      const int i = m.gl + k * G;
      gv[k] = ld4(b4 + (i < nvec ? i : nvec - 1));
    }
  }

  qv2_qparams qp;
  QP q{1.0f, 1.0f, 0.0f};
  double sx = 0.0, sx2_first = 0.0;
  if (ROLE != 1) {
    float mn = INFINITY, mx = -INFINITY;
    Acc4 as, as2;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      if (!on[k]) continue;
      mn = fminf(fminf(mn, xv[k].x), fminf(fminf(xv[k].y, xv[k].z), xv[k].w));
      mx = fmaxf(fmaxf(mx, xv[k].x), fmaxf(fmaxf(xv[k].y, xv[k].z), xv[k].w));
      as.add(xv[k]);
      // sum x^2 rides on the same conversion of x to fp64 (ROLE 2: the quantize step below then
      // leaves it out; same accumulators, same order, same bits as summing it there)
      if (ROLE != 1) as2.add_sq(xv[k].x, xv[k].y, xv[k].z, xv[k].w);
    }
    double v[2] = {as.total(), as2.total()};
    row_join<W, 2, true>(m, mn, mx, v, sf, sd1);
    if (ROLE == 0) {
      if (live && m.gl == 0) {
        StatPartial o;
        o.mn = mn; o.mx = mx; o.sx = v[0]; o.sx2 = v[1];
        static_cast<StatPartial*>(parts_any)[tl.part0 + r] = o;
      }
      return;
    }
    sx = v[0]; sx2_first = v[1];
    // rows are segments of a per-output-channel tensor: the scheme is symmetric and the zero-point 0
    make_params(mn, mx, QV2_SYM_CHANNEL, qp);
    q = QP{qp.scale, qp.inv_scale, 0.0f};
  } else if (live) {
    q = load_qp(params, tl.seg0 + r);
  }

  const gu32_ptr cw = (gu32_ptr)(tl.c + row_off);
  const bool has_c = tl.c != nullptr;
  Acc4 ae2, ax2, ad2, axh, axq;
#pragma unroll
  for (int k = 0; k < K; ++k) {
    if (!on[k]) continue;
    const uint32_t pk = ROLE == 2 ? quant4<COS, false, true>(xv[k], q, ae2, ax2, axh)
                                  : quant4<COS>(xv[k], q, ae2, ax2, axh);
    if (has_c) st_codes(cw + m.gl + k * G, pk);
    if (has_b) {
      ad2.add_sq(xv[k].x - gv[k].x, xv[k].y - gv[k].y, xv[k].z - gv[k].z, xv[k].w - gv[k].w);
      if (COS) axq.add_prod(xv[k], gv[k]);
    }
  }
  double e[NE];
  e[0] = ax2.total(); e[1] = ae2.total(); e[2] = ad2.total();
  if (COS) { e[NE - 2] = axh.total(); e[NE - 1] = axq.total(); }
  float u0 = 0.0f, u1 = 0.0f;
  row_join<W, NE, false>(m, u0, u1, e, sf, sd2);
  if (ROLE == 2) e[0] = sx2_first;
  if (live && m.gl == 0) {
    typename ErrRec<COS>::type o;
    o.sx2 = e[0]; o.se2 = e[1]; o.sd2 = e[2];
    set_cross(o, COS ? e[NE - 2] : 0.0, COS ? e[NE - 1] : 0.0);
    static_cast<typename ErrRec<COS>::type*>(parts_any)[tl.part0 + r] = o;
    if (ROLE == 2) {
      params_out[tl.seg0 + r] = qp;
      qv2_sums u;
      u.sum_x = sx; u.sum_x2 = e[0]; u.sum_e2 = e[1]; u.n = inner;
      sums_out[tl.seg0 + r] = u;
    }
  }
}

}  // namespace
