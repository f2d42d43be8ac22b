// HIP kernels (gfx950, wave64) and device entry points of the qv2 C ABI.
//
// Every pass is one flat launch over a tile table that spans all tensors of
// the plan: a workgroup owns one tile, reduces it and leaves one partial record
// per (tile, segment) in the workspace; a second small launch folds each
// segment's partials in a fixed order.  No floating-point atomics anywhere, so
// results are bit-stable.  The work is HBM-bound (4, 5, 8 and 9 bytes per
// element for the passes); MFMA has no role here.
//
// Compiled with -ffp-contract=off: the quantizer's fp32 steps (Sec. 2.1 Eq. 1-3,
// Sec. 4 Eq. 4-5) must each round once.  Fused multiply-adds appear only where
// written explicitly (fp64 energy accumulation).
//
// Two things the code generator needs to be told:
//  - tensor pointers come out of the tile table, so their address space is
//    unknown to the compiler; every access casts them to the global address
//    space, which turns flat_load into global_load and lets the wait-count
//    pass keep many loads in flight instead of draining them all;
//  - whether codes are stored as packed dwords, as bytes or not at all is
//    decided once per tile and selects a fully specialised loop, so the loop
//    body has no branches and all of a batch's loads are issued up front.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cfloat>
#include <cstdint>

#include "qv2_internal.h"

using namespace qv2;

namespace {

#define QV2_GLOBAL __attribute__((address_space(1)))

typedef float f4 __attribute__((ext_vector_type(4)));
typedef const QV2_GLOBAL f4* gf4_ptr;
typedef const QV2_GLOBAL float* gf_ptr;
typedef QV2_GLOBAL uint32_t* gu32_ptr;
typedef QV2_GLOBAL int8_t* gi8_ptr;

constexpr int kWave = 64;
#ifndef QV2_VEC_READ
#define QV2_VEC_READ 8              // 16-byte loads in flight per lane, read-only kernels
#endif
#ifndef QV2_NT_LOADS
#define QV2_NT_LOADS 1              // measured: +12 % HBM rate on the read-only passes
#endif
#ifndef QV2_NT_STORES
#define QV2_NT_STORES 1
#endif
constexpr int kVecRead = QV2_VEC_READ;
#ifndef QV2_VEC_QUANT_RO
#define QV2_VEC_QUANT_RO 4
#endif
constexpr int kVecQuantRO = QV2_VEC_QUANT_RO;     // 16-byte loads per lane in flight, quantize sweep without codes
constexpr int kFoldBlock = 1024;    // workgroup that folds one segment with many partials

// 16-byte streaming load of data that is read once per pass.
__device__ __forceinline__ f4 ld4(gf4_ptr p) {
#if QV2_NT_LOADS
  return __builtin_nontemporal_load(p);
#else
  return *p;
#endif
}

// Dword written once and not read again by the kernel that writes it: packed int8 codes, and
// the histogram pass's partial counts.
__device__ __forceinline__ void st_codes(gu32_ptr p, uint32_t v) {
#if QV2_NT_STORES
  __builtin_nontemporal_store(v, p);
#else
  *p = v;
#endif
}

// A tile's partial record, written by one lane.  NT: as 8-byte non-temporal stores - for
// kernels that otherwise only read (a plain store in a read-only sweep costs that sweep more
// than its bytes; the sweeps gain ~1 %); kernels that store codes keep plain stores (the fused
// quantize kernel lost 2 % with non-temporal ones).
template <bool NT, class T>
__device__ __forceinline__ void st_record(T* dst, const T& o) {
  if (NT) {
    static_assert(sizeof(T) % 8 == 0, "records are whole 8-byte words");
    typedef __attribute__((address_space(1))) unsigned long long* gu64_ptr;
    const unsigned long long* src = reinterpret_cast<const unsigned long long*>(&o);
    const gu64_ptr d = (gu64_ptr)dst;
#pragma unroll
    for (int i = 0; i < static_cast<int>(sizeof(T) / 8); ++i) __builtin_nontemporal_store(src[i], d + i);
  } else {
    *dst = o;
  }
}

// ---------------------------------------------------------------------------
// wavefront / workgroup reductions (fixed butterfly order => deterministic)
// ---------------------------------------------------------------------------
__device__ __forceinline__ float group_min(float v, int w) {
  for (int o = w >> 1; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ float group_max(float v, int w) {
  for (int o = w >> 1; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
  return v;
}
__device__ __forceinline__ double group_sum(double v, int w) {
  for (int o = w >> 1; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// Sums of N doubles over a workgroup of BLOCK threads; valid in thread 0.
template <int BLOCK, int N>
__device__ __forceinline__ void block_sum(double (&v)[N]) {
  constexpr int W = BLOCK / kWave;
#pragma unroll
  for (int k = 0; k < N; ++k) v[k] = group_sum(v[k], kWave);
  if (W == 1) return;
  __shared__ double s[N][W];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  if (lane == 0) {
#pragma unroll
    for (int k = 0; k < N; ++k) s[k][wave] = v[k];
  }
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int k = 0; k < N; ++k) {
      double t = s[k][0];
      for (int i = 1; i < W; ++i) t += s[k][i];
      v[k] = t;
    }
  }
}

template <int BLOCK>
__device__ __forceinline__ void block_sum3(double& a, double& b, double& c) {
  double v[3] = {a, b, c};
  block_sum<BLOCK, 3>(v);
  a = v[0]; b = v[1]; c = v[2];
}

template <int BLOCK>
__device__ __forceinline__ void block_minmax(float& mn, float& mx) {
  constexpr int W = BLOCK / kWave;
  mn = group_min(mn, kWave); mx = group_max(mx, kWave);
  if (W == 1) return;
  __shared__ float s[2][W];
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  if (lane == 0) { s[0][wave] = mn; s[1][wave] = mx; }
  __syncthreads();
  if (threadIdx.x == 0) {
    mn = s[0][0]; mx = s[1][0];
    for (int i = 1; i < W; ++i) { mn = fminf(mn, s[0][i]); mx = fmaxf(mx, s[1][i]); }
  }
}

// Four independent fp64 accumulators, one per vector component.  Energies are
// accumulated in fp64 from the first element on, so the whole fp32 range of
// inputs is safe (x*x can leave the fp32 range) and no fp32 rounding builds up.
struct Acc4 {
  double a = 0.0, b = 0.0, c = 0.0, d = 0.0;
  __device__ __forceinline__ void add(const f4& v) {
    a += static_cast<double>(v.x); b += static_cast<double>(v.y);
    c += static_cast<double>(v.z); d += static_cast<double>(v.w);
  }
  __device__ __forceinline__ void add_sq(float x, float y, float z, float w) {
    const double dx = x, dy = y, dz = z, dw = w;
    a = fma(dx, dx, a); b = fma(dy, dy, b); c = fma(dz, dz, c); d = fma(dw, dw, d);
  }
  __device__ __forceinline__ void add_prod(const f4& u, const f4& v) {
    a = fma(static_cast<double>(u.x), static_cast<double>(v.x), a);
    b = fma(static_cast<double>(u.y), static_cast<double>(v.y), b);
    c = fma(static_cast<double>(u.z), static_cast<double>(v.z), c);
    d = fma(static_cast<double>(u.w), static_cast<double>(v.w), d);
  }
  __device__ __forceinline__ double total() const { return (a + b) + (c + d); }
};

// Elements before the first 16-byte boundary of p (0..3, capped by len).
__device__ __forceinline__ int head_elems(const void* p, int len) {
  const int h = static_cast<int>(((16u - (reinterpret_cast<uintptr_t>(p) & 15u)) & 15u) >> 2);
  return h < len ? h : len;
}

// ---------------------------------------------------------------------------
// quantizer: Sec. 2.1 Eq. 1 / Sec. 4 Eq. 5 then Eq. 3, each step one fp32 rounding
// ---------------------------------------------------------------------------
struct QP { float scale, inv, zpf; };

// Returns the code as a float in [-128,127]; xhat is the dequantized value, err = x - xhat.
__device__ __forceinline__ float quant1(float x, const QP& q, float& err, float& xhat) {
  const float t = x * q.inv;                       // fp32 multiply
  const float r = rintf(t);                        // round half to even
  // integer add of the zero-point: exact in fp32 below 2^24, saturates above
  const float c = fminf(fmaxf(r + q.zpf, -128.0f), 127.0f);
  xhat = (c - q.zpf) * q.scale;                    // exact difference, one multiply
  err = x - xhat;
  return c;
}

// COS: also accumulate sum x*xhat (the cross term of the cosine similarity, Sec. 6.1 Eq. 8)
// X2 = false leaves sum x^2 out (the caller already has it from the calibration sweep)
template <bool COS, bool X2 = true>
__device__ __forceinline__ uint32_t quant4(const f4& v, const QP& q, Acc4& se2, Acc4& sx2, Acc4& sxh) {
  float e0, e1, e2, e3, h0, h1, h2, h3;
  const int c0 = static_cast<int>(quant1(v.x, q, e0, h0));
  const int c1 = static_cast<int>(quant1(v.y, q, e1, h1));
  const int c2 = static_cast<int>(quant1(v.z, q, e2, h2));
  const int c3 = static_cast<int>(quant1(v.w, q, e3, h3));
  const f4 h = {h0, h1, h2, h3};
  se2.add_sq(e0, e1, e2, e3);
  if (X2) sx2.add_sq(v.x, v.y, v.z, v.w);
  if (COS) sxh.add_prod(v, h);
  return (static_cast<uint32_t>(c0) & 0xffu) | ((static_cast<uint32_t>(c1) & 0xffu) << 8) |
         ((static_cast<uint32_t>(c2) & 0xffu) << 16) | (static_cast<uint32_t>(c3) << 24);
}

__device__ __forceinline__ QP load_qp(const qv2_qparams* __restrict__ params, int seg) {
  const qv2_qparams p = params[seg];
  return QP{p.scale, p.inv_scale, static_cast<float>(p.zp)};
}

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
template <int BLOCK, int V, bool WITHB, bool COS>
__device__ __forceinline__ void stats_body(gf4_ptr v4, gf4_ptr b4, int nvec, StatAcc& a) {
  const int tid = threadIdx.x;
  int base = 0;
  for (; base + V * BLOCK <= nvec; base += V * BLOCK) {          // uniform: whole batches
    f4 r[V], g[V];
#pragma unroll
    for (int u = 0; u < V; ++u) {
      r[u] = ld4(v4 + base + u * BLOCK + tid);
      if (WITHB) g[u] = ld4(b4 + base + u * BLOCK + tid);
    }
#pragma unroll
    for (int u = 0; u < V; ++u) {
      a.take(r[u]);
      if (WITHB) a.d2.add_sq(r[u].x - g[u].x, r[u].y - g[u].y, r[u].z - g[u].z, r[u].w - g[u].w);
      if (WITHB && COS) a.xq.add_prod(r[u], g[u]);
    }
  }
  for (int i = base + tid; i < nvec; i += BLOCK) {
    const f4 r = ld4(v4 + i);
    a.take(r);
    if (WITHB) {
      const f4 g = ld4(b4 + i);
      a.d2.add_sq(r.x - g.x, r.y - g.y, r.z - g.z, r.w - g.w);
      if (COS) a.xq.add_prod(r, g);
    }
  }
}

// PAIR: tiles whose tensor has a quantized-run partner also yield sum (x - qrun)^2 (Algorithm 2's
// D[i] against Q[i]) from the same visit: 8 B read per element, nothing but the partial written.
// COS: also sum x * qrun, the cross term of cos(x, qrun) (Sec. 6.1 Eq. 8).
template <int BLOCK, int V, bool PAIR, bool COS>
__global__ __launch_bounds__(BLOCK) void k_stats_stream(const Tile* __restrict__ tiles,
                                                        typename StatRec<PAIR, COS>::type* __restrict__ parts) {
  const Tile tl = tiles[blockIdx.x];
  const gf_ptr p = (gf_ptr)tl.x;
  const gf_ptr b = (gf_ptr)tl.q;
  const int len = tl.len, tid = threadIdx.x;
  const int head = head_elems(tl.x, len);
  const int body = len - head, nvec = body >> 2, tail = body & 3;
  const bool has_b = PAIR && tl.q != nullptr;
  // qrun at a different offset inside 16 bytes than x: its energy is taken element-wise
  const bool b_vec = has_b && (((reinterpret_cast<uintptr_t>(tl.x) ^ reinterpret_cast<uintptr_t>(tl.q)) & 15u) == 0);

  float mn = INFINITY, mx = -INFINITY;
  double sx = 0.0, sx2 = 0.0, sd2 = 0.0, sxq = 0.0;
  if (has_b && !b_vec) {
    for (int i = tid; i < len; i += BLOCK) {
      const float xv = p[i], qv = b[i];
      const double d = static_cast<double>(xv - qv);
      sd2 = fma(d, d, sd2);
      if (COS) sxq = fma(static_cast<double>(xv), static_cast<double>(qv), sxq);
    }
  }
  for (int k = 0; k < 2; ++k) {
    const bool on = k == 0 ? tid < head : tid < tail;
    if (!on) continue;
    const int idx = k == 0 ? tid : head + (nvec << 2) + tid;
    const float v = p[idx];
    mn = fminf(mn, v); mx = fmaxf(mx, v);
    sx += v; sx2 += static_cast<double>(v) * v;
    if (b_vec) {
      const float qv = b[idx], d = v - qv;
      sd2 += static_cast<double>(d) * d;
      if (COS) sxq = fma(static_cast<double>(v), static_cast<double>(qv), sxq);
    }
  }
  const gf4_ptr v4 = (gf4_ptr)(tl.x + head);
  const gf4_ptr b4 = (gf4_ptr)(tl.q + head);
  StatAcc a;
  if (PAIR && b_vec) stats_body<BLOCK, (V > 1 ? V / 2 : 1), true, COS>(v4, b4, nvec, a);
  else stats_body<BLOCK, V, false, false>(v4, b4, nvec, a);
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

// ---------------------------------------------------------------------------
// folds.  An item's partials (a segment's, or a tensor's for the pair sums) are folded in a
// fixed order: lane- (or thread-) strided, then a butterfly.  One launch of 1024-thread
// workgroups serves all items: the first n_wide workgroups take one listed item each (those
// with more than kFoldWaveMax partials) with all their threads, every other workgroup takes
// 16 items, one per wavefront, and leaves the listed ones alone.
// ---------------------------------------------------------------------------
constexpr int kFoldPerBlock = kFoldBlock / kWave;

struct FoldIdx {
  int id, lane, stride;
  bool wide, active;
  // b: index of the workgroup within its family of n_wide + ceil(n / 16) workgroups
  __device__ __forceinline__ FoldIdx(int b, const int* ids, int n_wide, int n) {
    wide = b < n_wide;
    if (wide) {
      id = ids[b]; lane = threadIdx.x; stride = kFoldBlock; active = true;
    } else {
      id = (b - n_wide) * kFoldPerBlock + (threadIdx.x >> 6); lane = threadIdx.x & (kWave - 1);
      stride = kWave; active = id < n;
    }
  }
};

int fold_blocks(int n_wide, int n) { return n_wide + (n + kFoldPerBlock - 1) / kFoldPerBlock; }

// `wide` is uniform over the workgroup (the wide form holds barriers)
__device__ __forceinline__ void fold_sum3(bool wide, double& a, double& b, double& c) {
  if (wide) {
    block_sum3<kFoldBlock>(a, b, c);
  } else {
    a = group_sum(a, kWave); b = group_sum(b, kWave); c = group_sum(c, kWave);
  }
}

// Calibration fold: range and sums of every segment, then its parameters (Eq. 2, Eq. 4).
template <class REC>
__device__ __forceinline__ void fold_stats_item(const FoldIdx& f, const Segment* __restrict__ segs,
                                                const REC* __restrict__ parts, qv2_qparams* __restrict__ params,
                                                qv2_sums* __restrict__ sums, int skip_below) {
  if (!f.active) return;
  const Segment sg = segs[f.id];
  if (!f.wide && sg.snp > kFoldWaveMax) return;    // left to its own workgroup
  if (sg.sp0 < skip_below) return;                 // row-group segment finished by its own kernel
  float mn = INFINITY, mx = -INFINITY;
  double sx = 0.0, sx2 = 0.0, unused = 0.0;
#pragma unroll 4
  for (int i = f.lane; i < sg.snp; i += f.stride) {
    const REC q = parts[sg.sp0 + i];
    mn = fminf(mn, q.mn); mx = fmaxf(mx, q.mx);
    sx += q.sx; sx2 += q.sx2;
  }
  if (f.wide) {
    block_minmax<kFoldBlock>(mn, mx);
    __syncthreads();
  } else {
    mn = group_min(mn, kWave); mx = group_max(mx, kWave);
  }
  fold_sum3(f.wide, sx, sx2, unused);
  if (f.lane == 0) {
    qv2_qparams qp;
    make_params(mn, mx, sg.scheme, qp);
    params[f.id] = qp;
    qv2_sums o;
    o.sum_x = sx; o.sum_x2 = sx2; o.sum_e2 = 0.0; o.n = sg.n;
    sums[f.id] = o;
  }
}

// pair energies of one tensor from calibration partials that carry them; tensors not listed
// there (n == 0) are left to the fold after the quantize pass
__device__ __forceinline__ double stat_cross(const StatPairPartial&) { return 0.0; }
__device__ __forceinline__ double stat_cross(const StatPairCosPartial& p) { return p.sxq; }

template <class REC>
__device__ __forceinline__ void fold_statpair_item(const FoldIdx& f, const PairTensor* __restrict__ pt,
                                                   const REC* __restrict__ parts,
                                                   qv2_pair_sums* __restrict__ out,
                                                   double* __restrict__ pair_xq) {
  if (!f.active) return;
  const PairTensor p = pt[f.id];
  if (p.n == 0) return;
  if (!f.wide && p.nparts > kFoldWaveMax) return;
  double sr2 = 0.0, sd2 = 0.0, sxq = 0.0;
#pragma unroll 4
  for (int i = f.lane; i < p.nparts; i += f.stride) {
    const REC q = parts[p.part0 + i];
    sr2 += q.sx2; sd2 += q.sd2; sxq += stat_cross(q);
  }
  fold_sum3(f.wide, sr2, sd2, sxq);
  if (f.lane == 0) {
    qv2_pair_sums o;
    o.sum_ref2 = sr2; o.sum_d2 = sd2; o.n = p.n; o._pad = 0;
    out[f.id] = o;
    if (pair_xq) pair_xq[f.id] = sxq;
  }
}

template <class REC>
struct StatFoldArgs {
  const Segment* segs; int nseg; const int* wide_segs; int n_wide_segs;
  const REC* parts; qv2_qparams* params; qv2_sums* sums; int skip_below;
  const PairTensor* pt; int nt; const int* wide_pt; int n_wide_pt;     // pair_out == null: none
  qv2_pair_sums* pair_out; double* pair_xq;
  int seg_blocks;
};

__device__ __forceinline__ void fold_statpair_family(const StatFoldArgs<StatPartial>&, int) {}
template <class REC>
__device__ __forceinline__ void fold_statpair_family(const StatFoldArgs<REC>& a, int b) {
  fold_statpair_item<REC>(FoldIdx(b, a.wide_pt, a.n_wide_pt, a.nt), a.pt, a.parts, a.pair_out, a.pair_xq);
}

template <class REC>
__global__ __launch_bounds__(kFoldBlock) void k_fold_stats(const StatFoldArgs<REC> a) {
  const int b = blockIdx.x;
  if (b < a.seg_blocks)
    fold_stats_item<REC>(FoldIdx(b, a.wide_segs, a.n_wide_segs, a.nseg), a.segs, a.parts, a.params, a.sums,
                         a.skip_below);
  else
    fold_statpair_family(a, b - a.seg_blocks);
}

// cross terms of a partial record (0 where the record has none)
__device__ __forceinline__ double cross_xh(const ErrPartial3&) { return 0.0; }
__device__ __forceinline__ double cross_xh(const ErrPartial5& p) { return p.sxh; }
__device__ __forceinline__ double cross_xq(const ErrPartial&) { return 0.0; }
__device__ __forceinline__ double cross_xq(const ErrPartial3&) { return 0.0; }
__device__ __forceinline__ double cross_xq(const ErrPartial5& p) { return p.sxq; }
// second energy of a partial record: the pair-noise energy
__device__ __forceinline__ double pair_energy(const ErrPartial& p) { return p.se2; }
__device__ __forceinline__ double pair_energy(const ErrPartial3& p) { return p.sd2; }
__device__ __forceinline__ double pair_energy(const ErrPartial5& p) { return p.sd2; }

// error energies of one segment
template <class P>
__device__ __forceinline__ void fold_err_item(const FoldIdx& f, const Segment* __restrict__ segs,
                                              const P* __restrict__ parts, qv2_sums* __restrict__ sums,
                                              double* __restrict__ seg_xxhat, int skip_below,
                                              bool keep_x2) {
  if (!f.active) return;
  const Segment sg = segs[f.id];
  if (!f.wide && sg.enp > kFoldWaveMax) return;
  if (sg.ep0 < skip_below) {         // a row its kernel has finished: only the cross term is left to copy
    if (seg_xxhat && f.lane == 0) seg_xxhat[f.id] = cross_xh(parts[sg.ep0]);
    return;
  }
  double sx2 = 0.0, se2 = 0.0, sxh = 0.0;
#pragma unroll 4
  for (int i = f.lane; i < sg.enp; i += f.stride) {
    const P q = parts[sg.ep0 + i];
    sx2 += q.sx2; se2 += q.se2; sxh += cross_xh(q);
  }
  fold_sum3(f.wide, sx2, se2, sxh);
  if (f.lane == 0) {
    if (!keep_x2) sums[f.id].sum_x2 = sx2;         // else the calibration sweep's sum stays
    sums[f.id].sum_e2 = se2; sums[f.id].n = sg.n;
    if (seg_xxhat) seg_xxhat[f.id] = sxh;
  }
}

// pair energies of one tensor
template <class P>
__device__ __forceinline__ void fold_pair_item(const FoldIdx& f, const PairTensor* __restrict__ pt,
                                               const P* __restrict__ parts, qv2_pair_sums* __restrict__ out,
                                               double* __restrict__ pair_xq,
                                               const PairTensor* __restrict__ done = nullptr) {
  if (!f.active) return;
  if (done && done[f.id].n != 0) return;           // already folded from the calibration partials
  const PairTensor p = pt[f.id];
  if (!f.wide && p.nparts > kFoldWaveMax) return;
  double sr2 = 0.0, sd2 = 0.0, sxq = 0.0;
#pragma unroll 4
  for (int i = f.lane; i < p.nparts; i += f.stride) {
    const P q = parts[p.part0 + i];
    sr2 += q.sx2; sd2 += pair_energy(q); sxq += cross_xq(q);
  }
  fold_sum3(f.wide, sr2, sd2, sxq);
  if (f.lane == 0) {
    qv2_pair_sums o;
    o.sum_ref2 = sr2; o.sum_d2 = sd2; o.n = p.n; o._pad = 0;
    out[f.id] = o;
    if (pair_xq) pair_xq[f.id] = sxq;
  }
}

// What a fold launch after a quantize pass works on: the segments, and (fused passes)
// the tensors with a quantized-run partner, whose workgroups follow those of the segments.
template <class P>
struct QuantFoldArgs {
  const Segment* segs; int nseg; const int* wide_segs; int n_wide_segs;
  qv2_sums* sums; double* seg_xxhat; int skip_below; bool keep_x2;
  const PairTensor* pt; int nt; const int* wide_pt; int n_wide_pt;     // pair_out == null: none
  qv2_pair_sums* pair_out; double* pair_xq;
  const PairTensor* pair_done;               // tensors with n != 0 here are skipped (may be null)
  const P* parts;
  int seg_blocks;
};

template <class P>
__global__ __launch_bounds__(kFoldBlock) void k_fold_quant(const QuantFoldArgs<P> a) {
  const int b = blockIdx.x;
  if (b < a.seg_blocks) {
    fold_err_item<P>(FoldIdx(b, a.wide_segs, a.n_wide_segs, a.nseg), a.segs, a.parts, a.sums,
                     a.seg_xxhat, a.skip_below, a.keep_x2);
  } else {
    fold_pair_item<P>(FoldIdx(b - a.seg_blocks, a.wide_pt, a.n_wide_pt, a.nt), a.pt, a.parts,
                      a.pair_out, a.pair_xq, a.pair_done);
  }
}

// fold of the separate pair pass
__global__ __launch_bounds__(kFoldBlock) void k_fold_pair(
    const PairTensor* __restrict__ pt, int nt, const int* __restrict__ ids, int n_wide,
    const ErrPartial* __restrict__ parts, qv2_pair_sums* __restrict__ out) {
  fold_pair_item<ErrPartial>(FoldIdx(blockIdx.x, ids, n_wide, nt), pt, parts, out, nullptr);
}

// ---------------------------------------------------------------------------
// pass 2 (Eq. 1, 3, 5 and the energies of Eq. 6-7), optionally with pass 3
// (Algorithm 2's D[i] vs Q[i]) in the same sweep: stream tiles.
// Per element 4 B read + 1 B code written (+ 4 B of qrun read when PAIR).
// ---------------------------------------------------------------------------
// STORE: 0 no code buffer, 1 packed dwords, 2 single bytes (misaligned code buffer)
template <int BLOCK, int V, int STORE, bool PAIR, bool COS, bool X2>
__device__ __forceinline__ void quant_body(gf4_ptr v4, gf4_ptr b4, gu32_ptr cw, gi8_ptr cb, int nvec,
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
      if (PAIR) g[u] = ld4(b4 + base + u * BLOCK + tid);
    }
#pragma unroll
    for (int u = 0; u < V; ++u) {
      put(base + u * BLOCK + tid, quant4<COS, X2>(r[u], q, ae2, ax2, axh));
      if (PAIR) ad2.add_sq(r[u].x - g[u].x, r[u].y - g[u].y, r[u].z - g[u].z, r[u].w - g[u].w);
      if (PAIR && COS) axq.add_prod(r[u], g[u]);
    }
  }
  for (int i = base + tid; i < nvec; i += BLOCK) {
    const f4 r = ld4(v4 + i);
    put(i, quant4<COS, X2>(r, q, ae2, ax2, axh));
    if (PAIR) {
      const f4 g = ld4(b4 + i);
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
__device__ __forceinline__ void set_cross(ErrPartial3&, double, double) {}
__device__ __forceinline__ void set_cross(ErrPartial5& o, double sxh, double sxq) { o.sxh = sxh; o.sxq = sxq; }

// RO: tiles of tensors without a code buffer (no store is compiled in; long tiles).
template <int BLOCK, int V, bool PAIR, bool COS, bool X2 = true, bool RO = false>
__global__ __launch_bounds__(BLOCK, (PAIR ? QV2_QUANT_WAVES_PER_EU : QV2_QUANT_PLAIN_WAVES_PER_EU)) void k_quant_stream(
    const Tile* __restrict__ tiles, const qv2_qparams* __restrict__ params,
    typename ErrRec<COS>::type* __restrict__ parts) {
  // Workgroups go to the 8 XCDs in turn.  The plain sweep (one read stream, one store stream)
  // runs 1.5 % faster (6 % without codes) when each XCD works through one contiguous eighth
  // of the tile table instead of every eighth tile; with qrun as a third stream it does not.
  int bt = blockIdx.x;
  if (!PAIR) {
    const int per = gridDim.x >> 3;
    if (bt < (per << 3)) bt = (bt & 7) * per + (bt >> 3);
  }
  const Tile tl = tiles[bt];
  const QP q = load_qp(params, tl.seg0);
  const gf_ptr p = (gf_ptr)tl.x;
  const gf_ptr b = (gf_ptr)tl.q;
  const gi8_ptr c = (gi8_ptr)tl.c;
  const bool has_c = !RO && tl.c != nullptr;
  const bool has_b = PAIR && tl.q != nullptr;
  const int len = tl.len, tid = threadIdx.x;
  double sx2 = 0.0, se2 = 0.0, sd2 = 0.0, sxh = 0.0, sxq = 0.0;

  // qrun at a different offset inside 16 bytes than x: its energy is taken element-wise
  const bool b_vec = has_b && (((reinterpret_cast<uintptr_t>(tl.x) ^ reinterpret_cast<uintptr_t>(tl.q)) & 15u) == 0);
  if (has_b && !b_vec) {
    for (int i = tid; i < len; i += BLOCK) {
      const float xv = p[i], qv = b[i];
      const double d = static_cast<double>(xv - qv);
      sd2 = fma(d, d, sd2);
      if (COS) sxq = fma(static_cast<double>(xv), static_cast<double>(qv), sxq);
    }
  }
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
    if (b_vec) {
      const float qv = b[idx], d = v - qv;
      sd2 += static_cast<double>(d) * d;
      if (COS) sxq = fma(static_cast<double>(v), static_cast<double>(qv), sxq);
    }
  }
  const gf4_ptr v4 = (gf4_ptr)(tl.x + head);
  const gf4_ptr b4 = (gf4_ptr)(tl.q + head);
  const gi8_ptr cb = c + head;
  const gu32_ptr cw = (gu32_ptr)(tl.c + head);
  const bool cw_ok = has_c && ((reinterpret_cast<uintptr_t>(tl.c + head) & 3u) == 0);
  Acc4 ae2, ax2, ad2, axh, axq;
  if (b_vec) {
    if (cw_ok) quant_body<BLOCK, V, 1, PAIR, COS, X2>(v4, b4, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
    else if (has_c) quant_body<BLOCK, V, 2, PAIR, COS, X2>(v4, b4, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
    else quant_body<BLOCK, V, 0, PAIR, COS, X2>(v4, b4, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
  } else {
    if (cw_ok) quant_body<BLOCK, V, 1, false, COS, X2>(v4, b4, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
    else if (has_c) quant_body<BLOCK, V, 2, false, COS, X2>(v4, b4, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
    else quant_body<BLOCK, V, 0, false, COS, X2>(v4, b4, cw, cb, nvec, q, ae2, ax2, ad2, axh, axq);
  }
  se2 += ae2.total(); sx2 += ax2.total(); sd2 += ad2.total();
  typename ErrRec<COS>::type o;
  if (COS) {
    double v[5] = {sx2, se2, sd2, sxh + axh.total(), sxq + axq.total()};
    block_sum<BLOCK, 5>(v);
    o.sx2 = v[0]; o.se2 = v[1]; o.sd2 = v[2];
    set_cross(o, v[3], v[4]);
  } else if (!X2 && !PAIR) {
    double v[1] = {se2};                            // the only energy this form takes
    block_sum<BLOCK, 1>(v);
    o.sx2 = 0.0; o.se2 = v[0]; o.sd2 = 0.0;
  } else {
    block_sum3<BLOCK>(sx2, se2, sd2);
    o.sx2 = sx2; o.se2 = se2; o.sd2 = sd2;
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
                                                    const Segment* __restrict__ segs,
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
  double sx = 0.0;
  if (ROLE != 1) {
    float mn = INFINITY, mx = -INFINITY;
    Acc4 as, as2;
#pragma unroll
    for (int k = 0; k < K; ++k) {
      if (!on[k]) continue;
      mn = fminf(fminf(mn, xv[k].x), fminf(fminf(xv[k].y, xv[k].z), xv[k].w));
      mx = fmaxf(fmaxf(mx, xv[k].x), fmaxf(fmaxf(xv[k].y, xv[k].z), xv[k].w));
      as.add(xv[k]);
      if (ROLE == 0) as2.add_sq(xv[k].x, xv[k].y, xv[k].z, xv[k].w);
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
    sx = v[0];
    make_params(mn, mx, segs[tl.seg0].scheme, qp);           // one tensor, one scheme per tile
    q = QP{qp.scale, qp.inv_scale, static_cast<float>(qp.zp)};
  } else if (live) {
    q = load_qp(params, tl.seg0 + r);
  }

  const gu32_ptr cw = (gu32_ptr)(tl.c + row_off);
  const bool has_c = tl.c != nullptr;
  Acc4 ae2, ax2, ad2, axh, axq;
#pragma unroll
  for (int k = 0; k < K; ++k) {
    if (!on[k]) continue;
    const uint32_t pk = quant4<COS>(xv[k], q, ae2, ax2, axh);
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

// ---------------------------------------------------------------------------
// pass 3 alone (Algorithm 2: CalculateSQNR / CalculateMSE on D[i] and Q[i])
// ---------------------------------------------------------------------------
template <int BLOCK, int V>
__global__ __launch_bounds__(BLOCK) void k_pair_stream(const Tile* __restrict__ tiles,
                                                       ErrPartial* __restrict__ parts) {
  const Tile tl = tiles[blockIdx.x];
  const gf_ptr a = (gf_ptr)tl.x;
  const gf_ptr b = (gf_ptr)tl.q;
  const int len = tl.len, tid = threadIdx.x;
  double sr2 = 0.0, sd2 = 0.0, unused = 0.0;

  if (((reinterpret_cast<uintptr_t>(tl.x) ^ reinterpret_cast<uintptr_t>(tl.q)) & 15u) != 0) {
    // the two tensors sit at different offsets within 16 bytes: element loads
    for (int i = tid; i < len; i += BLOCK) {
      const float x = a[i], d = x - b[i];
      sr2 = fma(static_cast<double>(x), static_cast<double>(x), sr2);
      sd2 = fma(static_cast<double>(d), static_cast<double>(d), sd2);
    }
  } else {
    const int head = head_elems(tl.x, len);
    const int body = len - head, nvec = body >> 2, tail = body & 3;
    if (tid < head) {
      const float x = a[tid], d = x - b[tid];
      sr2 += static_cast<double>(x) * x; sd2 += static_cast<double>(d) * d;
    }
    if (tid < tail) {
      const int idx = head + (nvec << 2) + tid;
      const float x = a[idx], d = x - b[idx];
      sr2 += static_cast<double>(x) * x; sd2 += static_cast<double>(d) * d;
    }
    const gf4_ptr a4 = (gf4_ptr)(tl.x + head);
    const gf4_ptr b4 = (gf4_ptr)(tl.q + head);
    Acc4 ar2, ad2;
    int base = 0;
    for (; base + V * BLOCK <= nvec; base += V * BLOCK) {
      f4 ra[V], rb[V];
#pragma unroll
      for (int u = 0; u < V; ++u) { ra[u] = ld4(a4 + base + u * BLOCK + tid); rb[u] = ld4(b4 + base + u * BLOCK + tid); }
#pragma unroll
      for (int u = 0; u < V; ++u) {
        ar2.add_sq(ra[u].x, ra[u].y, ra[u].z, ra[u].w);
        ad2.add_sq(ra[u].x - rb[u].x, ra[u].y - rb[u].y, ra[u].z - rb[u].z, ra[u].w - rb[u].w);
      }
    }
    for (int i = base + tid; i < nvec; i += BLOCK) {
      const f4 x = ld4(a4 + i), y = ld4(b4 + i);
      ar2.add_sq(x.x, x.y, x.z, x.w);
      ad2.add_sq(x.x - y.x, x.y - y.y, x.z - y.z, x.w - y.w);
    }
    sr2 += ar2.total(); sd2 += ad2.total();
  }
  block_sum3<BLOCK>(sr2, sd2, unused);
  if (tid == 0) {
    ErrPartial o;
    o.sx2 = sr2; o.se2 = sd2;
    st_record<true>(&parts[tl.part0], o);
  }
}

// ---------------------------------------------------------------------------
// calibration histograms (Sec. 5, calibration stage), the input of the KL
// divergence of Sec. 6.1 Eq. 9.  Integer counts only, so any order is exact.
// ---------------------------------------------------------------------------
// Per-tensor range from the per-segment calibration: one wavefront per tensor.
__global__ __launch_bounds__(256) void k_hist_range(const HistTensor* __restrict__ ht, int n,
                                                    const qv2_qparams* __restrict__ params,
                                                    float2* __restrict__ range) {
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & (kWave - 1);
  if (t >= n) return;
  const HistTensor h = ht[t];
  float lo = INFINITY, hi = -INFINITY;
  for (int i = lane; i < h.nseg; i += kWave) {
    lo = fminf(lo, params[h.seg0 + i].min);
    hi = fmaxf(hi, params[h.seg0 + i].max);
  }
  lo = group_min(lo, kWave); hi = group_max(hi, kWave);
  if (lane == 0) range[t] = make_float2(lo, hi);
}

struct Binner { float lo, inv_w, top; int idx0; };

// bin = clamp(floor((x - lo) * inv_w), 0, nbins - 1), each step one fp32 rounding
__device__ __forceinline__ int bin_of(float x, const Binner& b) {
  const float t = (x - b.lo) * b.inv_w;
  float f = floorf(t);
  f = fminf(fmaxf(f, 0.0f), b.top);                 // maxNum also turns NaN into 0
  return static_cast<int>(f);
}

// One stream of a chunk into an LDS histogram.  The bin that holds the value 0 (half of
// a post-ReLU tensor) is counted in a register and added once per wavefront.
template <int BLOCK>
__device__ __forceinline__ void hist_stream(const float* x, int len, const Binner& b, uint32_t* h) {
  const int tid = threadIdx.x;
  const gf_ptr p = (gf_ptr)x;
  const int head = head_elems(x, len);
  const int body = len - head, nvec = body >> 2, tail = body & 3;
  uint32_t zeros = 0;
  auto hit = [&](float v) {
    const int i = bin_of(v, b);
    if (i == b.idx0) ++zeros; else atomicAdd(&h[i], 1u);
  };
  if (tid < head) hit(p[tid]);
  if (tid < tail) hit(p[head + (nvec << 2) + tid]);
  const gf4_ptr v4 = (gf4_ptr)(x + head);
  constexpr int V = 4;
  int base = 0;
  for (; base + V * BLOCK <= nvec; base += V * BLOCK) {
    f4 r[V];
#pragma unroll
    for (int u = 0; u < V; ++u) r[u] = ld4(v4 + base + u * BLOCK + tid);
#pragma unroll
    for (int u = 0; u < V; ++u) { hit(r[u].x); hit(r[u].y); hit(r[u].z); hit(r[u].w); }
  }
  for (int i = base + tid; i < nvec; i += BLOCK) {
    const f4 r = ld4(v4 + i);
    hit(r.x); hit(r.y); hit(r.z); hit(r.w);
  }
  for (int o = kWave >> 1; o > 0; o >>= 1) zeros += __shfl_xor(zeros, o);
  if ((tid & (kWave - 1)) == 0 && zeros) atomicAdd(&h[b.idx0], zeros);
}

template <int BLOCK>
__global__ __launch_bounds__(BLOCK) void k_hist(const Tile* __restrict__ tiles,
                                                const float2* __restrict__ range, int nbins,
                                                uint32_t* __restrict__ partial) {
  __shared__ uint32_t h[2][kHistMaxBins];
  const Tile tl = tiles[blockIdx.x];
  const float2 r = range[tl.tensor];
  Binner b;
  b.lo = r.x;
  const float w = r.y - r.x;
  b.inv_w = (w > 0.0f && w <= FLT_MAX) ? static_cast<float>(nbins) / w : 0.0f;
  b.top = static_cast<float>(nbins - 1);
  b.idx0 = bin_of(0.0f, b);
  for (int i = threadIdx.x; i < nbins; i += BLOCK) { h[0][i] = 0; h[1][i] = 0; }
  __syncthreads();
  hist_stream<BLOCK>(tl.x, tl.len, b, h[0]);
  if (tl.q) hist_stream<BLOCK>(tl.q, tl.len, b, h[1]);
  __syncthreads();
  // non-temporal: these few stores ride in a read-only stream and cost it least that way
  const gu32_ptr out = (gu32_ptr)(partial + static_cast<size_t>(tl.part0) * 2 * nbins);
  for (int i = threadIdx.x; i < nbins; i += BLOCK) { st_codes(out + i, h[0][i]); st_codes(out + nbins + i, h[1][i]); }
}

// Sums a tensor's chunk histograms: ceil(nbins / 256) workgroups per tensor.
__global__ __launch_bounds__(256) void k_hist_fold(const HistTensor* __restrict__ ht, int nbins,
                                                   const uint32_t* __restrict__ partial,
                                                   unsigned long long* __restrict__ hist_x,
                                                   unsigned long long* __restrict__ hist_q) {
  const int per = (nbins + 255) / 256;
  const int t = blockIdx.x / per, i = (blockIdx.x % per) * 256 + threadIdx.x;
  if (i >= nbins) return;
  const HistTensor h = ht[t];
  unsigned long long a = 0, b = 0;
  const size_t pitch = static_cast<size_t>(2) * nbins;
  const uint32_t* src = partial + h.chunk0 * pitch + i;
  int c = 0;
  for (; c + 8 <= h.nchunks; c += 8, src += 8 * pitch) {        // 16 loads in flight; integer sums: any order
    uint32_t va[8], vb[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) { va[u] = src[u * pitch]; vb[u] = src[u * pitch + nbins]; }
#pragma unroll
    for (int u = 0; u < 8; ++u) { a += va[u]; b += vb[u]; }
  }
  for (; c < h.nchunks; ++c, src += pitch) { a += src[0]; b += src[nbins]; }
  hist_x[static_cast<size_t>(t) * nbins + i] = a;
  if (hist_q) hist_q[static_cast<size_t>(t) * nbins + i] = b;
}

// Per-tensor fold of the per-segment results: one 256-thread workgroup per tensor (thread-
// strided over the segments, butterfly per wavefront, then the four wavefronts in order).
__global__ __launch_bounds__(256) void k_tensor_fold(const HistTensor* __restrict__ ht, int n,
                                                     const qv2_qparams* __restrict__ params,
                                                     const qv2_sums* __restrict__ sums,
                                                     qv2_tensor_sums* __restrict__ out) {
  __shared__ long long scnt[256 / kWave];
  const int t = blockIdx.x, tid = threadIdx.x;
  const HistTensor h = ht[t];
  float mn = INFINITY, mx = -INFINITY;
  double sx = 0.0, sx2 = 0.0, se2 = 0.0;
  long long cnt = 0;
  for (int i = tid; i < h.nseg; i += 256) {
    const qv2_qparams p = params[h.seg0 + i];
    const qv2_sums u = sums[h.seg0 + i];
    mn = fminf(mn, p.min); mx = fmaxf(mx, p.max);
    sx += u.sum_x; sx2 += u.sum_x2; se2 += u.sum_e2; cnt += u.n;
  }
  for (int o = kWave >> 1; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
  if ((tid & (kWave - 1)) == 0) scnt[tid >> 6] = cnt;
  block_minmax<256>(mn, mx);                       // holds a barrier: scnt is visible after it
  block_sum3<256>(sx, sx2, se2);
  if (tid == 0) {
    qv2_tensor_sums o;
    o.sum_x = sx; o.sum_x2 = sx2; o.sum_e2 = se2; o.min = mn; o.max = mx;
    o.n = scnt[0] + scnt[1] + scnt[2] + scnt[3];
    o._pad[0] = o._pad[1] = 0;
    out[t] = o;
  }
}

// ---------------------------------------------------------------------------
// conv + BN folding (Sec. 6.3 Eq. 12): A = (gamma / sqrt(var)) * W per output channel,
// C = (gamma / sqrt(var)) * (B - mu) + beta.  One workgroup column per channel.
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_bn_fold(const float* w, long long inner,
                                                 const float* __restrict__ gamma,
                                                 const float* __restrict__ var,
                                                 const float* __restrict__ bias,
                                                 const float* __restrict__ mean,
                                                 const float* __restrict__ beta,
                                                 float* w_out, float* __restrict__ bias_out) {
  const long long c = blockIdx.y;
  const float f = gamma[c] / sqrtf(var[c]);          // correctly rounded sqrt and divide
  const float* src = w + c * inner;
  float* dst = w_out + c * inner;
  for (long long j = static_cast<long long>(blockIdx.x) * 256 + threadIdx.x; j < inner;
       j += static_cast<long long>(gridDim.x) * 256)
    dst[j] = f * src[j];
  if (bias_out && blockIdx.x == 0 && threadIdx.x == 0) {
    const float d = (bias ? bias[c] : 0.0f) - mean[c];
    const float p = f * d;
    bias_out[c] = p + beta[c];
  }
}

// ---------------------------------------------------------------------------
// host helpers
// ---------------------------------------------------------------------------
size_t align256(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

template <class T>
size_t bytes_of(const std::vector<T>& v) { return v.size() * sizeof(T); }

// First device call on a plan: one allocation holding all tables, blocking copies.
qv2_status ensure_uploaded(qv2_plan* p) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return QV2_ERR_HIP; }
  // the tables live on one device: a later call with another device current would hand its
  // kernels pointers they cannot use
  if (p->d_blob) return dev == p->device ? QV2_OK : QV2_ERR_HIP;
  size_t total = 256;
  auto reserve = [&](size_t n) { const size_t at = total; total += align256(n); return at; };
  const size_t o_read = reserve(bytes_of(p->read_tiles)), o_quant = reserve(bytes_of(p->quant_tiles));
  const size_t o_row = reserve(bytes_of(p->row_tiles)), o_pair = reserve(bytes_of(p->pair_tiles));
  const size_t o_seg = reserve(bytes_of(p->segments)), o_pt = reserve(bytes_of(p->pair_tensors));
  const size_t o_ft = reserve(bytes_of(p->fused_pair_tensors));
  const size_t o_bs = reserve(bytes_of(p->big_stat_segments)), o_be = reserve(bytes_of(p->big_err_segments));
  const size_t o_bp = reserve(bytes_of(p->big_pair_tensors)), o_bf = reserve(bytes_of(p->big_fused_pair_tensors));
  const size_t o_ht = reserve(bytes_of(p->hist_tiles)), o_hten = reserve(bytes_of(p->hist_tensors));
  const size_t o_st = reserve(bytes_of(p->stat_pair_tensors)), o_bst = reserve(bytes_of(p->big_stat_pair_tensors));
  const size_t o_reg = reserve(bytes_of(p->reg_tiles)), o_qro = reserve(bytes_of(p->quant_ro_tiles));
  char* blob = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&blob), total) != hipSuccess) {
    (void)hipGetLastError();
    return QV2_ERR_HIP;
  }
  bool ok = true;
  auto put = [&](size_t off, const void* h, size_t n) {
    if (n && hipMemcpy(blob + off, h, n, hipMemcpyHostToDevice) != hipSuccess) ok = false;
    return static_cast<void*>(blob + off);
  };
  p->d_read_tiles = static_cast<Tile*>(put(o_read, p->read_tiles.data(), bytes_of(p->read_tiles)));
  p->d_quant_tiles = static_cast<Tile*>(put(o_quant, p->quant_tiles.data(), bytes_of(p->quant_tiles)));
  p->d_row_tiles = static_cast<Tile*>(put(o_row, p->row_tiles.data(), bytes_of(p->row_tiles)));
  p->d_pair_tiles = static_cast<Tile*>(put(o_pair, p->pair_tiles.data(), bytes_of(p->pair_tiles)));
  p->d_segments = static_cast<Segment*>(put(o_seg, p->segments.data(), bytes_of(p->segments)));
  p->d_pair_tensors = static_cast<PairTensor*>(put(o_pt, p->pair_tensors.data(), bytes_of(p->pair_tensors)));
  p->d_fused_pair_tensors =
      static_cast<PairTensor*>(put(o_ft, p->fused_pair_tensors.data(), bytes_of(p->fused_pair_tensors)));
  p->d_big_stat_segments =
      static_cast<int32_t*>(put(o_bs, p->big_stat_segments.data(), bytes_of(p->big_stat_segments)));
  p->d_big_err_segments =
      static_cast<int32_t*>(put(o_be, p->big_err_segments.data(), bytes_of(p->big_err_segments)));
  p->d_big_pair_tensors =
      static_cast<int32_t*>(put(o_bp, p->big_pair_tensors.data(), bytes_of(p->big_pair_tensors)));
  p->d_big_fused_pair_tensors = static_cast<int32_t*>(
      put(o_bf, p->big_fused_pair_tensors.data(), bytes_of(p->big_fused_pair_tensors)));
  p->d_hist_tiles = static_cast<Tile*>(put(o_ht, p->hist_tiles.data(), bytes_of(p->hist_tiles)));
  p->d_hist_tensors =
      static_cast<HistTensor*>(put(o_hten, p->hist_tensors.data(), bytes_of(p->hist_tensors)));
  p->d_reg_tiles = static_cast<Tile*>(put(o_reg, p->reg_tiles.data(), bytes_of(p->reg_tiles)));
  p->d_quant_ro_tiles = static_cast<Tile*>(put(o_qro, p->quant_ro_tiles.data(), bytes_of(p->quant_ro_tiles)));
  p->d_stat_pair_tensors =
      static_cast<PairTensor*>(put(o_st, p->stat_pair_tensors.data(), bytes_of(p->stat_pair_tensors)));
  p->d_big_stat_pair_tensors = static_cast<int32_t*>(
      put(o_bst, p->big_stat_pair_tensors.data(), bytes_of(p->big_stat_pair_tensors)));
  if (!ok) { (void)hipGetLastError(); (void)hipFree(blob); return QV2_ERR_HIP; }
  p->d_blob = blob;
  p->device = dev;
  return QV2_OK;
}

qv2_status check_call(const qv2_plan* plan, const void* a, const void* b, const void* ws,
                      size_t ws_bytes) {
  if (!plan || !a || !b || !ws) return QV2_ERR_NULL;
  if (ws_bytes < plan->workspace_bytes) return QV2_ERR_WORKSPACE;
  if (reinterpret_cast<uintptr_t>(ws) & 15u) return QV2_ERR_ALIGN;
  if ((reinterpret_cast<uintptr_t>(a) & 7u) || (reinterpret_cast<uintptr_t>(b) & 7u)) return QV2_ERR_ALIGN;
  return QV2_OK;
}

qv2_status launch_status() { return hipGetLastError() == hipSuccess ? QV2_OK : QV2_ERR_HIP; }

// Brackets one kernel launch with the plan's HIP events when timing is enabled.
struct Timed {
  qv2_plan* p; int k; hipStream_t s;
  Timed(qv2_plan* plan, int kernel, hipStream_t st) : p(plan), k(kernel), s(st) {
    if (p->timing) { (void)hipEventRecord(static_cast<hipEvent_t>(p->ev_start[k]), s); p->ev_used[k] = true; }
  }
  ~Timed() { if (p->timing) (void)hipEventRecord(static_cast<hipEvent_t>(p->ev_stop[k]), s); }
};

int fold_grid(int n) { return (n + 3) / 4; }

// row-group tiles of a quantize pass, both forms; d_params_out != null: with calibration
template <bool PAIR, bool COS>
void launch_rows(qv2_plan* plan, const qv2_qparams* d_params, qv2_qparams* d_params_out, qv2_sums* d_sums,
                 typename ErrRec<COS>::type* parts, int n_rows, int n_regs, hipStream_t s) {
  const bool calib = d_params_out != nullptr;
  if (n_rows > 0) {
    if (calib)
      hipLaunchKernelGGL((k_quant_rows<kBlockRows, PAIR, COS, true>), dim3(n_rows), dim3(kBlockRows), 0, s,
                         plan->d_row_tiles, plan->d_segments, d_params, d_params_out, d_sums, parts);
    else
      hipLaunchKernelGGL((k_quant_rows<kBlockRows, PAIR, COS, false>), dim3(n_rows), dim3(kBlockRows), 0, s,
                         plan->d_row_tiles, plan->d_segments, d_params, d_params_out, d_sums, parts);
  }
  if (n_regs > 0) {
    if (calib)
      hipLaunchKernelGGL((k_rows_reg<kBlockRows, 2, PAIR, COS>), dim3(n_regs), dim3(kBlockRows), 0, s,
                         plan->d_reg_tiles, plan->d_segments, d_params, d_params_out, d_sums,
                         static_cast<void*>(parts));
    else
      hipLaunchKernelGGL((k_rows_reg<kBlockRows, 1, PAIR, COS>), dim3(n_regs), dim3(kBlockRows), 0, s,
                         plan->d_reg_tiles, plan->d_segments, d_params, d_params_out, d_sums,
                         static_cast<void*>(parts));
  }
}

// the stream tiles of a quantize pass: those with a code buffer, then those without
template <bool PAIR, bool COS, bool X2>
void launch_quant_stream(qv2_plan* plan, int n_stream, int n_ro, const qv2_qparams* d_params,
                         typename ErrRec<COS>::type* parts, hipStream_t s) {
  if (n_stream > 0)
    hipLaunchKernelGGL((k_quant_stream<kBlockQuant, kVecQuant, PAIR, COS, X2>), dim3(n_stream),
                       dim3(kBlockQuant), 0, s, plan->d_quant_tiles, d_params, parts);
  if (n_ro > 0)
    hipLaunchKernelGGL((k_quant_stream<kBlockRead, kVecQuantRO, PAIR, COS, X2, true>), dim3(n_ro),
                       dim3(kBlockRead), 0, s, plan->d_quant_ro_tiles, d_params, parts);
}

// quantize pass over stream and row-group tiles, then ONE fold launch for the segments'
// error sums and (d_pair_sums != null) the tensors' pair sums.  d_params_out != null: the
// row-group kernel also calibrates its rows (writes their parameter and sum records), and
// the fold leaves those segments alone.
template <bool PAIR, bool COS>
void launch_quant(qv2_plan* plan, const qv2_qparams* d_params, qv2_sums* d_sums,
                  typename ErrRec<COS>::type* parts, double* d_seg_xxhat, qv2_pair_sums* d_pair_sums,
                  double* d_pair_xq, hipStream_t s, qv2_qparams* d_params_out = nullptr,
                  bool pair_in_stats = false) {
  typedef typename ErrRec<COS>::type P;
  const bool calib_rows = d_params_out != nullptr;
  const int n_stream = static_cast<int>(plan->quant_tiles.size());
  const int n_ro = static_cast<int>(plan->quant_ro_tiles.size());
  const int n_rows = static_cast<int>(plan->row_tiles.size());
  if (n_stream + n_ro > 0) {
    // pair_in_stats: the calibration sweep already compared the stream tensors with their
    // partners, so the plain quantize kernel serves them
    Timed timed(plan, PAIR && !pair_in_stats ? QV2_K_QUANTPAIR_STREAM : QV2_K_QUANT_STREAM, s);
    if (PAIR && !pair_in_stats)
      launch_quant_stream<PAIR, COS, true>(plan, n_stream, n_ro, d_params, parts, s);
    else if (calib_rows)      // the calibration sweep of this same call already summed x^2
      launch_quant_stream<false, COS, false>(plan, n_stream, n_ro, d_params, parts, s);
    else
      launch_quant_stream<false, COS, true>(plan, n_stream, n_ro, d_params, parts, s);
  }
  const int n_regs = static_cast<int>(plan->reg_tiles.size());
  if (n_rows + n_regs > 0) {
    Timed timed(plan, calib_rows ? QV2_K_SINGLE_READ_ROWS : PAIR ? QV2_K_QUANTPAIR_ROWS : QV2_K_QUANT_ROWS, s);
    // the pair form of the row kernels costs registers: only when a row tensor has a partner
    if (PAIR && plan->rows_have_pair)
      launch_rows<true, COS>(plan, d_params, d_params_out, d_sums, parts, n_rows, n_regs, s);
    else
      launch_rows<false, COS>(plan, d_params, d_params_out, d_sums, parts, n_rows, n_regs, s);
  }
  QuantFoldArgs<P> a{};
  a.segs = plan->d_segments; a.nseg = static_cast<int>(plan->segments.size());
  a.wide_segs = plan->d_big_err_segments; a.n_wide_segs = static_cast<int>(plan->big_err_segments.size());
  a.sums = d_sums; a.seg_xxhat = d_seg_xxhat; a.skip_below = calib_rows ? plan->n_row_parts : 0;
  a.keep_x2 = calib_rows && (!PAIR || pair_in_stats);
  a.parts = parts;
  a.seg_blocks = fold_blocks(a.n_wide_segs, a.nseg);
  int blocks = a.seg_blocks;
  if (d_pair_sums) {
    a.pt = plan->d_fused_pair_tensors; a.nt = static_cast<int>(plan->fused_pair_tensors.size());
    a.wide_pt = plan->d_big_fused_pair_tensors;
    a.n_wide_pt = static_cast<int>(plan->big_fused_pair_tensors.size());
    a.pair_out = d_pair_sums; a.pair_xq = d_pair_xq;
    a.pair_done = pair_in_stats ? plan->d_stat_pair_tensors : nullptr;
    blocks += fold_blocks(a.n_wide_pt, a.nt);
  }
  hipLaunchKernelGGL(k_fold_quant<P>, dim3(blocks), dim3(kFoldBlock), 0, s, a);
}

// calibration over the stream tiles (and the row-group tiles unless their own single-read
// kernel will calibrate them), then the statistics fold.  PAIR: the same sweep compares the
// stream tensors with their quantized-run partners and the fold writes their pair sums.
template <bool PAIR, bool COS = false>
void launch_stats(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums,
                  typename StatRec<PAIR, COS>::type* parts, bool with_rows, qv2_pair_sums* d_pair_sums,
                  double* d_pair_xq, hipStream_t s) {
  typedef typename StatRec<PAIR, COS>::type REC;
  if (PAIR) with_rows = false;      // the row kernel of this pass writes 24-byte records: not in a PAIR sweep
  const int n_stream = static_cast<int>(plan->read_tiles.size());
  const int n_rows = static_cast<int>(plan->row_tiles.size());
  if (n_stream > 0) {
    Timed timed(plan, PAIR ? QV2_K_STATSPAIR_STREAM : QV2_K_STATS_STREAM, s);
    hipLaunchKernelGGL((k_stats_stream<kBlockRead, kVecRead, PAIR, COS>), dim3(n_stream), dim3(kBlockRead), 0, s,
                       plan->d_read_tiles, parts);
  }
  const int n_regs = static_cast<int>(plan->reg_tiles.size());
  if (with_rows && n_rows + n_regs > 0) {
    Timed timed(plan, QV2_K_STATS_ROWS, s);
    if (n_rows > 0)
      hipLaunchKernelGGL(k_stats_rows<kBlockRows>, dim3(n_rows), dim3(kBlockRows), 0, s,
                         plan->d_row_tiles, reinterpret_cast<StatPartial*>(parts));
    if (n_regs > 0)
      hipLaunchKernelGGL((k_rows_reg<kBlockRows, 0, false, false>), dim3(n_regs), dim3(kBlockRows), 0, s,
                         plan->d_reg_tiles, plan->d_segments, static_cast<const qv2_qparams*>(nullptr),
                         static_cast<qv2_qparams*>(nullptr), static_cast<qv2_sums*>(nullptr),
                         static_cast<void*>(parts));
  }
  if (with_rows || n_stream > 0) {
    StatFoldArgs<REC> a{};
    a.segs = plan->d_segments; a.nseg = static_cast<int>(plan->segments.size());
    a.wide_segs = plan->d_big_stat_segments; a.n_wide_segs = static_cast<int>(plan->big_stat_segments.size());
    a.parts = parts; a.params = d_params; a.sums = d_sums;
    a.skip_below = with_rows ? 0 : plan->n_row_parts;
    a.seg_blocks = fold_blocks(a.n_wide_segs, a.nseg);
    int blocks = a.seg_blocks;
    if (PAIR) {
      a.pt = plan->d_stat_pair_tensors; a.nt = static_cast<int>(plan->stat_pair_tensors.size());
      a.wide_pt = plan->d_big_stat_pair_tensors;
      a.n_wide_pt = static_cast<int>(plan->big_stat_pair_tensors.size());
      a.pair_out = d_pair_sums; a.pair_xq = d_pair_xq;
      blocks += fold_blocks(a.n_wide_pt, a.nt);
    }
    hipLaunchKernelGGL(k_fold_stats<REC>, dim3(blocks), dim3(kFoldBlock), 0, s, a);
  }
}

}  // namespace

extern "C" {

void qv2_plan_destroy(qv2_plan* plan) {
  if (!plan) return;
  if (plan->d_blob) (void)hipFree(plan->d_blob);
  for (int k = 0; k < QV2_K_COUNT; ++k) {
    if (plan->ev_start[k]) (void)hipEventDestroy(static_cast<hipEvent_t>(plan->ev_start[k]));
    if (plan->ev_stop[k]) (void)hipEventDestroy(static_cast<hipEvent_t>(plan->ev_stop[k]));
  }
  delete plan;
}

qv2_status qv2_plan_set_timing(qv2_plan* plan, int32_t enable) {
  if (!plan) return QV2_ERR_NULL;
  if (enable && !plan->ev_start[0]) {
    hipEvent_t ev[2 * QV2_K_COUNT] = {};
    for (int k = 0; k < 2 * QV2_K_COUNT; ++k) {
      if (hipEventCreate(&ev[k]) != hipSuccess) {      // all or none
        (void)hipGetLastError();
        for (int j = 0; j < k; ++j) (void)hipEventDestroy(ev[j]);
        return QV2_ERR_HIP;
      }
    }
    for (int k = 0; k < QV2_K_COUNT; ++k) { plan->ev_start[k] = ev[2 * k]; plan->ev_stop[k] = ev[2 * k + 1]; }
  }
  plan->timing = enable != 0;
  return QV2_OK;
}

qv2_status qv2_plan_kernel_ms(const qv2_plan* plan, int32_t kernel, float* ms_out) {
  if (!plan || !ms_out) return QV2_ERR_NULL;
  if (kernel < 0 || kernel >= QV2_K_COUNT) return QV2_ERR_SHAPE;
  *ms_out = 0.0f;
  if (!plan->ev_used[kernel]) return QV2_OK;
  if (hipEventElapsedTime(ms_out, static_cast<hipEvent_t>(plan->ev_start[kernel]),
                          static_cast<hipEvent_t>(plan->ev_stop[kernel])) != hipSuccess) {
    (void)hipGetLastError();
    return QV2_ERR_HIP;
  }
  return QV2_OK;
}

qv2_status qv2_plan_kernels_ms(const qv2_plan* plan, float* ms_out) {
  if (!plan || !ms_out) return QV2_ERR_NULL;
  for (int k = 0; k < QV2_K_COUNT; ++k) {
    const qv2_status st = qv2_plan_kernel_ms(plan, k, ms_out + k);
    if (st != QV2_OK) return st;
  }
  return QV2_OK;
}

qv2_status qv2_calibrate(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums,
                         void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  qv2_status st = check_call(plan, d_params, d_sums, d_workspace, workspace_bytes);
  if (st != QV2_OK) return st;
  if ((st = ensure_uploaded(plan)) != QV2_OK) return st;
  launch_stats<false>(plan, d_params, d_sums, static_cast<StatPartial*>(d_workspace), true, nullptr, nullptr,
                      static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

qv2_status qv2_fakequant_metrics(qv2_plan* plan, const qv2_qparams* d_params, qv2_sums* d_sums,
                                 void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  qv2_status st = check_call(plan, d_params, d_sums, d_workspace, workspace_bytes);
  if (st != QV2_OK) return st;
  if ((st = ensure_uploaded(plan)) != QV2_OK) return st;
  launch_quant<false, false>(plan, d_params, d_sums, static_cast<ErrPartial3*>(d_workspace), nullptr,
                             nullptr, nullptr, static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

qv2_status qv2_pair_metrics(qv2_plan* plan, qv2_pair_sums* d_pair_sums, void* d_workspace,
                            size_t workspace_bytes, void* hip_stream) {
  qv2_status st = check_call(plan, d_pair_sums, d_pair_sums, d_workspace, workspace_bytes);
  if (st != QV2_OK) return st;
  if ((st = ensure_uploaded(plan)) != QV2_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  ErrPartial* parts = static_cast<ErrPartial*>(d_workspace);
  const int n_tiles = static_cast<int>(plan->pair_tiles.size());
  const int nt = static_cast<int>(plan->pair_tensors.size());
  if (n_tiles > 0) {
    Timed timed(plan, QV2_K_PAIR_STREAM, s);
    hipLaunchKernelGGL((k_pair_stream<kBlockRead, kVecRead / 2>), dim3(n_tiles), dim3(kBlockRead), 0, s,
                       plan->d_pair_tiles, parts);
  }
  const int n_wide = static_cast<int>(plan->big_pair_tensors.size());
  hipLaunchKernelGGL(k_fold_pair, dim3(fold_blocks(n_wide, nt)), dim3(kFoldBlock), 0, s, plan->d_pair_tensors,
                     nt, plan->d_big_pair_tensors, n_wide, parts, d_pair_sums);
  return launch_status();
}

qv2_status qv2_fakequant_pair_metrics(qv2_plan* plan, const qv2_qparams* d_params, qv2_sums* d_sums,
                                      qv2_pair_sums* d_pair_sums, void* d_workspace,
                                      size_t workspace_bytes, void* hip_stream) {
  qv2_status st = check_call(plan, d_params, d_sums, d_workspace, workspace_bytes);
  if (st != QV2_OK) return st;
  if (!d_pair_sums) return QV2_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(d_pair_sums) & 7u) return QV2_ERR_ALIGN;
  if ((st = ensure_uploaded(plan)) != QV2_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  ErrPartial3* parts = static_cast<ErrPartial3*>(d_workspace);
  launch_quant<true, false>(plan, d_params, d_sums, parts, nullptr, d_pair_sums, nullptr, s);
  return launch_status();
}

qv2_status qv2_calibrate_fakequant_pair_metrics(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums,
                                                qv2_pair_sums* d_pair_sums, void* d_workspace,
                                                size_t workspace_bytes, void* hip_stream) {
  qv2_status st = check_call(plan, d_params, d_sums, d_workspace, workspace_bytes);
  if (st != QV2_OK) return st;
  if (d_pair_sums && (reinterpret_cast<uintptr_t>(d_pair_sums) & 7u)) return QV2_ERR_ALIGN;
  if ((st = ensure_uploaded(plan)) != QV2_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  // stream tiles: statistics (with the pair comparison: that sweep only reads, and read-only
  // sweeps run nearest to the HBM rate), fold (parameters), then the plain quantize sweep;
  // row-group tiles: one kernel, after the statistics fold because the partial records share
  // the workspace
  ErrPartial3* parts = static_cast<ErrPartial3*>(d_workspace);
  if (d_pair_sums) {
    launch_stats<true>(plan, d_params, d_sums, static_cast<StatPairPartial*>(d_workspace), false, d_pair_sums,
                       nullptr, s);
    launch_quant<true, false>(plan, d_params, d_sums, parts, nullptr, d_pair_sums, nullptr, s, d_params, true);
  } else {
    launch_stats<false>(plan, d_params, d_sums, static_cast<StatPartial*>(d_workspace), false, nullptr, nullptr, s);
    launch_quant<false, false>(plan, d_params, d_sums, parts, nullptr, nullptr, nullptr, s, d_params);
  }
  return launch_status();
}

qv2_status qv2_calibrate_fakequant_pair_metrics_cos(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums,
                                                    qv2_pair_sums* d_pair_sums, double* d_seg_xxhat,
                                                    double* d_pair_xq, void* d_workspace,
                                                    size_t workspace_bytes, void* hip_stream) {
  qv2_status st = check_call(plan, d_params, d_sums, d_workspace, workspace_bytes);
  if (st != QV2_OK) return st;
  if (!d_pair_sums || !d_seg_xxhat || !d_pair_xq) return QV2_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(d_pair_sums) | reinterpret_cast<uintptr_t>(d_seg_xxhat) |
       reinterpret_cast<uintptr_t>(d_pair_xq)) & 7u) return QV2_ERR_ALIGN;
  if ((st = ensure_uploaded(plan)) != QV2_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  // as the call without the cross terms: sum x * qrun rides on the read-only sweep, sum x * xhat
  // on the quantize sweep
  launch_stats<true, true>(plan, d_params, d_sums, static_cast<StatPairCosPartial*>(d_workspace), false,
                           d_pair_sums, d_pair_xq, s);
  launch_quant<true, true>(plan, d_params, d_sums, static_cast<ErrPartial5*>(d_workspace), d_seg_xxhat,
                           d_pair_sums, d_pair_xq, s, d_params, true);
  return launch_status();
}

qv2_status qv2_fakequant_pair_metrics_cos(qv2_plan* plan, const qv2_qparams* d_params, qv2_sums* d_sums,
                                          qv2_pair_sums* d_pair_sums, double* d_seg_xxhat,
                                          double* d_pair_xq, void* d_workspace, size_t workspace_bytes,
                                          void* hip_stream) {
  qv2_status st = check_call(plan, d_params, d_sums, d_workspace, workspace_bytes);
  if (st != QV2_OK) return st;
  if (!d_pair_sums || !d_seg_xxhat || !d_pair_xq) return QV2_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(d_pair_sums) | reinterpret_cast<uintptr_t>(d_seg_xxhat) |
       reinterpret_cast<uintptr_t>(d_pair_xq)) & 7u) return QV2_ERR_ALIGN;
  if ((st = ensure_uploaded(plan)) != QV2_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  ErrPartial5* parts = static_cast<ErrPartial5*>(d_workspace);
  launch_quant<true, true>(plan, d_params, d_sums, parts, d_seg_xxhat, d_pair_sums, d_pair_xq, s);
  return launch_status();
}

qv2_status qv2_tensor_sums_fold(qv2_plan* plan, const qv2_qparams* d_params, const qv2_sums* d_sums,
                                qv2_tensor_sums* d_tensor_sums, void* hip_stream) {
  if (!plan || !d_params || !d_sums || !d_tensor_sums) return QV2_ERR_NULL;
  if (reinterpret_cast<uintptr_t>(d_tensor_sums) & 7u) return QV2_ERR_ALIGN;
  qv2_status st = ensure_uploaded(plan);
  if (st != QV2_OK) return st;
  const int nt = static_cast<int>(plan->info.size());
  hipLaunchKernelGGL(k_tensor_fold, dim3(nt), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     plan->d_hist_tensors, nt, d_params, d_sums, d_tensor_sums);
  return launch_status();
}

qv2_status qv2_bn_fold(const float* d_w, int32_t channels, int64_t inner, const float* d_gamma,
                       const float* d_var, const float* d_bias, const float* d_mean,
                       const float* d_beta, float* d_w_out, float* d_bias_out, void* hip_stream) {
  if (!d_w || !d_gamma || !d_var || !d_w_out) return QV2_ERR_NULL;
  if (d_bias_out && (!d_mean || !d_beta)) return QV2_ERR_NULL;
  if (channels <= 0 || channels > 65535 || inner <= 0) return QV2_ERR_SHAPE;
  const int gx = static_cast<int>(std::min<int64_t>((inner + 255) / 256, 1024));
  hipLaunchKernelGGL(k_bn_fold, dim3(gx, channels), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     d_w, static_cast<long long>(inner), d_gamma, d_var, d_bias, d_mean, d_beta, d_w_out,
                     d_bias_out);
  return launch_status();
}

qv2_status qv2_histogram(qv2_plan* plan, const qv2_qparams* d_params, int32_t nbins,
                         uint64_t* d_hist_x, uint64_t* d_hist_q, void* d_workspace,
                         size_t workspace_bytes, void* hip_stream) {
  if (!plan || !d_params || !d_hist_x || !d_workspace) return QV2_ERR_NULL;
  if (nbins < 2 || nbins > kHistMaxBins) return QV2_ERR_SHAPE;
  if (workspace_bytes < qv2_histogram_workspace_bytes(plan, nbins)) return QV2_ERR_WORKSPACE;
  if ((reinterpret_cast<uintptr_t>(d_workspace) & 15u) || (reinterpret_cast<uintptr_t>(d_hist_x) & 7u) ||
      (reinterpret_cast<uintptr_t>(d_hist_q) & 7u)) return QV2_ERR_ALIGN;
  qv2_status st = ensure_uploaded(plan);
  if (st != QV2_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const int nt = static_cast<int>(plan->info.size());
  const int n_chunks = static_cast<int>(plan->hist_tiles.size());
  float2* range = static_cast<float2*>(d_workspace);
  uint32_t* partial = reinterpret_cast<uint32_t*>(static_cast<char*>(d_workspace) +
                                                  align256(static_cast<size_t>(nt) * sizeof(float2)));
  hipLaunchKernelGGL(k_hist_range, dim3(fold_grid(nt)), dim3(256), 0, s, plan->d_hist_tensors, nt,
                     d_params, range);
  {
    Timed timed(plan, QV2_K_HIST, s);
    hipLaunchKernelGGL(k_hist<kBlockRead>, dim3(n_chunks), dim3(kBlockRead), 0, s, plan->d_hist_tiles,
                       range, nbins, partial);
  }
  hipLaunchKernelGGL(k_hist_fold, dim3(((nbins + 255) / 256) * nt), dim3(256), 0, s, plan->d_hist_tensors,
                     nbins, partial, reinterpret_cast<unsigned long long*>(d_hist_x),
                     reinterpret_cast<unsigned long long*>(d_hist_q));
  return launch_status();
}

}  // extern "C"
