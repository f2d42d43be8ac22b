// HIP kernels (gfx950, wave64) and device entry points of the qv2 C ABI.
//
// Every pass is one flat launch over a tile table that spans all tensors of
// the plan: a workgroup owns one tile, reduces it and leaves one partial record
// per (tile, segment) in the workspace; a second small launch folds each
// segment's partials in a fixed order.  No floating-point atomics anywhere, so
// results are bit-stable.  The work is HBM-bound (4, 5 and 8 bytes per element
// for the three passes); MFMA has no role here.
//
// Compiled with -ffp-contract=off: the quantizer's fp32 steps (Sec. 2.1 Eq. 1-3,
// Sec. 4 Eq. 4-5) must each round once.  Fused multiply-adds appear only where
// written explicitly (energy accumulation).
#include <hip/hip_runtime.h>

#include <cfloat>
#include <cstdint>

#include "qv2_internal.h"

using namespace qv2;

namespace {

constexpr int kWave = 64;
constexpr int kWaves = kBlock / kWave;
#ifndef QV2_UNROLL
#define QV2_UNROLL 8
#endif
#ifndef QV2_NT_LOADS
#define QV2_NT_LOADS 1             // measured: +12 % HBM rate on the read-only passes
#endif
#ifndef QV2_NT_STORES
#define QV2_NT_STORES 1
#endif
#ifndef QV2_PAIR_UNROLL
#define QV2_PAIR_UNROLL (QV2_UNROLL / 2)
#endif
constexpr int kUnroll = QV2_UNROLL;  // independent 16-byte loads in flight per lane
constexpr int kPairUnroll = QV2_PAIR_UNROLL;  // per stream, in the two-stream kernels
#ifndef QV2_PIPELINE
#define QV2_PIPELINE 1
#endif
constexpr int kFoldBlock = 1024;    // workgroup that folds one segment with many partials
constexpr int kFoldWaves = kFoldBlock / kWave;

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

// Sum of two doubles over the workgroup; result valid in thread 0.
__device__ __forceinline__ void block_sum2(double& a, double& b) {
  __shared__ double sa[kWaves], sb[kWaves];
  a = group_sum(a, kWave);
  b = group_sum(b, kWave);
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  if (lane == 0) { sa[wave] = a; sb[wave] = b; }
  __syncthreads();
  if (threadIdx.x == 0) {
    a = sa[0]; b = sb[0];
    for (int i = 1; i < kWaves; ++i) { a += sa[i]; b += sb[i]; }
  }
}

__device__ __forceinline__ void block_minmax(float& mn, float& mx) {
  __shared__ float smn[kWaves], smx[kWaves];
  mn = group_min(mn, kWave);
  mx = group_max(mx, kWave);
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  if (lane == 0) { smn[wave] = mn; smx[wave] = mx; }
  __syncthreads();
  if (threadIdx.x == 0) {
    mn = smn[0]; mx = smx[0];
    for (int i = 1; i < kWaves; ++i) { mn = fminf(mn, smn[i]); mx = fmaxf(mx, smx[i]); }
  }
}

// Four independent fp64 accumulators, one per float4 component.  Energies are
// accumulated in fp64 from the first element on, so the whole fp32 range of
// inputs is safe (x*x can leave the fp32 range) and no fp32 rounding builds up.
struct Acc4 {
  double a = 0.0, b = 0.0, c = 0.0, d = 0.0;
  __device__ __forceinline__ void add(const float4& v) {
    a += static_cast<double>(v.x); b += static_cast<double>(v.y);
    c += static_cast<double>(v.z); d += static_cast<double>(v.w);
  }
  __device__ __forceinline__ void add_sq(float x, float y, float z, float w) {
    const double dx = x, dy = y, dz = z, dw = w;
    a = fma(dx, dx, a); b = fma(dy, dy, b); c = fma(dz, dz, c); d = fma(dw, dw, d);
  }
  __device__ __forceinline__ double total() const { return (a + b) + (c + d); }
};

// 16-byte streaming load of data that is read once per pass.
__device__ __forceinline__ float4 ld4(const float4* p) {
#if QV2_NT_LOADS
  typedef float vf4 __attribute__((ext_vector_type(4)));
  const vf4 v = __builtin_nontemporal_load(reinterpret_cast<const vf4*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
#else
  return *p;
#endif
}

// Packed int8 codes are written once and not read again by this library.
__device__ __forceinline__ void st_codes(uint32_t* p, uint32_t v) {
#if QV2_NT_STORES
  __builtin_nontemporal_store(v, p);
#else
  *p = v;
#endif
}

// Elements before the first 16-byte boundary of p (0..3, capped by len).
__device__ __forceinline__ int head_elems(const void* p, int len) {
  const int h = static_cast<int>(((16u - (reinterpret_cast<uintptr_t>(p) & 15u)) & 15u) >> 2);
  return h < len ? h : len;
}

// ---------------------------------------------------------------------------
// quantizer: Sec. 2.1 Eq. 1 / Sec. 4 Eq. 5 then Eq. 3, each step one fp32 rounding
// ---------------------------------------------------------------------------
struct QP { float scale, inv, zpf; };

// Returns the code as a float in [-128,127]; err receives x - xhat.
__device__ __forceinline__ float quant1(float x, const QP& q, float& err) {
  const float t = x * q.inv;                       // fp32 multiply
  const float r = rintf(t);                        // round half to even
  // integer add of the zero-point: exact in fp32 below 2^24, saturates above
  const float c = fminf(fmaxf(r + q.zpf, -128.0f), 127.0f);
  const float xhat = (c - q.zpf) * q.scale;        // exact difference, one multiply
  err = x - xhat;
  return c;
}

__device__ __forceinline__ uint32_t quant4(const float4& v, const QP& q, Acc4& se2, Acc4& sx2) {
  float e0, e1, e2, e3;
  const int c0 = static_cast<int>(quant1(v.x, q, e0));
  const int c1 = static_cast<int>(quant1(v.y, q, e1));
  const int c2 = static_cast<int>(quant1(v.z, q, e2));
  const int c3 = static_cast<int>(quant1(v.w, q, e3));
  se2.add_sq(e0, e1, e2, e3);
  sx2.add_sq(v.x, v.y, v.z, v.w);
  return (static_cast<uint32_t>(c0) & 0xffu) | ((static_cast<uint32_t>(c1) & 0xffu) << 8) |
         ((static_cast<uint32_t>(c2) & 0xffu) << 16) | (static_cast<uint32_t>(c3) << 24);
}

__device__ __forceinline__ QP load_qp(const qv2_qparams* params, int seg) {
  const qv2_qparams p = params[seg];
  return QP{p.scale, p.inv_scale, static_cast<float>(p.zp)};
}

// ---------------------------------------------------------------------------
// pass 1 (calibration stage, Sec. 5; x_min / x_max of Eq. 2): stream tiles
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_stats_stream(const TensorDesc* __restrict__ descs,
                                                         const Tile* __restrict__ tiles,
                                                         StatPartial* __restrict__ parts) {
  const Tile tl = tiles[blockIdx.x];
  const float* __restrict__ p = descs[tl.tensor].x + tl.off;
  const int len = tl.len, tid = threadIdx.x;
  const int head = head_elems(p, len);
  const int body = len - head, nvec = body >> 2, tail = body & 3;

  float mn = INFINITY, mx = -INFINITY;
  double sx = 0.0, sx2 = 0.0;
  if (tid < head) {
    const float v = p[tid];
    mn = fminf(mn, v); mx = fmaxf(mx, v);
    sx += v; sx2 += static_cast<double>(v) * v;
  }
  if (tid < tail) {
    const float v = p[head + (nvec << 2) + tid];
    mn = fminf(mn, v); mx = fmaxf(mx, v);
    sx += v; sx2 += static_cast<double>(v) * v;
  }
  const float4* __restrict__ v4 = reinterpret_cast<const float4*>(p + head);
  float4 mn4 = make_float4(INFINITY, INFINITY, INFINITY, INFINITY);
  float4 mx4 = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
  Acc4 as, as2;
  int i = tid;
  for (; i + (kUnroll - 1) * kBlock < nvec; i += kUnroll * kBlock) {
    float4 r[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) r[u] = ld4(&v4[i + u * kBlock]);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      mn4.x = fminf(mn4.x, r[u].x); mn4.y = fminf(mn4.y, r[u].y);
      mn4.z = fminf(mn4.z, r[u].z); mn4.w = fminf(mn4.w, r[u].w);
      mx4.x = fmaxf(mx4.x, r[u].x); mx4.y = fmaxf(mx4.y, r[u].y);
      mx4.z = fmaxf(mx4.z, r[u].z); mx4.w = fmaxf(mx4.w, r[u].w);
      as.add(r[u]); as2.add_sq(r[u].x, r[u].y, r[u].z, r[u].w);
    }
  }
  for (; i < nvec; i += kBlock) {
    const float4 r = ld4(&v4[i]);
    mn4.x = fminf(mn4.x, r.x); mn4.y = fminf(mn4.y, r.y);
    mn4.z = fminf(mn4.z, r.z); mn4.w = fminf(mn4.w, r.w);
    mx4.x = fmaxf(mx4.x, r.x); mx4.y = fmaxf(mx4.y, r.y);
    mx4.z = fmaxf(mx4.z, r.z); mx4.w = fmaxf(mx4.w, r.w);
    as.add(r); as2.add_sq(r.x, r.y, r.z, r.w);
  }
  sx += as.total(); sx2 += as2.total();
  mn = fminf(fminf(mn, mn4.x), fminf(fminf(mn4.y, mn4.z), mn4.w));
  mx = fmaxf(fmaxf(mx, mx4.x), fmaxf(fmaxf(mx4.y, mx4.z), mx4.w));

  block_minmax(mn, mx);
  block_sum2(sx, sx2);
  if (tid == 0) {
    StatPartial o;
    o.mn = mn; o.mx = mx; o.sx = sx; o.sx2 = sx2;
    parts[tl.part0] = o;
  }
}

// Copies a row-group tile into LDS with 16-byte transfers.  Element e of the
// tile lands at xs[e + shift]; returns shift (0..3).
__device__ __forceinline__ int stage_tile(const float* __restrict__ p, int len, float* xs) {
  const int tid = threadIdx.x;
  const int head = head_elems(p, len);
  const int shift = (4 - head) & 3;
  const int body = len - head, nvec = body >> 2, tail = body & 3;
  if (tid < head) xs[shift + tid] = p[tid];
  const float4* __restrict__ v4 = reinterpret_cast<const float4*>(p + head);
  float4* d4 = reinterpret_cast<float4*>(xs + shift + head);
  for (int i = tid; i < nvec; i += kBlock) d4[i] = v4[i];
  if (tid < tail) xs[shift + head + (nvec << 2) + tid] = p[head + (nvec << 2) + tid];
  return shift;
}

// Lanes per row of a row-group tile: the power of two >= inner, at most a wavefront.
__device__ __forceinline__ int row_width(int inner) {
  int w = 1;
  while (w < inner && w < kWave) w <<= 1;
  return w;
}

// pass 1, row-group tiles: many short segments (output channels) per workgroup
__global__ __launch_bounds__(kBlock) void k_stats_rows(const TensorDesc* __restrict__ descs,
                                                       const Tile* __restrict__ tiles,
                                                       StatPartial* __restrict__ parts) {
  __shared__ __attribute__((aligned(16))) float xs[kRowGroupCap + 4];
  const Tile tl = tiles[blockIdx.x];
  const int shift = stage_tile(descs[tl.tensor].x + tl.off, tl.len, xs);
  __syncthreads();

  const int inner = tl.inner, w = row_width(inner), gpw = kWave / w;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  const int g = lane >> __builtin_ctz(w), gl = lane & (w - 1);
  for (int rb = wave * gpw; rb < tl.rows; rb += kWaves * gpw) {     // uniform per wavefront
    const int r = rb + g;
    const bool live = r < tl.rows;
    float mn = INFINITY, mx = -INFINITY;
    double sx = 0.0, sx2 = 0.0;
    if (live) {
      const float* row = xs + shift + r * inner;
      for (int j = gl; j < inner; j += w) {
        const float v = row[j];
        mn = fminf(mn, v); mx = fmaxf(mx, v);
        sx += v; sx2 = fma(static_cast<double>(v), static_cast<double>(v), sx2);
      }
    }
    mn = group_min(mn, w); mx = group_max(mx, w);
    sx = group_sum(sx, w); sx2 = group_sum(sx2, w);
    if (live && gl == 0) {
      StatPartial o;
      o.mn = mn; o.mx = mx; o.sx = sx; o.sx2 = sx2;
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

// pass 1, fold: one wavefront per segment walks its partials in a fixed order
__global__ __launch_bounds__(kBlock) void k_fold_stats(const Segment* __restrict__ segs, int nseg,
                                                       const StatPartial* __restrict__ parts,
                                                       qv2_qparams* __restrict__ params,
                                                       qv2_sums* __restrict__ sums) {
  const int seg = blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  if (seg >= nseg) return;
  const Segment sg = segs[seg];
  if (sg.nparts > kFoldWaveMax) return;            // folded by k_fold_stats_big
  float mn = INFINITY, mx = -INFINITY;
  double sx = 0.0, sx2 = 0.0;
  for (int i = lane; i < sg.nparts; i += kWave) {
    const StatPartial q = parts[sg.part0 + i];
    mn = fminf(mn, q.mn); mx = fmaxf(mx, q.mx);
    sx += q.sx; sx2 += q.sx2;
  }
  mn = group_min(mn, kWave); mx = group_max(mx, kWave);
  sx = group_sum(sx, kWave); sx2 = group_sum(sx2, kWave);
  if (lane == 0) {
    qv2_qparams qp;
    make_params(mn, mx, sg.scheme, qp);
    params[seg] = qp;
    qv2_sums o;
    o.sum_x = sx; o.sum_x2 = sx2; o.sum_e2 = 0.0; o.n = sg.n;
    sums[seg] = o;
  }
}

// ---------------------------------------------------------------------------
// pass 2 (Eq. 1, 3, 5 and the energies of Eq. 6-7): stream tiles
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_quant_stream(const TensorDesc* __restrict__ descs,
                                                         const Tile* __restrict__ tiles,
                                                         const qv2_qparams* __restrict__ params,
                                                         ErrPartial* __restrict__ parts) {
  const Tile tl = tiles[blockIdx.x];
  const TensorDesc td = descs[tl.tensor];
  const float* __restrict__ p = td.x + tl.off;
  int8_t* __restrict__ c = td.codes ? td.codes + tl.off : nullptr;
  const QP q = load_qp(params, tl.seg0);
  const int len = tl.len, tid = threadIdx.x;
  const int head = head_elems(p, len);
  const int body = len - head, nvec = body >> 2, tail = body & 3;

  double sx2 = 0.0, se2 = 0.0;
  if (tid < head || tid < tail) {
    for (int k = 0; k < 2; ++k) {
      const bool on = k == 0 ? tid < head : tid < tail;
      if (!on) continue;
      const int idx = k == 0 ? tid : head + (nvec << 2) + tid;
      const float v = p[idx];
      float e;
      const float code = quant1(v, q, e);
      if (c) c[idx] = static_cast<int8_t>(static_cast<int>(code));
      sx2 += static_cast<double>(v) * v;
      se2 += static_cast<double>(e) * e;
    }
  }
  const float4* __restrict__ v4 = reinterpret_cast<const float4*>(p + head);
  // codes of the vector body go out as packed dwords when that address is 4-byte aligned
  const bool cw_ok = c && ((reinterpret_cast<uintptr_t>(c + head) & 3u) == 0);
  uint32_t* __restrict__ cw = reinterpret_cast<uint32_t*>(c + head);
  Acc4 ae2, ax2;
  int i = tid;
  for (; i + (kUnroll - 1) * kBlock < nvec; i += kUnroll * kBlock) {
    float4 r[kUnroll];
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) r[u] = ld4(&v4[i + u * kBlock]);
#pragma unroll
    for (int u = 0; u < kUnroll; ++u) {
      const uint32_t pk = quant4(r[u], q, ae2, ax2);
      if (cw_ok) {
        st_codes(&cw[i + u * kBlock], pk);
      } else if (c) {
        int8_t* d = c + head + ((i + u * kBlock) << 2);
        d[0] = static_cast<int8_t>(pk); d[1] = static_cast<int8_t>(pk >> 8);
        d[2] = static_cast<int8_t>(pk >> 16); d[3] = static_cast<int8_t>(pk >> 24);
      }
    }
  }
  for (; i < nvec; i += kBlock) {
    const float4 r = ld4(&v4[i]);
    const uint32_t pk = quant4(r, q, ae2, ax2);
    if (cw_ok) {
      st_codes(&cw[i], pk);
    } else if (c) {
      int8_t* d = c + head + (i << 2);
      d[0] = static_cast<int8_t>(pk); d[1] = static_cast<int8_t>(pk >> 8);
      d[2] = static_cast<int8_t>(pk >> 16); d[3] = static_cast<int8_t>(pk >> 24);
    }
  }
  se2 += ae2.total(); sx2 += ax2.total();
  block_sum2(sx2, se2);
  if (tid == 0) {
    ErrPartial o;
    o.sx2 = sx2; o.se2 = se2;
    parts[tl.part0] = o;
  }
}

// pass 2, row-group tiles
__global__ __launch_bounds__(kBlock) void k_quant_rows(const TensorDesc* __restrict__ descs,
                                                       const Tile* __restrict__ tiles,
                                                       const qv2_qparams* __restrict__ params,
                                                       ErrPartial* __restrict__ parts) {
  __shared__ __attribute__((aligned(16))) float xs[kRowGroupCap + 4];
  __shared__ __attribute__((aligned(16))) int8_t cs[kRowGroupCap + 8];
  const Tile tl = tiles[blockIdx.x];
  const TensorDesc td = descs[tl.tensor];
  const int shift = stage_tile(td.x + tl.off, tl.len, xs);
  int8_t* __restrict__ dst = td.codes ? td.codes + tl.off : nullptr;
  const int ca = static_cast<int>(reinterpret_cast<uintptr_t>(dst) & 3u);   // code e sits at cs[e + ca]
  __syncthreads();

  const int inner = tl.inner, w = row_width(inner), gpw = kWave / w;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  const int g = lane >> __builtin_ctz(w), gl = lane & (w - 1);
  for (int rb = wave * gpw; rb < tl.rows; rb += kWaves * gpw) {
    const int r = rb + g;
    const bool live = r < tl.rows;
    double sx2 = 0.0, se2 = 0.0;
    if (live) {
      const QP q = load_qp(params, tl.seg0 + r);
      const float* row = xs + shift + r * inner;
      int8_t* crow = cs + ca + r * inner;
      for (int j = gl; j < inner; j += w) {
        const float v = row[j];
        float e;
        const float code = quant1(v, q, e);
        crow[j] = static_cast<int8_t>(static_cast<int>(code));
        sx2 = fma(static_cast<double>(v), static_cast<double>(v), sx2);
        se2 = fma(static_cast<double>(e), static_cast<double>(e), se2);
      }
    }
    sx2 = group_sum(sx2, w); se2 = group_sum(se2, w);
    if (live && gl == 0) {
      ErrPartial o;
      o.sx2 = sx2; o.se2 = se2;
      parts[tl.part0 + r] = o;
    }
  }
  if (!dst) return;
  __syncthreads();
  // copy the codes out as whole dwords where the destination allows it
  const int total = tl.len + ca;
  int8_t* base = dst - ca;
  for (int k = threadIdx.x; (k << 2) < total; k += kBlock) {
    const int b0 = k << 2;
    if (b0 >= ca && b0 + 4 <= total) {
      *reinterpret_cast<uint32_t*>(base + b0) = *reinterpret_cast<const uint32_t*>(cs + b0);
    } else {
      const int lo = b0 > ca ? b0 : ca, hi = b0 + 4 < total ? b0 + 4 : total;
      for (int b = lo; b < hi; ++b) base[b] = cs[b];
    }
  }
}

// ---------------------------------------------------------------------------
// passes 2 + 3 in one sweep: x is read once for the fake-quant energies AND for
// the pair energies against qrun (Eq. 1, 3, 5, 6-7; Algorithm 2's D[i] vs Q[i]).
// Per element: 4 B (x) + 4 B (qrun) read, 1 B code written.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void put_codes4(int8_t* c, uint32_t* cw, bool cw_ok, int head, int i,
                                           uint32_t pk) {
  if (cw_ok) {
    st_codes(&cw[i], pk);
  } else if (c) {
    int8_t* d = c + head + (i << 2);
    d[0] = static_cast<int8_t>(pk); d[1] = static_cast<int8_t>(pk >> 8);
    d[2] = static_cast<int8_t>(pk >> 16); d[3] = static_cast<int8_t>(pk >> 24);
  }
}

__global__ __launch_bounds__(kBlock) void k_quantpair_stream(const TensorDesc* __restrict__ descs,
                                                             const Tile* __restrict__ tiles,
                                                             const qv2_qparams* __restrict__ params,
                                                             ErrPartial3* __restrict__ parts) {
  const Tile tl = tiles[blockIdx.x];
  const TensorDesc td = descs[tl.tensor];
  const float* __restrict__ p = td.x + tl.off;
  const float* __restrict__ b = td.qrun ? td.qrun + tl.off : nullptr;
  int8_t* __restrict__ c = td.codes ? td.codes + tl.off : nullptr;
  const QP q = load_qp(params, tl.seg0);
  const int len = tl.len, tid = threadIdx.x;
  double sx2 = 0.0, se2 = 0.0, sd2 = 0.0;

  // qrun at a different offset inside 16 bytes than x: its energy is taken element-wise
  const bool b_vec = b && (((reinterpret_cast<uintptr_t>(p) ^ reinterpret_cast<uintptr_t>(b)) & 15u) == 0);
  if (b && !b_vec) {
    for (int i = tid; i < len; i += kBlock) {
      const double d = static_cast<double>(p[i] - b[i]);
      sd2 = fma(d, d, sd2);
    }
  }
  const int head = head_elems(p, len);
  const int body = len - head, nvec = body >> 2, tail = body & 3;
  for (int k = 0; k < 2; ++k) {
    const bool on = k == 0 ? tid < head : tid < tail;
    if (!on) continue;
    const int idx = k == 0 ? tid : head + (nvec << 2) + tid;
    const float v = p[idx];
    float e;
    const float code = quant1(v, q, e);
    if (c) c[idx] = static_cast<int8_t>(static_cast<int>(code));
    sx2 += static_cast<double>(v) * v;
    se2 += static_cast<double>(e) * e;
    if (b_vec) { const float d = v - b[idx]; sd2 += static_cast<double>(d) * d; }
  }
  const float4* __restrict__ v4 = reinterpret_cast<const float4*>(p + head);
  const float4* __restrict__ b4 = reinterpret_cast<const float4*>(b + head);
  const bool cw_ok = c && ((reinterpret_cast<uintptr_t>(c + head) & 3u) == 0);
  uint32_t* __restrict__ cw = reinterpret_cast<uint32_t*>(c + head);
  Acc4 ae2, ax2, ad2;
#define PUT(ii, pk) put_codes4(c, cw, cw_ok, head, (ii), (pk))
  int i = tid;
  if (b_vec) {
    constexpr int U = kPairUnroll;
#if QV2_PIPELINE
    // Loads and stores share one in-order counter on this ISA: a wave that waits for its
    // next loads also waits for every store issued before them.  So the next round's loads
    // are issued BEFORE this round's code stores.
    if (i + (U - 1) * kBlock < nvec) {
      float4 r[U], g[U];
#pragma unroll
      for (int u = 0; u < U; ++u) { r[u] = ld4(&v4[i + u * kBlock]); g[u] = ld4(&b4[i + u * kBlock]); }
      for (;;) {
        const int inext = i + U * kBlock;
        const bool more = inext + (U - 1) * kBlock < nvec;
        float4 rn[U], gn[U];
        if (more) {
#pragma unroll
          for (int u = 0; u < U; ++u) { rn[u] = ld4(&v4[inext + u * kBlock]); gn[u] = ld4(&b4[inext + u * kBlock]); }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          PUT(i + u * kBlock, quant4(r[u], q, ae2, ax2));
          ad2.add_sq(r[u].x - g[u].x, r[u].y - g[u].y, r[u].z - g[u].z, r[u].w - g[u].w);
        }
        i = inext;
        if (!more) break;
#pragma unroll
        for (int u = 0; u < U; ++u) { r[u] = rn[u]; g[u] = gn[u]; }
      }
    }
#else
    for (; i + (U - 1) * kBlock < nvec; i += U * kBlock) {
      float4 r[U], g[U];
#pragma unroll
      for (int u = 0; u < U; ++u) { r[u] = ld4(&v4[i + u * kBlock]); g[u] = ld4(&b4[i + u * kBlock]); }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        PUT(i + u * kBlock, quant4(r[u], q, ae2, ax2));
        ad2.add_sq(r[u].x - g[u].x, r[u].y - g[u].y, r[u].z - g[u].z, r[u].w - g[u].w);
      }
    }
#endif
    for (; i < nvec; i += kBlock) {
      const float4 r = ld4(&v4[i]), g = ld4(&b4[i]);
      PUT(i, quant4(r, q, ae2, ax2));
      ad2.add_sq(r.x - g.x, r.y - g.y, r.z - g.z, r.w - g.w);
    }
  } else {
    for (; i + (kUnroll - 1) * kBlock < nvec; i += kUnroll * kBlock) {
      float4 r[kUnroll];
#pragma unroll
      for (int u = 0; u < kUnroll; ++u) r[u] = ld4(&v4[i + u * kBlock]);
#pragma unroll
      for (int u = 0; u < kUnroll; ++u)
        PUT(i + u * kBlock, quant4(r[u], q, ae2, ax2));
    }
    for (; i < nvec; i += kBlock)
      PUT(i, quant4(ld4(&v4[i]), q, ae2, ax2));
  }
#undef PUT
  se2 += ae2.total(); sx2 += ax2.total(); sd2 += ad2.total();
  double zero = 0.0;
  block_sum2(sx2, se2);
  __syncthreads();                                  // block_sum2's LDS slots are reused
  block_sum2(sd2, zero);
  if (tid == 0) {
    ErrPartial3 o;
    o.sx2 = sx2; o.se2 = se2; o.sd2 = sd2;
    parts[tl.part0] = o;
  }
}

// fused passes 2 + 3, row-group tiles
__global__ __launch_bounds__(kBlock) void k_quantpair_rows(const TensorDesc* __restrict__ descs,
                                                           const Tile* __restrict__ tiles,
                                                           const qv2_qparams* __restrict__ params,
                                                           ErrPartial3* __restrict__ parts) {
  __shared__ __attribute__((aligned(16))) float xs[kRowGroupCap + 4];
  __shared__ __attribute__((aligned(16))) int8_t cs[kRowGroupCap + 8];
  const Tile tl = tiles[blockIdx.x];
  const TensorDesc td = descs[tl.tensor];
  const int shift = stage_tile(td.x + tl.off, tl.len, xs);
  const float* __restrict__ b = td.qrun ? td.qrun + tl.off : nullptr;
  int8_t* __restrict__ dst = td.codes ? td.codes + tl.off : nullptr;
  const int ca = static_cast<int>(reinterpret_cast<uintptr_t>(dst) & 3u);
  __syncthreads();

  const int inner = tl.inner, w = row_width(inner), gpw = kWave / w;
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  const int g = lane >> __builtin_ctz(w), gl = lane & (w - 1);
  for (int rb = wave * gpw; rb < tl.rows; rb += kWaves * gpw) {
    const int r = rb + g;
    const bool live = r < tl.rows;
    double sx2 = 0.0, se2 = 0.0, sd2 = 0.0;
    if (live) {
      const QP q = load_qp(params, tl.seg0 + r);
      const float* row = xs + shift + r * inner;
      int8_t* crow = cs + ca + r * inner;
      for (int j = gl; j < inner; j += w) {
        const float v = row[j];
        float e;
        const float code = quant1(v, q, e);
        crow[j] = static_cast<int8_t>(static_cast<int>(code));
        sx2 = fma(static_cast<double>(v), static_cast<double>(v), sx2);
        se2 = fma(static_cast<double>(e), static_cast<double>(e), se2);
        if (b) {
          const double d = static_cast<double>(v - b[r * inner + j]);
          sd2 = fma(d, d, sd2);
        }
      }
    }
    sx2 = group_sum(sx2, w); se2 = group_sum(se2, w); sd2 = group_sum(sd2, w);
    if (live && gl == 0) {
      ErrPartial3 o;
      o.sx2 = sx2; o.se2 = se2; o.sd2 = sd2;
      parts[tl.part0 + r] = o;
    }
  }
  if (!dst) return;
  __syncthreads();
  const int total = tl.len + ca;
  int8_t* base = dst - ca;
  for (int k = threadIdx.x; (k << 2) < total; k += kBlock) {
    const int b0 = k << 2;
    if (b0 >= ca && b0 + 4 <= total) {
      *reinterpret_cast<uint32_t*>(base + b0) = *reinterpret_cast<const uint32_t*>(cs + b0);
    } else {
      const int lo = b0 > ca ? b0 : ca, hi = b0 + 4 < total ? b0 + 4 : total;
      for (int bb = lo; bb < hi; ++bb) base[bb] = cs[bb];
    }
  }
}

// second energy of a partial record: the pair-noise energy
__device__ __forceinline__ double pair_energy(const ErrPartial& p) { return p.se2; }
__device__ __forceinline__ double pair_energy(const ErrPartial3& p) { return p.sd2; }

template <class P>
__global__ __launch_bounds__(kBlock) void k_fold_err(const Segment* __restrict__ segs, int nseg,
                                                     const P* __restrict__ parts,
                                                     qv2_sums* __restrict__ sums) {
  const int seg = blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  if (seg >= nseg) return;
  const Segment sg = segs[seg];
  if (sg.nparts > kFoldWaveMax) return;            // folded by k_fold_err_big
  double sx2 = 0.0, se2 = 0.0;
  for (int i = lane; i < sg.nparts; i += kWave) {
    const P q = parts[sg.part0 + i];
    sx2 += q.sx2; se2 += q.se2;
  }
  sx2 = group_sum(sx2, kWave); se2 = group_sum(se2, kWave);
  if (lane == 0) {
    sums[seg].sum_x2 = sx2; sums[seg].sum_e2 = se2; sums[seg].n = sg.n;
  }
}

// ---------------------------------------------------------------------------
// pass 3 (Algorithm 2: CalculateSQNR / CalculateMSE on D[i] and Q[i])
// ---------------------------------------------------------------------------
__global__ __launch_bounds__(kBlock) void k_pair_stream(const TensorDesc* __restrict__ descs,
                                                        const Tile* __restrict__ tiles,
                                                        ErrPartial* __restrict__ parts) {
  const Tile tl = tiles[blockIdx.x];
  const TensorDesc td = descs[tl.tensor];
  const float* __restrict__ a = td.x + tl.off;
  const float* __restrict__ b = td.qrun + tl.off;
  const int len = tl.len, tid = threadIdx.x;
  double sr2 = 0.0, sd2 = 0.0;

  if (((reinterpret_cast<uintptr_t>(a) ^ reinterpret_cast<uintptr_t>(b)) & 15u) != 0) {
    // the two tensors sit at different offsets within 16 bytes: element loads
    for (int i = tid; i < len; i += kBlock) {
      const float x = a[i], d = x - b[i];
      sr2 = fma(static_cast<double>(x), static_cast<double>(x), sr2);
      sd2 = fma(static_cast<double>(d), static_cast<double>(d), sd2);
    }
  } else {
    const int head = head_elems(a, len);
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
    const float4* __restrict__ a4 = reinterpret_cast<const float4*>(a + head);
    const float4* __restrict__ b4 = reinterpret_cast<const float4*>(b + head);
    constexpr int U = kPairUnroll;                 // two streams: same bytes in flight
    Acc4 ar2, ad2;
    int i = tid;
    for (; i + (U - 1) * kBlock < nvec; i += U * kBlock) {
      float4 ra[U], rb[U];
#pragma unroll
      for (int u = 0; u < U; ++u) { ra[u] = ld4(&a4[i + u * kBlock]); rb[u] = ld4(&b4[i + u * kBlock]); }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        ar2.add_sq(ra[u].x, ra[u].y, ra[u].z, ra[u].w);
        ad2.add_sq(ra[u].x - rb[u].x, ra[u].y - rb[u].y, ra[u].z - rb[u].z, ra[u].w - rb[u].w);
      }
    }
    for (; i < nvec; i += kBlock) {
      const float4 x = ld4(&a4[i]), y = ld4(&b4[i]);
      ar2.add_sq(x.x, x.y, x.z, x.w);
      ad2.add_sq(x.x - y.x, x.y - y.y, x.z - y.z, x.w - y.w);
    }
    sr2 += ar2.total(); sd2 += ad2.total();
  }
  block_sum2(sr2, sd2);
  if (tid == 0) {
    ErrPartial o;
    o.sx2 = sr2; o.se2 = sd2;
    parts[tl.part0] = o;
  }
}

template <class P>
__global__ __launch_bounds__(kBlock) void k_fold_pair(const PairTensor* __restrict__ pt, int n,
                                                      const P* __restrict__ parts,
                                                      qv2_pair_sums* __restrict__ out) {
  const int t = blockIdx.x * kWaves + (threadIdx.x >> 6);
  const int lane = threadIdx.x & (kWave - 1);
  if (t >= n) return;
  const PairTensor p = pt[t];
  if (p.nparts > kFoldWaveMax) return;             // folded by k_fold_pair_big
  double sr2 = 0.0, sd2 = 0.0;
  for (int i = lane; i < p.nparts; i += kWave) {
    const P q = parts[p.part0 + i];
    sr2 += q.sx2; sd2 += pair_energy(q);
  }
  sr2 = group_sum(sr2, kWave); sd2 = group_sum(sd2, kWave);
  if (lane == 0) {
    qv2_pair_sums o;
    o.sum_ref2 = sr2; o.sum_d2 = sd2; o.n = p.n; o._pad = 0;
    out[t] = o;
  }
}

// ---------------------------------------------------------------------------
// folds of segments with many partials (large tensors): one 1024-thread
// workgroup per segment, thread-strided then a fixed tree => deterministic
// ---------------------------------------------------------------------------
__device__ __forceinline__ void fold_block_sum2(double& a, double& b) {
  __shared__ double sa[kFoldWaves], sb[kFoldWaves];
  a = group_sum(a, kWave);
  b = group_sum(b, kWave);
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  if (lane == 0) { sa[wave] = a; sb[wave] = b; }
  __syncthreads();
  if (threadIdx.x == 0) {
    a = sa[0]; b = sb[0];
    for (int i = 1; i < kFoldWaves; ++i) { a += sa[i]; b += sb[i]; }
  }
}

__global__ __launch_bounds__(kFoldBlock) void k_fold_stats_big(const Segment* __restrict__ segs,
                                                               const int* __restrict__ ids,
                                                               const StatPartial* __restrict__ parts,
                                                               qv2_qparams* __restrict__ params,
                                                               qv2_sums* __restrict__ sums) {
  __shared__ float smn[kFoldWaves], smx[kFoldWaves];
  const int seg = ids[blockIdx.x];
  const Segment sg = segs[seg];
  float mn = INFINITY, mx = -INFINITY;
  double sx = 0.0, sx2 = 0.0;
#pragma unroll 4
  for (int i = threadIdx.x; i < sg.nparts; i += kFoldBlock) {
    const StatPartial q = parts[sg.part0 + i];
    mn = fminf(mn, q.mn); mx = fmaxf(mx, q.mx);
    sx += q.sx; sx2 += q.sx2;
  }
  mn = group_min(mn, kWave); mx = group_max(mx, kWave);
  const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
  if (lane == 0) { smn[wave] = mn; smx[wave] = mx; }
  fold_block_sum2(sx, sx2);                         // contains the barrier
  if (threadIdx.x == 0) {
    for (int i = 1; i < kFoldWaves; ++i) { mn = fminf(mn, smn[i]); mx = fmaxf(mx, smx[i]); }
    qv2_qparams qp;
    make_params(mn, mx, sg.scheme, qp);
    params[seg] = qp;
    qv2_sums o;
    o.sum_x = sx; o.sum_x2 = sx2; o.sum_e2 = 0.0; o.n = sg.n;
    sums[seg] = o;
  }
}

template <class P>
__global__ __launch_bounds__(kFoldBlock) void k_fold_err_big(const Segment* __restrict__ segs,
                                                             const int* __restrict__ ids,
                                                             const P* __restrict__ parts,
                                                             qv2_sums* __restrict__ sums) {
  const int seg = ids[blockIdx.x];
  const Segment sg = segs[seg];
  double sx2 = 0.0, se2 = 0.0;
#pragma unroll 4
  for (int i = threadIdx.x; i < sg.nparts; i += kFoldBlock) {
    const P q = parts[sg.part0 + i];
    sx2 += q.sx2; se2 += q.se2;
  }
  fold_block_sum2(sx2, se2);
  if (threadIdx.x == 0) {
    sums[seg].sum_x2 = sx2; sums[seg].sum_e2 = se2; sums[seg].n = sg.n;
  }
}

template <class P>
__global__ __launch_bounds__(kFoldBlock) void k_fold_pair_big(const PairTensor* __restrict__ pt,
                                                              const int* __restrict__ ids,
                                                              const P* __restrict__ parts,
                                                              qv2_pair_sums* __restrict__ out) {
  const int t = ids[blockIdx.x];
  const PairTensor p = pt[t];
  double sr2 = 0.0, sd2 = 0.0;
#pragma unroll 4
  for (int i = threadIdx.x; i < p.nparts; i += kFoldBlock) {
    const P q = parts[p.part0 + i];
    sr2 += q.sx2; sd2 += pair_energy(q);
  }
  fold_block_sum2(sr2, sd2);
  if (threadIdx.x == 0) {
    qv2_pair_sums o;
    o.sum_ref2 = sr2; o.sum_d2 = sd2; o.n = p.n; o._pad = 0;
    out[t] = o;
  }
}

// ---------------------------------------------------------------------------
// host helpers
// ---------------------------------------------------------------------------
size_t align256(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

// First device call on a plan: one allocation holding all tables, blocking copies.
qv2_status ensure_uploaded(qv2_plan* p) {
  if (p->d_blob) return QV2_OK;
  const size_t b_desc = align256(p->descs.size() * sizeof(TensorDesc));
  const size_t b_tile = align256(p->tiles.size() * sizeof(Tile));
  const size_t b_seg = align256(p->segments.size() * sizeof(Segment));
  const size_t b_ptile = align256(p->pair_tiles.size() * sizeof(Tile));
  const size_t b_pten = align256(p->pair_tensors.size() * sizeof(PairTensor));
  const size_t b_bseg = align256(p->big_segments.size() * sizeof(int32_t));
  const size_t b_bpair = align256(p->big_pair_tensors.size() * sizeof(int32_t));
  const size_t b_ften = align256(p->fused_pair_tensors.size() * sizeof(PairTensor));
  const size_t b_bften = align256(p->big_fused_pair_tensors.size() * sizeof(int32_t));
  char* blob = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&blob), b_desc + b_tile + b_seg + b_ptile + b_pten +
                                                      b_bseg + b_bpair + b_ften + b_bften + 256) !=
      hipSuccess) { (void)hipGetLastError(); return QV2_ERR_HIP; }
  char* q = blob;
  p->d_descs = reinterpret_cast<TensorDesc*>(q); q += b_desc;
  p->d_tiles = reinterpret_cast<Tile*>(q); q += b_tile;
  p->d_segments = reinterpret_cast<Segment*>(q); q += b_seg;
  p->d_pair_tiles = reinterpret_cast<Tile*>(q); q += b_ptile;
  p->d_pair_tensors = reinterpret_cast<PairTensor*>(q); q += b_pten;
  p->d_big_segments = reinterpret_cast<int32_t*>(q); q += b_bseg;
  p->d_big_pair_tensors = reinterpret_cast<int32_t*>(q); q += b_bpair;
  p->d_fused_pair_tensors = reinterpret_cast<PairTensor*>(q); q += b_ften;
  p->d_big_fused_pair_tensors = reinterpret_cast<int32_t*>(q);
  bool ok = true;
  auto put = [&](void* d, const void* h, size_t n) {
    if (n && hipMemcpy(d, h, n, hipMemcpyHostToDevice) != hipSuccess) ok = false;
  };
  put(p->d_descs, p->descs.data(), p->descs.size() * sizeof(TensorDesc));
  put(p->d_tiles, p->tiles.data(), p->tiles.size() * sizeof(Tile));
  put(p->d_segments, p->segments.data(), p->segments.size() * sizeof(Segment));
  put(p->d_pair_tiles, p->pair_tiles.data(), p->pair_tiles.size() * sizeof(Tile));
  put(p->d_pair_tensors, p->pair_tensors.data(), p->pair_tensors.size() * sizeof(PairTensor));
  put(p->d_big_segments, p->big_segments.data(), p->big_segments.size() * sizeof(int32_t));
  put(p->d_big_pair_tensors, p->big_pair_tensors.data(), p->big_pair_tensors.size() * sizeof(int32_t));
  put(p->d_fused_pair_tensors, p->fused_pair_tensors.data(),
      p->fused_pair_tensors.size() * sizeof(PairTensor));
  put(p->d_big_fused_pair_tensors, p->big_fused_pair_tensors.data(),
      p->big_fused_pair_tensors.size() * sizeof(int32_t));
  if (!ok) { (void)hipGetLastError(); (void)hipFree(blob); return QV2_ERR_HIP; }
  p->d_blob = blob;
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
    for (int k = 0; k < QV2_K_COUNT; ++k) {
      hipEvent_t a = nullptr, b = nullptr;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) {
        (void)hipGetLastError();
        return QV2_ERR_HIP;
      }
      plan->ev_start[k] = a; plan->ev_stop[k] = b;
    }
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

qv2_status qv2_calibrate(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums,
                         void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  qv2_status st = check_call(plan, d_params, d_sums, d_workspace, workspace_bytes);
  if (st != QV2_OK) return st;
  if ((st = ensure_uploaded(plan)) != QV2_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  StatPartial* parts = static_cast<StatPartial*>(d_workspace);
  const int n_stream = static_cast<int>(plan->n_stream_tiles);
  const int n_rows = static_cast<int>(plan->tiles.size()) - n_stream;
  const int nseg = static_cast<int>(plan->segments.size());
  if (n_stream > 0) {
    Timed timed(plan, QV2_K_STATS_STREAM, s);
    hipLaunchKernelGGL(k_stats_stream, dim3(n_stream), dim3(kBlock), 0, s, plan->d_descs,
                       plan->d_tiles, parts);
  }
  if (n_rows > 0) {
    Timed timed(plan, QV2_K_STATS_ROWS, s);
    hipLaunchKernelGGL(k_stats_rows, dim3(n_rows), dim3(kBlock), 0, s, plan->d_descs,
                       plan->d_tiles + n_stream, parts);
  }
  hipLaunchKernelGGL(k_fold_stats, dim3((nseg + kWaves - 1) / kWaves), dim3(kBlock), 0, s,
                     plan->d_segments, nseg, parts, d_params, d_sums);
  if (const int nb = static_cast<int>(plan->big_segments.size()))
    hipLaunchKernelGGL(k_fold_stats_big, dim3(nb), dim3(kFoldBlock), 0, s, plan->d_segments,
                       plan->d_big_segments, parts, d_params, d_sums);
  return launch_status();
}

qv2_status qv2_fakequant_metrics(qv2_plan* plan, const qv2_qparams* d_params, qv2_sums* d_sums,
                                 void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  qv2_status st = check_call(plan, d_params, d_sums, d_workspace, workspace_bytes);
  if (st != QV2_OK) return st;
  if ((st = ensure_uploaded(plan)) != QV2_OK) return st;
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  ErrPartial* parts = static_cast<ErrPartial*>(d_workspace);
  const int n_stream = static_cast<int>(plan->n_stream_tiles);
  const int n_rows = static_cast<int>(plan->tiles.size()) - n_stream;
  const int nseg = static_cast<int>(plan->segments.size());
  if (n_stream > 0) {
    Timed timed(plan, QV2_K_QUANT_STREAM, s);
    hipLaunchKernelGGL(k_quant_stream, dim3(n_stream), dim3(kBlock), 0, s, plan->d_descs,
                       plan->d_tiles, d_params, parts);
  }
  if (n_rows > 0) {
    Timed timed(plan, QV2_K_QUANT_ROWS, s);
    hipLaunchKernelGGL(k_quant_rows, dim3(n_rows), dim3(kBlock), 0, s, plan->d_descs,
                       plan->d_tiles + n_stream, d_params, parts);
  }
  hipLaunchKernelGGL(k_fold_err<ErrPartial>, dim3((nseg + kWaves - 1) / kWaves), dim3(kBlock), 0, s,
                     plan->d_segments, nseg, parts, d_sums);
  if (const int nb = static_cast<int>(plan->big_segments.size()))
    hipLaunchKernelGGL(k_fold_err_big<ErrPartial>, dim3(nb), dim3(kFoldBlock), 0, s, plan->d_segments,
                       plan->d_big_segments, parts, d_sums);
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
    hipLaunchKernelGGL(k_pair_stream, dim3(n_tiles), dim3(kBlock), 0, s, plan->d_descs,
                       plan->d_pair_tiles, parts);
  }
  hipLaunchKernelGGL(k_fold_pair<ErrPartial>, dim3((nt + kWaves - 1) / kWaves), dim3(kBlock), 0, s,
                     plan->d_pair_tensors, nt, parts, d_pair_sums);
  if (const int nb = static_cast<int>(plan->big_pair_tensors.size()))
    hipLaunchKernelGGL(k_fold_pair_big<ErrPartial>, dim3(nb), dim3(kFoldBlock), 0, s, plan->d_pair_tensors,
                       plan->d_big_pair_tensors, parts, d_pair_sums);
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
  const int n_stream = static_cast<int>(plan->n_stream_tiles);
  const int n_rows = static_cast<int>(plan->tiles.size()) - n_stream;
  const int nseg = static_cast<int>(plan->segments.size());
  const int nt = static_cast<int>(plan->fused_pair_tensors.size());
  if (n_stream > 0) {
    Timed timed(plan, QV2_K_QUANTPAIR_STREAM, s);
    hipLaunchKernelGGL(k_quantpair_stream, dim3(n_stream), dim3(kBlock), 0, s, plan->d_descs,
                       plan->d_tiles, d_params, parts);
  }
  if (n_rows > 0) {
    Timed timed(plan, QV2_K_QUANTPAIR_ROWS, s);
    hipLaunchKernelGGL(k_quantpair_rows, dim3(n_rows), dim3(kBlock), 0, s, plan->d_descs,
                       plan->d_tiles + n_stream, d_params, parts);
  }
  hipLaunchKernelGGL(k_fold_err<ErrPartial3>, dim3((nseg + kWaves - 1) / kWaves), dim3(kBlock), 0, s,
                     plan->d_segments, nseg, parts, d_sums);
  if (const int nb = static_cast<int>(plan->big_segments.size()))
    hipLaunchKernelGGL(k_fold_err_big<ErrPartial3>, dim3(nb), dim3(kFoldBlock), 0, s,
                       plan->d_segments, plan->d_big_segments, parts, d_sums);
  hipLaunchKernelGGL(k_fold_pair<ErrPartial3>, dim3((nt + kWaves - 1) / kWaves), dim3(kBlock), 0, s,
                     plan->d_fused_pair_tensors, nt, parts, d_pair_sums);
  if (const int nb = static_cast<int>(plan->big_fused_pair_tensors.size()))
    hipLaunchKernelGGL(k_fold_pair_big<ErrPartial3>, dim3(nb), dim3(kFoldBlock), 0, s,
                       plan->d_fused_pair_tensors, plan->d_big_fused_pair_tensors, parts, d_pair_sums);
  return launch_status();
}

}  // extern "C"
