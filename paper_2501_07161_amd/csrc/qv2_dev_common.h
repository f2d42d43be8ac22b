// Device-side building blocks shared by all kernels: address-space typedefs, streaming loads
// and stores, wavefront / workgroup reductions in a fixed order, the quantizer of Eq. 1-5.
#pragma once
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
// the same 16-byte vector at an address that is only 4-byte aligned: the partner stream of a pair
// whose two tensors sit at different offsets inside 16 bytes (x decides where the vectors start)
typedef f4 f4u __attribute__((aligned(4)));
typedef const QV2_GLOBAL f4u* gf4u_ptr;
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

// Vector i of the partner stream that starts at float address b.  AL: the address is 16-byte
// aligned; otherwise only 4-byte aligned, which a dwordx4 load takes as well.
template <bool AL>
__device__ __forceinline__ f4 ld4b(gf_ptr b, int i) {
  if (AL) return ld4((gf4_ptr)b + i);
#if QV2_NT_LOADS
  return __builtin_nontemporal_load((gf4u_ptr)b + i);
#else
  return *((gf4u_ptr)b + i);
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
// ZP0: the zero-point is known to be 0 (a symmetric scheme whose parameters the kernel has just
// made itself), so its add and subtract are left out; codes, xhat and err^2 are the same.
template <bool ZP0 = false>
__device__ __forceinline__ float quant1(float x, const QP& q, float& err, float& xhat) {
  const float t = x * q.inv;                       // fp32 multiply
  const float r = rintf(t);                        // round half to even
  // integer add of the zero-point: exact in fp32 below 2^24, saturates above
  const float c = fminf(fmaxf(ZP0 ? r : r + q.zpf, -128.0f), 127.0f);
  xhat = (ZP0 ? c : c - q.zpf) * q.scale;          // exact difference, one multiply
  err = x - xhat;
  return c;
}

// COS: also accumulate sum x*xhat (the cross term of the cosine similarity, Sec. 6.1 Eq. 8)
// X2 = false leaves sum x^2 out (the caller already has it from the calibration sweep)
template <bool COS, bool X2 = true, bool ZP0 = false>
__device__ __forceinline__ uint32_t quant4(const f4& v, const QP& q, Acc4& se2, Acc4& sx2, Acc4& sxh) {
  float e0, e1, e2, e3, h0, h1, h2, h3;
  const int c0 = static_cast<int>(quant1<ZP0>(v.x, q, e0, h0));
  const int c1 = static_cast<int>(quant1<ZP0>(v.y, q, e1, h1));
  const int c2 = static_cast<int>(quant1<ZP0>(v.z, q, e2, h2));
  const int c3 = static_cast<int>(quant1<ZP0>(v.w, q, e3, h3));
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

}  // namespace
