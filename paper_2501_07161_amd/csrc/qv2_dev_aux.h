// Pass 3 alone (pair metrics), calibration histograms, the per-tensor fold and conv+BN folding.
#pragma once
#include "qv2_dev_quant.h"

namespace {

// ---------------------------------------------------------------------------
// pass 3 alone (Algorithm 2: CalculateSQNR / CalculateMSE on D[i] and Q[i])
// ---------------------------------------------------------------------------
// vector body of a pair tile (BAL: the partner's vectors are 16-byte aligned; otherwise only 4-byte)
template <int BLOCK, int V, bool BAL>
__device__ __forceinline__ void pair_body(gf4_ptr a4, gf_ptr b, int nvec, Acc4& ar2, Acc4& ad2) {
  const int tid = threadIdx.x;
  int base = 0;
  for (; base + V * BLOCK <= nvec; base += V * BLOCK) {
    f4 ra[V], rb[V];
#pragma unroll
    for (int u = 0; u < V; ++u) { ra[u] = ld4(a4 + base + u * BLOCK + tid); rb[u] = ld4b<BAL>(b, base + u * BLOCK + tid); }
#pragma unroll
    for (int u = 0; u < V; ++u) {
      ar2.add_sq(ra[u].x, ra[u].y, ra[u].z, ra[u].w);
      ad2.add_sq(ra[u].x - rb[u].x, ra[u].y - rb[u].y, ra[u].z - rb[u].z, ra[u].w - rb[u].w);
    }
  }
  if (base < nvec) {        // the last, partial batch, loaded like a whole one
    f4 ra[V], rb[V];
#pragma unroll
    for (int u = 0; u < V; ++u) {
      const int i = base + u * BLOCK + tid, j = i < nvec ? i : nvec - 1;
      ra[u] = ld4(a4 + j); rb[u] = ld4b<BAL>(b, j);
    }
#pragma unroll
    for (int u = 0; u < V; ++u) {
      if (base + u * BLOCK + tid >= nvec) continue;
      ar2.add_sq(ra[u].x, ra[u].y, ra[u].z, ra[u].w);
      ad2.add_sq(ra[u].x - rb[u].x, ra[u].y - rb[u].y, ra[u].z - rb[u].z, ra[u].w - rb[u].w);
    }
  }
}

template <int BLOCK, int V>
__global__ __launch_bounds__(BLOCK) void k_pair_stream(const StreamView tiles,
                                                       ErrPartial* __restrict__ parts) {
  const TileRef tl = decode_tile(tiles, blockIdx.x);
  const gf_ptr a = (gf_ptr)tl.x;
  const gf_ptr b = (gf_ptr)tl.q;
  const int len = tl.len, tid = threadIdx.x;
  double sr2 = 0.0, sd2 = 0.0, unused = 0.0;

  // the vectors start where x's alignment puts them; when the partner sits at another offset
  // inside 16 bytes its vectors are loaded from 4-byte aligned addresses
  const bool b_al = ((reinterpret_cast<uintptr_t>(tl.x) ^ reinterpret_cast<uintptr_t>(tl.q)) & 15u) == 0;
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
  Acc4 ar2, ad2;
  if (b_al) pair_body<BLOCK, V, true>(a4, b + head, nvec, ar2, ad2);
  else pair_body<BLOCK, V, false>(a4, b + head, nvec, ar2, ad2);
  sr2 += ar2.total(); sd2 += ad2.total();
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

// Per-tensor fold of the per-segment results: one workgroup per tensor; `list` (may be null)
// names the tensors to fold, else all n of them.
__global__ __launch_bounds__(kFoldBlock) void k_tensor_fold(const HistTensor* __restrict__ ht,
                                                            const int* __restrict__ list,
                                                            const qv2_qparams* __restrict__ params,
                                                            const qv2_sums* __restrict__ sums,
                                                            qv2_tensor_sums* __restrict__ out,
                                                            ptrdiff_t mirror) {
  const int t = list ? list[blockIdx.x] : blockIdx.x;
  tensor_record(ht[t], params, sums, out + t, mirror);
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

}  // namespace
