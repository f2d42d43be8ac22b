// Fold kernels: a segment's or tensor's partial records summed in a fixed order; the
// calibration fold also makes the quantization parameters (Eq. 2, Eq. 4).
#pragma once
#include "qv2_dev_calib.h"

namespace {

// ---------------------------------------------------------------------------
// folds.  An item's partials (a segment's, or a tensor's for the pair sums) are folded in a
// fixed order: lane- (or thread-) strided, then a butterfly.  One launch of 1024-thread
// workgroups serves all items: the first n_wide workgroups take one listed item each (those
// with more than kFoldWaveMax partials) with all their threads, every other workgroup takes
// 16 items, one per wavefront, and leaves the listed ones alone.
// ---------------------------------------------------------------------------
constexpr int kFoldPerBlock = kFoldBlock / kWave;

// A result record goes to its place in device memory and, when `mirror` is not 0, also to the
// address that many bytes further on: the same record in pinned host memory, mapped into the
// device's address space, so that a caller's results arrive without a copy after the kernels.
template <class T>
__device__ __forceinline__ void put_record(T* dst, const T& o, ptrdiff_t mirror) {
  *dst = o;
  if (mirror) *reinterpret_cast<T*>(reinterpret_cast<char*>(dst) + mirror) = o;
}

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
                                                   double* __restrict__ pair_xq, ptrdiff_t mirror) {
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
    put_record(out + f.id, o, mirror);
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
  ptrdiff_t mirror;                          // see put_record; 0 = none
};

__device__ __forceinline__ void fold_statpair_family(const StatFoldArgs<StatPartial>&, int) {}
template <class REC>
__device__ __forceinline__ void fold_statpair_family(const StatFoldArgs<REC>& a, int b) {
  fold_statpair_item<REC>(FoldIdx(b, a.wide_pt, a.n_wide_pt, a.nt), a.pt, a.parts, a.pair_out, a.pair_xq,
                          a.mirror);
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

// fields of a partial record (0 where the record has none)
__device__ __forceinline__ double part_sx2(const ErrPartial1&) { return 0.0; }
__device__ __forceinline__ double part_sx2(const ErrPartial3& p) { return p.sx2; }
__device__ __forceinline__ double part_sx2(const ErrPartial5& p) { return p.sx2; }
__device__ __forceinline__ double cross_xh(const ErrPartial1&) { return 0.0; }
__device__ __forceinline__ double cross_xh(const ErrPartial3&) { return 0.0; }
__device__ __forceinline__ double cross_xh(const ErrPartial5& p) { return p.sxh; }
__device__ __forceinline__ double cross_xq(const ErrPartial&) { return 0.0; }
__device__ __forceinline__ double cross_xq(const ErrPartial3&) { return 0.0; }
__device__ __forceinline__ double cross_xq(const ErrPartial5& p) { return p.sxq; }
// second energy of a partial record: the pair-noise energy
__device__ __forceinline__ double pair_energy(const ErrPartial& p) { return p.se2; }
__device__ __forceinline__ double pair_energy(const ErrPartial3& p) { return p.sd2; }
__device__ __forceinline__ double pair_energy(const ErrPartial5& p) { return p.sd2; }

// One tensor's record from its segments' records, by one workgroup of kFoldBlock threads: thread-
// strided over the segments, a butterfly per wavefront, then the wavefronts in order.
__device__ __forceinline__ void tensor_record(const HistTensor h, const qv2_qparams* __restrict__ params,
                                              const qv2_sums* __restrict__ sums,
                                              qv2_tensor_sums* __restrict__ out_rec, ptrdiff_t mirror) {
  __shared__ long long scnt[kFoldBlock / kWave];
  const int tid = threadIdx.x;
  float mn = INFINITY, mx = -INFINITY;
  double sx = 0.0, sx2 = 0.0, se2 = 0.0;
  long long cnt = 0;
  for (int i = tid; i < h.nseg; i += kFoldBlock) {
    const qv2_qparams p = params[h.seg0 + i];
    const qv2_sums u = sums[h.seg0 + i];
    mn = fminf(mn, p.min); mx = fmaxf(mx, p.max);
    sx += u.sum_x; sx2 += u.sum_x2; se2 += u.sum_e2; cnt += u.n;
  }
  for (int o = kWave >> 1; o > 0; o >>= 1) cnt += __shfl_xor(cnt, o);
  if ((tid & (kWave - 1)) == 0) scnt[tid >> 6] = cnt;
  block_minmax<kFoldBlock>(mn, mx);                // holds a barrier: scnt is visible after it
  block_sum3<kFoldBlock>(sx, sx2, se2);
  if (tid == 0) {
    qv2_tensor_sums o;
    o.sum_x = sx; o.sum_x2 = sx2; o.sum_e2 = se2; o.min = mn; o.max = mx;
    long long n = 0;
    for (int w = 0; w < kFoldBlock / kWave; ++w) n += scnt[w];
    o.n = n;
    o._pad[0] = o._pad[1] = 0;
    put_record(out_rec, o, mirror);
  }
}

// error energies of one segment.  ts != null (the last fold of a whole pass): a tensor that is this
// one segment gets its per-tensor record here as well - the same values tensor_record would give.
// P: the records of the row-group tiles; SP: those of the stream tiles (the same type, except
// in the last fold of a whole pass, whose quantize sweep leaves only one energy per tile).
template <class P, class SP>
__device__ __forceinline__ void fold_err_item(const FoldIdx& f, const Segment* __restrict__ segs,
                                              const P* __restrict__ parts, const SP* __restrict__ sparts,
                                              qv2_sums* __restrict__ sums,
                                              double* __restrict__ seg_xxhat, int skip_below,
                                              bool keep_x2, qv2_tensor_sums* __restrict__ ts = nullptr,
                                              const qv2_qparams* __restrict__ params = nullptr,
                                              const HistTensor* __restrict__ ht = nullptr, ptrdiff_t mirror = 0) {
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
    const SP q = sparts[sg.ep0 + i];
    sx2 += part_sx2(q); se2 += q.se2; sxh += cross_xh(q);
  }
  fold_sum3(f.wide, sx2, se2, sxh);
  if (f.lane == 0) {
    if (!keep_x2) sums[f.id].sum_x2 = sx2;         // else the calibration sweep's sum stays
    sums[f.id].sum_e2 = se2; sums[f.id].n = sg.n;
    if (seg_xxhat) seg_xxhat[f.id] = sxh;
    if (ts && ht[sg.tensor].nseg == 1) {
      const qv2_qparams p = params[f.id];
      qv2_tensor_sums o;                           // sums of one term; 0.0 + v as a fold would form it
      o.sum_x = 0.0 + sums[f.id].sum_x; o.sum_x2 = 0.0 + (keep_x2 ? sums[f.id].sum_x2 : sx2);
      o.sum_e2 = 0.0 + se2; o.n = sg.n; o.min = p.min; o.max = p.max;
      o._pad[0] = o._pad[1] = 0;
      put_record(ts + sg.tensor, o, mirror);
    }
  }
}

// pair energies of one tensor
template <class P>
__device__ __forceinline__ void fold_pair_item(const FoldIdx& f, const PairTensor* __restrict__ pt,
                                               const P* __restrict__ parts, qv2_pair_sums* __restrict__ out,
                                               double* __restrict__ pair_xq,
                                               const PairTensor* __restrict__ done = nullptr,
                                               ptrdiff_t mirror = 0) {
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
    put_record(out + f.id, o, mirror);
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
  const P* parts;                            // all records, or those of the row-group tiles when ...
  const void* sparts;                        // ... the stream tiles' are of another type (else == parts)
  int seg_blocks;
  // the last fold of a whole pass also leaves the per-tensor records (ts != null): single-segment
  // tensors with their segment, tensors made of row-group tiles by one more workgroup each
  qv2_tensor_sums* ts; const qv2_qparams* params; const HistTensor* ht;
  const int* row_tensors; int pair_blocks;
  ptrdiff_t mirror;                          // see put_record; 0 = none
};

template <class P, class SP>
__global__ __launch_bounds__(kFoldBlock) void k_fold_quant(const QuantFoldArgs<P> a) {
  const int b = blockIdx.x;
  if (b < a.seg_blocks) {
    fold_err_item<P, SP>(FoldIdx(b, a.wide_segs, a.n_wide_segs, a.nseg), a.segs, a.parts,
                         static_cast<const SP*>(a.sparts), a.sums,
                         a.seg_xxhat, a.skip_below, a.keep_x2, a.ts, a.params, a.ht, a.mirror);
  } else if (b < a.seg_blocks + a.pair_blocks) {
    fold_pair_item<P>(FoldIdx(b - a.seg_blocks, a.wide_pt, a.n_wide_pt, a.nt), a.pt, a.parts,
                      a.pair_out, a.pair_xq, a.pair_done, a.mirror);
  } else {
    const int t = a.row_tensors[b - a.seg_blocks - a.pair_blocks];
    tensor_record(a.ht[t], a.params, a.sums, a.ts + t, a.mirror);
  }
}

// fold of the separate pair pass
__global__ __launch_bounds__(kFoldBlock) void k_fold_pair(
    const PairTensor* __restrict__ pt, int nt, const int* __restrict__ ids, int n_wide,
    const ErrPartial* __restrict__ parts, qv2_pair_sums* __restrict__ out) {
  fold_pair_item<ErrPartial>(FoldIdx(blockIdx.x, ids, n_wide, nt), pt, parts, out, nullptr);
}

}  // namespace
