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
//
// The kernels live in the qv2_dev_*.h files beside this one (all part of this translation
// unit); this file holds the launches and the extern "C" device entry points.
#include <hip/hip_runtime.h>

#include <cstring>
#include <limits>
#include <mutex>

#include "qv2_dev_common.h"   // loads / stores, reductions, the quantizer
#include "qv2_dev_calib.h"    // pass 1: k_stats_stream, k_stats_rows
#include "qv2_dev_fold.h"     // k_fold_stats, k_fold_quant, k_fold_pair
#include "qv2_dev_quant.h"    // pass 2 (+3): k_quant_stream, k_quant_rows, k_rows_reg
#include "qv2_dev_aux.h"      // k_pair_stream, k_hist*, k_tensor_fold, k_bn_fold

namespace {

// ---------------------------------------------------------------------------
// host helpers
// ---------------------------------------------------------------------------
size_t align256(size_t v) { return (v + 255) & ~static_cast<size_t>(255); }

template <class T>
size_t bytes_of(const std::vector<T>& v) { return v.size() * sizeof(T); }

// Workspace of the one entry point that allocates nothing
// (qv2_calibrate_fakequant_pair_metrics_noalloc): a fixed array in device memory, one copy per
// GPU the library runs on, held until the process ends.  In host code the array's name only
// stands for the symbol; its device address is looked up once per device and kept.
constexpr size_t kStaticScratchBytes = QV2_STATIC_SCRATCH_BYTES;
static __device__ __attribute__((used)) __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mu;

// Device address of `scratch` on device `dev`, which must be the current device; null on failure.
void* scratch_on_device(int dev) {
  if (dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

// The plan's device blob: every table in one allocation, 256-byte aligned sections.  The host
// image is assembled first, so that one copy brings it over.
struct BlobBuilder {
  std::vector<char> image;
  BlobBuilder() : image(256, 0) {}
  template <class T>
  size_t put(const std::vector<T>& v) {
    const size_t at = image.size();
    image.resize(at + align256(v.size() * sizeof(T)), 0);
    if (!v.empty()) std::memcpy(image.data() + at, v.data(), v.size() * sizeof(T));
    return at;
  }
};

struct BlobLayout {
  size_t run[4], coarse[4], row, reg, wide, seg, pt, ft, st, bs, be, bp, bf, bst, ht, hten, rowt, latet;
};

const StreamTable* stream_tables(const qv2_plan* p, int i) {
  const StreamTable* t[4] = {&p->read_tiles, &p->quant_tiles, &p->quant_ro_tiles, &p->pair_tiles};
  return t[i];
}

BlobLayout build_blob(const qv2_plan* p, BlobBuilder& b) {
  BlobLayout o{};
  for (int i = 0; i < 4; ++i) {
    o.run[i] = b.put(stream_tables(p, i)->runs);
    o.coarse[i] = b.put(stream_tables(p, i)->coarse);
  }
  o.row = b.put(p->row_tiles); o.reg = b.put(p->reg_tiles); o.wide = b.put(p->wide_tiles);
  o.seg = b.put(p->segments); o.pt = b.put(p->pair_tensors); o.ft = b.put(p->fused_pair_tensors);
  o.st = b.put(p->stat_pair_tensors);
  o.bs = b.put(p->big_stat_segments); o.be = b.put(p->big_err_segments);
  o.bp = b.put(p->big_pair_tensors); o.bf = b.put(p->big_fused_pair_tensors);
  o.bst = b.put(p->big_stat_pair_tensors);
  o.ht = b.put(p->hist_tiles); o.hten = b.put(p->hist_tensors);
  o.rowt = b.put(p->row_tensors); o.latet = b.put(p->late_tensors);
  return o;
}

size_t blob_bytes(const qv2_plan* p) {
  auto sec = [](size_t n) { return align256(n); };
  size_t total = 256;
  for (int i = 0; i < 4; ++i)
    total += sec(bytes_of(stream_tables(p, i)->runs)) + sec(bytes_of(stream_tables(p, i)->coarse));
  total += sec(bytes_of(p->row_tiles)) + sec(bytes_of(p->reg_tiles)) + sec(bytes_of(p->wide_tiles)) +
           sec(bytes_of(p->segments)) +
           sec(bytes_of(p->pair_tensors)) + sec(bytes_of(p->fused_pair_tensors)) +
           sec(bytes_of(p->stat_pair_tensors)) + sec(bytes_of(p->big_stat_segments)) +
           sec(bytes_of(p->big_err_segments)) + sec(bytes_of(p->big_pair_tensors)) +
           sec(bytes_of(p->big_fused_pair_tensors)) + sec(bytes_of(p->big_stat_pair_tensors)) +
           sec(bytes_of(p->hist_tiles)) + sec(bytes_of(p->hist_tensors)) + sec(bytes_of(p->row_tensors)) +
           sec(bytes_of(p->late_tensors));
  return total;
}

// Puts the plan's tables on the current device: one allocation and one copy on `s`, which is
// then waited for.  A plan that is already on this device is left alone.
qv2_status upload(qv2_plan* p, hipStream_t s) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return QV2_ERR_HIP; }
  // the tables live on one device: a later call with another device current would hand its
  // kernels pointers they cannot use
  if (p->d_blob) return dev == p->device ? QV2_OK : QV2_ERR_HIP;
  BlobBuilder b;
  BlobLayout o;
  try {
    o = build_blob(p, b);
  } catch (...) {
    return QV2_ERR_NOMEM;
  }
  char* blob = nullptr;
  if (hipMalloc(reinterpret_cast<void**>(&blob), b.image.size()) != hipSuccess) {
    (void)hipGetLastError();
    return QV2_ERR_HIP;
  }
  if (hipMemcpyAsync(blob, b.image.data(), b.image.size(), hipMemcpyHostToDevice, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess) {
    (void)hipGetLastError();
    (void)hipFree(blob);
    return QV2_ERR_HIP;
  }
  StreamView* views[4] = {&p->d_read_tiles, &p->d_quant_tiles, &p->d_quant_ro_tiles, &p->d_pair_tiles};
  for (int i = 0; i < 4; ++i) {
    const StreamTable* t = stream_tables(p, i);
    *views[i] = StreamView{reinterpret_cast<const Run*>(blob + o.run[i]),
                           reinterpret_cast<const int32_t*>(blob + o.coarse[i]),
                           static_cast<int32_t>(t->runs.size()), t->shift};
  }
  p->d_row_tiles = reinterpret_cast<Tile*>(blob + o.row);
  p->d_reg_tiles = reinterpret_cast<Tile*>(blob + o.reg);
  p->d_wide_tiles = reinterpret_cast<Tile*>(blob + o.wide);
  p->d_segments = reinterpret_cast<Segment*>(blob + o.seg);
  p->d_pair_tensors = reinterpret_cast<PairTensor*>(blob + o.pt);
  p->d_fused_pair_tensors = reinterpret_cast<PairTensor*>(blob + o.ft);
  p->d_stat_pair_tensors = reinterpret_cast<PairTensor*>(blob + o.st);
  p->d_big_stat_segments = reinterpret_cast<int32_t*>(blob + o.bs);
  p->d_big_err_segments = reinterpret_cast<int32_t*>(blob + o.be);
  p->d_big_pair_tensors = reinterpret_cast<int32_t*>(blob + o.bp);
  p->d_big_fused_pair_tensors = reinterpret_cast<int32_t*>(blob + o.bf);
  p->d_big_stat_pair_tensors = reinterpret_cast<int32_t*>(blob + o.bst);
  p->d_hist_tiles = reinterpret_cast<Tile*>(blob + o.ht);
  p->d_hist_tensors = reinterpret_cast<HistTensor*>(blob + o.hten);
  p->d_row_tensors = reinterpret_cast<int32_t*>(blob + o.rowt);
  p->d_late_tensors = reinterpret_cast<int32_t*>(blob + o.latet);
  p->d_blob = blob;
  p->device = dev;
  (void)scratch_on_device(dev);      // set-up time: the entry point that allocates nothing finds it ready
  return QV2_OK;
}

// First device call on a plan that was not uploaded explicitly.
qv2_status ensure_uploaded(qv2_plan* p) { return upload(p, nullptr); }

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
  bool on;
  Timed(qv2_plan* plan, int kernel, hipStream_t st)
      : p(plan), k(kernel), s(st), on(plan->timing && (plan->time_only < 0 || plan->time_only == kernel)) {
    if (on) { (void)hipEventRecord(static_cast<hipEvent_t>(p->ev_start[k]), s); p->ev_used[k] = true; }
  }
  ~Timed() { if (on) (void)hipEventRecord(static_cast<hipEvent_t>(p->ev_stop[k]), s); }
};

int fold_grid(int n) { return (n + 3) / 4; }

// row-group tiles of a quantize pass, all forms; d_params_out != null: with calibration
template <bool PAIR, bool COS>
void launch_rows(qv2_plan* plan, const qv2_qparams* d_params, qv2_qparams* d_params_out, qv2_sums* d_sums,
                 typename ErrRec<COS>::type* parts, hipStream_t s) {
  const bool calib = d_params_out != nullptr;
  const int n_rows = static_cast<int>(plan->row_tiles.size());
  const int n_regs = static_cast<int>(plan->reg_tiles.size());
  const int n_wide = static_cast<int>(plan->wide_tiles.size());
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
                         plan->d_reg_tiles, d_params, d_params_out, d_sums,
                         static_cast<void*>(parts));
    else
      hipLaunchKernelGGL((k_rows_reg<kBlockRows, 1, PAIR, COS>), dim3(n_regs), dim3(kBlockRows), 0, s,
                         plan->d_reg_tiles, d_params, d_params_out, d_sums,
                         static_cast<void*>(parts));
  }
  if (n_wide > 0) {
    if (calib)
      hipLaunchKernelGGL((k_rows_reg<kBlockRowsWide, 2, PAIR, COS>), dim3(n_wide), dim3(kBlockRowsWide), 0, s,
                         plan->d_wide_tiles, d_params, d_params_out, d_sums,
                         static_cast<void*>(parts));
    else
      hipLaunchKernelGGL((k_rows_reg<kBlockRowsWide, 1, PAIR, COS>), dim3(n_wide), dim3(kBlockRowsWide), 0, s,
                         plan->d_wide_tiles, d_params, d_params_out, d_sums,
                         static_cast<void*>(parts));
  }
}

// the stream tiles of a quantize pass: those with a code buffer, then those without
template <bool PAIR, bool COS, bool X2>
void launch_quant_stream(qv2_plan* plan, int n_stream, int n_ro, const qv2_qparams* d_params,
                         typename StreamRec<PAIR, COS, X2>::type* parts, hipStream_t s) {
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
                  bool pair_in_stats = false, qv2_tensor_sums* d_ts = nullptr, ptrdiff_t mirror = 0) {
  typedef typename ErrRec<COS>::type P;
  typedef typename StreamRec<false, COS, false>::type SP;       // records of the sweep that keeps sum x^2
  const bool calib_rows = d_params_out != nullptr;
  const bool lean = calib_rows && (!PAIR || pair_in_stats);     // ... which is the sweep of this call
  // Where that sweep's records differ in size from the row-group tiles' (one double against
  // three) they start behind the rows' range of slots; slot numbers stay what the plan gave.
  SP* sparts = reinterpret_cast<SP*>(parts);
  if (sizeof(SP) != sizeof(P))
    sparts = reinterpret_cast<SP*>(reinterpret_cast<char*>(parts) + sizeof(P) * static_cast<size_t>(plan->n_row_parts)) -
             plan->n_row_parts;
  const int n_stream = static_cast<int>(plan->quant_tiles.n_tiles);
  const int n_ro = static_cast<int>(plan->quant_ro_tiles.n_tiles);
  const int n_rows = static_cast<int>(plan->row_tiles.size() + plan->reg_tiles.size() + plan->wide_tiles.size());
  if (n_stream + n_ro > 0) {
    // pair_in_stats: the calibration sweep already compared the stream tensors with their
    // partners, so the plain quantize kernel serves them
    Timed timed(plan, PAIR && !pair_in_stats ? QV2_K_QUANTPAIR_STREAM : QV2_K_QUANT_STREAM, s);
    if (PAIR && !pair_in_stats)
      launch_quant_stream<PAIR, COS, true>(plan, n_stream, n_ro, d_params, parts, s);
    else if (calib_rows)      // the calibration sweep of this same call already summed x^2
      launch_quant_stream<false, COS, false>(plan, n_stream, n_ro, d_params, sparts, s);
    else
      launch_quant_stream<false, COS, true>(plan, n_stream, n_ro, d_params, parts, s);
  }
  if (n_rows > 0) {
    Timed timed(plan, calib_rows ? QV2_K_SINGLE_READ_ROWS : PAIR ? QV2_K_QUANTPAIR_ROWS : QV2_K_QUANT_ROWS, s);
    // the pair form of the row kernels costs registers: only when a row tensor has a partner
    if (PAIR && plan->rows_have_pair)
      launch_rows<true, COS>(plan, d_params, d_params_out, d_sums, parts, s);
    else
      launch_rows<false, COS>(plan, d_params, d_params_out, d_sums, parts, s);
  }
  QuantFoldArgs<P> a{};
  a.segs = plan->d_segments; a.nseg = static_cast<int>(plan->segments.size());
  a.wide_segs = plan->d_big_err_segments; a.n_wide_segs = static_cast<int>(plan->big_err_segments.size());
  a.sums = d_sums; a.seg_xxhat = d_seg_xxhat; a.skip_below = calib_rows ? plan->n_row_parts : 0;
  a.keep_x2 = calib_rows && (!PAIR || pair_in_stats);
  a.parts = parts; a.sparts = lean ? static_cast<const void*>(sparts) : static_cast<const void*>(parts);
  a.seg_blocks = fold_blocks(a.n_wide_segs, a.nseg);
  int blocks = a.seg_blocks;
  if (d_pair_sums) {
    a.pt = plan->d_fused_pair_tensors; a.nt = static_cast<int>(plan->fused_pair_tensors.size());
    a.wide_pt = plan->d_big_fused_pair_tensors;
    a.n_wide_pt = static_cast<int>(plan->big_fused_pair_tensors.size());
    a.pair_out = d_pair_sums; a.pair_xq = d_pair_xq;
    a.pair_done = pair_in_stats ? plan->d_stat_pair_tensors : nullptr;
    a.pair_blocks = fold_blocks(a.n_wide_pt, a.nt);
    blocks += a.pair_blocks;
  }
  if (d_ts) {
    // the whole pass: this fold also leaves the per-tensor records.  The rows' segment records
    // are final by now (calib_rows), so the tensors made of them get one workgroup each here.
    a.ts = d_ts; a.params = d_params; a.ht = plan->d_hist_tensors; a.row_tensors = plan->d_row_tensors;
    a.mirror = mirror;
    blocks += static_cast<int>(plan->row_tensors.size());
  }
  if (lean) hipLaunchKernelGGL((k_fold_quant<P, SP>), dim3(blocks), dim3(kFoldBlock), 0, s, a);
  else hipLaunchKernelGGL((k_fold_quant<P, P>), dim3(blocks), dim3(kFoldBlock), 0, s, a);
  // tensors of several stream segments: their segment records were written by that very launch
  if (d_ts && !plan->late_tensors.empty())
    hipLaunchKernelGGL(k_tensor_fold, dim3(static_cast<int>(plan->late_tensors.size())), dim3(kFoldBlock), 0, s,
                       plan->d_hist_tensors, plan->d_late_tensors, d_params, d_sums, d_ts, mirror);
}

// calibration over the stream tiles (and the row-group tiles unless their own single-read
// kernel will calibrate them), then the statistics fold.  PAIR: the same sweep compares the
// stream tensors with their quantized-run partners and the fold writes their pair sums.
template <bool PAIR, bool COS = false>
void launch_stats(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums,
                  typename StatRec<PAIR, COS>::type* parts, bool with_rows, qv2_pair_sums* d_pair_sums,
                  double* d_pair_xq, hipStream_t s, ptrdiff_t mirror = 0) {
  typedef typename StatRec<PAIR, COS>::type REC;
  if (PAIR) with_rows = false;      // the row kernel of this pass writes 24-byte records: not in a PAIR sweep
  const int n_stream = static_cast<int>(plan->read_tiles.n_tiles);
  const int n_rows = static_cast<int>(plan->row_tiles.size());
  if (n_stream > 0) {
    Timed timed(plan, PAIR ? QV2_K_STATSPAIR_STREAM : QV2_K_STATS_STREAM, s);
    hipLaunchKernelGGL((k_stats_stream<kBlockRead, kVecRead, PAIR, COS>), dim3(n_stream), dim3(kBlockRead), 0, s,
                       plan->d_read_tiles, parts);
  }
  const int n_regs = static_cast<int>(plan->reg_tiles.size());
  const int n_wide = static_cast<int>(plan->wide_tiles.size());
  if (with_rows && n_rows + n_regs + n_wide > 0) {
    Timed timed(plan, QV2_K_STATS_ROWS, s);
    if (n_rows > 0)
      hipLaunchKernelGGL(k_stats_rows<kBlockRows>, dim3(n_rows), dim3(kBlockRows), 0, s,
                         plan->d_row_tiles, reinterpret_cast<StatPartial*>(parts));
    if (n_regs > 0)
      hipLaunchKernelGGL((k_rows_reg<kBlockRows, 0, false, false>), dim3(n_regs), dim3(kBlockRows), 0, s,
                         plan->d_reg_tiles, static_cast<const qv2_qparams*>(nullptr),
                         static_cast<qv2_qparams*>(nullptr), static_cast<qv2_sums*>(nullptr),
                         static_cast<void*>(parts));
    if (n_wide > 0)
      hipLaunchKernelGGL((k_rows_reg<kBlockRowsWide, 0, false, false>), dim3(n_wide), dim3(kBlockRowsWide), 0, s,
                         plan->d_wide_tiles, static_cast<const qv2_qparams*>(nullptr),
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
      a.pair_out = d_pair_sums; a.pair_xq = d_pair_xq; a.mirror = mirror;
      blocks += fold_blocks(a.n_wide_pt, a.nt);
    }
    hipLaunchKernelGGL(k_fold_stats<REC>, dim3(blocks), dim3(kFoldBlock), 0, s, a);
  }
}

// steps 1-3 of the single call, on a workspace of at least plan->workspace_bytes; d_ts != null
// (needs d_pair_sums): the per-tensor records as well, made inside the last fold
void single_call(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums, qv2_pair_sums* d_pair_sums,
                 void* d_workspace, hipStream_t s, qv2_tensor_sums* d_ts = nullptr, ptrdiff_t mirror = 0) {
  // stream tiles: statistics (with the pair comparison: that sweep only reads, and read-only
  // sweeps run nearest to the HBM rate), fold (parameters), then the plain quantize sweep;
  // row-group tiles: one kernel, after the statistics fold because the partial records share
  // the workspace
  ErrPartial3* parts = static_cast<ErrPartial3*>(d_workspace);
  if (d_pair_sums) {
    launch_stats<true>(plan, d_params, d_sums, static_cast<StatPairPartial*>(d_workspace), false, d_pair_sums,
                       nullptr, s, d_ts ? mirror : 0);
    launch_quant<true, false>(plan, d_params, d_sums, parts, nullptr, d_pair_sums, nullptr, s, d_params, true,
                              d_ts, d_ts ? mirror : 0);
  } else {
    launch_stats<false>(plan, d_params, d_sums, static_cast<StatPartial*>(d_workspace), false, nullptr, nullptr, s);
    launch_quant<false, false>(plan, d_params, d_sums, parts, nullptr, nullptr, nullptr, s, d_params);
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
  for (int k = 0; k < 2; ++k)
    if (plan->ev_done[k]) (void)hipEventDestroy(static_cast<hipEvent_t>(plan->ev_done[k]));
  delete plan;
}

qv2_status qv2_plan_upload(qv2_plan* plan, void* hip_stream) {
  if (!plan) return QV2_ERR_NULL;
  return upload(plan, static_cast<hipStream_t>(hip_stream));
}

size_t qv2_plan_device_bytes(const qv2_plan* plan) { return plan ? blob_bytes(plan) : 0; }

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

qv2_status qv2_plan_time_only(qv2_plan* plan, int32_t kernel) {
  if (!plan) return QV2_ERR_NULL;
  if (kernel < -1 || kernel >= QV2_K_COUNT) return QV2_ERR_SHAPE;
  plan->time_only = kernel;
  for (int k = 0; k < QV2_K_COUNT; ++k) plan->ev_used[k] = false;
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
  const int n_tiles = static_cast<int>(plan->pair_tiles.n_tiles);
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
  single_call(plan, d_params, d_sums, d_pair_sums, d_workspace, static_cast<hipStream_t>(hip_stream));
  return launch_status();
}

qv2_status qv2_calibrate_fakequant_pair_metrics_noalloc(qv2_plan* plan, qv2_qparams* d_params,
                                                        qv2_sums* d_sums, qv2_pair_sums* d_pair_sums,
                                                        void* hip_stream) {
  if (!plan || !d_params || !d_sums) return QV2_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(d_params) | reinterpret_cast<uintptr_t>(d_sums) |
       reinterpret_cast<uintptr_t>(d_pair_sums)) & 7u) return QV2_ERR_ALIGN;
  if (plan->workspace_bytes > kStaticScratchBytes) return QV2_ERR_WORKSPACE;
  // the tables must already be on this device: putting them there allocates
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return QV2_ERR_HIP; }
  if (!plan->d_blob) return QV2_ERR_STATE;
  if (dev != plan->device) return QV2_ERR_HIP;
  void* ws = scratch_on_device(dev);
  if (!ws) return QV2_ERR_HIP;
  // every partial record the folds read is written by this call's own sweeps first, so what the
  // previous call left in the array needs no clearing
  single_call(plan, d_params, d_sums, d_pair_sums, ws, static_cast<hipStream_t>(hip_stream));
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
  hipLaunchKernelGGL(k_tensor_fold, dim3(nt), dim3(kFoldBlock), 0, static_cast<hipStream_t>(hip_stream),
                     plan->d_hist_tensors, static_cast<const int*>(nullptr), d_params, d_sums, d_tensor_sums,
                     static_cast<ptrdiff_t>(0));
  return launch_status();
}

namespace {

// The device-side address of a host buffer when that buffer is pinned host memory the current
// device can write (hipHostMalloc), else null.  Asked anew at every call: an address that was
// pinned memory once may be something else by now.
const char* host_alias(void* h) {
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, h) != hipSuccess) {
    (void)hipGetLastError();                     // ordinary host memory is not known to the runtime
    return nullptr;
  }
  if (attr.type != hipMemoryTypeHost || !attr.devicePointer) return nullptr;
  return static_cast<const char*>(attr.devicePointer);
}

// device part of qv2_sensitivity_pass: the single call, the per-tensor fold and the copy of the
// per-tensor records to the host, all enqueued on hip_stream
qv2_status pass_enqueue(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums, void* d_records,
                        void* h_records, void* d_workspace, size_t workspace_bytes, void* hip_stream) {
  if (!plan || !d_records || !h_records) return QV2_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(d_records) | reinterpret_cast<uintptr_t>(h_records)) & 7u) return QV2_ERR_ALIGN;
  const size_t nt = plan->info.size();
  const size_t ts_bytes = nt * sizeof(qv2_tensor_sums);
  qv2_tensor_sums* d_ts = static_cast<qv2_tensor_sums*>(d_records);
  qv2_pair_sums* d_pair = reinterpret_cast<qv2_pair_sums*>(static_cast<char*>(d_records) + ts_bytes);
  qv2_status st = check_call(plan, d_params, d_sums, d_workspace, workspace_bytes);
  if (st != QV2_OK) return st;
  if ((st = ensure_uploaded(plan)) != QV2_OK) return st;
  // the single call; its last fold also makes the per-tensor records.  When h_records is pinned
  // host memory the device can address, the folds write every record there as well and no copy
  // follows; otherwise one copy brings them over.
  const char* alias = host_alias(h_records);
  const ptrdiff_t mirror = alias ? alias - static_cast<const char*>(d_records) : 0;
  single_call(plan, d_params, d_sums, d_pair, d_workspace, static_cast<hipStream_t>(hip_stream), d_ts, mirror);
  if ((st = launch_status()) != QV2_OK) return st;
  if (!mirror && hipMemcpyAsync(h_records, d_records, ts_bytes + nt * sizeof(qv2_pair_sums),
                                hipMemcpyDeviceToHost, static_cast<hipStream_t>(hip_stream)) != hipSuccess) {
    (void)hipGetLastError();
    return QV2_ERR_HIP;
  }
  return QV2_OK;
}

// host part: Eq. 6-7 for every tensor and pair, Eq. 16 and Algorithm 2, from records that have arrived
qv2_status pass_finish(const qv2_plan* plan, const void* h_records, const int32_t* layer_pos, int32_t n_layers,
                       const qv2_rank_config* cfg, qv2_metrics* h_metrics, double* h_pair_mse,
                       double* h_pair_sqnr_db, int32_t* order_out, double* score_out) {
  const int32_t nt = static_cast<int32_t>(plan->info.size());
  const qv2_tensor_sums* h_ts = static_cast<const qv2_tensor_sums*>(h_records);
  const qv2_pair_sums* h_pair = reinterpret_cast<const qv2_pair_sums*>(
      static_cast<const char*>(h_records) + static_cast<size_t>(nt) * sizeof(qv2_tensor_sums));
  bool finite = true;
  qv2_status st;
  if (h_metrics) {
    st = qv2_finalize_tensors(h_ts, nt, h_metrics);
    if (st == QV2_ERR_NONFINITE) finite = false; else if (st != QV2_OK) return st;
  }
  if (h_pair_mse && h_pair_sqnr_db) {
    st = qv2_pair_finalize(h_pair, nt, h_pair_mse, h_pair_sqnr_db);
    if (st == QV2_ERR_NONFINITE) finite = false; else if (st != QV2_OK) return st;
  }
  st = qv2_rank_tensors(plan, h_ts, h_pair, layer_pos, n_layers, cfg, order_out, score_out);
  if (st == QV2_ERR_NONFINITE) {
    // a NaN SQNR or a non-finite MSE in a series the ranking needs: no list can be made.  The
    // outputs still hold something defined - layer order and NaN scores.
    for (int32_t i = 0; i < n_layers; ++i) {
      order_out[i] = i;
      if (score_out) score_out[i] = std::numeric_limits<double>::quiet_NaN();
    }
  }
  if (st != QV2_OK) return st;
  return finite ? QV2_OK : QV2_ERR_NONFINITE;
}

}  // namespace

qv2_status qv2_sensitivity_pass(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums, void* d_records,
                                void* h_records, void* d_workspace, size_t workspace_bytes, void* hip_stream,
                                const int32_t* layer_pos, int32_t n_layers, const qv2_rank_config* cfg,
                                qv2_metrics* h_metrics, double* h_pair_mse, double* h_pair_sqnr_db,
                                int32_t* order_out, double* score_out) {
  if (!plan || !d_records || !h_records || !order_out) return QV2_ERR_NULL;
  if ((h_pair_mse == nullptr) != (h_pair_sqnr_db == nullptr)) return QV2_ERR_NULL;   // the two come together
  if (n_layers <= 0) return QV2_ERR_SHAPE;
  qv2_status st = pass_enqueue(plan, d_params, d_sums, d_records, h_records, d_workspace, workspace_bytes,
                               hip_stream);
  if (st != QV2_OK) return st;
  if (hipStreamSynchronize(static_cast<hipStream_t>(hip_stream)) != hipSuccess) {
    (void)hipGetLastError();
    return QV2_ERR_HIP;
  }
  return pass_finish(plan, h_records, layer_pos, n_layers, cfg, h_metrics, h_pair_mse, h_pair_sqnr_db,
                     order_out, score_out);
}

qv2_status qv2_sensitivity_pass_begin(qv2_plan* plan, qv2_qparams* d_params, qv2_sums* d_sums, void* d_records,
                                      void* h_records, void* d_workspace, size_t workspace_bytes,
                                      void* hip_stream, int32_t slot) {
  if (!plan) return QV2_ERR_NULL;
  if (slot < 0 || slot > 1) return QV2_ERR_SHAPE;
  if (!plan->ev_done[slot]) {
    hipEvent_t ev;
    if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); return QV2_ERR_HIP; }
    plan->ev_done[slot] = ev;
  }
  qv2_status st = pass_enqueue(plan, d_params, d_sums, d_records, h_records, d_workspace, workspace_bytes,
                               hip_stream);
  if (st != QV2_OK) return st;
  if (hipEventRecord(static_cast<hipEvent_t>(plan->ev_done[slot]), static_cast<hipStream_t>(hip_stream)) !=
      hipSuccess) {
    (void)hipGetLastError();
    return QV2_ERR_HIP;
  }
  return QV2_OK;
}

qv2_status qv2_sensitivity_pass_end(qv2_plan* plan, const void* h_records, int32_t slot, const int32_t* layer_pos,
                                    int32_t n_layers, const qv2_rank_config* cfg, qv2_metrics* h_metrics,
                                    double* h_pair_mse, double* h_pair_sqnr_db, int32_t* order_out,
                                    double* score_out) {
  if (!plan || !h_records || !order_out) return QV2_ERR_NULL;
  if ((h_pair_mse == nullptr) != (h_pair_sqnr_db == nullptr)) return QV2_ERR_NULL;
  if (slot < 0 || slot > 1 || n_layers <= 0) return QV2_ERR_SHAPE;
  if (reinterpret_cast<uintptr_t>(h_records) & 7u) return QV2_ERR_ALIGN;
  if (!plan->ev_done[slot]) return QV2_ERR_STATE;              // no pass was begun in this slot
  if (hipEventSynchronize(static_cast<hipEvent_t>(plan->ev_done[slot])) != hipSuccess) {
    (void)hipGetLastError();
    return QV2_ERR_HIP;
  }
  return pass_finish(plan, h_records, layer_pos, n_layers, cfg, h_metrics, h_pair_mse, h_pair_sqnr_db,
                     order_out, score_out);
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
