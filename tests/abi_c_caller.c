/*
 * A caller of the qv2 C ABI in plain C99: the header compiles as C, and the whole
 * sensitivity pass (Sec. 4 steps 1-4) runs with nothing but the HIP runtime's C API for
 * device memory - no Python, no torch.
 *
 *   abi_c_caller host           host-only entry points (needs no GPU); prints "host ok"
 *   abi_c_caller gpu <outfile>  one pass over a 4-tensor table on device 0; writes the
 *                               records and codes to <outfile> for the test to compare
 *                               with the CPU oracle on the same generated inputs
 *
 * Inputs come from a counter-based generator (splitmix64 of the element index) that the
 * test repeats in numpy; it holds none of the method's arithmetic.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "qv2.h"

/* the records cross the ABI as plain memory: their sizes are part of the contract */
typedef char size_qparams[sizeof(qv2_qparams) == 24 ? 1 : -1];
typedef char size_sums[sizeof(qv2_sums) == 32 ? 1 : -1];
typedef char size_pair[sizeof(qv2_pair_sums) == 32 ? 1 : -1];
typedef char size_tsums[sizeof(qv2_tensor_sums) == 48 ? 1 : -1];
typedef char size_metrics[sizeof(qv2_metrics) == 48 ? 1 : -1];
typedef char size_tensor[sizeof(qv2_tensor) == 48 ? 1 : -1];

#define REQUIRE(cond)                                                        \
  do {                                                                       \
    if (!(cond)) {                                                           \
      fprintf(stderr, "%s:%d: failed: %s\n", __FILE__, __LINE__, #cond);     \
      return 1;                                                              \
    }                                                                        \
  } while (0)

static uint64_t mix(uint64_t i, uint64_t seed) {
  uint64_t z = (i + 1u) * 0x9E3779B97F4A7C15ull + seed;
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  z ^= z >> 31;
  return z;
}
/* 24 random bits -> [0, 1), exact in fp32 */
static float unit(uint64_t i, uint64_t seed) { return (float)(mix(i, seed) >> 40) * (1.0f / 16777216.0f); }

typedef struct { int64_t numel; int32_t channels, scheme, kind, layer; uint64_t seed; } spec;

static const spec kTable[4] = {
  {64 * 147, 64, QV2_SYM_CHANNEL, 0, 0, 11},     /* conv weight, rows of 147 (not a multiple of 4) */
  {200707, 1, QV2_ASYM_TENSOR, 1, 0, 12},        /* post-ReLU activation with a ragged tail        */
  {32 * 512, 32, QV2_SYM_CHANNEL, 0, 1, 13},     /* weight with rows of 512                        */
  {50001, 1, QV2_ASYM_TENSOR, 1, 1, 14},         /* second activation                              */
};

static void fill(const spec* s, float* x, float* q) {
  for (int64_t i = 0; i < s->numel; ++i) {
    float v = (unit((uint64_t)i, s->seed) - 0.25f) * 3.0f;
    if (s->kind == 1 && v < 0.0f) v = 0.0f;
    x[i] = v;
    if (q) q[i] = v + (unit((uint64_t)i, s->seed + 100) - 0.5f) * 0.03125f;
  }
}

static int host_mode(void) {
  qv2_plan* plan = NULL;
  qv2_tensor rows[2];
  memset(rows, 0, sizeof rows);
  rows[0].x = (const float*)(uintptr_t)0x10000; rows[0].numel = 1000; rows[0].channels = 1;
  rows[0].scheme = QV2_ASYM_TENSOR;
  rows[1].x = (const float*)(uintptr_t)0x20000; rows[1].numel = 64 * 9; rows[1].channels = 64;
  rows[1].scheme = QV2_SYM_CHANNEL; rows[1].layer = 1;
  REQUIRE(qv2_plan_create(rows, 2, &plan) == QV2_OK && plan);
  REQUIRE(qv2_plan_num_tensors(plan) == 2 && qv2_plan_num_segments(plan) == 65);
  REQUIRE(qv2_workspace_bytes(plan) >= 256);
  REQUIRE(qv2_calibrate(plan, NULL, NULL, NULL, 0, NULL) == QV2_ERR_NULL);
  qv2_plan_destroy(plan);
  REQUIRE(qv2_plan_create(rows, 0, &plan) == QV2_ERR_SHAPE && plan == NULL);

  /* Eq. 16 + Algorithm 2 on an 8-layer example.  Deltas 0 -2 3 -11 5 1 -3 6, scores 0.6 x those;
     layer 2's MSE of 30 is above 5 x the mean 4.625, so it leads; the rest ascend by score. */
  const double w_sqnr[8] = {40.0, 38.0, 41.0, 30.0, 35.0, 36.0, 33.0, 39.0};
  const double w_mse[8] = {1.0, 1.0, 30.0, 1.0, 1.0, 1.0, 1.0, 1.0};
  const int32_t expect[8] = {2, 3, 6, 1, 0, 5, 4, 7};
  qv2_rank_config cfg;
  qv2_rank_config_default(&cfg);
  cfg.mse_source = 1;
  int32_t order[8];
  double score[8];
  REQUIRE(qv2_rank(w_sqnr, NULL, w_mse, NULL, NULL, 8, &cfg, order, score) == QV2_OK);
  REQUIRE(memcmp(order, expect, sizeof expect) == 0);
  REQUIRE(score[0] == 0.0 && score[3] < score[6] && score[7] > score[4]);

  /* Eq. 17: everything int8 saves 75 % */
  const double macs[3] = {1e6, 2e6, 3e6};
  const uint8_t none[3] = {0, 0, 0};
  double pct = 0.0;
  REQUIRE(qv2_bops_reduction_pct(macs, none, 3, &pct) == QV2_OK && pct == 75.0);
  REQUIRE(strcmp(qv2_status_string(QV2_OK), "ok") == 0);
  puts("host ok");
  return 0;
}

#define HIP(call) REQUIRE((call) == hipSuccess)
#define QV2(call) REQUIRE((call) == QV2_OK)

static int gpu_mode(const char* path) {
  enum { NT = 4, NL = 2 };
  float *hx[NT], *hq[NT], *dx[NT], *dq[NT];
  int8_t* dc[NT];
  qv2_tensor rows[NT];
  HIP(hipSetDevice(0));
  for (int t = 0; t < NT; ++t) {
    const spec* s = &kTable[t];
    const size_t bytes = (size_t)s->numel * sizeof(float);
    hx[t] = (float*)malloc(bytes);
    hq[t] = s->kind == 1 ? (float*)malloc(bytes) : NULL;
    REQUIRE(hx[t] && (s->kind == 0 || hq[t]));
    fill(s, hx[t], hq[t]);
    HIP(hipMalloc((void**)&dx[t], bytes));
    HIP(hipMemcpy(dx[t], hx[t], bytes, hipMemcpyHostToDevice));
    dq[t] = NULL;
    if (hq[t]) {
      HIP(hipMalloc((void**)&dq[t], bytes));
      HIP(hipMemcpy(dq[t], hq[t], bytes, hipMemcpyHostToDevice));
    }
    HIP(hipMalloc((void**)&dc[t], (size_t)s->numel));
    memset(&rows[t], 0, sizeof rows[t]);
    rows[t].x = dx[t]; rows[t].qrun = dq[t]; rows[t].codes = dc[t];
    rows[t].numel = s->numel; rows[t].channels = s->channels; rows[t].scheme = s->scheme;
    rows[t].kind = s->kind; rows[t].layer = s->layer;
  }
  qv2_plan* plan = NULL;
  QV2(qv2_plan_create(rows, NT, &plan));
  const int64_t nseg = qv2_plan_num_segments(plan);
  const size_t ws_bytes = qv2_workspace_bytes(plan);
  qv2_qparams* d_params; qv2_sums* d_sums; qv2_pair_sums* d_pair; qv2_tensor_sums* d_ts; void* d_ws;
  HIP(hipMalloc((void**)&d_params, (size_t)nseg * sizeof(qv2_qparams)));
  HIP(hipMalloc((void**)&d_sums, (size_t)nseg * sizeof(qv2_sums)));
  HIP(hipMalloc((void**)&d_pair, NT * sizeof(qv2_pair_sums)));
  HIP(hipMalloc((void**)&d_ts, NT * sizeof(qv2_tensor_sums)));
  HIP(hipMalloc(&d_ws, ws_bytes));
  hipStream_t stream;
  HIP(hipStreamCreate(&stream));
  /* set-up: the plan's tables go to the device now instead of inside the first device call */
  REQUIRE(qv2_plan_device_bytes(plan) >= 256);
  QV2(qv2_plan_upload(plan, stream));
  QV2(qv2_plan_upload(plan, stream));          /* already there: left alone */

  /* steps 1-3 in one call, per-tensor records folded on the device */
  QV2(qv2_calibrate_fakequant_pair_metrics(plan, d_params, d_sums, d_pair, d_ws, ws_bytes, stream));
  QV2(qv2_tensor_sums_fold(plan, d_params, d_sums, d_ts, stream));
  HIP(hipStreamSynchronize(stream));

  qv2_qparams* params = (qv2_qparams*)malloc((size_t)nseg * sizeof(qv2_qparams));
  qv2_sums* sums = (qv2_sums*)malloc((size_t)nseg * sizeof(qv2_sums));
  qv2_pair_sums pair[NT];
  qv2_tensor_sums ts[NT];
  REQUIRE(params && sums);
  HIP(hipMemcpy(params, d_params, (size_t)nseg * sizeof(qv2_qparams), hipMemcpyDeviceToHost));
  HIP(hipMemcpy(sums, d_sums, (size_t)nseg * sizeof(qv2_sums), hipMemcpyDeviceToHost));
  HIP(hipMemcpy(pair, d_pair, sizeof pair, hipMemcpyDeviceToHost));
  HIP(hipMemcpy(ts, d_ts, sizeof ts, hipMemcpyDeviceToHost));

  /* step 3 (Eq. 6-7) and step 4 (Eq. 16, Algorithm 2) on the host */
  qv2_metrics met[NT];
  double pmse[NT], psqnr[NT], score[NL];
  int32_t order[NL];
  QV2(qv2_finalize_tensors(ts, NT, met));
  QV2(qv2_pair_finalize(pair, NT, pmse, psqnr));
  QV2(qv2_rank_tensors(plan, ts, pair, NULL, NL, NULL, order, score));

  FILE* f = fopen(path, "wb");
  REQUIRE(f);
  const int64_t head[2] = {nseg, NT};
  REQUIRE(fwrite(head, sizeof head, 1, f) == 1);
  REQUIRE(fwrite(params, sizeof(qv2_qparams), (size_t)nseg, f) == (size_t)nseg);
  REQUIRE(fwrite(sums, sizeof(qv2_sums), (size_t)nseg, f) == (size_t)nseg);
  REQUIRE(fwrite(pair, sizeof pair, 1, f) == 1);
  REQUIRE(fwrite(met, sizeof met, 1, f) == 1);
  REQUIRE(fwrite(pmse, sizeof pmse, 1, f) == 1);
  REQUIRE(fwrite(psqnr, sizeof psqnr, 1, f) == 1);
  REQUIRE(fwrite(order, sizeof order, 1, f) == 1);
  REQUIRE(fwrite(score, sizeof score, 1, f) == 1);
  for (int t = 0; t < NT; ++t) {
    int8_t* codes = (int8_t*)malloc((size_t)kTable[t].numel);
    REQUIRE(codes);
    HIP(hipMemcpy(codes, dc[t], (size_t)kTable[t].numel, hipMemcpyDeviceToHost));
    REQUIRE(fwrite(codes, 1, (size_t)kTable[t].numel, f) == (size_t)kTable[t].numel);
    free(codes);
  }
  REQUIRE(fclose(f) == 0);

  /* the same again as ONE host call (it waits for the stream itself): same parameters, same list */
  {
    const size_t rec_bytes = NT * (sizeof(qv2_tensor_sums) + sizeof(qv2_pair_sums));
    void *d_rec, *h_rec = malloc(rec_bytes);
    qv2_qparams* params2 = (qv2_qparams*)malloc((size_t)nseg * sizeof(qv2_qparams));
    qv2_metrics met2[NT];
    double pmse2[NT], psqnr2[NT], score2[NL];
    int32_t order2[NL];
    REQUIRE(h_rec && params2);
    HIP(hipMalloc(&d_rec, rec_bytes));
    HIP(hipMemset(d_params, 0, (size_t)nseg * sizeof(qv2_qparams)));
    QV2(qv2_sensitivity_pass(plan, d_params, d_sums, d_rec, h_rec, d_ws, ws_bytes, stream, NULL, NL, NULL, met2,
                             pmse2, psqnr2, order2, score2));
    HIP(hipMemcpy(params2, d_params, (size_t)nseg * sizeof(qv2_qparams), hipMemcpyDeviceToHost));
    REQUIRE(memcmp(params2, params, (size_t)nseg * sizeof(qv2_qparams)) == 0);
    REQUIRE(memcmp(order2, order, sizeof order) == 0);
    for (int t = 0; t < NT; ++t) {
      REQUIRE(met2[t].min == met[t].min && met2[t].max == met[t].max);
      REQUIRE(met2[t].mse == met[t].mse && pmse2[t] == pmse[t]);   /* same kernels, same order of sums */
    }
    HIP(hipFree(d_rec));
    free(h_rec); free(params2);
  }

  qv2_plan_destroy(plan);
  HIP(hipStreamDestroy(stream));
  for (int t = 0; t < NT; ++t) {
    HIP(hipFree(dx[t])); HIP(hipFree(dc[t]));
    if (dq[t]) HIP(hipFree(dq[t]));
    free(hx[t]); free(hq[t]);
  }
  HIP(hipFree(d_params)); HIP(hipFree(d_sums)); HIP(hipFree(d_pair)); HIP(hipFree(d_ts)); HIP(hipFree(d_ws));
  free(params); free(sums);
  printf("gpu ok: %lld segments, order %d %d\n", (long long)nseg, order[0], order[1]);
  return 0;
}

int main(int argc, char** argv) {
  if (argc == 2 && strcmp(argv[1], "host") == 0) return host_mode();
  if (argc == 3 && strcmp(argv[1], "gpu") == 0) return gpu_mode(argv[2]);
  fprintf(stderr, "usage: %s host | gpu <outfile>\n", argv[0]);
  return 2;
}
