// qoda_probe: a torch-free driver of libqoda's C ABI for profilers and hardware counters.
//
//   qoda_probe <sizes.txt> <K> <S> <rounds> [adaptive=1] [copy_mib=1024] [time_classes=0xFFFFFFFF] [q_hat=0]
//              [norm_scope=0] [norm_kind=2]
//
// sizes.txt holds one layer size per line (python -m paper_2505_14371_amd.workloads <name> writes it).  The
// probe fills K gradient buffers with heavy-tailed synthetic values (one scale per layer), runs `rounds` rounds
// of fit -> quantize all nodes -> fused step, prints the per-kernel event timings, and finishes with three
// launches of the plain copy kernel over copy_mib MiB (the known-traffic kernel counters are scaled by).
// It is a measurement aid: it computes nothing of the method itself.

#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "../../include/qoda.h"

#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); return 1; } } while (0)
#define QK(x) do { int r_ = (x); if (r_ != QODA_OK) { fprintf(stderr, "%s -> %d: %s\n", #x, r_, qoda_last_error(ctx)); return 1; } } while (0)

__device__ inline uint32_t mix32(uint32_t x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}

// Student-t(3)-like values: z0 / sqrt((z1^2+z2^2+z3^2)/3), Box-Muller normals from hashed counters.
__global__ void fill_layer(float *p, long long n, float scale, uint32_t salt) {
  long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (; i < n; i += stride) {
    const uint32_t b = mix32((uint32_t)i * 4u + salt) ^ mix32((uint32_t)(i >> 30) + 0x9e3779b9u * salt);
    const float u0 = (mix32(b + 1u) + 0.5f) * 2.3283064e-10f, u1 = (mix32(b + 2u) + 0.5f) * 2.3283064e-10f;
    const float u2 = (mix32(b + 3u) + 0.5f) * 2.3283064e-10f, u3 = (mix32(b + 4u) + 0.5f) * 2.3283064e-10f;
    const float r0 = sqrtf(-2.0f * logf(u0)), r1 = sqrtf(-2.0f * logf(u2));
    const float z0 = r0 * cosf(6.2831853f * u1), z1 = r0 * sinf(6.2831853f * u1);
    const float z2 = r1 * cosf(6.2831853f * u3), z3 = r1 * sinf(6.2831853f * u3);
    p[i] = scale * z0 / sqrtf((z1 * z1 + z2 * z2 + z3 * z3) / 3.0f + 1e-12f);
  }
}

int main(int argc, char **argv) {
  if (argc < 5) { fprintf(stderr, "usage: %s sizes.txt K S rounds [adaptive=1] [copy_mib=1024] [time_classes=0xFFFFFFFF] [q_hat=0] [norm_scope=0] [norm_kind=2]\n", argv[0]); return 2; }
  std::vector<int64_t> sizes;
  FILE *f = fopen(argv[1], "r");
  if (!f) { perror(argv[1]); return 2; }
  long long v;
  while (fscanf(f, "%lld", &v) == 1) sizes.push_back(v);
  fclose(f);
  const int L = (int)sizes.size(), K = atoi(argv[2]), S = atoi(argv[3]), rounds = atoi(argv[4]);
  const bool adaptive = argc > 5 ? atoi(argv[5]) != 0 : true;
  const size_t copy_bytes = (size_t)(argc > 6 ? atoll(argv[6]) : 1024) << 20;
  const uint32_t time_classes = argc > 7 ? (uint32_t)strtoul(argv[7], nullptr, 0) : 0xFFFFFFFFu;
  const int scope = argc > 9 ? atoi(argv[9]) : QODA_SCOPE_LAYER;   // what one norm covers
  const int kind = argc > 10 ? atoi(argv[10]) : QODA_NORM_L2;   // the q of the normalisation (0: infinity)
  const double q_hat = argc > 8 ? atof(argv[8]) : 0.0;   // > 0: the step sizes of eq. (Alt) instead of the main rule
  if (L < 1 || K < 1 || S < 2 || rounds < 1) { fprintf(stderr, "bad arguments\n"); return 2; }

  std::vector<int32_t> types(L), points(L, S);
  std::vector<int64_t> off(L);
  int64_t total = 0, d = 0;
  for (int l = 0; l < L; ++l) { types[l] = l; off[l] = total; total += (sizes[l] + 63) / 64 * 64; d += sizes[l]; }
  if (total == 0) total = 64;
  qoda_config cfg = {L, sizes.data(), types.data(), L, points.data(), K, kind, 12345u, scope};
  qoda_ctx *ctx = nullptr;
  if (qoda_create(&cfg, &ctx) != QODA_OK) { fprintf(stderr, "qoda_create failed\n"); return 1; }
  const size_t mbytes = qoda_message_bytes(ctx);

  std::vector<float *> grad(K);
  std::vector<void *> msg(2 * K);
  float *x1, *y, *xh;
  double *acc;
  for (int k = 0; k < K; ++k) CK(hipMalloc(&grad[k], total * sizeof(float)));
  for (int i = 0; i < 2 * K; ++i) { CK(hipMalloc(&msg[i], mbytes)); CK(hipMemset(msg[i], 0, mbytes)); }
  CK(hipMalloc(&x1, total * sizeof(float)));
  CK(hipMalloc(&y, total * sizeof(float)));
  CK(hipMalloc(&xh, total * sizeof(float)));
  CK(hipMalloc(&acc, sizeof(double)));
  CK(hipMemset(y, 0, total * sizeof(float)));
  CK(hipMemset(xh, 0, total * sizeof(float)));
  CK(hipMemset(acc, 0, sizeof(double)));
  hipLaunchKernelGGL(fill_layer, dim3(4096), dim3(256), 0, 0, x1, (long long)total, 1.0f, 7u);
  for (int k = 0; k < K; ++k) {
    CK(hipMemset(grad[k], 0, total * sizeof(float)));
    for (int l = 0; l < L; ++l) {
      if (!sizes[l]) continue;
      const float scale = 1e-5f * powf(1000.0f, (float)((l * 2654435761u) % 1000u) / 1000.0f);
      const int blocks = (int)((sizes[l] + 1023) / 1024 < 4096 ? (sizes[l] + 1023) / 1024 : 4096);
      hipLaunchKernelGGL(fill_layer, dim3(blocks), dim3(256), 0, 0, grad[k] + off[l], (long long)sizes[l], scale,
                         (uint32_t)(1000003u * k + 31u * l + 1u));
    }
  }
  CK(hipDeviceSynchronize());

  std::vector<const float *> gp((size_t)K * L);
  std::vector<const float *> x1p(L);
  std::vector<float *> yp(L), xhp(L);
  for (int l = 0; l < L; ++l) {
    for (int k = 0; k < K; ++k) gp[(size_t)k * L + l] = grad[k] + off[l];
    x1p[l] = x1 + off[l]; yp[l] = y + off[l]; xhp[l] = xh + off[l];
  }
  qoda_state st = {x1p.data(), yp.data(), xhp.data(), nullptr, acc, nullptr};
  double *alt_sums;
  float *alt_eta;
  const float ones[2] = {1.0f, 1.0f};
  CK(hipMalloc(&alt_sums, 2 * sizeof(double)));
  CK(hipMalloc(&alt_eta, 2 * sizeof(float)));
  CK(hipMemset(alt_sums, 0, 2 * sizeof(double)));
  CK(hipMemcpy(alt_eta, ones, sizeof ones, hipMemcpyHostToDevice));
  qoda_alt_state ast = {x1p.data(), yp.data(), xhp.data(), nullptr, alt_sums, alt_eta};
  QK(qoda_profile_enable(ctx, time_classes));
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0));
  CK(hipEventCreate(&e1));
  float ms_total = 0.0f;
  auto one_round = [&](int t) -> int {
    const int cur = t & 1;
    // bucket scope: after the first round the fit uses the statistics gathered by the previous quantize pass
    if (adaptive) {
      if (scope == QODA_SCOPE_BUCKET && t > 1) QK(qoda_fit_levels(ctx, nullptr, (uint32_t)t, nullptr));
      else QK(qoda_fit_levels_keep_norms(ctx, gp.data(), (uint32_t)t, nullptr));   // the round's own vectors
    }
    QK(qoda_quantize_all(ctx, gp.data(), (uint32_t)t, msg.data() + cur * K,
                         (t > 1 && q_hat <= 0.0) ? (const void *const *)(msg.data() + (1 - cur) * K) : nullptr, nullptr));
    if (q_hat > 0.0) QK(qoda_step_alt(ctx, (const void *const *)(msg.data() + cur * K), &ast, q_hat, nullptr));
    else QK(qoda_step(ctx, (const void *const *)(msg.data() + cur * K), &st, nullptr));
    return 0;
  };
  for (int t = 1; t <= rounds + 1; ++t) {            // round 1 is a warm-up and is not reported
    if (t == 2) {
      double ms[QODA_NUM_KERNELS]; int64_t n[QODA_NUM_KERNELS];
      QK(qoda_profile_read(ctx, ms, n, nullptr));
      CK(hipEventRecord(e0, 0));
    }
    if (one_round(t)) return 1;
  }
  CK(hipEventRecord(e1, 0));
  CK(hipEventSynchronize(e1));
  CK(hipEventElapsedTime(&ms_total, e0, e1));
  double ms[QODA_NUM_KERNELS]; int64_t n[QODA_NUM_KERNELS];
  QK(qoda_profile_read(ctx, ms, n, nullptr));
  printf("workload: L=%d d=%lld K=%d S=%d adaptive=%d q_hat=%g norm_scope=%d norm_kind=%d message_bytes=%zu\n", L,
         (long long)d, K, S, (int)adaptive, q_hat, scope, kind, mbytes);
  printf("rounds=%d ms_per_round=%.4f fp32_gradient_GBps=%.1f\n", rounds, ms_total / rounds,
         4.0 * K * (double)d / (ms_total / rounds * 1e-3) / 1e9);
  for (int i = 0; i < QODA_NUM_KERNELS; ++i)
    if (n[i]) printf("  %-18s launches=%lld avg_ms=%.4f\n", qoda_kernel_name(i), (long long)n[i], ms[i] / n[i]);
  if (time_classes != 0u) {   // the same rounds once more with no launch bracketed by events
    float ms_plain = 0.0f;
    QK(qoda_profile_enable(ctx, 0u));
    CK(hipEventRecord(e0, 0));
    for (int t = rounds + 2; t <= 2 * rounds + 1; ++t)
      if (one_round(t)) return 1;
    CK(hipEventRecord(e1, 0));
    CK(hipEventSynchronize(e1));
    CK(hipEventElapsedTime(&ms_plain, e0, e1));
    printf("rounds=%d ms_per_round_without_kernel_events=%.4f fp32_gradient_GBps=%.1f\n", rounds, ms_plain / rounds,
           4.0 * K * (double)d / (ms_plain / rounds * 1e-3) / 1e9);
  }
  const int status = qoda_status(ctx, nullptr);
  printf("status=%d\n", status);

  QK(qoda_profile_enable(ctx, 0xFFFFFFFFu));
  size_t cb = copy_bytes;
  if (cb > (size_t)total * 4) cb = (size_t)total * 4 / 16 * 16;
  for (int i = 0; i < 3; ++i) QK(qoda_copy_calibration(ctx, y, xh, cb, nullptr));
  QK(qoda_profile_read(ctx, ms, n, nullptr));
  for (int i = 0; i < QODA_NUM_KERNELS; ++i)
    if (n[i]) printf("  %-18s launches=%lld avg_ms=%.4f bytes_read=%zu bytes_written=%zu\n", qoda_kernel_name(i),
                     (long long)n[i], ms[i] / n[i], cb, cb);
  qoda_destroy(ctx);
  return status == QODA_OK ? 0 : 1;
}
