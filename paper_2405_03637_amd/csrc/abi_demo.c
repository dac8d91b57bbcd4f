/* A consumer of the C ABI written in plain C99: no C++, no Python, no torch.  It allocates device buffers
 * with the HIP runtime, fills them with seeded bit patterns, runs Collage steps over two tensors through
 * mcf_plan_create / mcf_adamw_step (the last one with the fused EDQ, Def. 3.3), repoints the plan at a
 * second set of gradient buffers with mcf_plan_update on the way, and writes the final state to a file.
 * The GPU test suite runs it and compares the file with the oracle's result for the same inputs.
 *
 *   mcf_abi_demo OUT VARIANT N0 N1 STEPS
 *
 * Inputs: element i of stream s at step t is pattern(seed(s, t), i) below: a bf16 with a random sign,
 * significand and an exponent field in [lo, lo + span).
 * File layout: theta, dtheta, m, v (and dv for the plus variant), each N0 + N1 uint16_t, tensor 0 first,
 * then the four doubles {EDQ, S1, S2, lost} of the last step.                                            */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../include/mcf.h"

static uint64_t mix(uint64_t x) {
  x += 0x9E3779B97F4A7C15ull;
  x = (x ^ (x >> 30)) * 0xBF58476D1CE4E5B9ull;
  x = (x ^ (x >> 27)) * 0x94D049BB133111EBull;
  return x ^ (x >> 31);
}

static uint16_t pattern(uint64_t seed, uint64_t i, unsigned lo, unsigned span) {
  const uint64_t h = mix(seed * 0x100000001B3ull + i);
  const unsigned sign = (unsigned)(h >> 63), expo = lo + (unsigned)((h >> 32) % span), mant = (unsigned)(h & 0x7f);
  return (uint16_t)((sign << 15) | (expo << 7) | mant);
}

#define CHECK_HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_MCF(call) do { int r_ = (call); if (r_ != MCF_OK) { fprintf(stderr, "%s: %s\n", #call, mcf_status_string(r_)); return 3; } } while (0)

enum { TH, DTH, M, V, DV, G0, G1, STREAMS };

int main(int argc, char **argv) {
  if (argc != 6) { fprintf(stderr, "usage: %s OUT VARIANT N0 N1 STEPS\n", argv[0]); return 1; }
  const int variant = atoi(argv[2]);
  const uint64_t n[2] = {strtoull(argv[3], 0, 10), strtoull(argv[4], 0, 10)};
  const int steps = atoi(argv[5]);
  const uint64_t total = n[0] + n[1];
  const int plus = (variant & 0xff) == MCF_PLUS;
  /* every stream: one device buffer holding tensor 0, then tensor 1 right behind it (so tensor 1 starts
   * wherever N0 puts it: odd element offsets exercise the unaligned path), 3 elements into the allocation */
  const uint64_t lead = 3;
  uint16_t *dev[STREAMS];
  uint16_t *host = (uint16_t *)malloc(total * sizeof(uint16_t));
  if (!host) return 1;
  for (int s = 0; s < STREAMS; ++s) {
    CHECK_HIP(hipMalloc((void **)&dev[s], (total + lead) * sizeof(uint16_t)));
    CHECK_HIP(hipMemset(dev[s], 0, (total + lead) * sizeof(uint16_t)));
    dev[s] += lead;
  }
  for (uint64_t i = 0; i < total; ++i) host[i] = pattern(1, i, 118, 10);          /* theta: 2^-9 .. 2^0 */
  CHECK_HIP(hipMemcpy(dev[TH], host, total * 2, hipMemcpyHostToDevice));

  mcf_tensor t[2];
  for (int k = 0; k < 2; ++k) {
    const uint64_t o = k ? n[0] : 0;
    t[k].theta = dev[TH] + o; t[k].dtheta = dev[DTH] + o; t[k].m = dev[M] + o; t[k].v = dev[V] + o;
    t[k].dv = plus ? dev[DV] + o : NULL; t[k].grad = dev[G0] + o; t[k].n = n[k];
  }
  mcf_plan *plan = NULL;
  CHECK_MCF(mcf_plan_create(&plan, t, 2, variant));
  if (mcf_plan_params(plan) != total) { fprintf(stderr, "plan reports %llu parameters\n", (unsigned long long)mcf_plan_params(plan)); return 4; }
  hipStream_t stream;
  CHECK_HIP(hipStreamCreate(&stream));
  double *edq_dev;
  CHECK_HIP(hipMalloc((void **)&edq_dev, 4 * sizeof(double)));
  const mcf_hyper hyper = {1e-3, 0.9, 0.95, 1e-8, 0.1};
  for (int step = 1; step <= steps; ++step) {
    /* gradients alternate between two buffers, as they would if the caller's framework moved them */
    uint16_t *g = dev[(step & 1) ? G0 : G1];
    for (uint64_t i = 0; i < total; ++i) host[i] = pattern(100 + (uint64_t)step, i, 110, 12);   /* 2^-17 .. 2^-6 */
    CHECK_HIP(hipMemcpyAsync(g, host, total * 2, hipMemcpyHostToDevice, stream));
    CHECK_HIP(hipStreamSynchronize(stream));               /* host[] is reused next step */
    t[0].grad = g; t[1].grad = g + n[0];
    CHECK_MCF(mcf_plan_update(plan, t, 2, stream));
    CHECK_MCF(mcf_adamw_step(plan, &hyper, (uint64_t)step, stream, step == steps ? edq_dev : NULL));
  }
  CHECK_HIP(hipStreamSynchronize(stream));

  FILE *f = fopen(argv[1], "wb");
  if (!f) { perror(argv[1]); return 1; }
  const int outs[5] = {TH, DTH, M, V, DV};
  for (int k = 0; k < (plus ? 5 : 4); ++k) {
    CHECK_HIP(hipMemcpy(host, dev[outs[k]], total * 2, hipMemcpyDeviceToHost));
    if (fwrite(host, 2, total, f) != total) return 1;
  }
  double edq[4];
  CHECK_HIP(hipMemcpy(edq, edq_dev, sizeof(edq), hipMemcpyDeviceToHost));
  if (fwrite(edq, sizeof(double), 4, f) != 4) return 1;
  fclose(f);
  CHECK_MCF(mcf_plan_destroy(plan));
  for (int s = 0; s < STREAMS; ++s) CHECK_HIP(hipFree(dev[s] - lead));
  CHECK_HIP(hipFree(edq_dev));
  CHECK_HIP(hipStreamDestroy(stream));
  free(host);
  printf("mcf_abi_demo: %llu parameters, %d steps, EDQ %.6g\n", (unsigned long long)total, steps, edq[0]);
  return 0;
}
