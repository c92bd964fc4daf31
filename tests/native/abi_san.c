/* Sanitizer driver for the host half of the library (the library and this client are built with
 * -fsanitize=address,undefined on their host code): every entry point's validation and refusal paths, with
 * exact-size heap arrays of descriptors, and -- where a device is missing -- the error path of the first HIP
 * call.  No kernel is needed for any of it.  Prints "ok" and returns 0 when nothing trips. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "eco.h"

#define CHECK(c) do { if (!(c)) { printf("check failed at line %d: %s (last error: %s)\n", __LINE__, #c, eco_last_error()); return 1; } } while (0)

static eco_hparams_t hparams(void) {
  eco_hparams_t hp;
  memset(&hp, 0, sizeof hp);
  hp.opt = ECO_OPT_ADAM; hp.round = ECO_ROUND_SR; hp.mode = ECO_MODE_ECO; hp.block_size = 128;
  hp.lr = 1e-3; hp.beta1 = 0.9; hp.beta2 = 0.999; hp.eps = 1e-8; hp.step = 3; hp.seed = 7;
  return hp;
}

static eco_tensor_t tensor(uint64_t numel) {
  eco_tensor_t t;
  memset(&t, 0, sizeof t);
  t.weights = (void *)0x10000; t.scales = (void *)0x20000; t.grad = (void *)0x30000; t.m = (void *)0x40000; t.v = (void *)0x50000;
  t.numel = numel; t.fmt = ECO_FMT_FP8_E4M3;
  return t;
}

int main(void) {
  eco_hparams_t hp = hparams();
  eco_constants_t c;
  eco_plan_t *plan = (eco_plan_t *)0x1;
  CHECK(eco_version() >= 100 && strcmp(eco_status_string(ECO_OK), "ok") == 0 && strcmp(eco_status_string(-99), "unknown status") == 0);
  CHECK(eco_step_constants(&hp, &c) == ECO_OK && c.kappa < 0);
  CHECK(eco_step_constants(NULL, &c) == ECO_EINVAL && eco_step_constants(&hp, NULL) == ECO_EINVAL);
  hp.step = 0; CHECK(eco_step_constants(&hp, &c) == ECO_EINVAL); hp = hparams();
  hp.lr = 1e-42; CHECK(eco_step_constants(&hp, &c) == ECO_EINVAL); hp = hparams();
  hp.beta1 = 1.0; CHECK(eco_step_constants(&hp, &c) == ECO_EINVAL); hp = hparams();
  hp.mode = ECO_MODE_EXACT; CHECK(eco_step_constants(&hp, &c) == ECO_EUNSUPPORTED); hp = hparams();
  CHECK(strlen(eco_last_error()) > 0);

  /* plans: refusals come before any device work; exact-size descriptor arrays */
  for (size_t n = 1; n <= 65; n += 16) {
    eco_tensor_t *ts = malloc(sizeof *ts * n);
    CHECK(ts != NULL);
    for (size_t i = 0; i < n; i++) ts[i] = tensor(512 * (i + 1) + (i % 3));
    ts[n - 1].m = NULL;
    CHECK(eco_plan_create(ts, n, &hp, &plan) == ECO_EINVAL && plan == NULL);
    ts[n - 1].m = (void *)0x40004;
    CHECK(eco_plan_create(ts, n, &hp, &plan) == ECO_EALIGN && plan == NULL);
    ts[n - 1].m = (void *)0x40000; ts[n - 1].group_size = 100;
    CHECK(eco_plan_create(ts, n, &hp, &plan) == ECO_EUNSUPPORTED && plan == NULL);
    CHECK(eco_step_tensors(ts, n, &hp, NULL) == ECO_EUNSUPPORTED);
    CHECK(eco_step_tensors_noalloc(ts, n, &hp, NULL) == ECO_EUNSUPPORTED);
    ts[n - 1].group_size = 0; ts[n - 1].numel = 0;
    CHECK(eco_plan_create(ts, n, &hp, &plan) == ECO_EINVAL);
    free(ts);
  }
  CHECK(eco_plan_create(NULL, 1, &hp, &plan) == ECO_EINVAL && eco_plan_create((eco_tensor_t *)&hp, 0, &hp, &plan) == ECO_EINVAL);
  CHECK(eco_plan_destroy(NULL) == ECO_OK && eco_step(NULL, &hp, NULL) == ECO_EINVAL);
  {
    /* the limits of the allocation-free step: 4097 descriptors, and table entries beyond the static scratch */
    const size_t n = 4097;
    eco_tensor_t *ts = malloc(sizeof *ts * n);
    CHECK(ts != NULL);
    for (size_t i = 0; i < n; i++) ts[i] = tensor(512);
    CHECK(eco_step_tensors_noalloc(ts, n, &hp, NULL) == ECO_EUNSUPPORTED);
    ts[0].numel = (1ull << 29) + 512;
    CHECK(eco_step_tensors_noalloc(ts, 1, &hp, NULL) == ECO_EUNSUPPORTED);
    free(ts);
  }
  {
    /* a valid request: with a device it would create a plan; without one the first HIP call fails cleanly */
    eco_tensor_t t = tensor(4096);
    eco_status_t st = eco_plan_create(&t, 1, &hp, &plan);
    CHECK(st == ECO_OK || st == ECO_EHIP || st == ECO_ENOMEM);
    if (st == ECO_OK) CHECK(eco_plan_destroy(plan) == ECO_OK);
  }
  /* flat helpers */
  CHECK(eco_quantize_init(NULL, 0, 1024, 0, 128, 0, (void *)0x10000, (void *)0x20000, NULL) == ECO_EINVAL);
  CHECK(eco_quantize_init((void *)0x30000, 0, 1024, 0, 100, 0, (void *)0x10000, (void *)0x20000, NULL) == ECO_EUNSUPPORTED);
  CHECK(eco_quantize_init((void *)0x30000, 0, 1024, 0, 128, 0, (void *)0x10001, (void *)0x20000, NULL) == ECO_EALIGN);
  CHECK(eco_dequantize((void *)0x10000, (void *)0x20000, 0, 0, 128, 0, (float *)0x30000, NULL) == ECO_EINVAL);
  CHECK(eco_quantize_error((void *)0x30000, 0, (void *)0x10000, (void *)0x20000, 1024, 5, 128, 0, (float *)0x40000, NULL) == ECO_EINVAL);
  CHECK(eco_philox_fill(1, 1, 0, ~0ull, 2, (uint32_t *)0x10000, NULL) == ECO_EINVAL);
  CHECK(eco_bandwidth_probe(2, NULL, NULL, NULL, (void *)0x10000, (void *)0x20000, 1024, NULL) == ECO_EINVAL);
  CHECK(eco_bandwidth_probe(1, NULL, NULL, NULL, (void *)0x10000, (void *)0x20000, 1000, NULL) == ECO_EINVAL);
  CHECK(eco_arith_selftest(1, 1.0f, 0x30000000u, 0x30000010u, NULL, NULL) == ECO_EINVAL);
  CHECK(eco_arith_selftest(0, 0.0f, 1u, 2u, (uint64_t *)0x10000, NULL) == ECO_EINVAL);
  CHECK(eco_set_option(9, 0) == ECO_EINVAL && eco_set_option(0, -1) == ECO_EINVAL && eco_set_option(1, 4096) == ECO_OK && eco_set_option(1, -1) == ECO_OK);
  printf("ok\n");
  return 0;
}
