/* A plain C99 client of include/eco.h: checks that the header is valid C, that the library links by its
 * C names, and that the host-only entry points behave as documented.  No GPU work is issued. */
#include <stdio.h>
#include <string.h>
#include "eco.h"

int main(void) {
  eco_hparams_t hp;
  eco_constants_t c;
  eco_status_t st;
  memset(&hp, 0, sizeof hp);
  hp.opt = ECO_OPT_ADAM; hp.round = ECO_ROUND_SR; hp.mode = ECO_MODE_ECO; hp.block_size = 128;
  hp.state_dtype = ECO_DT_FP32; hp.scale_dtype = ECO_DT_FP32;
  hp.lr = 1e-3; hp.beta1 = 0.9; hp.beta2 = 0.999; hp.eps = 1e-8; hp.weight_decay = 0.0; hp.step = 3; hp.seed = 7;
  printf("version %d\n", eco_version());
  printf("sizes %u %u %u\n", (unsigned)sizeof(eco_tensor_t), (unsigned)sizeof(eco_hparams_t), (unsigned)sizeof(eco_constants_t));
  st = eco_step_constants(&hp, &c);
  printf("constants %d %.9g %.9g %.9g %.9g %.9g %.9g %.9g %.9g\n", (int)st, c.b1, c.omb1, c.b2, c.omb2, c.rbc2, c.c1, c.eps, c.kappa);
  hp.step = 0;
  st = eco_step_constants(&hp, &c);
  printf("step0 %d %s | %s\n", (int)st, eco_status_string(st), eco_last_error());
  st = eco_step(NULL, &hp, NULL);
  printf("nullplan %d\n", (int)st);
  st = eco_plan_destroy(NULL);
  printf("destroynull %d\n", (int)st);
  return 0;
}
