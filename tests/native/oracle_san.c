/* Sanitizer driver for the CPU oracle (oracle/eco_oracle.c is compiled into this program with
 * -fsanitize=address,undefined): small steps through every format, optimizer, rounding and mode, with ragged
 * lengths and odd block sizes, plus the argument checks.  Prints "ok" and returns 0 when nothing trips. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#ifndef REAL
#define REAL float
#endif

typedef struct {
  int32_t fmt, opt, round, mode;
  int32_t block_size, state_bf16, scale_bf16, reserved;
  double lr, beta1, beta2, eps, weight_decay;
  uint64_t step, seed, elem_offset;
  uint32_t tensor_id, pad;
} oracle_cfg;

int oracle_quantize_rtn(int fmt, int block_size, int scale_bf16, uint64_t numel, const REAL *x, uint8_t *codes, REAL *scales);
int oracle_dequantize(int fmt, int block_size, uint64_t numel, const uint8_t *codes, const REAL *scales, REAL *out);
int oracle_encode(int fmt, int round, uint64_t n, const REAL *y, const uint16_t *r16, uint8_t *out);
void oracle_philox_fill(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t first_word, uint64_t n_words, uint32_t *dst);
void oracle_random16(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t first_elem, uint64_t n, uint16_t *dst);
void oracle_decode_table(int fmt, REAL *out);
int oracle_eco_step(const oracle_cfg *cfg, uint64_t numel, uint8_t *codes, REAL *scales, REAL *wreal, const uint16_t *grad_bf16,
                    const REAL *grad_real, REAL *m, REAL *v, const REAL *xi, REAL *aux, REAL *dbg_theta, REAL *dbg_err);

static uint32_t lcg = 12345u;
static REAL rnd(void) { lcg = lcg * 1664525u + 1013904223u; return (REAL)((int32_t)lcg) / (REAL)2147483648.0; }

#define CHECK(c) do { if (!(c)) { printf("check failed at line %d: %s\n", __LINE__, #c); return 1; } } while (0)

int main(void) {
  const uint64_t sizes[] = {1, 7, 128, 129, 1000, 4099};
  const int blocks[] = {32, 128, 8, 5};
  int nrun = 0;
  for (unsigned si = 0; si < sizeof sizes / sizeof *sizes; si++)
    for (unsigned bi = 0; bi < sizeof blocks / sizeof *blocks; bi++)
      for (int fmt = 0; fmt < 2; fmt++)
        for (int variant = 0; variant < 8; variant++) {
          const uint64_t n = sizes[si];
          const int bs = blocks[bi];
          if (fmt == 1 && (bs & 1) && (uint64_t)bs < n) continue;          /* two INT4 blocks would share a byte */
          const uint64_t nb = (n + (uint64_t)bs - 1) / (uint64_t)bs;
          /* exact-size heap blocks: one byte too many read or written is an ASan report */
          REAL *x = malloc(sizeof(REAL) * n), *scales = malloc(sizeof(REAL) * nb), *m = malloc(sizeof(REAL) * n);
          REAL *v = malloc(sizeof(REAL) * n), *aux = malloc(sizeof(REAL) * n), *th = malloc(sizeof(REAL) * n), *out = malloc(sizeof(REAL) * n);
          uint8_t *codes = malloc(fmt == 0 ? n : (n + 1) / 2);
          uint16_t *g = malloc(sizeof(uint16_t) * n);
          CHECK(x && scales && m && v && aux && th && out && codes && g);
          for (uint64_t i = 0; i < n; i++) {
            x[i] = rnd() * (REAL)0.02; m[i] = rnd() * (REAL)1e-3; v[i] = rnd() * rnd() * (REAL)1e-6; aux[i] = x[i];
            float gf = (float)(rnd() * 1e-3); uint32_t u; memcpy(&u, &gf, 4); g[i] = (uint16_t)(u >> 16);
          }
          memset(codes, 0, fmt == 0 ? n : (n + 1) / 2);
          CHECK(oracle_quantize_rtn(fmt, bs, variant & 1, n, x, codes, scales) == 0);
          CHECK(oracle_dequantize(fmt, bs, n, codes, scales, out) == 0);
          oracle_cfg c;
          memset(&c, 0, sizeof c);
          c.fmt = fmt; c.block_size = bs; c.scale_bf16 = variant & 1; c.state_bf16 = (variant >> 1) & 1;
          c.opt = variant >= 4; c.round = (variant >> 2) & 1 ? 1 : 0;
          c.mode = (variant == 5) ? 2 : (variant == 6 || variant == 3) ? 3 : (variant == 7 ? 0 : 1);   /* exact needs SGDM */
          c.lr = c.opt ? 0.05 : 1e-3; c.beta1 = 0.9; c.beta2 = 0.999; c.eps = 1e-8; c.weight_decay = variant == 2 ? 0.1 : 0.0;
          c.seed = 99 + variant; c.tensor_id = (uint32_t)si; c.elem_offset = (uint64_t)bs * 3;
          for (c.step = 1; c.step <= 2; c.step++)
            CHECK(oracle_eco_step(&c, n, codes, scales, NULL, g, NULL, m, c.opt ? NULL : v, NULL, aux, th, out) == 0);
          nrun++;
          free(x); free(scales); free(m); free(v); free(aux); free(th); free(out); free(codes); free(g);
        }
  /* unquantized formats and the additive-noise quantizer of the Appendix C pins */
  for (int fmt = 2; fmt <= 4; fmt++) {
    const uint64_t n = 77;
    REAL *w = malloc(sizeof(REAL) * n), *gr = malloc(sizeof(REAL) * n), *m = calloc(n, sizeof(REAL)), *v = calloc(n, sizeof(REAL));
    REAL *xi = malloc(sizeof(REAL) * n);
    CHECK(w && gr && m && v && xi);
    for (uint64_t i = 0; i < n; i++) { w[i] = rnd(); gr[i] = rnd(); xi[i] = rnd() * (REAL)1e-3; }
    oracle_cfg c;
    memset(&c, 0, sizeof c);
    c.fmt = fmt; c.block_size = 16; c.mode = 1; c.lr = 1e-2; c.beta1 = 0.9; c.beta2 = 0.99; c.eps = 1e-8; c.step = 4;
    CHECK(oracle_eco_step(&c, n, NULL, NULL, w, NULL, gr, m, v, xi, NULL, NULL, NULL) == 0);
    c.opt = 1;
    CHECK(oracle_eco_step(&c, n, NULL, NULL, w, NULL, gr, m, NULL, xi, NULL, NULL, NULL) == 0);
    free(w); free(gr); free(m); free(v); free(xi);
  }
  /* helpers */
  {
    uint32_t words[37]; uint16_t r16[53]; REAL tab[256]; REAL y[53]; uint8_t enc[53];
    oracle_philox_fill(~0ull, 1ull << 40, 0xFFFFFFFFu, (1ull << 34) - 5, 37, words);
    oracle_random16(5, 6, 7, (1ull << 35) - 9, 53, r16);
    oracle_decode_table(0, tab); oracle_decode_table(1, tab);
    for (int i = 0; i < 53; i++) y[i] = rnd() * (REAL)500.0;
    CHECK(oracle_encode(0, 0, 53, y, r16, enc) == 0 && oracle_encode(1, 1, 53, y, NULL, enc) == 0 && oracle_encode(2, 0, 53, y, r16, enc) != 0);
  }
  /* refusals */
  {
    REAL m[8] = {0}, v[8] = {0}, s[1] = {1}; uint8_t cd[8] = {0}; uint16_t g[8] = {0};
    oracle_cfg c;
    memset(&c, 0, sizeof c);
    c.block_size = 8; c.mode = 1; c.lr = 1e-3; c.beta1 = 0.9; c.beta2 = 0.999; c.eps = 1e-8; c.step = 1;
    CHECK(oracle_eco_step(&c, 8, cd, s, NULL, g, NULL, m, v, NULL, NULL, NULL, NULL) == 0);
    c.step = 0; CHECK(oracle_eco_step(&c, 8, cd, s, NULL, g, NULL, m, v, NULL, NULL, NULL, NULL) != 0); c.step = 1;
    c.lr = 0; CHECK(oracle_eco_step(&c, 8, cd, s, NULL, g, NULL, m, v, NULL, NULL, NULL, NULL) != 0); c.lr = 1e-3;
    c.mode = 2; CHECK(oracle_eco_step(&c, 8, cd, s, NULL, g, NULL, m, v, NULL, m, NULL, NULL) != 0); c.mode = 1;
    CHECK(oracle_eco_step(&c, 8, NULL, s, NULL, g, NULL, m, v, NULL, NULL, NULL, NULL) != 0);
    CHECK(oracle_eco_step(&c, 8, cd, s, NULL, NULL, NULL, m, v, NULL, NULL, NULL, NULL) != 0);
    CHECK(oracle_quantize_rtn(3, 8, 0, 8, m, cd, s) != 0 && oracle_dequantize(0, 0, 8, cd, s, m) != 0);
  }
  printf("ok %d steps\n", nrun);
  return 0;
}
