/*
 * CPU oracle for the ECO optimizer step.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, scalar statement of
 * what one ECO step computes; it is called only by the tests, by the smoke
 * check and by the benchmark's CPU-baseline leg.  It shares no code, header,
 * table or constant with the HIP library and must never be reached from the
 * product path.
 *
 * What it follows (paper: "ECO: Quantized Training without Full-Precision
 * Master Weights"):
 *   - Sec. 3.1 "Quantization", Eq. (1) and the paragraph after it: symmetric
 *     abs-max quantizer  q(x) = (max|x|/rho) * round(rho*x/max|x|), zero point 0,
 *     round = round-to-nearest or stochastic rounding.
 *   - Alg. 1: theta~, s~ <- OPTIM_STEP(theta^, s^, H); then ECO_QUANTIZE.
 *   - Sec. 3.2 "Adam" display equations: the Adam update written with the
 *     element-wise step size eta_t = eta / ((1-b1^t)(sqrt(v/(1-b2^t))+eps));
 *     the update is formed the way the section writes it, theta~ = theta^ -
 *     eta_t (.) m~ with eta_t = (eta/(1-b1^t)) / (sqrt(v^)+eps) (one division,
 *     one multiplication).
 *   - Alg. 3 (ECO_QUANTIZE for Adam):  m^ = m~ + ((1-b1^t)/eta)(1-1/b1) *
 *     (sqrt(v/(1-b2^t))+eps) (.) e ,  e = theta~ - q(theta~);  v is returned
 *     unchanged.
 *   - Alg. 2 and Eqs. (m_tilde)...(alpha) of Sec. 3.3.1 (ECO for SGD with
 *     momentum, EMA form): m~ = b m^ + (1-b) g; theta~ = theta^ - eta m~;
 *     m^' = m~ + alpha e, alpha = (1/eta)(1 - 1/b).
 *
 * The arithmetic type is REAL (float or double, chosen at compile time).  The
 * double build is the one checked against closed forms and library routines;
 * the float build runs the same statements in fp32 because the quantized code
 * of an element is decided by fp32 arithmetic in the method as deployed, and a
 * decision must be taken in the same precision on both sides of a comparison.
 * Every floating-point statement below is a single IEEE operation (compile
 * with -ffp-contract=off); fused multiply-adds appear only where written.
 *
 * Readings of points the paper leaves open (each is restated in the design
 * document of this repository):
 *   - step counter k is 1-based (bias corrections 1-b^k), k = 0 is an error;
 *   - the scale group is a run of `block_size` consecutive elements of the
 *     flattened tensor; the scale is recomputed from theta~ at every step;
 *   - FP8 is OCP E4M3 (bias 7, no infinities, S.1111.111 = NaN), rho = 448;
 *     INT4 is two's complement restricted to [-7, 7], rho = 7, element 2j in
 *     the low nibble of byte j;
 *   - rounding acts on |y| and re-attaches the sign.  With lo <= |y| < hi the
 *     two neighbouring grid magnitudes: round-to-nearest takes the nearer one
 *     and, on an exact tie, the one with the even code.  Stochastic rounding
 *     forms f = (|y|-lo)/(hi-lo), F = rne(f * 2^20) (f * 2^20 is already an
 *     integer for fp32 y unless |y| lies in the E4M3 subnormal range), and
 *     goes up iff F + 16*r + 8 >= 2^20 with r the element's 16 random bits,
 *     so P(up) = floor((F+8)/16) / 2^16: f rounded to the nearest multiple of
 *     2^-16 (within 2^-17 of f, and with no preferred direction: Sec. 3.1
 *     calls stochastic rounding an unbiased estimator and Assumption 3.2 needs
 *     a zero-mean error; truncating F/16 instead would shrink every weight a
 *     little at every step).  On-grid values (F = 0) never move.  |y| >= rho
 *     saturates;
 *   - an all-zero block, or one whose abs-max is so small that rho/max
 *     overflows, is stored as scale 0 / codes 0 and its theta~ goes into e;
 *   - e is measured against the value the next step will reconstruct,
 *     fl(dec(code) * scale);
 *   - decoupled weight decay, when non-zero, is applied to theta^ inside the
 *     optimizer step, before quantization;
 *   - random bits: Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11), key =
 *     (seed lo, seed hi), counter = (q lo, q hi, step lo, tensor_id) with
 *     q = i >> 3 for element index i; element i takes the 16-bit field
 *     (i & 7) of the 128 output bits, low half of word (i&7)>>1 for even i.
 *
 * Parity pins are in tests/ (oracle_*): identity quantizer == library Adam,
 * codec round trips and boundaries, exhaustive stochastic-rounding counts,
 * Philox known answers, the SGDM virtual-sequence invariant (Lemma 3.4), the
 * one-step identity theta^' = theta^ - eta m^' - e/beta (proof of Lemma 3.4),
 * and the 1-D quadratic stationary second moments (Appendix C).
 * Parity unpinned: behaviour on NaN/Inf inputs (left undefined).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#ifndef REAL
#define REAL float
#endif

/* one IEEE operation each, in the width of REAL */
static inline REAL r_sqrt(REAL x) { return sizeof(REAL) == 4 ? (REAL)sqrtf((float)x) : (REAL)sqrt((double)x); }
static inline REAL r_fma(REAL a, REAL b, REAL c) {
  return sizeof(REAL) == 4 ? (REAL)fmaf((float)a, (float)b, (float)c) : (REAL)fma((double)a, (double)b, (double)c);
}
static inline REAL r_abs(REAL x) { return x < 0 ? -x : (x == 0 ? (REAL)0 : x); }

enum { FMT_E4M3 = 0, FMT_INT4 = 1, FMT_IDENTITY = 2, FMT_ADDNOISE = 3, FMT_BF16_PLAIN = 4 };
enum { OPT_ADAM = 0, OPT_SGDM = 1 };
enum { ROUND_SR = 0, ROUND_RTN = 1 };
enum { MODE_NAIVE = 0, MODE_ECO = 1, MODE_EXACT = 2, MODE_MASTER = 3 };

typedef struct {
  int32_t fmt, opt, round, mode;
  int32_t block_size, state_bf16, scale_bf16, reserved;
  double lr, beta1, beta2, eps, weight_decay;
  uint64_t step, seed, elem_offset;
  uint32_t tensor_id, pad;
} oracle_cfg;

/* ------------------------------------------------------------------ grids */

/* OCP E4M3: sign 1, exponent 4 (bias 7), mantissa 3; E = 0 is subnormal. */
static double e4m3_value(unsigned c) {
  unsigned s = c >> 7, E = (c >> 3) & 15u, M = c & 7u;
  double mag;
  if (E == 15u && M == 7u) return NAN;
  mag = (E == 0u) ? ldexp((double)M, -9) : ldexp((double)(8u + M), (int)E - 10);
  return s ? -mag : mag;
}

typedef struct { double mag[128]; int n; double rho; } grid_t;

static void make_grid(int fmt, grid_t *G) {
  int j;
  if (fmt == FMT_E4M3) {
    G->n = 127;
    for (j = 0; j < 127; j++) G->mag[j] = e4m3_value((unsigned)j);
    G->rho = 448.0;
  } else {
    G->n = 8;
    for (j = 0; j < 8; j++) G->mag[j] = (double)j;
    G->rho = 7.0;
  }
}

/* index of the grid magnitude chosen for |y| = ay (see header: rounding) */
static int encode_mag(const grid_t *G, double ay, int round, uint32_t r16) {
  int lo = 0, hi = G->n - 1, up;
  double f, F;
  if (ay >= G->rho) return G->n - 1;
  while (hi - lo > 1) {
    int mid = (lo + hi) / 2;
    if (G->mag[mid] <= ay) lo = mid; else hi = mid;
  }
  if (round == ROUND_SR) {
    f = (ay - G->mag[lo]) / (G->mag[lo + 1] - G->mag[lo]);
    F = nearbyint(f * 1048576.0);
    up = (F + 16.0 * (double)r16 + 8.0 >= 1048576.0);
  } else {
    double below = ay - G->mag[lo], above = G->mag[lo + 1] - ay;   /* exact for fp32 inputs */
    up = (below > above) || (below == above && (lo & 1));
  }
  return lo + up;
}

/* code of y: E4M3 byte, or INT4 value as a 4-bit two's-complement nibble */
static unsigned encode(int fmt, const grid_t *G, REAL y, int round, uint32_t r16) {
  int neg = signbit((double)y) ? 1 : 0;
  int mag = encode_mag(G, fabs((double)y), round, r16);
  if (fmt == FMT_E4M3) return (unsigned)mag | ((unsigned)neg << 7);
  return (unsigned)(neg ? -mag : mag) & 15u;
}

static REAL decode(int fmt, unsigned code) {
  if (fmt == FMT_E4M3) return (REAL)e4m3_value(code & 255u);
  return (REAL)((code & 8u) ? (int)(code & 15u) - 16 : (int)(code & 15u));
}

static unsigned get_code(int fmt, const uint8_t *codes, uint64_t i) {
  if (fmt == FMT_E4M3) return codes[i];
  return (i & 1) ? (unsigned)(codes[i >> 1] >> 4) : (unsigned)(codes[i >> 1] & 15u);
}

static void put_code(int fmt, uint8_t *codes, uint64_t i, unsigned code) {
  if (fmt == FMT_E4M3) { codes[i] = (uint8_t)code; return; }
  if (i & 1) codes[i >> 1] = (uint8_t)((codes[i >> 1] & 0x0Fu) | ((code & 15u) << 4));
  else       codes[i >> 1] = (uint8_t)((codes[i >> 1] & 0xF0u) | (code & 15u));
}

/* nearest bfloat16 (8 significant bits, fp32 exponent range), ties to even */
static REAL bf16_round_(REAL x) {
  double ax = (double)x;
  int ex, ue;
  if (ax == 0.0 || isnan(ax) || isinf(ax)) return x;
  (void)frexp(ax, &ex);            /* |ax| = fr * 2^ex, fr in [0.5, 1) */
  ue = ex - 8;                     /* exponent of the last kept bit */
  if (ue < -133) ue = -133;        /* bf16 subnormals: fixed spacing 2^-133 */
  return (REAL)scalbn(nearbyint(scalbn(ax, -ue)), ue);
}

static REAL bf16_bits_to_real(uint16_t h) {
  uint32_t u = (uint32_t)h << 16;
  float f;
  memcpy(&f, &u, 4);
  return (REAL)f;
}

/* ----------------------------------------------------------------- Philox */

static void philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
  uint32_t k0 = key[0], k1 = key[1];
  int r;
  for (r = 0; r < 10; r++) {
    uint64_t p0, p1;
    uint32_t n0, n1, n2, n3;
    if (r > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
    p0 = (uint64_t)0xD2511F53u * (uint64_t)c0;
    p1 = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
    n1 = (uint32_t)p1;
    n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
    n3 = (uint32_t)p0;
    c0 = n0; c1 = n1; c2 = n2; c3 = n3;
  }
  out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

static void philox_call(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t q, uint32_t out[4]) {
  uint32_t ctr[4], key[2];
  ctr[0] = (uint32_t)q; ctr[1] = (uint32_t)(q >> 32); ctr[2] = (uint32_t)step; ctr[3] = tensor_id;
  key[0] = (uint32_t)seed; key[1] = (uint32_t)(seed >> 32);
  philox4x32_10(ctr, key, out);
}

/* the 16 random bits of element i of a tensor */
static uint32_t random16(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t i) {
  uint32_t w[4], word;
  philox_call(seed, step, tensor_id, i >> 3, w);
  word = w[(i & 7) >> 1];
  return (i & 1) ? (word >> 16) : (word & 0xFFFFu);
}

/* ------------------------------------------------------- exported helpers */

int oracle_sizeof_real(void) { return (int)sizeof(REAL); }

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void oracle_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

void oracle_philox(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) { philox4x32_10(ctr, key, out); }

/* word j of the stream = output word (j & 3) of call (j >> 2) */
void oracle_philox_fill(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t first_word,
                        uint64_t n_words, uint32_t *dst) {
  uint64_t j;
  for (j = 0; j < n_words; j++) {
    uint32_t w[4];
    uint64_t g = first_word + j;
    philox_call(seed, step, tensor_id, g >> 2, w);
    dst[j] = w[g & 3];
  }
}

void oracle_random16(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t first_elem,
                     uint64_t n, uint16_t *dst) {
  uint64_t j;
  for (j = 0; j < n; j++) dst[j] = (uint16_t)random16(seed, step, tensor_id, first_elem + j);
}

/* decode every code: 256 entries for E4M3, 16 for INT4 */
void oracle_decode_table(int fmt, REAL *out) {
  int n = (fmt == FMT_E4M3) ? 256 : 16, c;
  for (c = 0; c < n; c++) out[c] = decode(fmt, (unsigned)c);
}

/* encode already-scaled values y (one output byte per element) */
int oracle_encode(int fmt, int round, uint64_t n, const REAL *y, const uint16_t *r16, uint8_t *out) {
  grid_t G;
  uint64_t i;
  if (fmt != FMT_E4M3 && fmt != FMT_INT4) return -1;
  make_grid(fmt, &G);
  for (i = 0; i < n; i++) out[i] = (uint8_t)encode(fmt, &G, y[i], round, r16 ? r16[i] : 0u);
  return 0;
}

REAL oracle_bf16_round(REAL x) { return bf16_round_(x); }

/* abs-max scale of one block and the multiplier that maps onto the code grid */
static void block_scale(const REAL *x, int n, double rho, int scale_bf16, REAL *s_out, REAL *inv_out) {
  REAL a = 0, s, inv;
  int j;
  for (j = 0; j < n; j++) { REAL t = r_abs(x[j]); if (t > a) a = t; }
  s = a / (REAL)rho;
  if (scale_bf16) { s = bf16_round_(s); inv = (REAL)1 / s; }
  else inv = (REAL)rho / a;
  if (!(inv < (REAL)INFINITY)) { s = 0; inv = 0; }   /* a == 0, or rho/a overflows */
  *s_out = s; *inv_out = inv;
}

/* q(x) with round-to-nearest: the initial quantization of a weight tensor */
int oracle_quantize_rtn(int fmt, int block_size, int scale_bf16, uint64_t numel, const REAL *x,
                        uint8_t *codes, REAL *scales) {
  grid_t G;
  uint64_t nb, b;
  if ((fmt != FMT_E4M3 && fmt != FMT_INT4) || block_size < 1) return -1;
  make_grid(fmt, &G);
  nb = (numel + (uint64_t)block_size - 1) / (uint64_t)block_size;
  for (b = 0; b < nb; b++) {
    uint64_t i0 = b * (uint64_t)block_size;
    int n = (int)((numel - i0 < (uint64_t)block_size) ? (numel - i0) : (uint64_t)block_size), j;
    REAL s, inv;
    block_scale(x + i0, n, G.rho, scale_bf16, &s, &inv);
    scales[b] = s;
    for (j = 0; j < n; j++) put_code(fmt, codes, i0 + (uint64_t)j, encode(fmt, &G, x[i0 + j] * inv, ROUND_RTN, 0u));
  }
  return 0;
}

int oracle_dequantize(int fmt, int block_size, uint64_t numel, const uint8_t *codes, const REAL *scales, REAL *out) {
  uint64_t i;
  if ((fmt != FMT_E4M3 && fmt != FMT_INT4) || block_size < 1) return -1;
  for (i = 0; i < numel; i++) out[i] = decode(fmt, get_code(fmt, codes, i)) * scales[i / (uint64_t)block_size];
  return 0;
}

/* ------------------------------------------------------------ the ECO step */

/*
 * One ECO step over `numel` consecutive elements of a tensor, starting at
 * element `cfg->elem_offset` of it (a multiple of block_size; the offset only
 * enters the random-number counter).  In place.
 *   codes / scales : quantized weights (FMT_E4M3, FMT_INT4)
 *   wreal          : weights held as REAL (FMT_IDENTITY, FMT_ADDNOISE, FMT_BF16_PLAIN)
 *   grad_bf16      : gradient as bfloat16 bit patterns, or NULL and then
 *   grad_real      : gradient as REAL
 *   m, v           : optimizer state (v unused for SGDM); if cfg->state_bf16
 *                    the values written are rounded to bfloat16
 *   xi             : FMT_ADDNOISE only, q(x) = x + xi
 *   aux            : MODE_EXACT: the stored error e_t, replaced by e_{t+1} (Appendix A, Eq. im_inject:
 *                    m <- m~ + e_t/eta - e_{t+1}/(eta beta), SGDM only);
 *                    MODE_MASTER: high-precision master weights (Sec. 3.1 "Quantization-Aware
 *                    Training with Master Weights"): the update is applied to them, the quantized
 *                    weights are q(master), and the momentum is left alone
 *   dbg_theta, dbg_err : optional outputs theta~ and e
 * cfg->mode: MODE_NAIVE (no injection), MODE_ECO (Alg. 2/3), MODE_EXACT, MODE_MASTER.
 */
int oracle_eco_step(const oracle_cfg *cfg, uint64_t numel, uint8_t *codes, REAL *scales, REAL *wreal,
                    const uint16_t *grad_bf16, const REAL *grad_real, REAL *m, REAL *v, const REAL *xi,
                    REAL *aux, REAL *dbg_theta, REAL *dbg_err) {
  const int fmt = cfg->fmt, bs = cfg->block_size;
  const int quantized = (fmt == FMT_E4M3 || fmt == FMT_INT4);
  const int adam = (cfg->opt == OPT_ADAM);
  const int mode = (fmt == FMT_BF16_PLAIN) ? MODE_NAIVE : cfg->mode;
  const int inject = (mode == MODE_ECO || mode == MODE_EXACT);
  grid_t G;
  double bc1, bc2;
  REAL b1, omb1, b2, omb2, rbc2, c1, epsf, kap, wdf, lrf, alpha, ca, cb;
  int64_t nb, b;
  int bad = 0;

  if (bs < 1 || cfg->step == 0 || fmt < 0 || fmt > FMT_BF16_PLAIN) return -1;
  if (!(cfg->lr > 0.0) && inject) return -1;                          /* kappa, alpha divide by eta  */
  if (inject && !(cfg->beta1 > 0.0 && cfg->beta1 < 1.0)) return -1;   /* ... and by beta             */
  if (quantized && (!codes || !scales)) return -1;
  if (!quantized && !wreal) return -1;
  if (fmt == FMT_ADDNOISE && !xi) return -1;
  if (fmt == FMT_INT4 && (bs & 1) && (uint64_t)bs < numel) return -1;   /* two blocks would share a byte */
  if (cfg->elem_offset % (uint64_t)bs) return -1;
  if (!m || (adam && !v) || (!grad_bf16 && !grad_real)) return -1;
  if (mode < MODE_NAIVE || mode > MODE_MASTER) return -1;
  if ((mode == MODE_EXACT || mode == MODE_MASTER) && !aux) return -1;
  if (mode == MODE_EXACT && adam) return -1;                          /* Appendix A is stated for SGDM */
  if (quantized) make_grid(fmt, &G); else { G.n = 0; G.rho = 1.0; }

  /* scalars: formed in double, rounded once to REAL */
  bc1 = 1.0 - pow(cfg->beta1, (double)cfg->step);
  bc2 = 1.0 - pow(cfg->beta2, (double)cfg->step);
  b1 = (REAL)cfg->beta1;  omb1 = (REAL)(1.0 - cfg->beta1);
  b2 = (REAL)cfg->beta2;  omb2 = (REAL)(1.0 - cfg->beta2);
  rbc2 = (REAL)(1.0 / bc2);
  c1 = (REAL)(cfg->lr / bc1);
  epsf = (REAL)cfg->eps;
  kap = (REAL)((bc1 / cfg->lr) * (1.0 - 1.0 / cfg->beta1));          /* Alg. 3, injection line */
  lrf = (REAL)cfg->lr;
  alpha = (REAL)((1.0 / cfg->lr) * (1.0 - 1.0 / cfg->beta1));        /* Eq. (alpha)            */
  wdf = (REAL)(cfg->lr * cfg->weight_decay);
  ca = (REAL)(1.0 / cfg->lr);                                        /* Eq. (im_inject)        */
  cb = (REAL)(1.0 / (cfg->lr * cfg->beta1));

  nb = (int64_t)((numel + (uint64_t)bs - 1) / (uint64_t)bs);
#ifdef _OPENMP
#pragma omp parallel for schedule(static)
#endif
  for (b = 0; b < nb; b++) {
    const uint64_t i0 = (uint64_t)b * (uint64_t)bs;
    const int n = (int)((numel - i0 < (uint64_t)bs) ? (numel - i0) : (uint64_t)bs);
    REAL *th = (REAL *)malloc(sizeof(REAL) * (size_t)n * 3), *dd, *mt;
    REAL s_new = 0, inv = 0;
    uint32_t rw[4] = {0, 0, 0, 0};
    uint64_t rq = ~(uint64_t)0;
    int j;
    if (!th) { bad = 1; continue; }
    dd = th + n; mt = dd + n;

    /* OPTIM_STEP on the de-quantized weights (Alg. 1, first line) */
    for (j = 0; j < n; j++) {
      const uint64_t i = i0 + (uint64_t)j;
      REAL w, g, u;
      if (mode == MODE_MASTER) w = aux[i];
      else if (quantized) w = decode(fmt, get_code(fmt, codes, i)) * scales[b];
      else w = wreal[i];
      g = grad_bf16 ? bf16_bits_to_real(grad_bf16[i]) : grad_real[i];
      mt[j] = r_fma(b1, m[i], omb1 * g);
      if (adam) {
        REAL vt = r_fma(b2, v[i], omb2 * (g * g));
        dd[j] = r_sqrt(vt * rbc2) + epsf;
        u = (c1 / dd[j]) * mt[j];                        /* eta_t (.) m~: the element-wise step size of Sec. 3.2 */
        v[i] = cfg->state_bf16 ? bf16_round_(vt) : vt;   /* v is final after the gradient */
      } else {
        dd[j] = 0;
        u = lrf * mt[j];
      }
      if (cfg->weight_decay != 0.0) w = w - wdf * w;
      th[j] = w - u;
    }

    /* ECO_QUANTIZE (Alg. 2 / Alg. 3) */
    if (quantized) block_scale(th, n, G.rho, cfg->scale_bf16, &s_new, &inv);
    for (j = 0; j < n; j++) {
      const uint64_t i = i0 + (uint64_t)j;
      REAL q, e, mh;
      if (quantized) {
        const uint64_t gi = cfg->elem_offset + i;
        uint32_t r16 = 0;
        unsigned code;
        if (cfg->round == ROUND_SR) {
          uint32_t word;
          if ((gi >> 3) != rq) { rq = gi >> 3; philox_call(cfg->seed, cfg->step, cfg->tensor_id, rq, rw); }
          word = rw[(gi & 7) >> 1];
          r16 = (gi & 1) ? (word >> 16) : (word & 0xFFFFu);
        }
        code = encode(fmt, &G, th[j] * inv, cfg->round, r16);
        put_code(fmt, codes, i, code);
        q = decode(fmt, code) * s_new;
      } else if (fmt == FMT_ADDNOISE) {
        q = th[j] + xi[i];
      } else if (fmt == FMT_BF16_PLAIN) {
        q = bf16_round_(th[j]);
      } else {
        q = th[j];
      }
      e = th[j] - q;
      if (!quantized) wreal[i] = q;
      if (mode == MODE_ECO) mh = adam ? r_fma(kap * dd[j], e, mt[j]) : r_fma(alpha, e, mt[j]);
      else if (mode == MODE_EXACT) { mh = r_fma(-cb, e, r_fma(ca, aux[i], mt[j])); aux[i] = e; }
      else mh = mt[j];
      if (mode == MODE_MASTER) aux[i] = th[j];
      m[i] = cfg->state_bf16 ? bf16_round_(mh) : mh;
      if (dbg_theta) dbg_theta[i] = th[j];
      if (dbg_err) dbg_err[i] = e;
    }
    if (quantized) scales[b] = s_new;
    free(th);
  }
  return bad ? -2 : 0;
}
