// C ABI of the ECO library (see include/eco.h): argument validation, derivation of the fp32 step
// constants, launch plans (device tables mapping tiles to tensors) and kernel dispatch.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "../../include/eco.h"
#include "eco_internal.hpp"

namespace {

thread_local std::string g_last_error;
int64_t g_wgs_per_cu = 0;   // 0 = default
int64_t g_lds_bytes = -1;    // -1 = default; dynamic LDS per workgroup of the step kernel (occupancy limiter)

eco_status_t fail(eco_status_t st, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return st;
}

eco_status_t fail_hip(hipError_t e, const char *what) {
  return fail(ECO_EHIP, "%s: %s", what, hipGetErrorString(e));
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int log2_exact(uint32_t x) {
  for (int s = 0; s < 32; ++s)
    if ((1u << s) == x) return s;
  return -1;
}

eco_status_t check_block_size(uint32_t bs, int *shift) {
  if (bs == 0) return fail(ECO_EINVAL, "block_size must be positive");
  const int s = log2_exact(bs);
  if (s < 5 || s > 9) return fail(ECO_EUNSUPPORTED, "block_size %u: supported sizes are 32, 64, 128, 256, 512", bs);
  *shift = s;
  return ECO_OK;
}

bool is_dtype(int32_t d) { return d == ECO_DT_FP32 || d == ECO_DT_BF16; }

// Validation of everything eco_step reads from the hyper-parameters.
eco_status_t check_hparams(const eco_hparams_t *hp) {
  if (!hp) return fail(ECO_EINVAL, "hyper-parameters: null pointer");
  if (hp->opt != ECO_OPT_ADAM && hp->opt != ECO_OPT_SGDM) return fail(ECO_EINVAL, "opt %d: unknown optimizer", hp->opt);
  if (hp->round != ECO_ROUND_SR && hp->round != ECO_ROUND_RTN) return fail(ECO_EINVAL, "round %d: unknown rounding", hp->round);
  if (hp->mode < ECO_MODE_NAIVE || hp->mode > ECO_MODE_MASTER) return fail(ECO_EINVAL, "mode %d: unknown mode", hp->mode);
  if (hp->mode == ECO_MODE_EXACT && hp->opt != ECO_OPT_SGDM)
    return fail(ECO_EUNSUPPORTED, "exact stored-error injection is defined for SGDM only");
  if (!is_dtype(hp->state_dtype) || !is_dtype(hp->scale_dtype)) return fail(ECO_EINVAL, "unknown state or scale dtype");
  if (hp->step == 0) return fail(ECO_EINVAL, "step is 1-based: step == 0 has no bias correction");
  if (!std::isfinite(hp->lr) || hp->lr < 0.0) return fail(ECO_EINVAL, "lr must be finite and >= 0");
  if (!std::isfinite(hp->weight_decay) || hp->weight_decay < 0.0) return fail(ECO_EINVAL, "weight_decay must be finite and >= 0");
  if (!(hp->beta1 >= 0.0 && hp->beta1 < 1.0)) return fail(ECO_EINVAL, "beta1 must lie in [0, 1)");
  if (hp->mode == ECO_MODE_ECO || hp->mode == ECO_MODE_EXACT) {
    // the injection strength divides by the learning rate and by beta (Eq. alpha; Alg. 3 line 5; Eq. im_inject)
    if (!(hp->lr > 0.0)) return fail(ECO_EINVAL, "error injection needs lr > 0");
    if (!(hp->beta1 > 0.0)) return fail(ECO_EINVAL, "error injection needs beta1 in (0, 1)");
  }
  if (hp->opt == ECO_OPT_ADAM) {
    if (!(hp->beta2 >= 0.0 && hp->beta2 < 1.0)) return fail(ECO_EINVAL, "beta2 must lie in [0, 1)");
    if (!std::isfinite(hp->eps) || hp->eps < 0.0) return fail(ECO_EINVAL, "eps must be finite and >= 0");
  }
  return ECO_OK;
}

void derive_constants(const eco_hparams_t *hp, eco_constants_t *c) {
  const double k = static_cast<double>(hp->step);
  const double bc1 = 1.0 - std::pow(hp->beta1, k);
  const double bc2 = 1.0 - std::pow(hp->beta2, k);
  std::memset(c, 0, sizeof *c);
  c->b1 = static_cast<float>(hp->beta1);
  c->omb1 = static_cast<float>(1.0 - hp->beta1);
  c->b2 = static_cast<float>(hp->beta2);
  c->omb2 = static_cast<float>(1.0 - hp->beta2);
  c->rbc2 = static_cast<float>(1.0 / bc2);
  c->c1 = static_cast<float>(hp->lr / bc1);
  c->eps = static_cast<float>(hp->eps);
  c->lr = static_cast<float>(hp->lr);
  c->wd = static_cast<float>(hp->lr * hp->weight_decay);
  if (hp->mode == ECO_MODE_ECO) {
    c->kappa = static_cast<float>((bc1 / hp->lr) * (1.0 - 1.0 / hp->beta1));
    c->alpha = static_cast<float>((1.0 / hp->lr) * (1.0 - 1.0 / hp->beta1));
  }
  if (hp->mode == ECO_MODE_EXACT) {
    c->inv_lr = static_cast<float>(1.0 / hp->lr);
    c->inv_lr_beta = static_cast<float>(1.0 / (hp->lr * hp->beta1));
  }
}

struct Group {
  std::vector<eco::TensorDesc> descs;
  std::vector<uint32_t> tile_tensor;     // one entry per full tile
  std::vector<uint32_t> ragged_tensor;   // tensors whose last tile is partial
  eco::TensorDesc *d_descs = nullptr;
  uint32_t *d_tiles = nullptr;           // tile_tensor followed by ragged_tensor
};

int num_compute_units() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
  return cus;
}

// Default: one workgroup per tile.  The hardware dispatcher then hands out tiles in address order,
// which keeps the set of DRAM pages in flight compact; grid-stride loops over a resident grid
// measured 10-15 % slower on MI355X.  Option 0 overrides with a resident grid.
unsigned grid_for(uint64_t tiles, int cus) {
  uint64_t g = tiles;
  if (g_wgs_per_cu > 0) {
    const uint64_t cap = static_cast<uint64_t>(cus) * static_cast<uint64_t>(g_wgs_per_cu);
    if (g > cap) g = cap;
  }
  if (g > 0x7FFFFFFFull) g = 0x7FFFFFFFull;
  if (g == 0) g = 1;
  return static_cast<unsigned>(g);
}

}  // namespace

struct eco_plan {
  uint32_t block_size = 0;
  int bs_shift = 0;
  int32_t state_dtype = 0, scale_dtype = 0, opt = 0, mode = 0;
  int cus = 256;
  Group groups[4];   // indexed by eco_format_t
};

extern "C" {

const char *eco_status_string(eco_status_t s) {
  switch (s) {
    case ECO_OK: return "ok";
    case ECO_EINVAL: return "invalid argument";
    case ECO_EALIGN: return "misaligned pointer";
    case ECO_EUNSUPPORTED: return "unsupported combination";
    case ECO_EHIP: return "HIP runtime error";
    case ECO_ENOMEM: return "out of memory";
  }
  return "unknown status";
}

const char *eco_last_error(void) { return g_last_error.c_str(); }

int eco_version(void) { return 100; }

eco_status_t eco_set_option(int32_t option, int64_t value) {
  if (option == 0) {
    if (value < 0 || value > 65536) return fail(ECO_EINVAL, "workgroups per compute unit must lie in [0, 65536]");
    g_wgs_per_cu = value;
    return ECO_OK;
  }
  if (option == 1) {
    if (value < -1 || value > 65536) return fail(ECO_EINVAL, "LDS bytes per workgroup must lie in [-1, 65536]");
    g_lds_bytes = value;
    return ECO_OK;
  }
  return fail(ECO_EINVAL, "unknown option %d", option);
}

eco_status_t eco_step_constants(const eco_hparams_t *hp, eco_constants_t *out) {
  if (!out) return fail(ECO_EINVAL, "constants: null output");
  const eco_status_t st = check_hparams(hp);
  if (st != ECO_OK) return st;
  derive_constants(hp, out);
  return ECO_OK;
}

eco_status_t eco_plan_destroy(eco_plan_t *plan) {
  if (!plan) return ECO_OK;
  bool any = false;
  for (Group &g : plan->groups) any = any || g.d_descs || g.d_tiles;
  eco_status_t st = ECO_OK;
  if (any) {
    const hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) st = fail_hip(e, "hipDeviceSynchronize");
  }
  for (Group &g : plan->groups) {
    if (g.d_descs) (void)hipFree(g.d_descs);
    if (g.d_tiles) (void)hipFree(g.d_tiles);
  }
  delete plan;
  return st;
}

eco_status_t eco_plan_create(const eco_tensor_t *tensors, size_t n, const eco_hparams_t *layout, eco_plan_t **out) {
  if (!out) return fail(ECO_EINVAL, "plan: null output pointer");
  *out = nullptr;
  if (!tensors || n == 0) return fail(ECO_EINVAL, "plan: empty tensor list");
  if (!layout) return fail(ECO_EINVAL, "plan: null layout");
  if (layout->opt != ECO_OPT_ADAM && layout->opt != ECO_OPT_SGDM) return fail(ECO_EINVAL, "opt %d: unknown optimizer", layout->opt);
  if (!is_dtype(layout->state_dtype) || !is_dtype(layout->scale_dtype)) return fail(ECO_EINVAL, "unknown state or scale dtype");
  if (layout->mode < ECO_MODE_NAIVE || layout->mode > ECO_MODE_MASTER) return fail(ECO_EINVAL, "mode %d: unknown mode", layout->mode);
  if (layout->mode == ECO_MODE_EXACT && layout->opt != ECO_OPT_SGDM)
    return fail(ECO_EUNSUPPORTED, "exact stored-error injection is defined for SGDM only");
  const bool needs_aux = layout->mode == ECO_MODE_EXACT || layout->mode == ECO_MODE_MASTER;
  int shift = 0;
  eco_status_t st = check_block_size(layout->block_size, &shift);
  if (st != ECO_OK) return st;

  eco_plan *plan = new (std::nothrow) eco_plan;
  if (!plan) return fail(ECO_ENOMEM, "plan: host allocation failed");
  plan->block_size = layout->block_size;
  plan->bs_shift = shift;
  plan->state_dtype = layout->state_dtype;
  plan->scale_dtype = layout->scale_dtype;
  plan->opt = layout->opt;
  plan->mode = layout->mode;

  try {
    for (size_t i = 0; i < n; ++i) {
      const eco_tensor_t &t = tensors[i];
      if (t.fmt < ECO_FMT_FP8_E4M3 || t.fmt > ECO_FMT_FP32_IDENTITY) { st = fail(ECO_EINVAL, "tensor %zu: unknown format %d", i, t.fmt); break; }
      if (t.numel == 0) { st = fail(ECO_EINVAL, "tensor %zu: numel == 0", i); break; }
      const bool quantized = t.fmt == ECO_FMT_FP8_E4M3 || t.fmt == ECO_FMT_INT4;
      if (!t.weights || !t.grad || !t.m) { st = fail(ECO_EINVAL, "tensor %zu: null weights, grad or m", i); break; }
      if (quantized && !t.scales) { st = fail(ECO_EINVAL, "tensor %zu: quantized format needs scales", i); break; }
      if (layout->opt == ECO_OPT_ADAM && !t.v) { st = fail(ECO_EINVAL, "tensor %zu: Adam needs v", i); break; }
      if (quantized && needs_aux && !t.aux) { st = fail(ECO_EINVAL, "tensor %zu: this mode needs the aux buffer", i); break; }
      if (!aligned16(t.weights) || !aligned16(t.grad) || !aligned16(t.m) || (quantized && !aligned16(t.scales)) ||
          (layout->opt == ECO_OPT_ADAM && !aligned16(t.v)) || (quantized && needs_aux && !aligned16(t.aux))) {
        st = fail(ECO_EALIGN, "tensor %zu: every data pointer must be 16-byte aligned", i);
        break;
      }
      Group &g = plan->groups[t.fmt];
      const uint64_t ntiles = t.numel / eco::TILE_ELEMS;   // full tiles
      if (g.tile_tensor.size() + ntiles > 0xFFFFFFF0ull) { st = fail(ECO_EUNSUPPORTED, "plan: more than 2^32 tiles in one format"); break; }
      eco::TensorDesc d;
      std::memset(&d, 0, sizeof d);
      d.w = t.weights; d.s = t.scales; d.g = t.grad; d.m = t.m; d.v = t.v; d.aux = t.aux;
      d.numel = t.numel;
      d.first_tile = static_cast<uint32_t>(g.tile_tensor.size());
      d.tensor_id = t.tensor_id;
      const uint32_t idx = static_cast<uint32_t>(g.descs.size());
      g.descs.push_back(d);
      g.tile_tensor.insert(g.tile_tensor.end(), static_cast<size_t>(ntiles), idx);
      if (t.numel % eco::TILE_ELEMS) g.ragged_tensor.push_back(idx);
    }
  } catch (const std::bad_alloc &) {
    st = fail(ECO_ENOMEM, "plan: host allocation failed");
  }
  if (st != ECO_OK) { delete plan; return st; }

  plan->cus = num_compute_units();
  for (Group &g : plan->groups) {
    if (g.descs.empty()) continue;
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&g.d_descs), g.descs.size() * sizeof(eco::TensorDesc));
    const size_t nt = g.tile_tensor.size(), nr = g.ragged_tensor.size();
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&g.d_tiles), (nt + nr) * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMemcpy(g.d_descs, g.descs.data(), g.descs.size() * sizeof(eco::TensorDesc), hipMemcpyHostToDevice);
    if (e == hipSuccess && nt) e = hipMemcpy(g.d_tiles, g.tile_tensor.data(), nt * sizeof(uint32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess && nr) e = hipMemcpy(g.d_tiles + nt, g.ragged_tensor.data(), nr * sizeof(uint32_t), hipMemcpyHostToDevice);
    if (e != hipSuccess) {
      st = (e == hipErrorOutOfMemory) ? fail(ECO_ENOMEM, "plan: device allocation failed") : fail_hip(e, "plan upload");
      (void)eco_plan_destroy(plan);
      return st;
    }
  }
  *out = plan;
  return ECO_OK;
}

eco_status_t eco_step(eco_plan_t *plan, const eco_hparams_t *hp, void *stream) {
  if (!plan) return fail(ECO_EINVAL, "step: null plan");
  eco_status_t st = check_hparams(hp);
  if (st != ECO_OK) return st;
  if (hp->block_size != plan->block_size || hp->state_dtype != plan->state_dtype || hp->scale_dtype != plan->scale_dtype ||
      hp->opt != plan->opt || hp->mode != plan->mode)
    return fail(ECO_EINVAL, "step: block_size, state_dtype, scale_dtype, opt and mode must equal the plan's");

  eco_constants_t c;
  derive_constants(hp, &c);
  for (int f = 0; f < 4; ++f) {
    Group &g = plan->groups[f];
    if (g.descs.empty()) continue;
    eco::StepArgs a;
    a.tensors = g.d_descs;
    a.tile_tensor = g.d_tiles;
    a.ragged_tensor = g.d_tiles + g.tile_tensor.size();
    a.num_tiles = static_cast<uint32_t>(g.tile_tensor.size());
    a.num_ragged = static_cast<uint32_t>(g.ragged_tensor.size());
    a.bs_shift = static_cast<uint32_t>(plan->bs_shift);
    a.b1 = c.b1; a.omb1 = c.omb1; a.b2 = c.b2; a.omb2 = c.omb2; a.rbc2 = c.rbc2; a.c1 = c.c1; a.eps = c.eps;
    a.kappa = c.kappa; a.lr = c.lr; a.alpha = c.alpha; a.wd = c.wd; a.inv_lr = c.inv_lr; a.inv_lr_beta = c.inv_lr_beta;
    a.seed_lo = static_cast<uint32_t>(hp->seed);
    a.seed_hi = static_cast<uint32_t>(hp->seed >> 32);
    a.step_lo = static_cast<uint32_t>(hp->step);
    // fp32 state: 20 B per parameter, bound by HBM -> cap the resident waves; bf16 state: 11-12 B per
    // parameter, bound by vector-ALU issue -> full occupancy
    a.lds_bytes = g_lds_bytes >= 0 ? static_cast<uint32_t>(g_lds_bytes)
                                   : (hp->state_dtype == ECO_DT_FP32 ? eco::DEFAULT_STEP_LDS_BYTES : 0u);
    eco::KernelVariant kv;
    kv.fmt = f;
    kv.state_bf16 = hp->state_dtype == ECO_DT_BF16;
    kv.scale_bf16 = hp->scale_dtype == ECO_DT_BF16;
    if (hp->mode == ECO_MODE_MASTER) kv.algo = hp->opt == ECO_OPT_ADAM ? eco::ALGO_ADAM_MASTER : eco::ALGO_SGDM_MASTER;
    else if (hp->mode == ECO_MODE_EXACT) kv.algo = eco::ALGO_SGDM_EXACT;
    else kv.algo = hp->opt == ECO_OPT_ADAM ? eco::ALGO_ADAM : eco::ALGO_SGDM;
    kv.round = hp->round;
    const hipError_t e = eco::launch_step(kv, a, grid_for(a.num_tiles, plan->cus), static_cast<hipStream_t>(stream));
    if (e != hipSuccess) return fail_hip(e, "step kernel launch");
  }
  return ECO_OK;
}

eco_status_t eco_step_tensors(const eco_tensor_t *tensors, size_t n, const eco_hparams_t *hp, void *stream) {
  eco_status_t st = check_hparams(hp);
  if (st != ECO_OK) return st;
  eco_plan_t *plan = nullptr;
  st = eco_plan_create(tensors, n, hp, &plan);
  if (st != ECO_OK) return st;
  st = eco_step(plan, hp, stream);
  const hipError_t e = hipStreamSynchronize(static_cast<hipStream_t>(stream));
  const eco_status_t st2 = eco_plan_destroy(plan);
  if (st != ECO_OK) return st;
  if (e != hipSuccess) return fail_hip(e, "hipStreamSynchronize");
  return st2;
}

static eco_status_t check_flat(const void *weights, const void *scales, uint64_t numel, int32_t fmt, uint32_t block_size,
                               int32_t scale_dtype, int *shift) {
  if (fmt != ECO_FMT_FP8_E4M3 && fmt != ECO_FMT_INT4) return fail(ECO_EINVAL, "format %d is not a quantized format", fmt);
  if (!is_dtype(scale_dtype)) return fail(ECO_EINVAL, "unknown scale dtype");
  if (numel == 0) return fail(ECO_EINVAL, "numel == 0");
  if (!weights || !scales) return fail(ECO_EINVAL, "null weights or scales");
  if (!aligned16(weights) || !aligned16(scales)) return fail(ECO_EALIGN, "weights and scales must be 16-byte aligned");
  return check_block_size(block_size, shift);
}

eco_status_t eco_quantize_init(const void *src, int32_t src_dtype, uint64_t numel, int32_t fmt, uint32_t block_size,
                               int32_t scale_dtype, void *weights, void *scales, void *stream) {
  int shift = 0;
  eco_status_t st = check_flat(weights, scales, numel, fmt, block_size, scale_dtype, &shift);
  if (st != ECO_OK) return st;
  if (!src) return fail(ECO_EINVAL, "null source");
  if (!is_dtype(src_dtype)) return fail(ECO_EINVAL, "unknown source dtype");
  if (!aligned16(src)) return fail(ECO_EALIGN, "source must be 16-byte aligned");
  const uint64_t tiles = (numel + eco::TILE_ELEMS - 1) / eco::TILE_ELEMS;
  const hipError_t e = eco::launch_quantize_init(src, src_dtype == ECO_DT_BF16, numel, fmt, static_cast<uint32_t>(shift),
                                                 scale_dtype == ECO_DT_BF16, weights, scales,
                                                 grid_for(tiles, num_compute_units()), static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ECO_OK : fail_hip(e, "quantize kernel launch");
}

eco_status_t eco_dequantize(const void *weights, const void *scales, uint64_t numel, int32_t fmt, uint32_t block_size,
                            int32_t scale_dtype, float *dst, void *stream) {
  int shift = 0;
  eco_status_t st = check_flat(weights, scales, numel, fmt, block_size, scale_dtype, &shift);
  if (st != ECO_OK) return st;
  if (!dst) return fail(ECO_EINVAL, "null destination");
  if (!aligned16(dst)) return fail(ECO_EALIGN, "destination must be 16-byte aligned");
  const uint64_t tiles = (numel + eco::TILE_ELEMS - 1) / eco::TILE_ELEMS;
  const hipError_t e = eco::launch_dequantize(weights, scales, numel, fmt, static_cast<uint32_t>(shift),
                                              scale_dtype == ECO_DT_BF16, dst, grid_for(tiles, num_compute_units()),
                                              static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ECO_OK : fail_hip(e, "dequantize kernel launch");
}

eco_status_t eco_philox_fill(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t first_word, uint64_t n_words,
                             uint32_t *dst, void *stream) {
  if (!dst) return fail(ECO_EINVAL, "null destination");
  if (n_words == 0) return fail(ECO_EINVAL, "n_words == 0");
  if (first_word + n_words < first_word) return fail(ECO_EINVAL, "word range overflows");
  const hipError_t e = eco::launch_philox_fill(seed, step, tensor_id, first_word, n_words, dst, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ECO_OK : fail_hip(e, "philox kernel launch");
}

}  // extern "C"
