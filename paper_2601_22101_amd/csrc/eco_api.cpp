// C ABI of the ECO library (see include/eco.h): argument validation, derivation of the fp32 step
// constants, launch plans (device tables mapping tiles to tensors) and kernel dispatch.
#include <hip/hip_runtime.h>

#include <atomic>
#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/eco.h"
#include "eco_internal.hpp"

namespace {

thread_local std::string g_last_error;
// launch tuning (eco_set_option): read by every eco_step, possibly from other host threads
std::atomic<int64_t> g_wgs_per_cu{0};        // 0 = default
std::atomic<int64_t> g_max_launch_threads{-1};   // -1 = the runtime's limit; smaller values make the step launch in chunks
std::atomic<int64_t> g_lds_bytes{-1};        // -1 = default; dynamic LDS per workgroup of the step kernel (occupancy limiter)
std::atomic<int64_t> g_lds_bytes_wave{-1};   // -1 = default; the same per wave of the wide-group and tensor-wise kernels

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

// hparams.block_size is the default scale group of a plan: a power of two in [32, 512] (tensors may
// override it with their own group_size)
eco_status_t check_block_size(uint32_t bs) {
  if (bs == 0) return fail(ECO_EINVAL, "block_size must be positive");
  const int s = eco::log2_exact(bs);
  if (s < 5 || s > 9) return fail(ECO_EUNSUPPORTED, "block_size %u: supported sizes are 32, 64, 128, 256, 512", bs);
  return ECO_OK;
}

bool is_dtype(int32_t d) { return d == ECO_DT_FP32 || d == ECO_DT_BF16; }

void derive_constants(const eco_hparams_t *hp, eco_constants_t *c);

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
  // valid doubles can still leave the fp32 range once combined (a tiny lr makes the injection strength
  // (1/lr)(1 - 1/beta) overflow): the step would then write non-finite state
  eco_constants_t c;
  derive_constants(hp, &c);
  const float all[] = {c.b1, c.omb1, c.b2, c.omb2, c.rbc2, c.c1, c.eps, c.kappa, c.lr, c.alpha, c.wd, c.inv_lr, c.inv_lr_beta};
  for (float x : all)
    if (!std::isfinite(x)) return fail(ECO_EINVAL, "a step constant derived from lr, the betas and the step index is not finite in fp32");
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

struct Group {                           // the tensors of one storage format
  std::vector<eco::TensorDesc> descs;
  std::vector<uint32_t> tile_tensor;     // block-scaled: one entry per full tile
  std::vector<uint32_t> ragged_tensor;   // block-scaled: tensors whose last tile is partial
  std::vector<uint32_t> wide[eco::MAX_WIDE_WAVES + 1];   // wide groups, by waves per group: one entry per group
  std::vector<uint32_t> tw_tile_tensor;  // tensor-wise: one entry per tile (full or partial)
  std::vector<uint32_t> tw_tensor;       // tensor-wise: the tensors
  eco::TensorDesc *d_descs = nullptr;
  uint32_t *d_tables = nullptr;          // all the lists above, back to back, then the abs-max slots
  uint32_t *d_tile_max = nullptr;        // scratch of the tensor-wise passes: one entry per tensor-wise tile
  size_t off_ragged = 0, off_wide[eco::MAX_WIDE_WAVES + 1] = {0}, off_tw_tiles = 0, off_tw_tensor = 0, off_slots = 0;
};

int num_compute_units() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess) return 256;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
  return cus;
}

// Resident waves per compute unit at which the full-tile step kernel measured fastest on MI355X, by bytes
// moved per 512-element tile (fp32 state: the kernel is bound by HBM, which delivers most with roughly
// 100-120 KB of tile traffic in flight per compute unit; bf16 state: bound by instruction issue, no cap: 0).
int default_waves(const eco::KernelVariant &kv) {
  if (kv.state_bf16 || kv.fmt == eco::FMT_BF16_PLAIN || kv.fmt == eco::FMT_FP32_ID) return 0;
  switch (kv.algo) {
    case eco::ALGO_ADAM: return 12;          // 20.1 B/parameter
    case eco::ALGO_ADAM_MASTER: return 8;    // 27.0
    case eco::ALGO_SGDM: return 14;          // 12.1
    case eco::ALGO_SGDM_MASTER: return 8;    // 19.0
    default: return 11;                      // SGDM with a stored error: 20.1
  }
}

// The cap is expressed as a dynamic-LDS request the kernels never touch (160 KB of LDS per compute unit).
// For Adam the wide-group kernel measured best at the same cap, the two tensor-wise passes with four waves more.
uint32_t lds_for_waves(int waves, int granule) {
  return waves > 0 ? static_cast<uint32_t>(163840 / waves / granule * granule) : 0u;
}

// Default: one workgroup per tile.  The hardware dispatcher then hands out tiles in address order,
// which keeps the set of DRAM pages in flight compact; grid-stride loops over a resident grid
// measured 10-15 % slower on MI355X.  Option 0 overrides with a resident grid.
unsigned grid_for(uint64_t tiles, int cus) {
  uint64_t g = tiles;
  const int64_t wgs_per_cu = g_wgs_per_cu.load(std::memory_order_relaxed);
  if (wgs_per_cu > 0) {
    const uint64_t cap = static_cast<uint64_t>(cus) * static_cast<uint64_t>(wgs_per_cu);
    if (g > cap) g = cap;
  }
  if (g > 0x7FFFFFFFull) g = 0x7FFFFFFFull;
  if (g == 0) g = 1;
  return static_cast<unsigned>(g);
}

// Validation of one tensor descriptor against the layout part of the hyper-parameters; on success *gsz is the
// tensor's scale group and *cls its class (eco::GROUP_*).
eco_status_t check_tensor(const eco_tensor_t &t, size_t i, const eco_hparams_t *layout, uint64_t *gsz, int *cls) {
  const bool needs_aux = layout->mode == ECO_MODE_EXACT || layout->mode == ECO_MODE_MASTER;
  if (t.fmt < ECO_FMT_FP8_E4M3 || t.fmt > ECO_FMT_FP32_IDENTITY) return fail(ECO_EINVAL, "tensor %zu: unknown format %d", i, t.fmt);
  if (t.numel == 0) return fail(ECO_EINVAL, "tensor %zu: numel == 0", i);
  const bool quantized = t.fmt == ECO_FMT_FP8_E4M3 || t.fmt == ECO_FMT_INT4;
  if (!t.weights || !t.grad || !t.m) return fail(ECO_EINVAL, "tensor %zu: null weights, grad or m", i);
  if (quantized && !t.scales) return fail(ECO_EINVAL, "tensor %zu: quantized format needs scales", i);
  if (layout->opt == ECO_OPT_ADAM && !t.v) return fail(ECO_EINVAL, "tensor %zu: Adam needs v", i);
  if (quantized && needs_aux && !t.aux) return fail(ECO_EINVAL, "tensor %zu: this mode needs the aux buffer", i);
  if (!aligned16(t.weights) || !aligned16(t.grad) || !aligned16(t.m) || (quantized && !aligned16(t.scales)) ||
      (layout->opt == ECO_OPT_ADAM && !aligned16(t.v)) || (quantized && needs_aux && !aligned16(t.aux)))
    return fail(ECO_EALIGN, "tensor %zu: every data pointer must be 16-byte aligned", i);
  *gsz = t.group_size ? t.group_size : layout->block_size;
  *cls = quantized ? eco::classify_group(*gsz, t.numel) : eco::GROUP_BLOCK;
  if (*cls == eco::GROUP_UNSUPPORTED)
    return fail(ECO_EUNSUPPORTED, "tensor %zu: scale group of %llu elements: supported are powers of two in [32, 512], "
                "multiples of 8 up to 8192, and the whole tensor", i, (unsigned long long)*gsz);
  return ECO_OK;
}

// The layout part of the hyper-parameters (what eco_plan_create reads).
eco_status_t check_layout(const eco_hparams_t *layout) {
  if (!layout) return fail(ECO_EINVAL, "plan: null layout");
  if (layout->opt != ECO_OPT_ADAM && layout->opt != ECO_OPT_SGDM) return fail(ECO_EINVAL, "opt %d: unknown optimizer", layout->opt);
  if (!is_dtype(layout->state_dtype) || !is_dtype(layout->scale_dtype)) return fail(ECO_EINVAL, "unknown state or scale dtype");
  if (layout->mode < ECO_MODE_NAIVE || layout->mode > ECO_MODE_MASTER) return fail(ECO_EINVAL, "mode %d: unknown mode", layout->mode);
  if (layout->mode == ECO_MODE_EXACT && layout->opt != ECO_OPT_SGDM)
    return fail(ECO_EUNSUPPORTED, "exact stored-error injection is defined for SGDM only");
  return check_block_size(layout->block_size);
}

// The kernel variant of a step with these hyper-parameters on tensors of format f.
eco::KernelVariant variant_for(const eco_hparams_t *hp, int f) {
  eco::KernelVariant kv;
  kv.fmt = f;
  kv.state_bf16 = hp->state_dtype == ECO_DT_BF16;
  kv.scale_bf16 = hp->scale_dtype == ECO_DT_BF16;
  if (hp->mode == ECO_MODE_MASTER) kv.algo = hp->opt == ECO_OPT_ADAM ? eco::ALGO_ADAM_MASTER : eco::ALGO_SGDM_MASTER;
  else if (hp->mode == ECO_MODE_EXACT) kv.algo = eco::ALGO_SGDM_EXACT;
  else kv.algo = hp->opt == ECO_OPT_ADAM ? eco::ALGO_ADAM : eco::ALGO_SGDM;
  kv.round = hp->round;
  return kv;
}

// The scalar part of the kernel arguments: step constants, random-stream key, launch options.
void fill_step_scalars(const eco_hparams_t *hp, const eco_constants_t &c, const eco::KernelVariant &kv, eco::StepArgs *a) {
  a->b1 = c.b1; a->omb1 = c.omb1; a->b2 = c.b2; a->omb2 = c.omb2; a->rbc2 = c.rbc2; a->c1 = c.c1; a->eps = c.eps;
  a->kappa = c.kappa; a->lr = c.lr; a->alpha = c.alpha; a->wd = c.wd; a->inv_lr = c.inv_lr; a->inv_lr_beta = c.inv_lr_beta;
  a->seed_lo = static_cast<uint32_t>(hp->seed);
  a->seed_hi = static_cast<uint32_t>(hp->seed >> 32);
  a->step_lo = static_cast<uint32_t>(hp->step);
  a->div_mid = (c.c1 >= 0x1p-40f && c.c1 <= 0x1p40f && c.eps <= 1.0f) ? 1u : 0u;
  const int64_t opt_threads = g_max_launch_threads.load(std::memory_order_relaxed);
  a->max_launch_threads = opt_threads > 0 ? static_cast<uint64_t>(opt_threads) : eco::MAX_LAUNCH_THREADS;
  a->unit_base = 0;
  const int waves = default_waves(kv);
  const int waves_wide = kv.algo == eco::ALGO_ADAM ? waves : 0;     // measured for Adam only; SGDM ran best uncapped
  const int64_t opt_lds = g_lds_bytes.load(std::memory_order_relaxed);
  const int64_t opt_lds_wave = g_lds_bytes_wave.load(std::memory_order_relaxed);
  a->lds_bytes = opt_lds >= 0 ? static_cast<uint32_t>(opt_lds) : lds_for_waves(waves, 512);
  a->lds_bytes_wave = opt_lds_wave >= 0 ? static_cast<uint32_t>(opt_lds_wave) : lds_for_waves(waves_wide, 256);
  a->lds_bytes_tw = opt_lds_wave >= 0 ? static_cast<uint32_t>(opt_lds_wave) : lds_for_waves(waves_wide ? waves_wide + 4 : 0, 256);
}


// ------------------------------------------------------------------------------------------------------------
// eco_step_tensors_noalloc: the plan-less step for callers that cannot allocate.  What eco_step_tensors puts
// into freshly allocated device memory -- the tensor descriptors, the tile -> tensor launch tables, and the
// abs-max slots and per-tile maxima of tensor-wise scaling -- lives in one static device array here; the tables
// are written by a small kernel from descriptors passed as kernel arguments, so nothing is copied from host
// memory either.  Every call on a GPU shares that GPU's array: calls that overlap on one GPU race.
namespace noalloc {

constexpr uint32_t MAX_TENSORS = ECO_NOALLOC_MAX_TENSORS;
constexpr uint32_t MAX_UNITS = ECO_NOALLOC_MAX_UNITS;
constexpr size_t OFF_DESCS = 0;
constexpr size_t OFF_TABLES = OFF_DESCS + sizeof(eco::TensorDesc) * MAX_TENSORS;       // launch lists, back to back
constexpr size_t OFF_SLOTS = OFF_TABLES + sizeof(uint32_t) * MAX_UNITS;                // one per tensor-wise tensor
constexpr size_t OFF_TILE_MAX = OFF_SLOTS + sizeof(uint32_t) * MAX_TENSORS;            // one per tensor-wise tile
constexpr size_t SCRATCH_BYTES = OFF_TILE_MAX + sizeof(uint32_t) * MAX_UNITS;
static_assert(OFF_TABLES % 256 == 0 && OFF_SLOTS % 256 == 0 && OFF_TILE_MAX % 256 == 0, "scratch sections stay aligned");

static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];

// The array's device address, per device: in host code the array's name is only a handle for
// hipGetSymbolAddress, never an address a kernel could use.
constexpr int MAX_DEVICES = 32;
std::mutex g_mu;
unsigned char *g_scratch_ptr[MAX_DEVICES] = {nullptr};

eco_status_t scratch_for_current_device(unsigned char **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail_hip(e, "hipGetDevice");
  if (dev < 0 || dev >= MAX_DEVICES) return fail(ECO_EUNSUPPORTED, "device %d: only devices 0..%d are supported", dev, MAX_DEVICES - 1);
  std::lock_guard<std::mutex> lock(g_mu);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail_hip(e, "hipGetSymbolAddress(scratch)");
    g_scratch_ptr[dev] = static_cast<unsigned char *>(p);
  }
  *out = g_scratch_ptr[dev];
  return ECO_OK;
}

// One launch of the table builder carries up to BUILD_CHUNK descriptors by value.
constexpr int BUILD_CHUNK = 32;
struct BuildArgs {
  eco::TensorDesc desc[BUILD_CHUNK];
  uint32_t list_pos[BUILD_CHUNK];    // index into the tables of the first of this tensor's `units` entries
  uint32_t units[BUILD_CHUNK];       // entries (tiles or groups) the tensor adds to its launch list
  uint32_t extra_pos[BUILD_CHUNK];   // index of one more entry (ragged-tail list, tensor-wise tensor list), or NO_ENTRY
  uint32_t first_index;              // descriptor index of desc[0]
  uint32_t count;
  unsigned char *scratch;
};
constexpr uint32_t NO_ENTRY = 0xFFFFFFFFu;
static_assert(sizeof(BuildArgs) <= 4096, "kernel arguments are limited to 4 KB");

constexpr int BUILD_THREADS = 256, BUILD_BLOCKS_PER_TENSOR = 32;
__global__ __launch_bounds__(BUILD_THREADS) void eco_noalloc_build_kernel(const BuildArgs a) {
  const uint32_t k = blockIdx.x;
  if (k >= a.count) return;
  const uint32_t index = a.first_index + k;
  uint32_t *tables = reinterpret_cast<uint32_t *>(a.scratch + OFF_TABLES);
  if (blockIdx.y == 0 && threadIdx.x < sizeof(eco::TensorDesc) / sizeof(uint64_t)) {
    const uint64_t *src = reinterpret_cast<const uint64_t *>(&a.desc[k]);
    reinterpret_cast<uint64_t *>(a.scratch + OFF_DESCS)[(size_t)index * (sizeof(eco::TensorDesc) / sizeof(uint64_t)) + threadIdx.x] =
        src[threadIdx.x];
  }
  if (blockIdx.y == 0 && threadIdx.x == 0 && a.extra_pos[k] != NO_ENTRY) tables[a.extra_pos[k]] = index;
  const uint32_t pos = a.list_pos[k], n = a.units[k];
  for (uint32_t i = blockIdx.y * BUILD_THREADS + threadIdx.x; i < n; i += BUILD_BLOCKS_PER_TENSOR * BUILD_THREADS)
    tables[pos + i] = index;
}

// Launch lists of one storage format, in the order they are laid out in the tables.
enum : int { L_TILE = 0, L_RAGGED = 1, L_WIDE1 = 2, L_TW_TILES = L_WIDE1 + eco::MAX_WIDE_WAVES, L_TW_TENSORS, L_COUNT };

struct ListOf { int list; int extra; uint64_t units; uint64_t group; };
// Which lists a tensor enters, and with how many entries (mirrors eco_plan_create).
ListOf lists_of(const eco_tensor_t &t, uint64_t gsz, int cls) {
  ListOf r = {L_TILE, -1, 0, 0};
  if (cls == eco::GROUP_BLOCK) {
    r.units = t.numel / eco::TILE_ELEMS;
    if (t.numel % eco::TILE_ELEMS) r.extra = L_RAGGED;
    r.group = gsz;
  } else if (cls == eco::GROUP_WIDE) {
    r.group = gsz < t.numel ? gsz : t.numel;
    const eco::WideGeometry wg = eco::wide_geometry(t.numel, r.group);
    r.units = wg.units;
    r.list = L_WIDE1 + static_cast<int>(wg.waves) - 1;
  } else {
    r.group = t.numel;
    r.units = (t.numel + eco::TILE_ELEMS - 1) / eco::TILE_ELEMS;
    r.list = L_TW_TILES;
    r.extra = L_TW_TENSORS;
  }
  return r;
}

}  // namespace noalloc

}  // namespace

struct eco_plan {
  uint32_t block_size = 0;
  int32_t state_dtype = 0, scale_dtype = 0, opt = 0, mode = 0;
  int cus = 256;
  int device = 0;    // the device that was current when the plan was created (its tables live there)
  Group groups[4];   // indexed by eco_format_t
};

extern "C" {

const char *eco_status_string(int s) {
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

int eco_version(void) { return 200; }

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
  if (option == 2) {
    if (value < -1 || value > 32768) return fail(ECO_EINVAL, "LDS bytes per wave must lie in [-1, 32768]");
    g_lds_bytes_wave = value;
    return ECO_OK;
  }
  if (option == 3) {
    if (value != -1 && (value < 1024 || value > static_cast<int64_t>(eco::MAX_LAUNCH_THREADS)))
      return fail(ECO_EINVAL, "threads per launch must be -1 or lie in [1024, 2^32 - 1]");
    g_max_launch_threads = value;
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
  for (Group &g : plan->groups) any = any || g.d_descs || g.d_tables;
  eco_status_t st = ECO_OK;
  if (any) {
    // steps may still be running on the plan's device: wait for that device, whichever is current
    int cur = -1;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    if (have_cur && cur != plan->device) (void)hipSetDevice(plan->device);
    const hipError_t e = hipDeviceSynchronize();
    if (e != hipSuccess) st = fail_hip(e, "hipDeviceSynchronize");
    for (Group &g : plan->groups) {
      if (g.d_descs) (void)hipFree(g.d_descs);
      if (g.d_tables) (void)hipFree(g.d_tables);
      if (g.d_tile_max) (void)hipFree(g.d_tile_max);
    }
    if (have_cur && cur != plan->device) (void)hipSetDevice(cur);
  }
  delete plan;
  return st;
}

eco_status_t eco_plan_create(const eco_tensor_t *tensors, size_t n, const eco_hparams_t *layout, eco_plan_t **out) {
  if (!out) return fail(ECO_EINVAL, "plan: null output pointer");
  *out = nullptr;
  if (!tensors || n == 0) return fail(ECO_EINVAL, "plan: empty tensor list");
  eco_status_t st = check_layout(layout);
  if (st != ECO_OK) return st;

  eco_plan *plan = new (std::nothrow) eco_plan;
  if (!plan) return fail(ECO_ENOMEM, "plan: host allocation failed");
  plan->block_size = layout->block_size;
  plan->state_dtype = layout->state_dtype;
  plan->scale_dtype = layout->scale_dtype;
  plan->opt = layout->opt;
  plan->mode = layout->mode;

  try {
    for (size_t i = 0; i < n; ++i) {
      const eco_tensor_t &t = tensors[i];
      uint64_t gsz = 0;
      int cls = 0;
      st = check_tensor(t, i, layout, &gsz, &cls);
      if (st != ECO_OK) break;
      const bool quantized = t.fmt == ECO_FMT_FP8_E4M3 || t.fmt == ECO_FMT_INT4;
      Group &g = plan->groups[t.fmt];
      eco::TensorDesc d;
      std::memset(&d, 0, sizeof d);
      d.w = t.weights; d.s = t.scales; d.g = t.grad; d.m = t.m; d.v = t.v; d.aux = t.aux;
      d.numel = t.numel;
      d.tensor_id = t.tensor_id;
      const uint32_t idx = static_cast<uint32_t>(g.descs.size());
      uint64_t units = 0;                 // tiles or groups this tensor adds to its launch list
      std::vector<uint32_t> *list = nullptr;
      if (cls == eco::GROUP_BLOCK) {
        d.group_size = quantized ? gsz : layout->block_size;
        d.bs_shift = static_cast<uint32_t>(eco::log2_exact(d.group_size));
        units = t.numel / eco::TILE_ELEMS;              // full tiles
        list = &g.tile_tensor;
        if (t.numel % eco::TILE_ELEMS) g.ragged_tensor.push_back(idx);
      } else if (cls == eco::GROUP_WIDE) {
        d.group_size = gsz < t.numel ? gsz : t.numel;
        const eco::WideGeometry wg = eco::wide_geometry(t.numel, d.group_size);
        d.slot = wg.rows;
        units = wg.units;
        list = &g.wide[wg.waves];
      } else {
        d.group_size = t.numel;
        d.slot = static_cast<uint32_t>(g.tw_tensor.size());
        units = (t.numel + eco::TILE_ELEMS - 1) / eco::TILE_ELEMS;
        list = &g.tw_tile_tensor;
        g.tw_tensor.push_back(idx);
      }
      if (list->size() + units > 0x7FFFFFF0ull) { st = fail(ECO_EUNSUPPORTED, "plan: more than 2^31 tiles in one launch"); break; }
      d.first_unit = static_cast<uint32_t>(list->size());
      list->insert(list->end(), static_cast<size_t>(units), idx);
      g.descs.push_back(d);
    }
  } catch (const std::bad_alloc &) {
    st = fail(ECO_ENOMEM, "plan: host allocation failed");
  }
  if (st != ECO_OK) { delete plan; return st; }

  {
    const hipError_t e = hipGetDevice(&plan->device);
    if (e != hipSuccess) { delete plan; return fail_hip(e, "hipGetDevice"); }
  }
  plan->cus = num_compute_units();
  for (Group &g : plan->groups) {
    if (g.descs.empty()) continue;
    // one device buffer: [full tiles | ragged | wide lists 1..16 | tensor-wise tiles | tensor-wise tensors | slots]
    std::vector<uint32_t> host;
    try {
      host = g.tile_tensor;
      g.off_ragged = host.size();
      host.insert(host.end(), g.ragged_tensor.begin(), g.ragged_tensor.end());
      for (int nw = 1; nw <= eco::MAX_WIDE_WAVES; ++nw) {
        g.off_wide[nw] = host.size();
        host.insert(host.end(), g.wide[nw].begin(), g.wide[nw].end());
      }
      g.off_tw_tiles = host.size();
      host.insert(host.end(), g.tw_tile_tensor.begin(), g.tw_tile_tensor.end());
      g.off_tw_tensor = host.size();
      host.insert(host.end(), g.tw_tensor.begin(), g.tw_tensor.end());
      g.off_slots = host.size();
      host.insert(host.end(), g.tw_tensor.size() + 1, 0u);      // abs-max slots start at zero
    } catch (const std::bad_alloc &) {
      (void)eco_plan_destroy(plan);
      return fail(ECO_ENOMEM, "plan: host allocation failed");
    }
    hipError_t e = hipMalloc(reinterpret_cast<void **>(&g.d_descs), g.descs.size() * sizeof(eco::TensorDesc));
    if (e == hipSuccess) e = hipMalloc(reinterpret_cast<void **>(&g.d_tables), host.size() * sizeof(uint32_t));
    if (e == hipSuccess && !g.tw_tile_tensor.empty())
      e = hipMalloc(reinterpret_cast<void **>(&g.d_tile_max), g.tw_tile_tensor.size() * sizeof(uint32_t));
    if (e == hipSuccess) e = hipMemcpy(g.d_descs, g.descs.data(), g.descs.size() * sizeof(eco::TensorDesc), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(g.d_tables, host.data(), host.size() * sizeof(uint32_t), hipMemcpyHostToDevice);
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
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev != plan->device)
    return fail(ECO_EINVAL, "step: the plan was created on device %d, which is not the current device (%d)", plan->device, dev);
  (void)hipGetLastError();   // an error left behind by the caller's earlier HIP work is not this call's

  eco_constants_t c;
  derive_constants(hp, &c);
  for (int f = 0; f < 4; ++f) {
    Group &g = plan->groups[f];
    if (g.descs.empty()) continue;
    if (!g.d_descs || !g.d_tables) return fail(ECO_EINVAL, "step: the plan's device tables are missing");
    eco::StepArgs a;
    std::memset(&a, 0, sizeof a);
    a.tensors = g.d_descs;
    a.tile_tensor = g.d_tables;
    a.ragged_tensor = g.d_tables + g.off_ragged;
    a.num_tiles = static_cast<uint32_t>(g.tile_tensor.size());
    a.num_ragged = static_cast<uint32_t>(g.ragged_tensor.size());
    a.wide_base = g.d_tables;
    for (int nw = 1; nw <= eco::MAX_WIDE_WAVES; ++nw) {
      a.wide_offset[nw] = static_cast<uint32_t>(g.off_wide[nw]);
      a.num_wide[nw] = static_cast<uint32_t>(g.wide[nw].size());
    }
    a.tw_tile_tensor = g.d_tables + g.off_tw_tiles;
    a.tw_tensor = g.d_tables + g.off_tw_tensor;
    a.slots = g.d_tables + g.off_slots;
    a.tile_max = g.d_tile_max;
    a.num_tw_tiles = static_cast<uint32_t>(g.tw_tile_tensor.size());
    a.num_tw_tensors = static_cast<uint32_t>(g.tw_tensor.size());
    const eco::KernelVariant kv = variant_for(hp, f);
    fill_step_scalars(hp, c, kv, &a);
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

eco_status_t eco_step_tensors_noalloc(const eco_tensor_t *tensors, size_t n, const eco_hparams_t *hp, void *stream) {
  using namespace noalloc;
  eco_status_t st = check_hparams(hp);
  if (st != ECO_OK) return st;
  st = check_layout(hp);
  if (st != ECO_OK) return st;
  if (!tensors || n == 0) return fail(ECO_EINVAL, "step: empty tensor list");
  if (n > MAX_TENSORS)
    return fail(ECO_EUNSUPPORTED, "eco_step_tensors_noalloc: %zu tensors, the static scratch holds %u (use a plan)", n, MAX_TENSORS);

  // pass 1: validate, count the entries of every launch list
  uint64_t count[4][L_COUNT] = {{0}};
  uint64_t total = 0;
  for (size_t i = 0; i < n; ++i) {
    uint64_t gsz = 0;
    int cls = 0;
    st = check_tensor(tensors[i], i, hp, &gsz, &cls);
    if (st != ECO_OK) return st;
    const ListOf lo = lists_of(tensors[i], gsz, cls);
    if (lo.units > MAX_UNITS) return fail(ECO_EUNSUPPORTED, "eco_step_tensors_noalloc: tensor %zu alone exceeds the static scratch", i);
    count[tensors[i].fmt][lo.list] += lo.units;
    if (lo.extra >= 0) count[tensors[i].fmt][lo.extra] += 1;
    total += lo.units + (lo.extra >= 0 ? 1 : 0);
    if (total > MAX_UNITS)
      return fail(ECO_EUNSUPPORTED, "eco_step_tensors_noalloc: more than %u launch-table entries (512-element tiles, or scale "
                  "groups wider than 512): the static scratch does not hold them (use a plan)", MAX_UNITS);
  }
  uint32_t start[4][L_COUNT], tw_tile_start[4], tw_tensor_start[4];
  {
    uint32_t pos = 0, tw_tiles = 0, tw_tensors = 0;
    for (int f = 0; f < 4; ++f) {
      for (int l = 0; l < L_COUNT; ++l) { start[f][l] = pos; pos += static_cast<uint32_t>(count[f][l]); }
      tw_tile_start[f] = tw_tiles; tw_tiles += static_cast<uint32_t>(count[f][L_TW_TILES]);
      tw_tensor_start[f] = tw_tensors; tw_tensors += static_cast<uint32_t>(count[f][L_TW_TENSORS]);
    }
  }

  unsigned char *sp = nullptr;
  st = scratch_for_current_device(&sp);
  if (st != ECO_OK) return st;
  (void)hipGetLastError();
  hipStream_t hs = static_cast<hipStream_t>(stream);

  // pass 2: descriptors and tables, BUILD_CHUNK tensors per launch of the builder
  uint32_t fill[4][L_COUNT] = {{0}};
  BuildArgs ba;
  std::memset(&ba, 0, sizeof ba);
  ba.scratch = sp;
  for (size_t i = 0; i < n; ++i) {
    const eco_tensor_t &t = tensors[i];
    uint64_t gsz = 0;
    int cls = 0;
    (void)check_tensor(t, i, hp, &gsz, &cls);
    const ListOf lo = lists_of(t, gsz, cls);
    const uint32_t k = ba.count++;
    if (k == 0) ba.first_index = static_cast<uint32_t>(i);
    eco::TensorDesc &d = ba.desc[k];
    std::memset(&d, 0, sizeof d);
    d.w = t.weights; d.s = t.scales; d.g = t.grad; d.m = t.m; d.v = t.v; d.aux = t.aux;
    d.numel = t.numel;
    d.tensor_id = t.tensor_id;
    const bool quantized = t.fmt == ECO_FMT_FP8_E4M3 || t.fmt == ECO_FMT_INT4;
    d.group_size = (cls == eco::GROUP_BLOCK && !quantized) ? hp->block_size : lo.group;
    if (cls == eco::GROUP_BLOCK) d.bs_shift = static_cast<uint32_t>(eco::log2_exact(d.group_size));
    if (cls == eco::GROUP_WIDE) d.slot = eco::wide_geometry(t.numel, lo.group).rows;
    d.first_unit = fill[t.fmt][lo.list];
    ba.list_pos[k] = start[t.fmt][lo.list] + fill[t.fmt][lo.list];
    ba.units[k] = static_cast<uint32_t>(lo.units);
    fill[t.fmt][lo.list] += static_cast<uint32_t>(lo.units);
    ba.extra_pos[k] = NO_ENTRY;
    if (lo.extra >= 0) {
      if (lo.extra == L_TW_TENSORS) d.slot = fill[t.fmt][lo.extra];
      ba.extra_pos[k] = start[t.fmt][lo.extra] + fill[t.fmt][lo.extra]++;
    }
    if (ba.count == BUILD_CHUNK || i + 1 == n) {
      hipLaunchKernelGGL(eco_noalloc_build_kernel, dim3(ba.count, BUILD_BLOCKS_PER_TENSOR), dim3(BUILD_THREADS), 0, hs, ba);
      const hipError_t e = hipGetLastError();
      if (e != hipSuccess) return fail_hip(e, "table kernel launch");
      ba.count = 0;
    }
  }

  eco_constants_t c;
  derive_constants(hp, &c);
  const int cus = num_compute_units();
  const eco::TensorDesc *descs = reinterpret_cast<const eco::TensorDesc *>(sp + OFF_DESCS);
  uint32_t *tables = reinterpret_cast<uint32_t *>(sp + OFF_TABLES);
  for (int f = 0; f < 4; ++f) {
    uint64_t any = 0;
    for (int l = 0; l < L_COUNT; ++l) any += count[f][l];
    if (!any) continue;
    eco::StepArgs a;
    std::memset(&a, 0, sizeof a);
    a.tensors = descs;
    a.tile_tensor = tables + start[f][L_TILE];
    a.ragged_tensor = tables + start[f][L_RAGGED];
    a.num_tiles = static_cast<uint32_t>(count[f][L_TILE]);
    a.num_ragged = static_cast<uint32_t>(count[f][L_RAGGED]);
    a.wide_base = tables;
    for (int nw = 1; nw <= eco::MAX_WIDE_WAVES; ++nw) {
      a.wide_offset[nw] = start[f][L_WIDE1 + nw - 1];
      a.num_wide[nw] = static_cast<uint32_t>(count[f][L_WIDE1 + nw - 1]);
    }
    a.tw_tile_tensor = tables + start[f][L_TW_TILES];
    a.tw_tensor = tables + start[f][L_TW_TENSORS];
    a.slots = reinterpret_cast<uint32_t *>(sp + OFF_SLOTS) + tw_tensor_start[f];
    a.tile_max = reinterpret_cast<uint32_t *>(sp + OFF_TILE_MAX) + tw_tile_start[f];
    a.num_tw_tiles = static_cast<uint32_t>(count[f][L_TW_TILES]);
    a.num_tw_tensors = static_cast<uint32_t>(count[f][L_TW_TENSORS]);
    const eco::KernelVariant kv = variant_for(hp, f);
    fill_step_scalars(hp, c, kv, &a);
    const hipError_t e = eco::launch_step(kv, a, grid_for(a.num_tiles, cus), hs);
    if (e != hipSuccess) return fail_hip(e, "step kernel launch");
  }
  return ECO_OK;
}

static eco_status_t check_flat(const void *weights, const void *scales, uint64_t numel, int32_t fmt, uint64_t group_size,
                               int32_t scale_dtype) {
  if (fmt != ECO_FMT_FP8_E4M3 && fmt != ECO_FMT_INT4) return fail(ECO_EINVAL, "format %d is not a quantized format", fmt);
  if (!is_dtype(scale_dtype)) return fail(ECO_EINVAL, "unknown scale dtype");
  if (numel == 0) return fail(ECO_EINVAL, "numel == 0");
  if (numel > (1ull << 40)) return fail(ECO_EUNSUPPORTED, "more than 2^40 elements in one call");
  if (group_size == 0) return fail(ECO_EINVAL, "group_size must be positive");
  if (!weights || !scales) return fail(ECO_EINVAL, "null weights or scales");
  if (!aligned16(weights) || !aligned16(scales)) return fail(ECO_EALIGN, "weights and scales must be 16-byte aligned");
  if (!eco::flat_call_fits(numel, group_size))
    return fail(ECO_EUNSUPPORTED, "%llu elements in groups of %llu: one call handles what one launch can (about 2^35 elements); "
                "call it on slices of whole scale groups", (unsigned long long)numel, (unsigned long long)group_size);
  return ECO_OK;
}

eco_status_t eco_quantize_init(const void *src, int32_t src_dtype, uint64_t numel, int32_t fmt, uint64_t group_size,
                               int32_t scale_dtype, void *weights, void *scales, void *stream) {
  eco_status_t st = check_flat(weights, scales, numel, fmt, group_size, scale_dtype);
  if (st != ECO_OK) return st;
  if (!src) return fail(ECO_EINVAL, "null source");
  if (!is_dtype(src_dtype)) return fail(ECO_EINVAL, "unknown source dtype");
  if (!aligned16(src)) return fail(ECO_EALIGN, "source must be 16-byte aligned");
  if (eco::classify_group(group_size, numel) == eco::GROUP_UNSUPPORTED)
    return fail(ECO_EUNSUPPORTED, "scale group of %llu elements: supported are powers of two in [32, 512], multiples of 8 "
                "up to 8192, and the whole tensor", (unsigned long long)group_size);
  (void)hipGetLastError();
  const hipError_t e = eco::launch_quantize_init(src, src_dtype == ECO_DT_BF16, numel, fmt, group_size,
                                                 scale_dtype == ECO_DT_BF16, weights, scales, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ECO_OK : fail_hip(e, "quantize kernel launch");
}

eco_status_t eco_dequantize(const void *weights, const void *scales, uint64_t numel, int32_t fmt, uint64_t group_size,
                            int32_t scale_dtype, float *dst, void *stream) {
  eco_status_t st = check_flat(weights, scales, numel, fmt, group_size, scale_dtype);
  if (st != ECO_OK) return st;
  if (!dst) return fail(ECO_EINVAL, "null destination");
  if (!aligned16(dst)) return fail(ECO_EALIGN, "destination must be 16-byte aligned");
  if (group_size < 8 && group_size < numel)      // a single group over a tiny tensor is fine
    return fail(ECO_EUNSUPPORTED, "scale groups of fewer than 8 elements are not supported");
  (void)hipGetLastError();
  const hipError_t e = eco::launch_dequantize(weights, scales, numel, fmt, group_size, scale_dtype == ECO_DT_BF16, nullptr, 0,
                                              dst, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ECO_OK : fail_hip(e, "dequantize kernel launch");
}

eco_status_t eco_quantize_error(const void *src, int32_t src_dtype, const void *weights, const void *scales, uint64_t numel,
                                int32_t fmt, uint64_t group_size, int32_t scale_dtype, float *err, void *stream) {
  eco_status_t st = check_flat(weights, scales, numel, fmt, group_size, scale_dtype);
  if (st != ECO_OK) return st;
  if (!src || !err) return fail(ECO_EINVAL, "null source or destination");
  if (!is_dtype(src_dtype)) return fail(ECO_EINVAL, "unknown source dtype");
  if (!aligned16(src) || !aligned16(err)) return fail(ECO_EALIGN, "source and destination must be 16-byte aligned");
  if (group_size < 8 && group_size < numel)
    return fail(ECO_EUNSUPPORTED, "scale groups of fewer than 8 elements are not supported");
  (void)hipGetLastError();
  const hipError_t e = eco::launch_dequantize(weights, scales, numel, fmt, group_size, scale_dtype == ECO_DT_BF16, src,
                                              src_dtype == ECO_DT_BF16 ? 2 : 1, err, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ECO_OK : fail_hip(e, "quantization-error kernel launch");
}

eco_status_t eco_bandwidth_probe(int32_t kind, void *codes, void *scales, const void *grad, void *m, void *v, uint64_t numel,
                                 void *stream) {
  if (kind != 0 && kind != 1) return fail(ECO_EINVAL, "probe kind %d: 0 = byte-mix copy, 1 = plain copy", kind);
  if (!m || !v || (kind == 0 && (!codes || !scales || !grad))) return fail(ECO_EINVAL, "null array");
  if (!aligned16(m) || !aligned16(v) || (kind == 0 && (!aligned16(codes) || !aligned16(scales) || !aligned16(grad))))
    return fail(ECO_EALIGN, "every array must be 16-byte aligned");
  if (numel == 0 || numel % 1024 != 0 || numel / eco::ELEMS_PER_LANE > eco::MAX_LAUNCH_THREADS)
    return fail(ECO_EINVAL, "numel must be a positive multiple of 1024 below 2^35");
  eco::KernelVariant kv;
  kv.fmt = eco::FMT_FP8; kv.state_bf16 = 0; kv.scale_bf16 = 0; kv.algo = eco::ALGO_ADAM; kv.round = eco::ROUND_SR;
  const int64_t opt_lds = g_lds_bytes.load(std::memory_order_relaxed);
  const uint32_t lds = opt_lds >= 0 ? static_cast<uint32_t>(opt_lds) : lds_for_waves(default_waves(kv), 512);
  (void)hipGetLastError();
  const hipError_t e = eco::launch_bandwidth_probe(kind, codes, scales, grad, m, v, numel, lds, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ECO_OK : fail_hip(e, "probe kernel launch");
}

eco_status_t eco_arith_selftest(int32_t kind, float numerator, uint32_t bits_lo, uint32_t bits_hi, uint64_t *mismatches,
                                void *stream) {
  if (kind != 0 && kind != 1) return fail(ECO_EINVAL, "self-test kind %d: 0 = square root, 1 = division", kind);
  if (!mismatches || (reinterpret_cast<uintptr_t>(mismatches) & 7u)) return fail(ECO_EINVAL, "mismatch counter: null or not 8-byte aligned");
  if (bits_hi <= bits_lo) return fail(ECO_EINVAL, "empty range of bit patterns");
  // the ranges the short forms are used in (bit patterns of positive floats)
  const uint32_t lo = kind == 0 ? 0x0F800000u : 0x27800000u, hi = kind == 0 ? 0x6F800001u : 0x58000001u;   // 2^-96..2^96 | 2^-48..2^49
  if (bits_lo < lo || bits_hi > hi) return fail(ECO_EINVAL, "bit patterns outside the range the short form is used in");
  if (kind == 1 && !(std::fabs(numerator) >= 0x1p-40f && std::fabs(numerator) <= 0x1p40f))
    return fail(ECO_EINVAL, "numerator outside [2^-40, 2^40]");
  (void)hipGetLastError();
  const hipError_t e = eco::launch_arith_selftest(kind, numerator, bits_lo, bits_hi, reinterpret_cast<unsigned long long *>(mismatches),
                                                  static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ECO_OK : fail_hip(e, "self-test kernel launch");
}

eco_status_t eco_philox_fill(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t first_word, uint64_t n_words,
                             uint32_t *dst, void *stream) {
  if (!dst) return fail(ECO_EINVAL, "null destination");
  if (n_words == 0) return fail(ECO_EINVAL, "n_words == 0");
  if (first_word + n_words < first_word) return fail(ECO_EINVAL, "word range overflows");
  (void)hipGetLastError();
  const hipError_t e = eco::launch_philox_fill(seed, step, tensor_id, first_word, n_words, dst, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? ECO_OK : fail_hip(e, "philox kernel launch");
}

}  // extern "C"
