// Host/device shared declarations of the ECO library: launch tables and launcher entry points.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stdint.h>

namespace eco {

enum : int { FMT_FP8 = 0, FMT_INT4 = 1, FMT_BF16_PLAIN = 2, FMT_FP32_ID = 3 };
enum : int { ROUND_SR = 0, ROUND_RTN = 1 };
// optimizer x treatment of the quantization error: Adam / SGDM with the memory-free injection (or none,
// when the injection constants are zero), SGDM with the exact stored-error injection, and the
// master-weight baselines
enum : int { ALGO_ADAM = 0, ALGO_SGDM = 1, ALGO_SGDM_EXACT = 2, ALGO_ADAM_MASTER = 3, ALGO_SGDM_MASTER = 4 };
constexpr bool algo_is_adam(int a) { return a == ALGO_ADAM || a == ALGO_ADAM_MASTER; }
constexpr bool algo_is_master(int a) { return a == ALGO_ADAM_MASTER || a == ALGO_SGDM_MASTER; }

// A tile is TILE_ELEMS consecutive elements of one tensor, processed by one workgroup of one wave,
// 8 consecutive elements per lane.  A scale group of B elements therefore occupies B/8 consecutive
// lanes (B = 32..512 fits inside the 64-lane wave).
#ifndef ECO_WG_THREADS
#define ECO_WG_THREADS 64
#endif
constexpr int WG_THREADS = ECO_WG_THREADS;
constexpr int ELEMS_PER_LANE = 8;
constexpr int TILE_ELEMS = WG_THREADS * ELEMS_PER_LANE;
// Dynamic LDS requested per workgroup of the full-tile step kernel.  The kernel does not touch it:
// the request only caps how many waves a compute unit (160 KB of LDS) holds at once.  The step is
// bound by HBM, and on MI355X the memory system delivers most when about 12 waves per compute
// unit have their 5.6 KB of loads in flight; with more resident waves the achieved bandwidth
// drops (measured: 32 waves 5.2 TB/s, 12 waves 5.7 TB/s, 8 waves 5.1 TB/s).  Used for fp32 optimizer
// state only: with bf16 state the step moves half the bytes and is bound by instruction issue.
constexpr uint32_t DEFAULT_STEP_LDS_BYTES = 13312;

// Limits of the allocation-free plan-less step (its tables live in a static device array): tensors per call,
// and launch-table entries per call (one per 512-element tile; one per scale group for groups wider than that).
#define ECO_NOALLOC_MAX_TENSORS 4096
#define ECO_NOALLOC_MAX_UNITS (1u << 20)

constexpr int MAX_WIDE_WAVES = 16;          // widest single-workgroup scale group: 16 waves * 512 = 8192 elements
constexpr uint64_t MAX_WIDE_GROUP = 8192;

struct TensorDesc {          // 80 bytes, device table entry
  void *w;                   // weights / codes
  void *s;                   // scales
  const void *g;             // bf16 gradient
  void *m;
  void *v;
  void *aux;                 // fp32: stored error (exact injection) or master weights
  uint64_t numel;
  uint64_t group_size;       // elements per scale group
  uint32_t first_unit;       // index of this tensor's first tile (or first group) in its launch list
  uint32_t tensor_id;
  uint32_t bs_shift;         // log2(group_size) for power-of-two groups of 32..512 elements
  uint32_t slot;             // tensor-wise scaling: index of the tensor's abs-max slot; wide groups: groups per workgroup
};
static_assert(sizeof(TensorDesc) == 80, "TensorDesc layout");

struct StepArgs {            // by-value kernel argument: everything wave-uniform
  const TensorDesc *tensors;
  const uint32_t *tile_tensor;     // block-scaled tensors: full tile -> index into tensors
  const uint32_t *ragged_tensor;   //   ... tensors that end in a partial tile
  const uint32_t *wide_tensor;     // wide groups of the launch in flight: group -> index into tensors
  const uint32_t *tw_tile_tensor;  // tensor-wise scaling: tile (full or partial) -> index into tensors
  const uint32_t *tw_tensor;       //   ... the tensors themselves
  uint32_t *slots;                 //   ... one abs-max slot (fp32 bit pattern) per such tensor
  uint32_t *tile_max;              //   ... scratch: the abs-max of every such tile, written and consumed within a step
  uint32_t num_tiles, num_ragged, num_tw_tiles, num_tw_tensors;
  float b1, omb1, b2, omb2, rbc2, c1, eps, kappa, lr, alpha, wd, inv_lr, inv_lr_beta;
  uint32_t seed_lo, seed_hi, step_lo;
  uint32_t div_mid;                // c1 and eps allow the short division (see div_rn_midrange) after a short square root
  uint32_t unit_base;              // first work item (group, tile, tensor) of the launch in flight, see launch_in_chunks
  // host side only
  uint64_t max_launch_threads;     // most threads one launch may have (the runtime's limit, or a smaller one set for tests)
  uint32_t lds_bytes;              // dynamic LDS per workgroup of the full-tile kernel (occupancy cap)
  uint32_t lds_bytes_wave;         // the same per wave of the wide-group kernel
  uint32_t lds_bytes_tw;           // the same per (one-wave) workgroup of the two tensor-wise passes
  const uint32_t *wide_base;       // wide-group lists, one per workgroup size, back to back
  uint32_t wide_offset[MAX_WIDE_WAVES + 1];
  uint32_t num_wide[MAX_WIDE_WAVES + 1];
};

struct KernelVariant {
  int fmt;          // FMT_*
  int state_bf16;   // m, v stored as bfloat16
  int scale_bf16;
  int algo;         // ALGO_*
  int round;        // ROUND_*
};

// Each launcher enqueues its kernels on `stream`, checks every launch, and returns the first error.
hipError_t launch_step(const KernelVariant &kv, const StepArgs &args, unsigned grid, hipStream_t stream);
hipError_t launch_quantize_init(const void *src, int src_bf16, uint64_t numel, int fmt, uint64_t group_size,
                                int scale_bf16, void *weights, void *scales, hipStream_t stream);
hipError_t launch_dequantize(const void *weights, const void *scales, uint64_t numel, int fmt, uint64_t group_size,
                             int scale_bf16, const void *src, int src_kind, float *dst, hipStream_t stream);

hipError_t launch_bandwidth_probe(int kind, void *codes, void *scales, const void *grad, void *m, void *v, uint64_t numel,
                                  uint32_t lds_bytes, hipStream_t stream);

hipError_t launch_arith_selftest(int kind, float numerator, uint32_t bits_lo, uint32_t bits_hi, unsigned long long *mismatches,
                                 hipStream_t stream);

// Scale-group classes (how the abs-max of a group is reduced)
enum : int { GROUP_BLOCK = 0, GROUP_WIDE = 1, GROUP_TENSOR = 2, GROUP_UNSUPPORTED = -1 };
inline int classify_group(uint64_t group_size, uint64_t numel) {
  if (group_size >= 32 && group_size <= 512 && (group_size & (group_size - 1)) == 0) return GROUP_BLOCK;
  const uint64_t g = group_size < numel ? group_size : numel;       // a group never exceeds the tensor
  if (g <= MAX_WIDE_GROUP && g % 8 == 0) return GROUP_WIDE;
  if (group_size >= numel) return GROUP_TENSOR;
  return GROUP_UNSUPPORTED;
}
// The helper kernels (initial quantizer, de-quantizer, error) take one launch with one workgroup per tile or per
// wide group, and the runtime wants grid x block below 2^32: about 2^35 elements a call.
constexpr uint64_t MAX_LAUNCH_THREADS = 0xFFFFFFFFull;
inline bool flat_call_fits(uint64_t numel, uint64_t group_size) {
  if (numel > (1ull << 40)) return false;
  uint64_t threads = (numel + TILE_ELEMS - 1) / TILE_ELEMS * WG_THREADS;
  if (classify_group(group_size, numel) == GROUP_WIDE) {
    const uint64_t g = group_size < numel ? group_size : numel;
    threads = (numel + g - 1) / g * 64 * ((g + TILE_ELEMS - 1) / TILE_ELEMS);
  }
  return threads <= MAX_LAUNCH_THREADS;
}
// Wide groups (a multiple of 8 up to 8192 elements, not a power of two in [32, 512]): one workgroup of `waves` waves
// steps `rows` consecutive groups.  One group a workgroup in general; groups of more than 512 elements whose length is
// not a multiple of 512 leave lanes of their last wave idle, so where 2..8 of them together fill a whole number of
// waves exactly (1408 = 2.75 waves: four rows in 11 waves; 576: eight rows in 9 waves) and the tensor is a whole number
// of such bundles, a workgroup takes the bundle.
struct WideGeometry { uint32_t rows; uint32_t waves; uint64_t units; };
inline WideGeometry wide_geometry(uint64_t numel, uint64_t g) {          // g = min(group size, numel)
  const uint64_t ngroups = (numel + g - 1) / g;
  WideGeometry w = {1u, static_cast<uint32_t>((g + TILE_ELEMS - 1) / TILE_ELEMS), ngroups};
  if (g > TILE_ELEMS && g % TILE_ELEMS != 0 && numel % g == 0) {
    for (uint32_t k = 2; k <= 8; ++k) {
      if ((k * g) % TILE_ELEMS == 0 && k * g / TILE_ELEMS <= MAX_WIDE_WAVES && ngroups % k == 0) {
        w.rows = k;
        w.waves = static_cast<uint32_t>(k * g / TILE_ELEMS);
        w.units = ngroups / k;
        break;
      }
    }
  }
  return w;
}
inline int log2_exact(uint64_t x) {
  for (int s = 0; s < 64; ++s)
    if ((1ull << s) == x) return s;
  return -1;
}
hipError_t launch_philox_fill(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t first_word, uint64_t n_words,
                              uint32_t *dst, hipStream_t stream);

// per-(fmt, state) translation units of the quantized step kernel
hipError_t launch_step_fp8_f32(const KernelVariant &, const StepArgs &, unsigned, hipStream_t);
hipError_t launch_step_fp8_bf16(const KernelVariant &, const StepArgs &, unsigned, hipStream_t);
hipError_t launch_step_int4_f32(const KernelVariant &, const StepArgs &, unsigned, hipStream_t);
hipError_t launch_step_int4_bf16(const KernelVariant &, const StepArgs &, unsigned, hipStream_t);
hipError_t launch_step_plain(const KernelVariant &, const StepArgs &, unsigned, hipStream_t);

}  // namespace eco
