// Kernels beside the fused quantized step: the unquantized ("plain") optimizer step for bf16 /
// fp32 weights, the round-to-nearest initial quantizer, the dequantizer, and the raw Philox
// stream.  They share the tile geometry and the 8-element access helpers of the step kernel.
#include <mutex>

#include "eco_step_kernel.hpp"

namespace eco {

// ------------------------------------------------------------------------ plain optimizer step
// Adam / SGDM on weights that are not quantized.  FMT_BF16_PLAIN: bf16 weights, result rounded to
// nearest even, no injection (the method is applied to linear layers only; norm weights take the
// ordinary optimizer).  FMT_FP32_ID: fp32 weights under the identity quantizer, for which the
// quantization error is zero and Alg. 2/3 add nothing to the momentum.
template <int FMT, bool STATE_BF16, bool ADAM, int ACC>
__device__ __forceinline__ void plain_tile(const StepArgs &a, const TensorDesc &td, uint64_t e0) {
  const int nvalid = ACC == ACC_FULL ? 8 : valid_from(e0, td.numel);
  float w[8], g[8], m[8], v[8];
  load_state8<FMT == FMT_BF16_PLAIN, ACC>(td.w, e0, nvalid, w);
  load_bf16x8<ACC>(static_cast<const uint16_t *>(td.g) + e0, nvalid, g);
  load_state8<STATE_BF16, ACC>(td.m, e0, nvalid, m);
  if (ADAM) load_state8<STATE_BF16, ACC>(td.v, e0, nvalid, v);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    float wj = w[j];
    m[j] = fmaf(a.b1, m[j], a.omb1 * g[j]);
    float u;
    if (ADAM) {
      v[j] = fmaf(a.b2, v[j], a.omb2 * (g[j] * g[j]));
      const float d = sqrtf(v[j] * a.rbc2) + a.eps;
      u = (a.c1 / d) * m[j];          // the element-wise step size of Sec. 3.2 times the first moment
    } else {
      u = a.lr * m[j];
    }
    if (a.wd != 0.0f) wj = wj - a.wd * wj;
    w[j] = wj - u;
  }
  store_state8<FMT == FMT_BF16_PLAIN, ACC>(td.w, e0, nvalid, w);
  store_state8<STATE_BF16, ACC>(td.m, e0, nvalid, m);
  if (ADAM) store_state8<STATE_BF16, ACC>(td.v, e0, nvalid, v);
}

template <int FMT, bool STATE_BF16, bool ADAM>
__global__ __launch_bounds__(WG_THREADS) void eco_plain_kernel(const StepArgs a) {
  for (uint32_t tile = blockIdx.x; tile < a.num_tiles; tile += gridDim.x) {
    const TensorDesc td = load_tensor_desc(a, load_table(a.tile_tensor, tile));
    const uint64_t tile_off = (uint64_t)(tile - td.first_unit) * TILE_ELEMS;
    plain_tile<FMT, STATE_BF16, ADAM, ACC_FULL>(a, td, tile_off + (uint64_t)threadIdx.x * ELEMS_PER_LANE);
  }
}

template <int FMT, bool STATE_BF16, bool ADAM>
__global__ __launch_bounds__(WG_THREADS) void eco_plain_ragged_kernel(const StepArgs a) {
  const TensorDesc td = load_tensor_desc(a, load_table(a.ragged_tensor, blockIdx.x + a.unit_base));
  const uint64_t tile_off = td.numel / TILE_ELEMS * TILE_ELEMS;
  plain_tile<FMT, STATE_BF16, ADAM, ACC_GUARDED>(a, td, tile_off + (uint64_t)threadIdx.x * ELEMS_PER_LANE);
}

hipError_t launch_step_plain(const KernelVariant &kv, const StepArgs &args, unsigned grid, hipStream_t stream) {
#define ECO_LAUNCH(F, ST, AD)                                                                                  \
  do {                                                                                                         \
    if (args.num_tiles)                                                                                        \
      ECO_LAUNCH_CHECKED((eco_plain_kernel<F, ST, AD>), dim3(capped_grid(grid, args)), dim3(WG_THREADS), 0,    \
                         stream, args);                                                                        \
    if (args.num_ragged)                                                                                       \
      ECO_CHUNKS_CHECKED((eco_plain_ragged_kernel<F, ST, AD>), args.num_ragged, WG_THREADS, 0, stream, args);  \
  } while (0)
  const int key = (kv.fmt == FMT_FP32_ID ? 4 : 0) | (kv.state_bf16 ? 2 : 0) | (algo_is_adam(kv.algo) ? 0 : 1);
  switch (key) {
    case 0: ECO_LAUNCH(FMT_BF16_PLAIN, false, true); break;
    case 1: ECO_LAUNCH(FMT_BF16_PLAIN, false, false); break;
    case 2: ECO_LAUNCH(FMT_BF16_PLAIN, true, true); break;
    case 3: ECO_LAUNCH(FMT_BF16_PLAIN, true, false); break;
    case 4: ECO_LAUNCH(FMT_FP32_ID, false, true); break;
    case 5: ECO_LAUNCH(FMT_FP32_ID, false, false); break;
    case 6: ECO_LAUNCH(FMT_FP32_ID, true, true); break;
    default: ECO_LAUNCH(FMT_FP32_ID, true, false); break;
  }
#undef ECO_LAUNCH
  return hipSuccess;
}

hipError_t launch_step(const KernelVariant &kv, const StepArgs &args, unsigned grid, hipStream_t stream) {
  if (kv.fmt == FMT_FP8) return kv.state_bf16 ? launch_step_fp8_bf16(kv, args, grid, stream) : launch_step_fp8_f32(kv, args, grid, stream);
  if (kv.fmt == FMT_INT4) return kv.state_bf16 ? launch_step_int4_bf16(kv, args, grid, stream) : launch_step_int4_f32(kv, args, grid, stream);
  return launch_step_plain(kv, args, grid, stream);
}

// ------------------------------------------------------------------------ initial quantizer
// q(x) of Sec. 3.1 with nearest-even rounding over one flat tensor, for the three classes of scale
// groups (in-wave blocks, one workgroup per wide group, one scale for the whole tensor in two passes).
// The two-pass form keeps its abs-max, between its kernels, in one of QUANT_SLOTS file-scope slots; the host
// hands the slots out in turn and makes a call wait (on its own stream) for the previous user of its slot, so
// calls on different streams never share a slot that is in use.
constexpr int QUANT_SLOTS = 64;
__device__ uint32_t g_quantize_slots[QUANT_SLOTS];     // zero at load; every call leaves its slot at zero again

template <int FMT, bool SCALE_BF16, bool SRC_BF16, int ACC, int RED>
__device__ __forceinline__ void quantize_lane(const void *src, void *weights, void *scales, uint64_t e0, int nvalid,
                                              uint64_t sg, int shift, bool scale_writer, uint32_t slot = 0) {
  float x[8];
  load_state8<SRC_BF16, ACC>(src, e0, nvalid, x);
  const float amax = group_absmax<RED>(absmax8(x), shift, &g_quantize_slots[slot]);
  if (RED == RED_ATOMIC) return;
  float s_new, inv;
  block_scale<FMT, SCALE_BF16>(amax, s_new, inv);
  uint32_t c[2];
  const Philox4 none = {0, 0, 0, 0};
  float q[8];
  encode8<FMT, ROUND_RTN, false>(x, inv, none, c, q);
  store_codes8<FMT, ACC>(weights, e0, nvalid, c);
  if (RED != RED_SLOT && scale_writer && (ACC == ACC_FULL || nvalid > 0)) {
    if (SCALE_BF16) static_cast<uint16_t *>(scales)[sg] = (uint16_t)(f2u(s_new) >> 16);
    else static_cast<float *>(scales)[sg] = s_new;
  }
}

template <int FMT, bool SCALE_BF16, bool SRC_BF16>
__global__ __launch_bounds__(WG_THREADS) void eco_quantize_kernel(const void *src, uint64_t numel, uint32_t bs_shift,
                                                                  void *weights, void *scales) {
  const uint64_t e0 = (uint64_t)blockIdx.x * TILE_ELEMS + (uint64_t)threadIdx.x * ELEMS_PER_LANE;
  const bool writer = (threadIdx.x & ((1u << (bs_shift - 3)) - 1u)) == 0;
  if ((uint64_t)(blockIdx.x + 1) * TILE_ELEMS <= numel)
    quantize_lane<FMT, SCALE_BF16, SRC_BF16, ACC_FULL, RED_BLOCK>(src, weights, scales, e0, 8, e0 >> bs_shift, (int)bs_shift, writer);
  else
    quantize_lane<FMT, SCALE_BF16, SRC_BF16, ACC_GUARDED, RED_BLOCK>(src, weights, scales, e0, valid_from(e0, numel),
                                                                     e0 >> bs_shift, (int)bs_shift, writer);
}

template <int FMT, bool SCALE_BF16, bool SRC_BF16>
__global__ __launch_bounds__(1024) void eco_quantize_wide_kernel(const void *src, uint64_t numel, uint64_t group_size,
                                                                 void *weights, void *scales) {
  const uint64_t start = (uint64_t)blockIdx.x * group_size;
  const uint64_t end = start + group_size < numel ? start + group_size : numel;
  const uint64_t e0 = start + (uint64_t)threadIdx.x * ELEMS_PER_LANE;
  quantize_lane<FMT, SCALE_BF16, SRC_BF16, ACC_LANE, RED_WG>(src, weights, scales, e0, valid_from(e0, end), blockIdx.x, 0,
                                                             threadIdx.x == 0);
}

template <int FMT, bool SCALE_BF16, bool SRC_BF16, int RED>
__global__ __launch_bounds__(WG_THREADS) void eco_quantize_tensorwise_kernel(const void *src, uint64_t numel, void *weights,
                                                                             void *scales, uint32_t slot) {
  const uint64_t e0 = (uint64_t)blockIdx.x * TILE_ELEMS + (uint64_t)threadIdx.x * ELEMS_PER_LANE;
  quantize_lane<FMT, SCALE_BF16, SRC_BF16, ACC_LANE, RED>(src, weights, scales, e0, valid_from(e0, numel), 0, 0, false, slot);
}

template <int FMT, bool SCALE_BF16>
__global__ void eco_quantize_tensorwise_scale_kernel(void *scales, uint32_t slot) {
  float s_new, inv;
  block_scale<FMT, SCALE_BF16>(u2f(g_quantize_slots[slot]), s_new, inv);
  if (SCALE_BF16) static_cast<uint16_t *>(scales)[0] = (uint16_t)(f2u(s_new) >> 16);
  else static_cast<float *>(scales)[0] = s_new;
  g_quantize_slots[slot] = 0;
}

// Hands out the abs-max slots of the two-pass quantizer.  A slot is free again once the scale kernel of its
// last user has run; the event recorded behind that kernel is what the next user of the slot waits for.
struct QuantSlotRing {
  static constexpr int MAX_DEVICES = 32;
  std::mutex mu;
  unsigned next[MAX_DEVICES] = {0};
  hipEvent_t done[MAX_DEVICES][QUANT_SLOTS] = {{nullptr}};
};
static QuantSlotRing g_quant_ring;

template <int FMT, bool SC, bool SR>
static hipError_t launch_quantize_t(const void *src, uint64_t numel, uint64_t group_size, void *weights, void *scales,
                                    hipStream_t stream) {
  const uint64_t tiles = (numel + TILE_ELEMS - 1) / TILE_ELEMS;
  const int cls = classify_group(group_size, numel);
  if (cls == GROUP_BLOCK) {
    ECO_LAUNCH_CHECKED((eco_quantize_kernel<FMT, SC, SR>), dim3((unsigned)tiles), dim3(WG_THREADS), 0, stream, src, numel,
                       (uint32_t)log2_exact(group_size), weights, scales);
  } else if (cls == GROUP_WIDE) {
    const uint64_t g = group_size < numel ? group_size : numel;
    const unsigned nw = (unsigned)((g + TILE_ELEMS - 1) / TILE_ELEMS);
    ECO_LAUNCH_CHECKED((eco_quantize_wide_kernel<FMT, SC, SR>), dim3((unsigned)((numel + g - 1) / g)), dim3(64 * nw), 0,
                       stream, src, numel, g, weights, scales);
  } else {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= QuantSlotRing::MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_quant_ring.mu);
    const uint32_t slot = g_quant_ring.next[dev]++ % QUANT_SLOTS;
    hipEvent_t &done = g_quant_ring.done[dev][slot];
    if (done) {
      e = hipStreamWaitEvent(stream, done, 0);          // the slot's previous user, on whatever stream it ran
      if (e != hipSuccess) return e;
    } else {
      e = hipEventCreateWithFlags(&done, hipEventDisableTiming);
      if (e != hipSuccess) { done = nullptr; return e; }
    }
    ECO_LAUNCH_CHECKED((eco_quantize_tensorwise_kernel<FMT, SC, SR, RED_ATOMIC>), dim3((unsigned)tiles), dim3(WG_THREADS), 0,
                       stream, src, numel, weights, scales, slot);
    ECO_LAUNCH_CHECKED((eco_quantize_tensorwise_kernel<FMT, SC, SR, RED_SLOT>), dim3((unsigned)tiles), dim3(WG_THREADS), 0,
                       stream, src, numel, weights, scales, slot);
    ECO_LAUNCH_CHECKED((eco_quantize_tensorwise_scale_kernel<FMT, SC>), dim3(1), dim3(1), 0, stream, scales, slot);
    e = hipEventRecord(done, stream);
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_quantize_init(const void *src, int src_bf16, uint64_t numel, int fmt, uint64_t group_size, int scale_bf16,
                                void *weights, void *scales, hipStream_t stream) {
  const int key = (fmt == FMT_INT4 ? 4 : 0) | (scale_bf16 ? 2 : 0) | (src_bf16 ? 1 : 0);
  switch (key) {
    case 0: return launch_quantize_t<FMT_FP8, false, false>(src, numel, group_size, weights, scales, stream);
    case 1: return launch_quantize_t<FMT_FP8, false, true>(src, numel, group_size, weights, scales, stream);
    case 2: return launch_quantize_t<FMT_FP8, true, false>(src, numel, group_size, weights, scales, stream);
    case 3: return launch_quantize_t<FMT_FP8, true, true>(src, numel, group_size, weights, scales, stream);
    case 4: return launch_quantize_t<FMT_INT4, false, false>(src, numel, group_size, weights, scales, stream);
    case 5: return launch_quantize_t<FMT_INT4, false, true>(src, numel, group_size, weights, scales, stream);
    case 6: return launch_quantize_t<FMT_INT4, true, false>(src, numel, group_size, weights, scales, stream);
    default: return launch_quantize_t<FMT_INT4, true, true>(src, numel, group_size, weights, scales, stream);
  }
}

// ------------------------------------------------------------------------ dequantizer, quantization error
// SRC == 0: dst[i] = dec(code_i) * scale[i / group_size] (Sec. 3.1, x^ = s*y).
// SRC == 1 / 2: dst[i] = src[i] - dec(code_i) * scale[i / group_size] for an fp32 / bf16 source: the
// quantization error e = theta - q(theta) of the notation paragraph of Sec. 3.1 (one multiplication, one
// subtraction, each rounded to fp32).
// A lane's 8 elements may straddle two groups when the group size is not a multiple of 8, so the scale
// index is taken per element.
template <int FMT, bool SCALE_BF16, int SRC>
__global__ __launch_bounds__(WG_THREADS) void eco_dequantize_kernel(const void *weights, const void *scales,
                                                                    uint64_t numel, uint64_t group_size, const void *src,
                                                                    float *dst) {
  const uint64_t e0 = (uint64_t)blockIdx.x * TILE_ELEMS + (uint64_t)threadIdx.x * ELEMS_PER_LANE;
  const int nvalid = valid_from(e0, numel);
  if (nvalid == 0) return;
  uint32_t c[2];
  load_codes8<FMT, ACC_LANE>(weights, e0, nvalid, c);
  const uint64_t sg = e0 / group_size;
  const uint64_t boundary = (sg + 1) * group_size - e0;     // elements of this lane before the next group starts
  const float s0 = load_scale<SCALE_BF16>(scales, sg);
  const float s1 = boundary < (uint64_t)nvalid ? load_scale<SCALE_BF16>(scales, sg + 1) : s0;
  float x[8];
  x[0] = decode_elem<FMT, 0>(c); x[1] = decode_elem<FMT, 1>(c); x[2] = decode_elem<FMT, 2>(c); x[3] = decode_elem<FMT, 3>(c);
  x[4] = decode_elem<FMT, 4>(c); x[5] = decode_elem<FMT, 5>(c); x[6] = decode_elem<FMT, 6>(c); x[7] = decode_elem<FMT, 7>(c);
#pragma unroll
  for (int j = 0; j < 8; ++j) x[j] *= ((uint64_t)j < boundary ? s0 : s1);
  if (SRC != 0) {
    float t[8];
    load_state8<SRC == 2, ACC_LANE>(src, e0, nvalid, t);
#pragma unroll
    for (int j = 0; j < 8; ++j) x[j] = t[j] - x[j];
  }
  store_f32x8<ACC_LANE>(dst + e0, nvalid, x);
}

// src_kind: 0 = no source (plain de-quantization), 1 = fp32 source, 2 = bf16 source (dst = src - q)
hipError_t launch_dequantize(const void *weights, const void *scales, uint64_t numel, int fmt, uint64_t group_size,
                             int scale_bf16, const void *src, int src_kind, float *dst, hipStream_t stream) {
  const unsigned tiles = (unsigned)((numel + TILE_ELEMS - 1) / TILE_ELEMS);
#define ECO_LAUNCH(F, SC, SK)                                                                                          \
  ECO_LAUNCH_CHECKED((eco_dequantize_kernel<F, SC, SK>), dim3(tiles), dim3(WG_THREADS), 0, stream, weights, scales, numel, \
                     group_size, src, dst)
#define ECO_LAUNCH_SRC(F, SC)                                                                                          \
  do {                                                                                                                 \
    if (src_kind == 0) ECO_LAUNCH(F, SC, 0); else if (src_kind == 1) ECO_LAUNCH(F, SC, 1); else ECO_LAUNCH(F, SC, 2);  \
  } while (0)
  if (fmt == FMT_FP8) { if (scale_bf16) ECO_LAUNCH_SRC(FMT_FP8, true); else ECO_LAUNCH_SRC(FMT_FP8, false); }
  else { if (scale_bf16) ECO_LAUNCH_SRC(FMT_INT4, true); else ECO_LAUNCH_SRC(FMT_INT4, false); }
#undef ECO_LAUNCH_SRC
#undef ECO_LAUNCH
  return hipSuccess;
}

// ------------------------------------------------------------------------ bandwidth probes
// Measurement aids: what the memory system delivers for the step's own access pattern with the arithmetic
// taken out.  MIX: every lane loads what a lane of the FP8 / fp32-state Adam step loads for its 8 elements
// (8 B codes, 16 B gradient, 2 x 16 B m, 2 x 16 B v, the block's scale) and stores what it stores (codes, m, v,
// scale), in the same tile geometry and under the same occupancy cap: 11.03 bytes read and 9.03 written per
// element.  COPY: the plain two-stream copy, 16 B per lane and instruction (4 B read, 4 B written per element).
__global__ __launch_bounds__(WG_THREADS, 8) void eco_probe_mix_kernel(const uint2 *codes, float *scales, const uint4 *grad,
                                                                      float4 *m, float4 *v, uint2 *codes_out) {
  const uint64_t i = (uint64_t)blockIdx.x * WG_THREADS + threadIdx.x;        // the lane's 8-element piece
  __builtin_amdgcn_s_setprio(3);
  const uint4 g = grad[i];
  float4 m0 = m[2 * i], m1 = m[2 * i + 1], v0 = v[2 * i], v1 = v[2 * i + 1];
  uint2 c = codes[i];
  const float s = scales[i >> 4];
  __builtin_amdgcn_s_setprio(0);
  // every loaded value reaches a store, so that no load can be dropped
  c.x ^= g.x ^ g.z; c.y ^= g.y ^ g.w;
  m0.x += s * 0.0f;
  codes_out[i] = c;
  m[2 * i] = v0; m[2 * i + 1] = v1; v[2 * i] = m0; v[2 * i + 1] = m1;
  if ((threadIdx.x & 15) == 0) scales[i >> 4] = s;
}

__global__ __launch_bounds__(256) void eco_probe_copy_kernel(const float4 *src, float4 *dst) {
  const uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x;
  dst[i] = src[i];
}

hipError_t launch_bandwidth_probe(int kind, void *codes, void *scales, const void *grad, void *m, void *v, uint64_t numel,
                                  uint32_t lds_bytes, hipStream_t stream) {
  if (kind == 0) {
    ECO_LAUNCH_CHECKED(eco_probe_mix_kernel, dim3((unsigned)(numel / TILE_ELEMS)), dim3(WG_THREADS), lds_bytes, stream,
                       static_cast<const uint2 *>(codes), static_cast<float *>(scales), static_cast<const uint4 *>(grad),
                       static_cast<float4 *>(m), static_cast<float4 *>(v), static_cast<uint2 *>(codes));
  } else {
    ECO_LAUNCH_CHECKED(eco_probe_copy_kernel, dim3((unsigned)(numel / 1024)), dim3(256), 0, stream,
                       static_cast<const float4 *>(m), static_cast<float4 *>(v));
  }
  return hipSuccess;
}

// ------------------------------------------------------------------------ arithmetic self-test
// The step kernels replace sqrtf() and `/` by shorter sequences inside stated operand ranges; these kernels
// compare the short forms with the long ones for every fp32 bit pattern of [bits_lo, bits_hi) and count the
// patterns on which they differ (expected: none).
template <int KIND>
__global__ __launch_bounds__(256) void eco_selftest_kernel(float numerator, uint32_t bits_lo, uint32_t bits_hi,
                                                           unsigned long long *mismatches) {
  const uint64_t n = (uint64_t)bits_hi - bits_lo;
  unsigned bad = 0;
  for (uint64_t i = (uint64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (uint64_t)gridDim.x * 256) {
    const float x = u2f(bits_lo + (uint32_t)i);
    float fast, ref;
    if (KIND == 0) { fast = sqrt_rn_midrange(x); ref = sqrtf(x); }
    else { fast = div_rn_midrange(numerator, x); ref = numerator / x; }
    bad += f2u(fast) != f2u(ref);
  }
  if (bad) atomicAdd(mismatches, (unsigned long long)bad);
}

hipError_t launch_arith_selftest(int kind, float numerator, uint32_t bits_lo, uint32_t bits_hi, unsigned long long *mismatches,
                                 hipStream_t stream) {
  if (kind == 0)
    ECO_LAUNCH_CHECKED(eco_selftest_kernel<0>, dim3(256 * 16), dim3(256), 0, stream, numerator, bits_lo, bits_hi, mismatches);
  else
    ECO_LAUNCH_CHECKED(eco_selftest_kernel<1>, dim3(256 * 16), dim3(256), 0, stream, numerator, bits_lo, bits_hi, mismatches);
  return hipSuccess;
}

// ------------------------------------------------------------------------ raw Philox stream
__global__ __launch_bounds__(WG_THREADS) void eco_philox_kernel(uint32_t seed_lo, uint32_t seed_hi, uint32_t step_lo,
                                                                uint32_t tensor_id, uint64_t first_word,
                                                                uint64_t n_words, uint32_t *dst) {
  // thread t produces call (first_word >> 2) + t and writes those of its four words that are in range
  const uint64_t first_call = first_word >> 2;
  const uint64_t last_word = first_word + n_words;   // exclusive
  const uint64_t ncalls = ((last_word + 3) >> 2) - first_call;
  for (uint64_t t = (uint64_t)blockIdx.x * WG_THREADS + threadIdx.x; t < ncalls; t += (uint64_t)gridDim.x * WG_THREADS) {
    const uint64_t q = first_call + t;
    const Philox4 r = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), step_lo, tensor_id, seed_lo, seed_hi);
    const uint32_t w[4] = {r.w0, r.w1, r.w2, r.w3};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uint64_t j = q * 4 + k;
      if (j >= first_word && j < last_word) dst[j - first_word] = w[k];
    }
  }
}

hipError_t launch_philox_fill(uint64_t seed, uint64_t step, uint32_t tensor_id, uint64_t first_word, uint64_t n_words,
                              uint32_t *dst, hipStream_t stream) {
  const uint64_t ncalls = ((first_word + n_words + 3) >> 2) - (first_word >> 2);
  uint64_t grid = (ncalls + WG_THREADS - 1) / WG_THREADS;
  if (grid > 65536) grid = 65536;
  if (grid == 0) grid = 1;
  hipLaunchKernelGGL(eco_philox_kernel, dim3((unsigned)grid), dim3(WG_THREADS), 0, stream, (uint32_t)seed,
                     (uint32_t)(seed >> 32), (uint32_t)step, tensor_id, first_word, n_words, dst);
  return hipGetLastError();
}

}  // namespace eco
