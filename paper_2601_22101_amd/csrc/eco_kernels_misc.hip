// Kernels beside the fused quantized step: the unquantized ("plain") optimizer step for bf16 /
// fp32 weights, the round-to-nearest initial quantizer, the dequantizer, and the raw Philox
// stream.  They share the tile geometry and the 8-element access helpers of the step kernel.
#include "eco_step_kernel.hpp"

namespace eco {

// ------------------------------------------------------------------------ plain optimizer step
// Adam / SGDM on weights that are not quantized.  FMT_BF16_PLAIN: bf16 weights, result rounded to
// nearest even, no injection (the method is applied to linear layers only; norm weights take the
// ordinary optimizer).  FMT_FP32_ID: fp32 weights under the identity quantizer, for which the
// quantization error is zero and Alg. 2/3 add nothing to the momentum.
template <int FMT, bool STATE_BF16, bool ADAM, bool FULL>
__device__ __forceinline__ void plain_tile(const StepArgs &a, const TensorDesc &td, uint64_t e0) {
  int nvalid = 8;
  if (!FULL) {
    const int64_t left = (int64_t)td.numel - (int64_t)e0;
    nvalid = left >= 8 ? 8 : (left <= 0 ? 0 : (int)left);
  }
  float w[8], g[8], m[8], v[8];
  load_state8<FMT == FMT_BF16_PLAIN, FULL>(td.w, e0, nvalid, w);
  load_bf16x8<FULL>(static_cast<const uint16_t *>(td.g) + e0, nvalid, g);
  load_state8<STATE_BF16, FULL>(td.m, e0, nvalid, m);
  if (ADAM) load_state8<STATE_BF16, FULL>(td.v, e0, nvalid, v);
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    float wj = w[j];
    m[j] = fmaf(a.b1, m[j], a.omb1 * g[j]);
    float u;
    if (ADAM) {
      v[j] = fmaf(a.b2, v[j], a.omb2 * (g[j] * g[j]));
      const float d = sqrtf(v[j] * a.rbc2) + a.eps;
      u = (a.c1 * m[j]) / d;
    } else {
      u = a.lr * m[j];
    }
    if (a.wd != 0.0f) wj = wj - a.wd * wj;
    w[j] = wj - u;
  }
  store_state8<FMT == FMT_BF16_PLAIN, FULL>(td.w, e0, nvalid, w);
  store_state8<STATE_BF16, FULL>(td.m, e0, nvalid, m);
  if (ADAM) store_state8<STATE_BF16, FULL>(td.v, e0, nvalid, v);
}

template <int FMT, bool STATE_BF16, bool ADAM>
__global__ __launch_bounds__(WG_THREADS) void eco_plain_kernel(const StepArgs a) {
  for (uint32_t tile = blockIdx.x; tile < a.num_tiles; tile += gridDim.x) {
    const TensorDesc td = load_tensor_desc(a, load_tile_tensor(a, tile));
    const uint64_t tile_off = (uint64_t)(tile - td.first_tile) * TILE_ELEMS;
    plain_tile<FMT, STATE_BF16, ADAM, true>(a, td, tile_off + (uint64_t)threadIdx.x * ELEMS_PER_LANE);
  }
}

template <int FMT, bool STATE_BF16, bool ADAM>
__global__ __launch_bounds__(WG_THREADS) void eco_plain_ragged_kernel(const StepArgs a) {
  const ECO_CONST_AS uint32_t *rt = (const ECO_CONST_AS uint32_t *)(uintptr_t)a.ragged_tensor;
  const TensorDesc td = load_tensor_desc(a, rt[blockIdx.x]);
  const uint64_t tile_off = td.numel / TILE_ELEMS * TILE_ELEMS;
  plain_tile<FMT, STATE_BF16, ADAM, false>(a, td, tile_off + (uint64_t)threadIdx.x * ELEMS_PER_LANE);
}

hipError_t launch_step_plain(const KernelVariant &kv, const StepArgs &args, unsigned grid, hipStream_t stream) {
#define ECO_LAUNCH(F, ST, OP)                                                                                  \
  do {                                                                                                         \
    if (args.num_tiles)                                                                                        \
      hipLaunchKernelGGL((eco_plain_kernel<F, ST, OP>), dim3(grid), dim3(WG_THREADS), 0, stream, args);        \
    if (args.num_ragged)                                                                                       \
      hipLaunchKernelGGL((eco_plain_ragged_kernel<F, ST, OP>), dim3(args.num_ragged), dim3(WG_THREADS), 0,     \
                         stream, args);                                                                        \
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
  return hipGetLastError();
}

hipError_t launch_step(const KernelVariant &kv, const StepArgs &args, unsigned grid, hipStream_t stream) {
  if (kv.fmt == FMT_FP8) return kv.state_bf16 ? launch_step_fp8_bf16(kv, args, grid, stream) : launch_step_fp8_f32(kv, args, grid, stream);
  if (kv.fmt == FMT_INT4) return kv.state_bf16 ? launch_step_int4_bf16(kv, args, grid, stream) : launch_step_int4_f32(kv, args, grid, stream);
  return launch_step_plain(kv, args, grid, stream);
}

// ------------------------------------------------------------------------ initial quantizer
// q(x) of Sec. 3.1 with nearest-even rounding over one flat tensor.
template <int FMT, bool SCALE_BF16, bool SRC_BF16, bool FULL>
__device__ __forceinline__ void quantize_tile(const void *src, uint64_t numel, uint32_t bs_shift, void *weights,
                                              void *scales, uint64_t e0) {
  int nvalid = 8;
  if (!FULL) {
    const int64_t left = (int64_t)numel - (int64_t)e0;
    nvalid = left >= 8 ? 8 : (left <= 0 ? 0 : (int)left);
  }
  float x[8];
  load_state8<SRC_BF16, FULL>(src, e0, nvalid, x);
  const float amax = u2f(group_umax(f2u(absmax8(x)), 1 << (bs_shift - 3)));
  float s_new, inv;
  block_scale<FMT, SCALE_BF16>(amax, s_new, inv);
  uint32_t c[2];
  const Philox4 none = {0, 0, 0, 0};
  encode8<FMT, ROUND_RTN, false>(x, inv, none, c);
  store_codes8<FMT, FULL>(weights, e0, nvalid, c);
  const uint64_t blk = e0 >> bs_shift;
  const uint32_t lanes_mask = (1u << (bs_shift - 3)) - 1u;
  if ((threadIdx.x & lanes_mask) == 0 && (FULL || nvalid > 0)) {
    if (SCALE_BF16) static_cast<uint16_t *>(scales)[blk] = (uint16_t)(f2u(s_new) >> 16);
    else static_cast<float *>(scales)[blk] = s_new;
  }
}

template <int FMT, bool SCALE_BF16, bool SRC_BF16>
__global__ __launch_bounds__(WG_THREADS) void eco_quantize_kernel(const void *src, uint64_t numel, uint32_t bs_shift,
                                                                  void *weights, void *scales) {
  const uint64_t ntiles = (numel + TILE_ELEMS - 1) / TILE_ELEMS;
  for (uint64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint64_t tile_off = tile * TILE_ELEMS;
    const uint64_t e0 = tile_off + (uint64_t)threadIdx.x * ELEMS_PER_LANE;
    if (tile_off + TILE_ELEMS <= numel) quantize_tile<FMT, SCALE_BF16, SRC_BF16, true>(src, numel, bs_shift, weights, scales, e0);
    else quantize_tile<FMT, SCALE_BF16, SRC_BF16, false>(src, numel, bs_shift, weights, scales, e0);
  }
}

hipError_t launch_quantize_init(const void *src, int src_bf16, uint64_t numel, int fmt, uint32_t bs_shift, int scale_bf16,
                                void *weights, void *scales, unsigned grid, hipStream_t stream) {
#define ECO_LAUNCH(F, SC, SR)                                                                              \
  hipLaunchKernelGGL((eco_quantize_kernel<F, SC, SR>), dim3(grid), dim3(WG_THREADS), 0, stream, src, numel, \
                     bs_shift, weights, scales)
  const int key = (fmt == FMT_INT4 ? 4 : 0) | (scale_bf16 ? 2 : 0) | (src_bf16 ? 1 : 0);
  switch (key) {
    case 0: ECO_LAUNCH(FMT_FP8, false, false); break;
    case 1: ECO_LAUNCH(FMT_FP8, false, true); break;
    case 2: ECO_LAUNCH(FMT_FP8, true, false); break;
    case 3: ECO_LAUNCH(FMT_FP8, true, true); break;
    case 4: ECO_LAUNCH(FMT_INT4, false, false); break;
    case 5: ECO_LAUNCH(FMT_INT4, false, true); break;
    case 6: ECO_LAUNCH(FMT_INT4, true, false); break;
    default: ECO_LAUNCH(FMT_INT4, true, true); break;
  }
#undef ECO_LAUNCH
  return hipGetLastError();
}

// ------------------------------------------------------------------------ dequantizer
template <int FMT, bool SCALE_BF16, bool FULL>
__device__ __forceinline__ void dequantize_tile(const void *weights, const void *scales, uint64_t numel,
                                                uint32_t bs_shift, float *dst, uint64_t e0) {
  int nvalid = 8;
  if (!FULL) {
    const int64_t left = (int64_t)numel - (int64_t)e0;
    nvalid = left >= 8 ? 8 : (left <= 0 ? 0 : (int)left);
  }
  uint32_t c[2];
  load_codes8<FMT, FULL>(weights, e0, nvalid, c);
  const float s = (FULL || nvalid > 0) ? load_scale<SCALE_BF16>(scales, e0 >> bs_shift) : 0.0f;
  float x[8];
  x[0] = decode_elem<FMT, 0>(c) * s; x[1] = decode_elem<FMT, 1>(c) * s; x[2] = decode_elem<FMT, 2>(c) * s;
  x[3] = decode_elem<FMT, 3>(c) * s; x[4] = decode_elem<FMT, 4>(c) * s; x[5] = decode_elem<FMT, 5>(c) * s;
  x[6] = decode_elem<FMT, 6>(c) * s; x[7] = decode_elem<FMT, 7>(c) * s;
  store_f32x8<FULL>(dst + e0, nvalid, x);
}

template <int FMT, bool SCALE_BF16>
__global__ __launch_bounds__(WG_THREADS) void eco_dequantize_kernel(const void *weights, const void *scales,
                                                                    uint64_t numel, uint32_t bs_shift, float *dst) {
  const uint64_t ntiles = (numel + TILE_ELEMS - 1) / TILE_ELEMS;
  for (uint64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint64_t tile_off = tile * TILE_ELEMS;
    const uint64_t e0 = tile_off + (uint64_t)threadIdx.x * ELEMS_PER_LANE;
    if (tile_off + TILE_ELEMS <= numel) dequantize_tile<FMT, SCALE_BF16, true>(weights, scales, numel, bs_shift, dst, e0);
    else dequantize_tile<FMT, SCALE_BF16, false>(weights, scales, numel, bs_shift, dst, e0);
  }
}

hipError_t launch_dequantize(const void *weights, const void *scales, uint64_t numel, int fmt, uint32_t bs_shift,
                             int scale_bf16, float *dst, unsigned grid, hipStream_t stream) {
#define ECO_LAUNCH(F, SC)                                                                                  \
  hipLaunchKernelGGL((eco_dequantize_kernel<F, SC>), dim3(grid), dim3(WG_THREADS), 0, stream, weights, scales, \
                     numel, bs_shift, dst)
  if (fmt == FMT_FP8) { if (scale_bf16) ECO_LAUNCH(FMT_FP8, true); else ECO_LAUNCH(FMT_FP8, false); }
  else { if (scale_bf16) ECO_LAUNCH(FMT_INT4, true); else ECO_LAUNCH(FMT_INT4, false); }
#undef ECO_LAUNCH
  return hipGetLastError();
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
