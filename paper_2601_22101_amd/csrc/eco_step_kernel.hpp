// The fused ECO step kernel for quantized tensors (FP8-E4M3 or INT4 codes with per-block scales).
//
// One pass over memory per step: every lane owns 8 consecutive elements, loads their codes,
// gradient and optimizer state, de-quantizes, applies the optimizer update (Alg. 1 line 1 with
// the Adam form of Sec. 3.2, or the SGDM recurrences of Sec. 3.3.1), reduces the block's abs-max
// across the B/8 lanes that share a scale (Sec. 3.1, s = max|x|/rho), re-quantizes with
// stochastic or nearest-even rounding, forms the quantization error and injects it into the
// first moment (Alg. 3 line 5 / Alg. 2 line 5), and stores codes, scale, m and v.
//
// The arithmetic is a fixed sequence of single IEEE fp32 operations (the build disables
// contraction; fused multiply-adds are explicit), so that the codes and scales it produces can
// be reproduced bit for bit elsewhere:
//   w  = dec(code) * s_old            g = f32(bf16 gradient)
//   m~ = fma(b1, m, omb1*g)           v~ = fma(b2, v, omb2*(g*g))
//   d  = sqrt(v~ * rbc2) + eps        eta_t = c1 / d;  u = eta_t * m~   [SGDM: u = lr * m~]
//   theta~ = w - u                    [with decay: (w - wd*w) - u]
//   a = max|theta~| over the block;   s' = a / rho;  inv = rho / a
//       [bf16 scales: s' = bf16(a/rho), inv = 1/s'];  if inv is not finite: s' = inv = 0
//   y = theta~ * inv;  code' = round(y);  q = dec(code') * s';  e = theta~ - q
//   m^ = fma(kappa*d, e, m~)          [SGDM: fma(alpha, e, m~)]
// Variants (template parameter ALGO):
//   exact injection (Appendix A, SGDM):  m^ = fma(-inv_lr_beta, e, fma(inv_lr, e_old, m~)), e stored for the next step
//   master weights (Sec. 3.1):           w is read from / theta~ written to an fp32 master copy, m^ = m~
#pragma once
#include "eco_device.hpp"
#include "eco_internal.hpp"

namespace eco {

template <int FMT> struct FmtTraits;
template <> struct FmtTraits<FMT_FP8> { static constexpr float RHO = 448.0f; };
template <> struct FmtTraits<FMT_INT4> { static constexpr float RHO = 7.0f; };

// ------------------------------------------------------------------ 8-element loads and stores
// Access modes of a lane's 8 consecutive elements:
//   ACC_FULL    all 8 exist in every lane: vector access, no checks (full tiles)
//   ACC_GUARDED only the first `nvalid` (possibly <= 0) exist: element-wise access in every lane; missing
//               elements read as zero and are not written (the ragged tail of a tensor)
//   ACC_LANE    decided per lane: vector access where nvalid == 8, element-wise elsewhere (wide groups,
//               whose last lanes may lie beyond the group)
enum : int { ACC_FULL = 0, ACC_GUARDED = 1, ACC_LANE = 2 };

template <int ACC>
__device__ __forceinline__ bool use_vector(int nvalid) {
  return ACC == ACC_FULL || (ACC == ACC_LANE && nvalid == 8);
}

template <int ACC>
__device__ __forceinline__ void load_f32x8(const float *p, int nvalid, float (&out)[8]) {
  if (use_vector<ACC>(nvalid)) {
    const float4 a = reinterpret_cast<const float4 *>(p)[0];
    const float4 b = reinterpret_cast<const float4 *>(p)[1];
    out[0] = a.x; out[1] = a.y; out[2] = a.z; out[3] = a.w;
    out[4] = b.x; out[5] = b.y; out[6] = b.z; out[7] = b.w;
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) out[j] = j < nvalid ? p[j] : 0.0f;
  }
}

template <int ACC>
__device__ __forceinline__ void load_bf16x8(const uint16_t *p, int nvalid, float (&out)[8]) {
  if (use_vector<ACC>(nvalid)) {
    const uint4 q = *reinterpret_cast<const uint4 *>(p);
    out[0] = bf16_lo(q.x); out[1] = bf16_hi(q.x); out[2] = bf16_lo(q.y); out[3] = bf16_hi(q.y);
    out[4] = bf16_lo(q.z); out[5] = bf16_hi(q.z); out[6] = bf16_lo(q.w); out[7] = bf16_hi(q.w);
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j) out[j] = j < nvalid ? u2f((uint32_t)p[j] << 16) : 0.0f;
  }
}

// Tuning builds only (-DECO_NT_STORES): full-tile vector stores carry the non-temporal hint.
typedef float eco_f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t eco_u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t eco_u32x2_t __attribute__((ext_vector_type(2)));
template <class V>
__device__ __forceinline__ void store_vec(V *p, V x) {
#ifdef ECO_NT_STORES
  __builtin_nontemporal_store(x, p);
#else
  *p = x;
#endif
}

template <int ACC>
__device__ __forceinline__ void store_f32x8(float *p, int nvalid, const float (&x)[8]) {
  if (use_vector<ACC>(nvalid)) {
    store_vec(reinterpret_cast<eco_f32x4_t *>(p), eco_f32x4_t{x[0], x[1], x[2], x[3]});
    store_vec(reinterpret_cast<eco_f32x4_t *>(p) + 1, eco_f32x4_t{x[4], x[5], x[6], x[7]});
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < nvalid) p[j] = x[j];
  }
}

template <int ACC>
__device__ __forceinline__ void store_bf16x8(uint16_t *p, int nvalid, const float (&x)[8]) {
  uint32_t h[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) h[j] = f32x2_to_bf16x2_rne(x[2 * j], x[2 * j + 1]);
  if (use_vector<ACC>(nvalid)) {
    store_vec(reinterpret_cast<eco_u32x4_t *>(p), eco_u32x4_t{h[0], h[1], h[2], h[3]});
  } else {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < nvalid) p[j] = (uint16_t)(h[j >> 1] >> (16 * (j & 1)));
  }
}

template <bool BF16, int ACC>
__device__ __forceinline__ void load_state8(const void *base, uint64_t e0, int nvalid, float (&out)[8]) {
  if (BF16) load_bf16x8<ACC>(static_cast<const uint16_t *>(base) + e0, nvalid, out);
  else load_f32x8<ACC>(static_cast<const float *>(base) + e0, nvalid, out);
}

template <bool BF16, int ACC>
__device__ __forceinline__ void store_state8(void *base, uint64_t e0, int nvalid, const float (&x)[8]) {
  if (BF16) store_bf16x8<ACC>(static_cast<uint16_t *>(base) + e0, nvalid, x);
  else store_f32x8<ACC>(static_cast<float *>(base) + e0, nvalid, x);
}

// 8 codes of one lane: two dwords of E4M3 bytes, or one dword of INT4 nibbles (in c[0]).
template <int FMT, int ACC>
__device__ __forceinline__ void load_codes8(const void *base, uint64_t e0, int nvalid, uint32_t (&c)[2]) {
  const uint8_t *p = static_cast<const uint8_t *>(base) + (FMT == FMT_FP8 ? e0 : (e0 >> 1));
  if (use_vector<ACC>(nvalid)) {
    if (FMT == FMT_FP8) {
      const uint2 q = *reinterpret_cast<const uint2 *>(p);
      c[0] = q.x; c[1] = q.y;
    } else {
      c[0] = *reinterpret_cast<const uint32_t *>(p); c[1] = 0;
    }
  } else {
    c[0] = 0; c[1] = 0;
    const int nbytes = FMT == FMT_FP8 ? nvalid : (nvalid + 1) >> 1;
    constexpr int MAXB = FMT == FMT_FP8 ? 8 : 4;
#pragma unroll
    for (int k = 0; k < MAXB; ++k)
      if (k < nbytes) c[k >> 2] |= (uint32_t)p[k] << (8 * (k & 3));
  }
}

template <int FMT, int ACC>
__device__ __forceinline__ void store_codes8(void *base, uint64_t e0, int nvalid, const uint32_t (&c)[2]) {
  uint8_t *p = static_cast<uint8_t *>(base) + (FMT == FMT_FP8 ? e0 : (e0 >> 1));
  if (use_vector<ACC>(nvalid)) {
    if (FMT == FMT_FP8) store_vec(reinterpret_cast<eco_u32x2_t *>(p), eco_u32x2_t{c[0], c[1]});
    else store_vec(reinterpret_cast<uint32_t *>(p), c[0]);
  } else {
    const int nbytes = FMT == FMT_FP8 ? nvalid : (nvalid + 1) >> 1;
    constexpr int MAXB = FMT == FMT_FP8 ? 8 : 4;
#pragma unroll
    for (int k = 0; k < MAXB; ++k)
      if (k < nbytes) p[k] = (uint8_t)(c[k >> 2] >> (8 * (k & 3)));
  }
}

template <int FMT, int J>
__device__ __forceinline__ float decode_elem(const uint32_t (&c)[2]) {
  if (FMT == FMT_FP8) return e4m3_decode<(J & 3)>(c[J >> 2]);
  return int4_decode_sixteenth<J>(c[0], c[0] >> 4) * 16.0f;
}

// The decoded values dq_j of a lane's 8 codes and the factor sc with w_j = dq_j * sc (INT4 decodes to
// sixteenths, so sc = 16 s there: exact, see int4_decode_sixteenth).
template <int FMT>
__device__ __forceinline__ float decode8(const uint32_t (&c)[2], float s, float (&dq)[8]) {
  if (FMT == FMT_FP8) {
    dq[0] = e4m3_decode<0>(c[0]); dq[1] = e4m3_decode<1>(c[0]); dq[2] = e4m3_decode<2>(c[0]); dq[3] = e4m3_decode<3>(c[0]);
    dq[4] = e4m3_decode<0>(c[1]); dq[5] = e4m3_decode<1>(c[1]); dq[6] = e4m3_decode<2>(c[1]); dq[7] = e4m3_decode<3>(c[1]);
    return s;
  }
  uint32_t hi = c[0] >> 4;
  asm volatile("" : "+v"(hi));          // keep the shifted copy in a register: each nibble is then one byte-select away
  dq[0] = int4_decode_sixteenth<0>(c[0], hi); dq[1] = int4_decode_sixteenth<1>(c[0], hi);
  dq[2] = int4_decode_sixteenth<2>(c[0], hi); dq[3] = int4_decode_sixteenth<3>(c[0], hi);
  dq[4] = int4_decode_sixteenth<4>(c[0], hi); dq[5] = int4_decode_sixteenth<5>(c[0], hi);
  dq[6] = int4_decode_sixteenth<6>(c[0], hi); dq[7] = int4_decode_sixteenth<7>(c[0], hi);
  return s * 16.0f;
}

template <bool BF16>
__device__ __forceinline__ float load_scale(const void *scales, uint64_t blk) {
  if (BF16) return u2f((uint32_t)static_cast<const uint16_t *>(scales)[blk] << 16);
  return static_cast<const float *>(scales)[blk];
}

// abs-max scale of a block from a = max|x| (identical in all lanes of the block)
template <int FMT, bool SCALE_BF16>
__device__ __forceinline__ void block_scale(float a, float &s_new, float &inv) {
  constexpr float RHO = FmtTraits<FMT>::RHO;
  s_new = a / RHO;
  if (SCALE_BF16) {
    s_new = u2f(f32_to_bf16_rne(s_new) << 16);
    inv = 1.0f / s_new;
  } else {
    inv = RHO / a;
  }
  if (!(inv < __builtin_inff())) { s_new = 0.0f; inv = 0.0f; }   // a == 0, or rho/a overflows
}

__device__ __forceinline__ float absmax8(const float (&x)[8]) {
  float a = __builtin_fmaxf(__builtin_fabsf(x[0]), __builtin_fabsf(x[1]));
#pragma unroll
  for (int j = 2; j < 8; ++j) a = __builtin_fmaxf(a, __builtin_fabsf(x[j]));
  return a;
}

__device__ __forceinline__ float absmin8(const float (&x)[8]) {
  float a = __builtin_fminf(__builtin_fabsf(x[0]), __builtin_fabsf(x[1]));
#pragma unroll
  for (int j = 2; j < 8; ++j) a = __builtin_fminf(a, __builtin_fabsf(x[j]));
  return a;
}

// Encode y_j = x_j * inv (j = 0..7) onto the grid: packed codes in c, and in q the values the new codes decode
// to (before scaling).  r = the lane's Philox words.
template <int FMT, int ROUND, bool NORMAL_ONLY>
__device__ __forceinline__ void encode8(const float (&x)[8], float inv, const Philox4 &r, uint32_t (&c)[2], float (&q)[8]) {
  const uint32_t rw[4] = {r.w0, r.w1, r.w2, r.w3};
  c[1] = 0;
  if (FMT == FMT_FP8) {
    // inv >= 0, so the sign of y is the sign of x
    uint32_t t[8];
#define ECO_FP8_ELEM(J) t[J] = e4m3_encode_top<ROUND, NORMAL_ONLY, (J & 1)>(__builtin_fabsf(x[J]) * inv, rw[J >> 1], f2u(x[J]));
    ECO_FP8_ELEM(0) ECO_FP8_ELEM(1) ECO_FP8_ELEM(2) ECO_FP8_ELEM(3)
    ECO_FP8_ELEM(4) ECO_FP8_ELEM(5) ECO_FP8_ELEM(6) ECO_FP8_ELEM(7)
#undef ECO_FP8_ELEM
    c[0] = pack_top_bytes4(t[0], t[1], t[2], t[3]);
    c[1] = pack_top_bytes4(t[4], t[5], t[6], t[7]);
    q[0] = e4m3_decode<0>(c[0]); q[1] = e4m3_decode<1>(c[0]); q[2] = e4m3_decode<2>(c[0]); q[3] = e4m3_decode<3>(c[0]);
    q[4] = e4m3_decode<0>(c[1]); q[5] = e4m3_decode<1>(c[1]); q[6] = e4m3_decode<2>(c[1]); q[7] = e4m3_decode<3>(c[1]);
  } else {
    uint32_t even = 0, odd = 0;
#define ECO_INT4_ELEM(J)                                                                              \
    q[J] = int4_round<ROUND, (J & 1)>(x[J] * inv, rw[J >> 1]);                                        \
    int4_insert<J>(q[J], even, odd);
    ECO_INT4_ELEM(0) ECO_INT4_ELEM(1) ECO_INT4_ELEM(2) ECO_INT4_ELEM(3)
    ECO_INT4_ELEM(4) ECO_INT4_ELEM(5) ECO_INT4_ELEM(6) ECO_INT4_ELEM(7)
#undef ECO_INT4_ELEM
    c[0] = int4_pack(even, odd);
  }
}

// d_j = sqrt(x_j) + eps for eight non-negative x.  When every x of the wave lies in the range of
// sqrt_rn_midrange the short sequence is used; both branches return the correctly rounded root.
// Returns whether the short sequence was used (wave-uniform): then every x of the wave lies in [2^-96, 2^96].
__device__ __forceinline__ bool sqrt_plus_eps8(const float (&x)[8], float eps, float (&d)[8]) {
  uint32_t lo = f2u(x[0]), hi = f2u(x[0]);
#pragma unroll
  for (int j = 1; j < 8; ++j) {
    const uint32_t b = f2u(x[j]);
    lo = lo < b ? lo : b;
    hi = hi > b ? hi : b;
  }
  if (wave_all(lo >= SQRT_MID_LO && hi <= SQRT_MID_HI)) {
#pragma unroll
    for (int j = 0; j < 8; ++j) d[j] = sqrt_rn_midrange(x[j]) + eps;
    return true;
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) d[j] = sqrtf(x[j]) + eps;
  return false;
}

// ------------------------------------------------------------------ the step of one lane
// How the abs-max of a scale group is obtained:
//   RED_BLOCK  the group is 2^shift elements inside one wave: DPP/swizzle all-reduce over its lanes
//   RED_WG     the group is the whole workgroup (1..16 waves): wave all-reduce, then an LDS combine
//   RED_WG_ROWS the workgroup holds 2..8 whole groups of more than 512 elements each (a wave meets at most two of
//              them): per wave one all-reduce for each of its groups, LDS atomic max into the group's entry
//   RED_ATOMIC first pass of a group larger than a workgroup, one group at a time (the initial quantizer):
//              wave all-reduce, one atomic max per wave into the group's slot; nothing else is written
//   RED_TILE   first pass of the step for such groups (tensor-wise scaling): wave all-reduce, the wave's
//              maximum goes to its tile's entry of a scratch array, which a small kernel folds into the
//              tensor's slot (tens of thousands of atomics on one address serialize in the memory system)
//   RED_SLOT   second pass: the abs-max is read from that slot; everything is recomputed and written
//              except the scale (a last, tiny kernel writes it once every tile has used the old one)
enum : int { RED_BLOCK = 0, RED_WG = 1, RED_ATOMIC = 2, RED_SLOT = 3, RED_TILE = 4, RED_WG_ROWS = 5 };

// arg: RED_BLOCK: log2(group size); RED_WG_ROWS: which of the workgroup's groups the lane belongs to.
template <int RED>
__device__ __forceinline__ float group_absmax(float lane_max, int arg, uint32_t *slot) {
  if (RED == RED_BLOCK) return u2f(group_umax(f2u(lane_max), 1 << (arg - 3)));
  if (RED == RED_SLOT) return u2f(*slot);
  if (RED == RED_WG_ROWS) {
    __shared__ uint32_t row_max[8];
    if (threadIdx.x < 8) row_max[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t x = f2u(lane_max);
    const int first = __builtin_amdgcn_readfirstlane(arg), last = __builtin_amdgcn_readlane(arg, 63);
    const uint32_t m_first = group_umax(arg == first ? x : 0u, 64);
    if ((threadIdx.x & 63) == 0) atomicMax(&row_max[first], m_first);
    if (last != first) {                                      // wave-uniform
      const uint32_t m_last = group_umax(arg == last ? x : 0u, 64);
      if ((threadIdx.x & 63) == 0) atomicMax(&row_max[last], m_last);
    }
    __syncthreads();
    return u2f(row_max[arg]);
  }
  const uint32_t wmax = group_umax(f2u(lane_max), 64);
  if (RED == RED_ATOMIC) {
    // the slot only grows, so a wave whose maximum does not exceed what the slot already holds has
    // nothing to add; the read goes to the device-coherent cache level, and the atomic is what decides
    if ((threadIdx.x & 63) == 0 && wmax > __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT))
      atomicMax(slot, wmax);
    return 0.0f;
  }
  if (RED == RED_TILE) {
    if ((threadIdx.x & 63) == 0) *slot = wmax;
    return 0.0f;
  }
  // RED_WG
  __shared__ uint32_t wave_max[16];
  const int nwaves = (int)(blockDim.x >> 6);
  if (nwaves == 1) return u2f(wmax);
  if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = wmax;
  __syncthreads();
  uint32_t r = wave_max[0];
  for (int k = 1; k < nwaves; ++k) { const uint32_t o = wave_max[k]; r = r > o ? r : o; }
  return u2f(r);
}

// One lane's 8 consecutive elements, starting at element e0 of tensor td, of which the first nvalid exist;
// scale group number sg; bs_shift = log2(group size) for RED_BLOCK; row = the lane's group within the workgroup for
// RED_WG_ROWS.
template <int FMT, bool STATE_BF16, bool SCALE_BF16, int ALGO, int ROUND, int ACC, int RED>
__device__ __forceinline__ void step_lane(const StepArgs &a, const TensorDesc &td, uint64_t e0, int nvalid,
                                          uint64_t sg, bool scale_writer, uint32_t *slot, int row = 0) {
  constexpr bool ADAM = algo_is_adam(ALGO);
  constexpr bool MASTER = algo_is_master(ALGO);
  constexpr bool WRITE = RED != RED_ATOMIC && RED != RED_TILE;   // the first pass of a two-pass group writes nothing
  const bool any = ACC == ACC_FULL || nvalid > 0;

  // A bf16 scale has 8 significant bits and a decoded code at most 4, so dec(c) * s is exact in fp32 (also where
  // it is subnormal: its lowest bit is at least 2^-142) and theta~ = w - u and e = theta~ - dec(c') s' may be
  // formed by one fused multiply-add each: the same real number is rounded once either way.  Until then w holds
  // the decoded values and sc the factor.
  constexpr bool EXACT_SCALE = SCALE_BF16 && !MASTER;
  float g[8], m[8], v[8], w[8], sc = 1.0f;
  load_bf16x8<ACC>(static_cast<const uint16_t *>(td.g) + e0, nvalid, g);
  load_state8<STATE_BF16, ACC>(td.m, e0, nvalid, m);
  if (ADAM) load_state8<STATE_BF16, ACC>(td.v, e0, nvalid, v);
  if (MASTER) {
    load_f32x8<ACC>(static_cast<const float *>(td.aux) + e0, nvalid, w);
  } else {
    uint32_t c[2];
    load_codes8<FMT, ACC>(td.w, e0, nvalid, c);
    const float s_old = any ? load_scale<SCALE_BF16>(td.s, sg) : 0.0f;
    sc = decode8<FMT>(c, s_old, w);
    if (!EXACT_SCALE) {
#pragma unroll
      for (int j = 0; j < 8; ++j) w[j] *= sc;
    }
  }

  __builtin_amdgcn_s_setprio(0);      // loads issued: back to the default priority (see eco_step_kernel)

  // OPTIM_STEP on the de-quantized (or master) weights
  float th[8], d[8], eta[8];
  if (ADAM) {
    float x[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      m[j] = fmaf(a.b1, m[j], a.omb1 * g[j]);
      v[j] = fmaf(a.b2, v[j], a.omb2 * (g[j] * g[j]));
      x[j] = v[j] * a.rbc2;
    }
    if (WRITE) store_state8<STATE_BF16, ACC>(td.v, e0, nvalid, v);   // v is final (Alg. 3 returns it unchanged)
    // the element-wise step size of Sec. 3.2, eta_t = (eta / (1 - b1^k)) / (sqrt(v^) + eps).  After the short square
    // root every d of the wave lies in [2^-48, 2^48 + eps], and div_mid says that eps <= 1 and c1 is in range
    if (sqrt_plus_eps8(x, a.eps, d) && a.div_mid) {
#pragma unroll
      for (int j = 0; j < 8; ++j) eta[j] = div_rn_midrange(a.c1, d[j]);
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) eta[j] = a.c1 / d[j];
    }
  }
  float u[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    if (ADAM) {
      u[j] = eta[j] * m[j];
    } else {
      m[j] = fmaf(a.b1, m[j], a.omb1 * g[j]);
      d[j] = 0.0f;
      u[j] = a.lr * m[j];
    }
  }
  // decoupled decay is off in most runs, so it is kept a (wave-uniform) branch: the empty asm statements stop
  // the compiler from turning the blocks into multiply-subtract-select triples
  if (EXACT_SCALE && a.wd == 0.0f) {
    asm volatile("" ::: "memory");
#pragma unroll
    for (int j = 0; j < 8; ++j) th[j] = fmaf(w[j], sc, -u[j]);
  } else {
    if (EXACT_SCALE) {
#pragma unroll
      for (int j = 0; j < 8; ++j) w[j] *= sc;
    }
    if (a.wd != 0.0f) {
      asm volatile("" ::: "memory");
#pragma unroll
      for (int j = 0; j < 8; ++j) w[j] = w[j] - a.wd * w[j];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) th[j] = w[j] - u[j];
  }
  if (ACC != ACC_FULL) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j >= nvalid) th[j] = 0.0f;
  }

  // ECO_QUANTIZE
  const float amax = group_absmax<RED>(absmax8(th), RED == RED_WG_ROWS ? row : (int)td.bs_shift, slot);
  if (!WRITE) return;
  if (MASTER) store_f32x8<ACC>(static_cast<float *>(td.aux) + e0, nvalid, th);
  float s_new, inv;
  block_scale<FMT, SCALE_BF16>(amax, s_new, inv);

  Philox4 r = {0, 0, 0, 0};
  if (ROUND == ROUND_SR) {
    const uint64_t q = e0 >> 3;
    // tensors of up to 2^35 elements (a wave-uniform, scalar test): the high counter word is zero, so the words
    // that enter the first two rounds beside q are all wave-uniform and their products are scalar work (the
    // empty asm statement keeps the two calls apart: merged, the zero would become a per-lane select)
    if (td.numel <= (1ull << 35)) {
      r = philox4x32_10((uint32_t)q, 0u, a.step_lo, td.tensor_id, a.seed_lo, a.seed_hi);
      asm volatile("" ::: "memory");
    } else {
      r = philox4x32_10((uint32_t)q, (uint32_t)(q >> 32), a.step_lo, td.tensor_id, a.seed_lo, a.seed_hi);
    }
  }
  uint32_t cn[2];
  float qn[8];
  if (FMT == FMT_FP8) {
    // the E4M3 subnormal range (|y| < 2^-6) needs a second formula; it is rare, so decide per wave
    // (multiplication by inv >= 0 is monotone, so the smallest |y| is fl(min|theta~| * inv))
    if (wave_any(absmin8(th) * inv < 0x1p-6f)) encode8<FMT, ROUND, false>(th, inv, r, cn, qn);
    else encode8<FMT, ROUND, true>(th, inv, r, cn, qn);
  } else {
    encode8<FMT, ROUND, true>(th, inv, r, cn, qn);
  }
  store_codes8<FMT, ACC>(td.w, e0, nvalid, cn);

  if (!MASTER) {
    float eo[8];
    if (ALGO == ALGO_SGDM_EXACT) load_f32x8<ACC>(static_cast<const float *>(td.aux) + e0, nvalid, eo);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float e = SCALE_BF16 ? fmaf(-qn[j], s_new, th[j]) : th[j] - qn[j] * s_new;   // exact product, see above
      if (ALGO == ALGO_ADAM) m[j] = fmaf(a.kappa * d[j], e, m[j]);
      else if (ALGO == ALGO_SGDM) m[j] = fmaf(a.alpha, e, m[j]);
      else { m[j] = fmaf(-a.inv_lr_beta, e, fmaf(a.inv_lr, eo[j], m[j])); eo[j] = e; }
    }
    if (ALGO == ALGO_SGDM_EXACT) store_f32x8<ACC>(static_cast<float *>(td.aux) + e0, nvalid, eo);
  }
  store_state8<STATE_BF16, ACC>(td.m, e0, nvalid, m);

  if (RED != RED_SLOT && scale_writer && any) {
    if (SCALE_BF16) static_cast<uint16_t *>(td.s)[sg] = (uint16_t)(f2u(s_new) >> 16);
    else static_cast<float *>(td.s)[sg] = s_new;
  }
}

// The launch tables are read-only for the lifetime of a launch; reading them through the constant
// address space lets the compiler fetch them with scalar loads (one per wave, into SGPRs) even
// though the kernel also writes global memory.
#define ECO_CONST_AS __attribute__((address_space(4)))

__device__ __forceinline__ uint32_t load_table(const uint32_t *table, uint32_t i) {
  const ECO_CONST_AS uint32_t *p = (const ECO_CONST_AS uint32_t *)(uintptr_t)table;
  return p[i];
}

__device__ __forceinline__ TensorDesc load_tensor_desc(const StepArgs &a, uint32_t ti) {
  const ECO_CONST_AS uint64_t *p = (const ECO_CONST_AS uint64_t *)(uintptr_t)(a.tensors + ti);
  TensorDesc td;
  td.w = (void *)(uintptr_t)p[0];
  td.s = (void *)(uintptr_t)p[1];
  td.g = (const void *)(uintptr_t)p[2];
  td.m = (void *)(uintptr_t)p[3];
  td.v = (void *)(uintptr_t)p[4];
  td.aux = (void *)(uintptr_t)p[5];
  td.numel = p[6];
  td.group_size = p[7];
  const uint64_t a8 = p[8], a9 = p[9];
  td.first_unit = (uint32_t)a8;
  td.tensor_id = (uint32_t)(a8 >> 32);
  td.bs_shift = (uint32_t)a9;
  td.slot = (uint32_t)(a9 >> 32);
  return td;
}

// ------------------------------------------------------------------ kernels
// (1) Block-scaled tensors (group = 32..512 elements, a power of two): one workgroup of one wave per
// full 512-element tile, dispatched in address order (or, when the host caps the grid, looping with
// the grid as stride).  The tile -> tensor table and the descriptors are wave-uniform scalar loads.
template <int FMT, bool STATE_BF16, bool SCALE_BF16, int ALGO, int ROUND>
__global__ __launch_bounds__(WG_THREADS, 8) void eco_step_kernel(const StepArgs a) {
  for (uint32_t tile = blockIdx.x; tile < a.num_tiles; tile += gridDim.x) {
    // A wave that has not issued its loads yet goes first: its address arithmetic and load instructions
    // are not queued behind the arithmetic of the waves that already have their data (the priority is
    // dropped again in step_lane, once the loads are issued).  Measured: +0.3 % and a flatter optimum
    // over the occupancy cap.
    __builtin_amdgcn_s_setprio(3);
    const TensorDesc td = load_tensor_desc(a, load_table(a.tile_tensor, tile));
    const uint64_t e0 = (uint64_t)(tile - td.first_unit) * TILE_ELEMS + (uint64_t)threadIdx.x * ELEMS_PER_LANE;
    const bool writer = (threadIdx.x & ((1u << (td.bs_shift - 3)) - 1u)) == 0;
    step_lane<FMT, STATE_BF16, SCALE_BF16, ALGO, ROUND, ACC_FULL, RED_BLOCK>(a, td, e0, 8, e0 >> td.bs_shift, writer, nullptr);
  }
}

// (2) The last, partial tile of each block-scaled tensor whose length is not a multiple of TILE_ELEMS:
// one workgroup per such tensor, element-wise guarded accesses.  A separate kernel keeps the guards'
// registers and branches out of the full-tile kernel.
__device__ __forceinline__ int valid_from(uint64_t e0, uint64_t end) {
  const int64_t left = (int64_t)end - (int64_t)e0;
  return left >= 8 ? 8 : (left <= 0 ? 0 : (int)left);
}

template <int FMT, bool STATE_BF16, bool SCALE_BF16, int ALGO, int ROUND>
__global__ __launch_bounds__(WG_THREADS) void eco_step_ragged_kernel(const StepArgs a) {
  const TensorDesc td = load_tensor_desc(a, load_table(a.ragged_tensor, blockIdx.x + a.unit_base));
  const uint64_t e0 = td.numel / TILE_ELEMS * TILE_ELEMS + (uint64_t)threadIdx.x * ELEMS_PER_LANE;
  const bool writer = (threadIdx.x & ((1u << (td.bs_shift - 3)) - 1u)) == 0;
  step_lane<FMT, STATE_BF16, SCALE_BF16, ALGO, ROUND, ACC_GUARDED, RED_BLOCK>(a, td, e0, valid_from(e0, td.numel),
                                                                              e0 >> td.bs_shift, writer, nullptr);
}

// (3) Wide groups (any multiple of 8 up to 8192 elements: row-wise scaling, Sec. 4.1): one workgroup of
// ceil(group/512) waves per group, abs-max by wave all-reduce plus an LDS combine across the waves -- or, where the
// plan found that 2..8 groups fill a whole number of waves exactly (TensorDesc::slot, see wide_geometry), one
// workgroup per such bundle of groups, every lane busy.
template <int FMT, bool STATE_BF16, bool SCALE_BF16, int ALGO, int ROUND>
__global__ __launch_bounds__(1024) void eco_step_wide_kernel(const StepArgs a) {
  __builtin_amdgcn_s_setprio(3);      // as in eco_step_kernel: loading waves first
  const uint32_t unit = blockIdx.x + a.unit_base;
  const TensorDesc td = load_tensor_desc(a, load_table(a.wide_tensor, unit));
  const uint32_t rows = td.slot;
  const uint64_t grp = (uint64_t)(unit - td.first_unit) * rows;       // the workgroup's first group
  const uint64_t start = grp * td.group_size;
  const uint32_t lane_elem = threadIdx.x * ELEMS_PER_LANE;
  const uint64_t e0 = start + lane_elem;
  if (rows > 1) {
    const uint32_t gs = (uint32_t)td.group_size;
    uint32_t row = 0;
    for (uint32_t k = 1; k < rows; ++k) row += lane_elem >= k * gs ? 1u : 0u;
    step_lane<FMT, STATE_BF16, SCALE_BF16, ALGO, ROUND, ACC_FULL, RED_WG_ROWS>(a, td, e0, 8, grp + row, lane_elem == row * gs, nullptr,
                                                                               (int)row);
    return;
  }
  const uint64_t end = start + td.group_size < td.numel ? start + td.group_size : td.numel;
  // a group that fills every lane of the workgroup (e.g. rows of 1024, 2048, 4096) needs no per-lane guards
  if (end - start == (uint64_t)blockDim.x * ELEMS_PER_LANE)
    step_lane<FMT, STATE_BF16, SCALE_BF16, ALGO, ROUND, ACC_FULL, RED_WG>(a, td, e0, 8, grp, threadIdx.x == 0, nullptr);
  else
    step_lane<FMT, STATE_BF16, SCALE_BF16, ALGO, ROUND, ACC_LANE, RED_WG>(a, td, e0, valid_from(e0, end), grp,
                                                                          threadIdx.x == 0, nullptr);
}

// (4) One scale per tensor (tensor-wise scaling, Sec. 4.4), tensors too large for one workgroup: two passes
// over 512-element tiles.  Pass 1 recomputes theta~ and leaves each tile's abs-max in a scratch array, which
// a reduction kernel (one workgroup per tensor) folds into the tensor's slot; pass 2 recomputes theta~ again
// (the inputs are untouched so far), quantizes against the slot's value and writes codes and state; a last
// kernel writes the new scales.
template <int FMT, bool STATE_BF16, bool SCALE_BF16, int ALGO, int ROUND, int RED>
__global__ __launch_bounds__(WG_THREADS) void eco_step_tensorwise_kernel(const StepArgs a) {
  __builtin_amdgcn_s_setprio(3);      // as in eco_step_kernel: loading waves first
  const uint32_t unit = blockIdx.x + a.unit_base;
  const TensorDesc td = load_tensor_desc(a, load_table(a.tw_tile_tensor, unit));
  const uint64_t tile_off = (uint64_t)(unit - td.first_unit) * TILE_ELEMS;
  const uint64_t e0 = tile_off + (uint64_t)threadIdx.x * ELEMS_PER_LANE;
  uint32_t *slot = RED == RED_TILE ? a.tile_max + unit : a.slots + td.slot;
  if (tile_off + TILE_ELEMS <= td.numel)
    step_lane<FMT, STATE_BF16, SCALE_BF16, ALGO, ROUND, ACC_FULL, RED>(a, td, e0, 8, 0, false, slot);
  else
    step_lane<FMT, STATE_BF16, SCALE_BF16, ALGO, ROUND, ACC_GUARDED, RED>(a, td, e0, valid_from(e0, td.numel), 0, false, slot);
}

constexpr int TW_REDUCE_THREADS = 1024;
template <int FMT>   // a template only so that every translation unit may hold its own copy
__global__ __launch_bounds__(TW_REDUCE_THREADS) void eco_tensorwise_reduce_kernel(const StepArgs a) {
  const TensorDesc td = load_tensor_desc(a, a.tw_tensor[blockIdx.x + a.unit_base]);
  const uint64_t ntiles = (td.numel + TILE_ELEMS - 1) / TILE_ELEMS;
  const uint32_t *tm = a.tile_max + td.first_unit;
  uint32_t r = 0;
  for (uint64_t i = threadIdx.x; i < ntiles; i += TW_REDUCE_THREADS) { const uint32_t x = tm[i]; r = r > x ? r : x; }
  r = group_umax(r, 64);
  __shared__ uint32_t wave_max[TW_REDUCE_THREADS / 64];
  if ((threadIdx.x & 63) == 0) wave_max[threadIdx.x >> 6] = r;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int k = 1; k < TW_REDUCE_THREADS / 64; ++k) { const uint32_t o = wave_max[k]; r = r > o ? r : o; }
    a.slots[td.slot] = r;
  }
}

template <int FMT, bool SCALE_BF16>
__global__ __launch_bounds__(WG_THREADS) void eco_tensorwise_scale_kernel(const StepArgs a) {
  const uint32_t i = (blockIdx.x + a.unit_base) * WG_THREADS + threadIdx.x;
  if (i >= a.num_tw_tensors) return;
  const TensorDesc td = load_tensor_desc(a, a.tw_tensor[i]);
  float s_new, inv;
  block_scale<FMT, SCALE_BF16>(u2f(a.slots[td.slot]), s_new, inv);
  if (SCALE_BF16) static_cast<uint16_t *>(td.s)[0] = (uint16_t)(f2u(s_new) >> 16);
  else static_cast<float *>(td.s)[0] = s_new;
}

inline unsigned lds_cap(unsigned bytes) { return bytes < 65536u ? bytes : 65536u; }   // per-workgroup request limit

// Every launch is followed by its own error check, so that a failed launch stops the sequence and is the
// error that is reported.
#define ECO_LAUNCH_CHECKED(kernel, grid, block, lds, stream, ...)                                                 \
  do {                                                                                                            \
    hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                                            \
    const hipError_t launch_err_ = hipGetLastError();                                                             \
    if (launch_err_ != hipSuccess) return launch_err_;                                                            \
  } while (0)

// One work item per workgroup, `units` of them: as many launches as the limit on the threads of one launch asks
// for (the runtime wants grid x block below 2^32), each told where it starts through StepArgs::unit_base.
template <class Kernel>
hipError_t launch_in_chunks(Kernel kernel, uint64_t units, unsigned block, unsigned lds, hipStream_t stream, StepArgs args) {
  const uint64_t per_launch = args.max_launch_threads / block ? args.max_launch_threads / block : 1;
  for (uint64_t base = 0; base < units; base += per_launch) {
    args.unit_base = static_cast<uint32_t>(base);
    const uint64_t n = units - base < per_launch ? units - base : per_launch;
    ECO_LAUNCH_CHECKED(kernel, dim3(static_cast<unsigned>(n)), dim3(block), lds, stream, args);
  }
  return hipSuccess;
}
#define ECO_CHUNKS_CHECKED(...)                                  \
  do {                                                           \
    const hipError_t chunk_err_ = launch_in_chunks(__VA_ARGS__); \
    if (chunk_err_ != hipSuccess) return chunk_err_;             \
  } while (0)

// The full-tile kernels loop over tiles with the grid as stride, so they take one launch with a capped grid.
inline unsigned capped_grid(unsigned grid, const StepArgs &args) {
  const uint64_t most = args.max_launch_threads / WG_THREADS ? args.max_launch_threads / WG_THREADS : 1;
  return grid > most ? static_cast<unsigned>(most) : grid;
}

template <int FMT, bool STATE_BF16, bool SC, int RD, int AL>
hipError_t launch_step_kernels(const StepArgs &args, unsigned grid, hipStream_t stream) {
  if (args.num_tiles)
    ECO_LAUNCH_CHECKED((eco_step_kernel<FMT, STATE_BF16, SC, AL, RD>), dim3(capped_grid(grid, args)), dim3(WG_THREADS),
                       args.lds_bytes, stream, args);
  if (args.num_ragged)
    ECO_CHUNKS_CHECKED((eco_step_ragged_kernel<FMT, STATE_BF16, SC, AL, RD>), args.num_ragged, WG_THREADS, 0, stream, args);
  for (int nw = 1; nw <= MAX_WIDE_WAVES; ++nw) {
    if (!args.num_wide[nw]) continue;
    StepArgs wa = args;
    wa.wide_tensor = args.wide_base + args.wide_offset[nw];
    ECO_CHUNKS_CHECKED((eco_step_wide_kernel<FMT, STATE_BF16, SC, AL, RD>), args.num_wide[nw], 64 * nw,
                       lds_cap(args.lds_bytes_wave * nw), stream, wa);
  }
  if (args.num_tw_tiles) {
    ECO_CHUNKS_CHECKED((eco_step_tensorwise_kernel<FMT, STATE_BF16, SC, AL, RD, RED_TILE>), args.num_tw_tiles, WG_THREADS,
                       args.lds_bytes_tw, stream, args);
    ECO_CHUNKS_CHECKED((eco_tensorwise_reduce_kernel<FMT>), args.num_tw_tensors, TW_REDUCE_THREADS, 0, stream, args);
    ECO_CHUNKS_CHECKED((eco_step_tensorwise_kernel<FMT, STATE_BF16, SC, AL, RD, RED_SLOT>), args.num_tw_tiles, WG_THREADS,
                       args.lds_bytes_tw, stream, args);
    ECO_CHUNKS_CHECKED((eco_tensorwise_scale_kernel<FMT, SC>), (args.num_tw_tensors + WG_THREADS - 1) / WG_THREADS, WG_THREADS,
                       0, stream, args);
  }
  return hipSuccess;
}

template <int FMT, bool STATE_BF16, bool SC, int RD>
hipError_t launch_step_algos(const KernelVariant &kv, const StepArgs &args, unsigned grid, hipStream_t stream) {
  switch (kv.algo) {
    case ALGO_ADAM: return launch_step_kernels<FMT, STATE_BF16, SC, RD, ALGO_ADAM>(args, grid, stream);
    case ALGO_SGDM: return launch_step_kernels<FMT, STATE_BF16, SC, RD, ALGO_SGDM>(args, grid, stream);
    case ALGO_SGDM_EXACT: return launch_step_kernels<FMT, STATE_BF16, SC, RD, ALGO_SGDM_EXACT>(args, grid, stream);
    case ALGO_ADAM_MASTER: return launch_step_kernels<FMT, STATE_BF16, SC, RD, ALGO_ADAM_MASTER>(args, grid, stream);
    default: return launch_step_kernels<FMT, STATE_BF16, SC, RD, ALGO_SGDM_MASTER>(args, grid, stream);
  }
}

template <int FMT, bool STATE_BF16>
hipError_t launch_step_variants(const KernelVariant &kv, const StepArgs &args, unsigned grid, hipStream_t stream) {
  const int key = (kv.scale_bf16 ? 2 : 0) | (kv.round == ROUND_RTN ? 1 : 0);
  switch (key) {
    case 0: return launch_step_algos<FMT, STATE_BF16, false, ROUND_SR>(kv, args, grid, stream);
    case 1: return launch_step_algos<FMT, STATE_BF16, false, ROUND_RTN>(kv, args, grid, stream);
    case 2: return launch_step_algos<FMT, STATE_BF16, true, ROUND_SR>(kv, args, grid, stream);
    default: return launch_step_algos<FMT, STATE_BF16, true, ROUND_RTN>(kv, args, grid, stream);
  }
}

}  // namespace eco
