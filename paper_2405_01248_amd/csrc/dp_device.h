// Device-side helpers shared by the gfx950 kernels: vector types, MFMA and
// transposing-LDS-read wrappers, guarded 16-byte global loads, wave reductions,
// activation functions.  gfx950 (CDNA4) only; wave size is 64.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dp {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

#define DP_LDS __attribute__((address_space(3)))

// D[32x32] += A[32x16] * B[16x32], bf16 in, fp32 accumulate.
// Operand layout (lane l, g = l / 32): A: row l % 32, k = 8g..8g+7; B: column l % 32, k = 8g..8g+7;
// D: column l % 32, register r holds row 8 * (r / 4) + 4g + (r % 4).
__device__ __forceinline__ f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row index inside a 32x32 accumulator tile held by register r of a lane in half g.
__device__ __forceinline__ int acc_row(int r, int g) { return 8 * (r >> 2) + 4 * g + (r & 3); }

// Transposing LDS read (ds_read_b64_tr_b16).  Inside each block of 16 lanes the 16
// addresses describe a 4 x 16 tile (lanes 4r..4r+3 supply the four 4-element pieces of
// row r); lane j of the block receives column j of that tile (4 values, rows 0..3).
__device__ __forceinline__ bf16x4 lds_read_tr(const bf16* p) {
  s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16((DP_LDS s16x4*)(p));
  return __builtin_bit_cast(bf16x4, v);
}

// Fetch an MFMA A/B fragment (8 contraction values per lane) from an LDS tile stored
// [k][mn] (the non-contracted index contiguous).  `tile` points at element (k0, mn0);
// ld is the row stride in elements.  Slot u of the result is k = k0 + 8g + u.
__device__ __forceinline__ bf16x8 frag_from_mc(const bf16* tile, int ld, int lane) {
  const int b = lane >> 4, j = lane & 15;
  const bf16* p = tile + (8 * (b >> 1) + (j >> 2)) * ld + 16 * (b & 1) + 4 * (j & 3);
  bf16x4 lo = lds_read_tr(p);
  bf16x4 hi = lds_read_tr(p + 4 * ld);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Fragment fetch from an unpadded [k][mn] tile (row length ld elements, a multiple of 128) whose
// 16-byte chunks are permuted inside each k-row: chunk c of row k sits at chunk position
// c ^ (4 * (k & 3)).  The four k-rows a 32-lane half of the transposing read touches then fall
// into four different 64-byte bank groups, so the read is conflict-free without padding.
// col0 (a multiple of 32) is the first column of the fragment, k0 (a multiple of 16) its first k.
__device__ __forceinline__ int mc_swizzle(int chunk, int k) { return chunk ^ (4 * (k & 3)); }
__device__ __forceinline__ bf16x8 frag_from_mc_swz(const bf16* tile, int ld, int k0, int col0, int lane) {
  const int b = lane >> 4, j = lane & 15;
  const int k = k0 + 8 * (b >> 1) + (j >> 2);
  const int c = col0 / 8 + 2 * (b & 1) + ((j & 3) >> 1);
  const bf16* q = tile + k * ld + mc_swizzle(c, k) * 8 + 4 * (j & 1);
  bf16x4 lo = lds_read_tr(q);
  bf16x4 hi = lds_read_tr(q + 4 * ld);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Same, but the 8 contraction slots follow the accumulator row order of a 32x32 tile:
// slot u is k = k0 + 8 * (u / 4) + 4g + (u % 4)  (16 k values: two groups of 8 per g).
// This lets a C-layout register block (after conversion to bf16) act as the other operand.
__device__ __forceinline__ bf16x8 frag_from_mc_accorder(const bf16* tile, int ld, int lane) {
  const int b = lane >> 4, j = lane & 15;
  const bf16* p = tile + (4 * (b >> 1) + (j >> 2)) * ld + 16 * (b & 1) + 4 * (j & 3);
  bf16x4 lo = lds_read_tr(p);
  bf16x4 hi = lds_read_tr(p + 8 * ld);
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Asynchronous global -> LDS copy: every lane fetches 16 bytes from its own global address and the
// wave's 64 x 16 bytes land contiguously at lds_base (wave-uniform).  Completion is tracked by vmcnt.
__device__ __forceinline__ void async_copy_16B(const void* gptr, void* lds_base) {
  __builtin_amdgcn_global_load_lds(gptr, (DP_LDS void*)lds_base, 16, 0, 0);
}
// The same copy through a buffer descriptor: the source is base + lane_off + wave_off (bytes; wave_off
// wave-uniform).  Preferred over the flat-address form inside pipelined loops: with a flat-address LDS
// copy in flight the compiler treats the LDS counter as unordered and turns every wait for an LDS read
// into a wait for all of them, which defeats fragment prefetching.
typedef __amdgpu_buffer_rsrc_t rsrc_t;
__device__ __forceinline__ rsrc_t make_rsrc(const void* base, uint32_t bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}
__device__ __forceinline__ void async_copy_16B_buf(rsrc_t r, uint32_t lane_off, uint32_t wave_off, void* lds_base) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(r, (DP_LDS void*)lds_base, 16, lane_off, wave_off, 0, 0);
}
// Wait until at most N of this wave's vector-memory operations are outstanding (lgkmcnt / expcnt untouched).
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}
// Wait for all of this wave's LDS / scalar-memory operations (vmcnt / expcnt untouched).
__device__ __forceinline__ void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }
// Workgroup barrier without the memory fence of __syncthreads() (which would also wait for every
// outstanding asynchronous copy); the empty asm statements keep the compiler from moving memory
// accesses across it.
__device__ __forceinline__ void barrier_nofence() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

__device__ __forceinline__ bf16x8 zero8() {
  u32x4 z = {0, 0, 0, 0};
  return __builtin_bit_cast(bf16x8, z);
}

// 16-byte global load of 8 bf16, or zeros when !ok.
__device__ __forceinline__ bf16x8 ld8(const bf16* p, bool ok) {
  if (ok) return *reinterpret_cast<const bf16x8*>(p);
  return zero8();
}

// Branch-free guarded load: p must be a valid address in any case (the caller clamps it);
// the value is replaced by zeros when !ok.
__device__ __forceinline__ bf16x8 ld8_sel(const bf16* p, bool ok) {
  u32x4 v = *reinterpret_cast<const u32x4*>(p);
  const u32x4 z = {0, 0, 0, 0};
  v = ok ? v : z;
  return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// ---- storage conversion -------------------------------------------------
template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16>(bf16 v) { return (float)v; }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f<bf16>(float v) { return (bf16)v; }

// ---- activations (fp32) ----------------------------------------------------
enum Act { ACT_NONE = 0, ACT_GELU_ERF = 1, ACT_GELU_TANH = 2, ACT_QUICK_GELU = 3 };

// erf by the rational-times-Gaussian formula 7.1.26 of Abramowitz & Stegun (absolute error below 1.5e-7,
// i.e. about one fp32 ulp of the values it is added to here): one reciprocal, one exponential and a
// degree-5 Horner chain instead of the library routine's branches.  ex2 receives exp(-x^2) for callers
// that need the Gaussian as well.
__device__ __forceinline__ float erf_fast(float x, float& ex2) {
  const float ax = fabsf(x);
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, ax, 1.0f));
  float poly = fmaf(1.061405429f, t, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  ex2 = __builtin_amdgcn_exp2f(-1.4426950408889634f * ax * ax);
  const float r = fmaf(-poly * t, ex2, 1.0f);
  return copysignf(r, x);
}
__device__ __forceinline__ float gelu_erf_f(float z) {
  float e;
  return 0.5f * z * (1.0f + erf_fast(z * 0.70710678118654752f, e));
}
__device__ __forceinline__ float gelu_erf_grad_f(float z) {
  float e;   // exp(-z^2 / 2), the Gaussian of the density term
  const float erfv = erf_fast(z * 0.70710678118654752f, e);
  return 0.5f * (1.0f + erfv) + z * e * 0.3989422804014327f;
}
// Logistic function through the hardware exp2 and reciprocal (1 ulp each): the division of the
// textbook form costs ten instructions in IEEE mode and these functions sit in GEMM epilogues.
__device__ __forceinline__ float sigmoid_f(float z) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}
// tanh-form GELU: 0.5 z (1 + tanh(u)) = z sigmoid(2u), u = sqrt(2/pi) (z + 0.044715 z^3)
__device__ __forceinline__ float gelu_tanh_f(float z) {
  const float u2 = z * fmaf(0.0713548162726f, z * z, 1.5957691216057308f);   // 2u
  return z * sigmoid_f(u2);
}
__device__ __forceinline__ float gelu_tanh_grad_f(float z) {
  const float z2 = z * z;
  const float u2 = z * fmaf(0.0713548162726f, z2, 1.5957691216057308f);
  const float r = sigmoid_f(u2);
  const float du2 = fmaf(0.2140644488178f, z2, 1.5957691216057308f);          // d(2u)/dz
  return fmaf(z * r * (1.0f - r), du2, r);
}
__device__ __forceinline__ float quick_gelu_f(float z) { return z * sigmoid_f(1.702f * z); }
__device__ __forceinline__ float silu_f(float z) { return z * sigmoid_f(z); }
__device__ __forceinline__ float silu_grad_f(float z) {
  float s = sigmoid_f(z);
  return s * (1.0f + z * (1.0f - s));
}
__device__ __forceinline__ float act_apply(int act, float z) {
  switch (act) {
    case ACT_GELU_ERF: return gelu_erf_f(z);
    case ACT_GELU_TANH: return gelu_tanh_f(z);
    case ACT_QUICK_GELU: return quick_gelu_f(z);
    default: return z;
  }
}
__device__ __forceinline__ float act_grad(int act, float z) {
  switch (act) {
    case ACT_GELU_ERF: return gelu_erf_grad_f(z);
    case ACT_GELU_TANH: return gelu_tanh_grad_f(z);
    default: return 1.0f;
  }
}

}  // namespace dp
