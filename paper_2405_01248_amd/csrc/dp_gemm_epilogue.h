// Epilogue shared by the MFMA GEMM kernels and the implicit-GEMM convolution: what happens to a
// tile of fp32 accumulators on its way to memory (bias, saved pre-activation, activation and its
// derivative, gate, residual, GeGLU forward / backward, split-K partial tiles, fp32 or storage-dtype
// output), and the XCD-aware map from workgroup id to output tile.  Device code only; included by the kernel translation units.
#pragma once
#include "dp_device.h"

namespace dp {

template <typename T>
struct EpiParams {
  int M, N;
  T* out; int ldo;
  float* out32; int ldo32; int accumulate;
  float* partial;                 // split-K partial tiles [z][M][N] when gridDim.z > 1
  const T* bias;
  T* pre_out; int ld_pre;
  int act;
  const T* dact_pre; int ld_dact; int dact_kind;
  const T* gate; int gate_ld; int rows_per_batch;
  const void* residual; int ld_res; int residual_f32; int out_fused_f32;
  int geglu, geglu_inner; const T* geglu_u; int ld_geglu;
  float out_scale;                // the accumulators are multiplied by this before anything else (1 except for fp8 operands)
};

// Scalar epilogue (fp32 path).
template <typename T>
__device__ __forceinline__ void epi_store(const EpiParams<T>& e, int m, int n, float v) {
  if (m < e.M && n < e.N) {
    if (e.partial) e.partial[((size_t)blockIdx.z * e.M + m) * e.N + n] = v;
    else if (e.out32) {
      float* p = e.out32 + (size_t)m * e.ldo32 + n;
      *p = e.accumulate ? (*p + v) : v;
    } else {
      if (e.bias) v += to_f<T>(e.bias[n]);
      if (e.pre_out) e.pre_out[(size_t)m * e.ld_pre + n] = from_f<T>(v);
      if (e.act) v = act_apply(e.act, v);
      if (e.dact_pre) v *= act_grad(e.dact_kind, to_f<T>(e.dact_pre[(size_t)m * e.ld_dact + n]));
      if (e.gate) v *= to_f<T>(e.gate[(size_t)(m / e.rows_per_batch) * e.gate_ld + n]);
      if (e.residual) v += to_f<T>(((const T*)e.residual)[(size_t)m * e.ld_res + n]);
      e.out[(size_t)m * e.ldo + n] = from_f<T>(v);
    }
  }
}

// Vector epilogue (bf16 path): 8 consecutive columns of row m starting at column n, all in bounds.
__device__ __forceinline__ void epi_vec8(const EpiParams<bf16>& e, int m, int n, float* v) {
  if (e.partial || e.out32) {
    float* o = e.partial ? e.partial + ((size_t)blockIdx.z * e.M + m) * e.N + n : e.out32 + (size_t)m * e.ldo32 + n;
    if (!e.partial && e.accumulate) {
      const f32x4 o0 = *reinterpret_cast<const f32x4*>(o), o1 = *reinterpret_cast<const f32x4*>(o + 4);
#pragma unroll
      for (int t = 0; t < 4; ++t) { v[t] += o0[t]; v[4 + t] += o1[t]; }
    }
    *reinterpret_cast<f32x4*>(o) = *reinterpret_cast<const f32x4*>(&v[0]);
    *reinterpret_cast<f32x4*>(o + 4) = *reinterpret_cast<const f32x4*>(&v[4]);
    return;
  }
  if (e.out_scale != 1.0f) {
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] *= e.out_scale;
  }
  if (e.bias) {
    const bf16x8 bv = *reinterpret_cast<const bf16x8*>(e.bias + n);
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] += (float)bv[t];
  }
  if (e.geglu == 2) {
    // v is dg[m, n .. n + 7]; the two halves of du come from the saved projection u = [value | gate]
    const bf16* up = e.geglu_u + (size_t)m * e.ld_geglu + n;
    const bf16x8 uv = *reinterpret_cast<const bf16x8*>(up), ug = *reinterpret_cast<const bf16x8*>(up + e.geglu_inner);
    bf16x8 o0, o1;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const float gt = (float)ug[t];
      o0[t] = (bf16)(v[t] * gelu_erf_f(gt));
      o1[t] = (bf16)(v[t] * (float)uv[t] * gelu_erf_grad_f(gt));
    }
    bf16* op = e.out + (size_t)m * e.ldo + n;
    *reinterpret_cast<bf16x8*>(op) = o0;
    *reinterpret_cast<bf16x8*>(op + e.geglu_inner) = o1;
    return;
  }
  if (e.pre_out) {
    bf16x8 o;
#pragma unroll
    for (int t = 0; t < 8; ++t) o[t] = (bf16)v[t];
    *reinterpret_cast<bf16x8*>(e.pre_out + (size_t)m * e.ld_pre + n) = o;
  }
  if (e.act) {
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] = act_apply(e.act, v[t]);
  }
  if (e.dact_pre) {
    const bf16x8 pv = *reinterpret_cast<const bf16x8*>(e.dact_pre + (size_t)m * e.ld_dact + n);
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] *= act_grad(e.dact_kind, (float)pv[t]);
  }
  if (e.gate) {
    const bf16x8 gv = *reinterpret_cast<const bf16x8*>(e.gate + (size_t)(m / e.rows_per_batch) * e.gate_ld + n);
#pragma unroll
    for (int t = 0; t < 8; ++t) v[t] *= (float)gv[t];
  }
  if (e.residual) {
    if (e.residual_f32) {
      const float* rp = (const float*)e.residual + (size_t)m * e.ld_res + n;
      const f32x4 r0 = *reinterpret_cast<const f32x4*>(rp), r1 = *reinterpret_cast<const f32x4*>(rp + 4);
#pragma unroll
      for (int t = 0; t < 4; ++t) { v[t] += r0[t]; v[4 + t] += r1[t]; }
    } else {
      const bf16x8 rv = *reinterpret_cast<const bf16x8*>((const bf16*)e.residual + (size_t)m * e.ld_res + n);
#pragma unroll
      for (int t = 0; t < 8; ++t) v[t] += (float)rv[t];
    }
  }
  if (e.out_fused_f32) {
    float* op = reinterpret_cast<float*>(e.out) + (size_t)m * e.ldo + n;
    *reinterpret_cast<f32x4*>(op) = *reinterpret_cast<const f32x4*>(&v[0]);
    *reinterpret_cast<f32x4*>(op + 4) = *reinterpret_cast<const f32x4*>(&v[4]);
  } else {
    bf16x8 o;
#pragma unroll
    for (int t = 0; t < 8; ++t) o[t] = (bf16)v[t];
    *reinterpret_cast<bf16x8*>(e.out + (size_t)m * e.ldo + n) = o;
  }
}

// Epilogue shared by the MFMA kernels.  A wave stages one 32-row slab of its accumulators at a time
// through its own fp32 LDS region Cw ([32][C_LD], reusing the operand tiles once every wave of the
// workgroup is past its last fragment read) and re-reads it as 8 consecutive columns per lane, so
// bias / residual / saved pre-activation loads and all stores are 16-byte accesses.  LDS requests
// of one wave are served in order, so no barrier is needed between a slab's writes and reads; the
// empty asm statements only stop the compiler from reordering them.  The store loop is kept rolled:
// unrolled, the activation and gradient variants would be replicated per 8-column group and the
// kernel would outgrow the instruction cache.
template <int TM, int TN, int WN, int C_LD>
__device__ __forceinline__ void wave_epilogue(const f32x16 (&acc)[TM][TN], float* Cw, const EpiParams<bf16>& e, int row0,
                                              int col0, int lane) {
  const int g = lane >> 5, l32 = lane & 31;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) Cw[(8 * (r >> 2) + 4 * g + (r & 3)) * C_LD + j * 32 + l32] = acc[i][j][r];
    asm volatile("" ::: "memory");
    if (WN == 64 && e.geglu == 1) {
      // Forward GeGLU: the tile's columns are permuted so that this wave's first 32 columns are values
      // and its last 32 the gates of the same outputs j0 .. j0 + 31 (see the B loader).
      const int j0 = col0 / 2;
#pragma unroll 1
      for (int it = 0; it < 2; ++it) {
        const int id = it * 64 + lane;
        const int lr = id >> 2, lc = (id & 3) * 8;
        const int m = row0 + i * 32 + lr, j = j0 + lc;
        if (m < e.M && j < e.geglu_inner) {
          float va[8], ga[8];
          *reinterpret_cast<f32x4*>(&va[0]) = *reinterpret_cast<const f32x4*>(&Cw[lr * C_LD + lc]);
          *reinterpret_cast<f32x4*>(&va[4]) = *reinterpret_cast<const f32x4*>(&Cw[lr * C_LD + lc + 4]);
          *reinterpret_cast<f32x4*>(&ga[0]) = *reinterpret_cast<const f32x4*>(&Cw[lr * C_LD + 32 + lc]);
          *reinterpret_cast<f32x4*>(&ga[4]) = *reinterpret_cast<const f32x4*>(&Cw[lr * C_LD + 32 + lc + 4]);
          if (e.bias) {
            const bf16x8 bv = *reinterpret_cast<const bf16x8*>(e.bias + j), bg = *reinterpret_cast<const bf16x8*>(e.bias + e.geglu_inner + j);
#pragma unroll
            for (int t = 0; t < 8; ++t) { va[t] += (float)bv[t]; ga[t] += (float)bg[t]; }
          }
          bf16x8 uv, ug, o;
#pragma unroll
          for (int t = 0; t < 8; ++t) {
            uv[t] = (bf16)va[t]; ug[t] = (bf16)ga[t];
            o[t] = (bf16)((float)uv[t] * gelu_erf_f((float)ug[t]));
          }
          if (e.pre_out) {
            bf16* up = e.pre_out + (size_t)m * e.ld_pre + j;
            *reinterpret_cast<bf16x8*>(up) = uv;
            *reinterpret_cast<bf16x8*>(up + e.geglu_inner) = ug;
          }
          *reinterpret_cast<bf16x8*>(e.out + (size_t)m * e.ldo + j) = o;
        }
      }
      asm volatile("" ::: "memory");
      continue;
    }
#pragma unroll 1
    for (int it = 0; it < 32 * WN / 8 / 64; ++it) {
      const int id = it * 64 + lane;
      const int lr = id / (WN / 8), lc = (id % (WN / 8)) * 8;
      const int m = row0 + i * 32 + lr, n = col0 + lc;
      if (m < e.M && n < e.N) {
        float v[8];
        *reinterpret_cast<f32x4*>(&v[0]) = *reinterpret_cast<const f32x4*>(&Cw[lr * C_LD + lc]);
        *reinterpret_cast<f32x4*>(&v[4]) = *reinterpret_cast<const f32x4*>(&Cw[lr * C_LD + lc + 4]);
        epi_vec8(e, m, n, v);
      }
    }
    asm volatile("" ::: "memory");
  }
}

// Maps the linear workgroup id to an output tile.  Hardware deals consecutive ids round-robin
// to the 8 XCDs; the remap gives each XCD a contiguous range of tiles, ordered in groups of
// `group_m` tile-rows (walked down the rows, then to the next column) so that concurrently running
// tiles share A and B panels in that XCD's L2.
// First half: position of workgroup pid in an order of n items in which every XCD owns a contiguous range.
__device__ __forceinline__ int xcd_contiguous_id(int pid, int n) {
  const int ppx = (n + 7) / 8, tall = n % 8;
  const int xcd = pid % 8, local = pid / 8;
  return (tall == 0 || xcd < tall) ? xcd * ppx + local : tall * ppx + (xcd - tall) * (ppx - 1) + local;
}
// Second half: tile of position id in the grouped order.
__device__ __forceinline__ void tile_of_id(int id, int tiles_m, int tiles_n, int group_m, int& tm, int& tn) {
  const int in_group = group_m * tiles_n;
  const int first_m = (id / in_group) * group_m;
  const int gsz = min(tiles_m - first_m, group_m);
  tm = first_m + (id % in_group) % gsz;
  tn = (id % in_group) / gsz;
}
__device__ __forceinline__ void tile_of_block(int pid, int tiles_m, int tiles_n, int group_m, int& tm, int& tn) {
  tile_of_id(xcd_contiguous_id(pid, tiles_m * tiles_n), tiles_m, tiles_n, group_m, tm, tn);
}

}  // namespace dp
