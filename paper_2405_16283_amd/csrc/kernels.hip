// gfx950 task kernels of the memgraph runtime: tile GEMMs, blocked attention with online
// softmax, attention combine, RMSNorm (statistic + apply), rotary embedding, SiLU*mul, add, their
// reverse-mode counterparts for the fine-tuning workload, transposition, and grouped copies.
//
// The paper runs such vertices through a vendor tensor library plus a few hand-written kernels
// (Appendix A); here every vertex kind has its own kernel, written for 64-wide wavefronts and
// the MFMA units.  All kernels are grouped (see kernels.h) and deterministic: fixed summation
// order, no atomics, so any dispatch order gives the same bits.
#include "kernels.h"

#include <climits>
#include <mutex>
#include <type_traits>

namespace tn {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef unsigned short bf16_t;  // storage of a bf16 value

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float((uint32_t)b << 16); }
// round to nearest, ties to even: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32)
__device__ __forceinline__ bf16_t f2bf(float f) { return __builtin_bit_cast(bf16_t, (__bf16)f); }
// two values at once, the first in the low half
__device__ __forceinline__ uint32_t f2bf2(float a, float b) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){a, b}, bf16x2_t));
}
template <typename T> __device__ __forceinline__ float ld(const T* p);
template <> __device__ __forceinline__ float ld<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ld<bf16_t>(const bf16_t* p) { return bf2f(*p); }
template <typename T> __device__ __forceinline__ void st(T* p, float v);
template <> __device__ __forceinline__ void st<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void st<bf16_t>(bf16_t* p, float v) { *p = f2bf(v); }

// ---------------------------------------------------------------------------------------------
// elementwise: add, silu*mul
// ---------------------------------------------------------------------------------------------
// zeros, the value a sum's output starts from; 16 bytes per lane, the tail element by element
template <typename T>
__global__ void __launch_bounds__(256) zero_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  T* o = (T*)d.out;
  const int n = d.rows * d.cols;
  constexpr int V = 16 / (int)sizeof(T);
  const int i0 = (blockIdx.x * 256 + threadIdx.x) * V;
  if (i0 + V <= n) {
    *(uint4*)(o + i0) = make_uint4(0, 0, 0, 0);
  } else {
    for (int i = i0; i < n; ++i) o[i] = T(0);
  }
}

template <typename T, bool SILU>
__global__ void __launch_bounds__(256) ewise2_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const T* x = (const T*)t.ptrs[d.ptr0];
  const T* y = (const T*)t.ptrs[d.ptr0 + 1];
  T* o = (T*)d.out;
  const int n = d.rows * d.cols;
  const int i0 = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (i0 >= n) return;
  float a[8], c[8];
  if (i0 + 8 <= n) {
    if constexpr (sizeof(T) == 2) {
      uint4 va = *(const uint4*)(x + i0), vb = *(const uint4*)(y + i0);
      const bf16_t* pa = (const bf16_t*)&va;
      const bf16_t* pb = (const bf16_t*)&vb;
#pragma unroll
      for (int k = 0; k < 8; ++k) { a[k] = bf2f(pa[k]); c[k] = bf2f(pb[k]); }
    } else {
      float4 a0 = *(const float4*)(x + i0), a1 = *(const float4*)(x + i0 + 4);
      float4 c0 = *(const float4*)(y + i0), c1 = *(const float4*)(y + i0 + 4);
      a[0] = a0.x; a[1] = a0.y; a[2] = a0.z; a[3] = a0.w; a[4] = a1.x; a[5] = a1.y; a[6] = a1.z; a[7] = a1.w;
      c[0] = c0.x; c[1] = c0.y; c[2] = c0.z; c[3] = c0.w; c[4] = c1.x; c[5] = c1.y; c[6] = c1.z; c[7] = c1.w;
    }
#pragma unroll
    for (int k = 0; k < 8; ++k) a[k] = SILU ? a[k] / (1.f + __expf(-a[k])) * c[k] : a[k] + c[k];
    if constexpr (sizeof(T) == 2) {
      uint4 vo;
      bf16_t* po = (bf16_t*)&vo;
#pragma unroll
      for (int k = 0; k < 8; ++k) po[k] = f2bf(a[k]);
      *(uint4*)(o + i0) = vo;
    } else {
      *(float4*)(o + i0) = make_float4(a[0], a[1], a[2], a[3]);
      *(float4*)(o + i0 + 4) = make_float4(a[4], a[5], a[6], a[7]);
    }
  } else {
    for (int i = i0; i < n; ++i) {
      float u = ld(x + i), v = ld(y + i);
      st(o + i, SILU ? u / (1.f + __expf(-u)) * v : u + v);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// RMSNorm statistic: one wavefront per row, over all column tiles of the row block
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) rms_stat_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= d.rows) return;
  float ss = 0.f;
  for (int j = 0; j < d.n_in; ++j) {
    const int cols = t.aux[d.aux0 + j];
    const T* x = (const T*)t.ptrs[d.ptr0 + j] + (size_t)row * cols;
    for (int c = lane * 8; c < cols; c += 512) {
      if (c + 8 <= cols && (cols & 7) == 0) {
        if constexpr (sizeof(T) == 2) {
          uint4 v = *(const uint4*)(x + c);
          const bf16_t* p = (const bf16_t*)&v;
#pragma unroll
          for (int k = 0; k < 8; ++k) { float f = bf2f(p[k]); ss += f * f; }
        } else {
          float4 v0 = *(const float4*)(x + c), v1 = *(const float4*)(x + c + 4);
          ss += v0.x * v0.x; ss += v0.y * v0.y; ss += v0.z * v0.z; ss += v0.w * v0.w;
          ss += v1.x * v1.x; ss += v1.y * v1.y; ss += v1.z * v1.z; ss += v1.w * v1.w;
        }
      } else {
        for (int k = c; k < min(c + 8, cols); ++k) { float f = ld(x + k); ss += f * f; }
      }
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
  if (lane == 0) ((float*)d.out)[row] = 1.0f / sqrtf(ss / (float)d.p.d + d.p.eps);
}

// Softmax over materialised scores, first portion: one wavefront per row walks over the score
// tiles of the row block twice (maximum, then the sum of exponentials), columns counted across
// the tiles.  aux: the tiles' widths.
template <typename T>
__global__ void __launch_bounds__(256) softmax_stat_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= d.rows) return;
  const float scale = d.p.scale;
  const int last = d.p.causal ? d.p.q_pos0 + row - d.p.k_pos0 : INT_MAX;  // last visible column
  float m = -INFINITY;
  for (int j = 0, c0 = 0; j < d.n_in; ++j) {
    const int cols = t.aux[d.aux0 + j];
    const T* x = (const T*)t.ptrs[d.ptr0 + j] + (size_t)row * cols;
    for (int c = lane; c < cols && c0 + c <= last; c += 64) m = fmaxf(m, ld(x + c) * scale);
    c0 += cols;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  const float msafe = m == -INFINITY ? 0.f : m;
  float l = 0.f;
  for (int j = 0, c0 = 0; j < d.n_in; ++j) {
    const int cols = t.aux[d.aux0 + j];
    const T* x = (const T*)t.ptrs[d.ptr0 + j] + (size_t)row * cols;
    for (int c = lane; c < cols && c0 + c <= last; c += 64) l += __expf(ld(x + c) * scale - msafe);
    c0 += cols;
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) l += __shfl_xor(l, off, 64);
  if (lane == 0) {
    float* out = (float*)d.out + (size_t)row * 2;
    out[0] = m;
    out[1] = l;
  }
}

// second portion: the probabilities of one score tile, 8 columns per thread
template <typename T>
__global__ void __launch_bounds__(256) softmax_apply_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const T* x = (const T*)t.ptrs[d.ptr0];
  const float* stat = (const float*)t.ptrs[d.ptr0 + 1];
  T* o = (T*)d.out;
  const int segs = (d.cols + 7) / 8;
  const int id = blockIdx.x * 256 + threadIdx.x;
  if (id >= d.rows * segs) return;
  const int row = id / segs, c0 = (id % segs) * 8;
  const float m = stat[row * 2], inv = 1.f / stat[row * 2 + 1], scale = d.p.scale;
  const float msafe = m == -INFINITY ? 0.f : m;
  const int last = d.p.causal ? d.p.q_pos0 + row - d.p.k_pos0 : INT_MAX;
  for (int c = c0; c < min(c0 + 8, d.cols); ++c) {
    const size_t e = (size_t)row * d.cols + c;
    st(o + e, c <= last ? __expf(ld(x + e) * scale - msafe) * inv : 0.f);
  }
}

// RMSNorm apply: out = x * stat[row] * gain[col]
template <typename T>
__global__ void __launch_bounds__(256) rms_apply_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const T* x = (const T*)t.ptrs[d.ptr0];
  const float* stat = (const float*)t.ptrs[d.ptr0 + 1];
  const T* g = (const T*)t.ptrs[d.ptr0 + 2];
  T* o = (T*)d.out;
  const int segs = (d.cols + 7) / 8;
  const int id = blockIdx.x * 256 + threadIdx.x;
  if (id >= d.rows * segs) return;
  const int row = id / segs, c0 = (id % segs) * 8;
  const float s = stat[row];
  if ((d.cols & 7) == 0) {  // whole 16-byte (bf16) or 32-byte (fp32) pieces
    const size_t e = (size_t)row * d.cols + c0;
    float v[8], gv[8];
    if constexpr (sizeof(T) == 2) {
      const uint4 u = *(const uint4*)(x + e), ug = *(const uint4*)(g + c0);
      const bf16_t* pu = (const bf16_t*)&u;
      const bf16_t* pg = (const bf16_t*)&ug;
#pragma unroll
      for (int k = 0; k < 8; ++k) { v[k] = bf2f(pu[k]); gv[k] = bf2f(pg[k]); }
      uint4 r;
      bf16_t* pr = (bf16_t*)&r;
#pragma unroll
      for (int k = 0; k < 8; ++k) pr[k] = f2bf(v[k] * s * gv[k]);
      *(uint4*)(o + e) = r;
    } else {
      const float4 a = *(const float4*)(x + e), b2 = *(const float4*)(x + e + 4);
      const float4 ga = *(const float4*)(g + c0), gb = *(const float4*)(g + c0 + 4);
      *(float4*)(o + e) = make_float4(a.x * s * ga.x, a.y * s * ga.y, a.z * s * ga.z, a.w * s * ga.w);
      *(float4*)(o + e + 4) = make_float4(b2.x * s * gb.x, b2.y * s * gb.y, b2.z * s * gb.z, b2.w * s * gb.w);
    }
    return;
  }
  for (int c = c0; c < min(c0 + 8, d.cols); ++c)
    st(o + (size_t)row * d.cols + c, ld(x + (size_t)row * d.cols + c) * s * ld(g + c));
}

// Rotary embedding on interleaved pairs; the angle is formed and reduced in double so that long
// sequences lose no accuracy, then the single-precision sincos is taken of the reduced angle
// Tiles that hold whole heads take the fast path: a thread owns 4 pairs (8 elements, one 16-byte
// piece for bf16) of a row and walks over the heads of the tile, so the angles and their sines and
// cosines -- the expensive part -- are formed once per row and pair, not once per head.
__host__ __device__ __forceinline__ bool rope_whole_heads(const OpDesc& d) {
  return d.p.head_dim % 8 == 0 && d.p.col0 % d.p.head_dim == 0 && d.cols % d.p.head_dim == 0;
}
template <typename T>
__global__ void __launch_bounds__(256) rope_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const T* x = (const T*)t.ptrs[d.ptr0];
  T* o = (T*)d.out;
  const int id = blockIdx.x * 256 + threadIdx.x;
  if (rope_whole_heads(d)) {
    const int hd = d.p.head_dim, per_row = hd / 8;
    if (id >= d.rows * per_row) return;
    const int row = id / per_row, q8 = id % per_row;
    float cs[4], sn[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      double ang = (double)(d.p.pos0 + row) * t.rope_theta[d.aux0 + 4 * q8 + k];
      ang -= 6.283185307179586476925 * rint(ang * 0.15915494309189533577);
      sincosf((float)ang, &sn[k], &cs[k]);
      if (d.p.mode) sn[k] = -sn[k];  // the inverse rotation
    }
    for (int c0 = 8 * q8; c0 < d.cols; c0 += hd) {
      const size_t e = (size_t)row * d.cols + c0;
      float v[8];
      if constexpr (sizeof(T) == 2) {
        const uint4 u = *(const uint4*)(x + e);
        const bf16_t* pu = (const bf16_t*)&u;
#pragma unroll
        for (int k = 0; k < 8; ++k) v[k] = bf2f(pu[k]);
      } else {
        const float4 a = *(const float4*)(x + e), c = *(const float4*)(x + e + 4);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = c.x; v[5] = c.y; v[6] = c.z; v[7] = c.w;
      }
      float r[8];
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        r[2 * k] = v[2 * k] * cs[k] - v[2 * k + 1] * sn[k];
        r[2 * k + 1] = v[2 * k] * sn[k] + v[2 * k + 1] * cs[k];
      }
      if constexpr (sizeof(T) == 2) {
        uint4 u;
        bf16_t* pu = (bf16_t*)&u;
#pragma unroll
        for (int k = 0; k < 8; ++k) pu[k] = f2bf(r[k]);
        *(uint4*)(o + e) = u;
      } else {
        *(float4*)(o + e) = make_float4(r[0], r[1], r[2], r[3]);
        *(float4*)(o + e + 4) = make_float4(r[4], r[5], r[6], r[7]);
      }
    }
    return;
  }
  const int pairs = d.cols / 2;
  if (id >= d.rows * pairs) return;
  const int row = id / pairs, pc = id % pairs;
  const int i = ((d.p.col0 + 2 * pc) % d.p.head_dim) / 2;
  double ang = (double)(d.p.pos0 + row) * t.rope_theta[d.aux0 + i];
  ang -= 6.283185307179586476925 * rint(ang * 0.15915494309189533577);
  float sn, cs;
  sincosf((float)ang, &sn, &cs);
  if (d.p.mode) sn = -sn;  // the inverse rotation
  const size_t e = (size_t)row * d.cols + 2 * pc;
  const float xe = ld(x + e), xo = ld(x + e + 1);
  st(o + e, xe * cs - xo * sn);
  st(o + e + 1, xe * sn + xo * cs);
}

// Attention combine: merge the partials of one query block (j ascending) and normalise.  Where the
// shapes allow, a thread forms 4 neighbouring columns of a row (one head, so one set of weights).
__host__ __device__ __forceinline__ bool combine_by_four(const OpDesc& d) {
  return d.cols % 4 == 0 && d.p.col0 % 4 == 0 && d.p.head_dim % 4 == 0;
}
template <typename T>
__global__ void __launch_bounds__(256) attn_combine_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const int id = blockIdx.x * 256 + threadIdx.x;
  const int hd = d.p.head_dim, hpg = d.p.hpg, gw = hd * hpg, ldp = gw + 2 * hpg;
  if (combine_by_four(d)) {
    const int per_row = d.cols / 4;
    if (id >= d.rows * per_row) return;
    const int row = id / per_row, c = (id % per_row) * 4;
    const int col = d.p.col0 + c, h = col / hd;
    const size_t r = (size_t)(d.p.row0 + row) * ldp;
    const bool wide = (ldp & 3) == 0;  // rows of a partial are 16-byte aligned
    float mstar = -INFINITY;
    for (int j = 0; j < d.n_in; ++j) mstar = fmaxf(mstar, ((const float*)t.ptrs[d.ptr0 + j])[r + gw + h]);
    float num[4] = {0.f, 0.f, 0.f, 0.f}, den = 0.f;
#pragma unroll 4
    for (int j = 0; j < d.n_in; ++j) {
      const float* p = (const float*)t.ptrs[d.ptr0 + j];
      const float w = __expf(p[r + gw + h] - mstar);
      float v[4];
      if (wide) {
        const float4 u = *(const float4*)(p + r + col);
        v[0] = u.x; v[1] = u.y; v[2] = u.z; v[3] = u.w;
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) v[k] = p[r + col + k];
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) num[k] += v[k] * w;
      den += p[r + gw + hpg + h] * w;
    }
    T* out = (T*)d.out + (size_t)row * d.cols + c;
    if constexpr (sizeof(T) == 2) {
      uint2 u;
      u.x = (uint32_t)f2bf(num[0] / den) | ((uint32_t)f2bf(num[1] / den) << 16);
      u.y = (uint32_t)f2bf(num[2] / den) | ((uint32_t)f2bf(num[3] / den) << 16);
      *(uint2*)out = u;
    } else {
      *(float4*)out = make_float4(num[0] / den, num[1] / den, num[2] / den, num[3] / den);
    }
    return;
  }
  if (id >= d.rows * d.cols) return;
  const int row = id / d.cols, c = id % d.cols;
  const int col = d.p.col0 + c, h = col / hd;
  const size_t r = (size_t)(d.p.row0 + row) * ldp;
  float mstar = -INFINITY;
  for (int j = 0; j < d.n_in; ++j) mstar = fmaxf(mstar, ((const float*)t.ptrs[d.ptr0 + j])[r + gw + h]);
  float num = 0.f, den = 0.f;
  for (int j = 0; j < d.n_in; ++j) {
    const float* p = (const float*)t.ptrs[d.ptr0 + j];
    const float w = __expf(p[r + gw + h] - mstar);
    num += p[r + col] * w;
    den += p[r + gw + hpg + h] * w;
  }
  st((T*)d.out + (size_t)row * d.cols + c, num / den);
}

// ---------------------------------------------------------------------------------------------
// reverse-mode elementwise and RMSNorm kernels (fine-tuning workload)
// ---------------------------------------------------------------------------------------------
// gradient of silu(gate) * up with respect to gate (mode 0) or up (mode 1)
template <typename T>
__global__ void __launch_bounds__(256) silu_bwd_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const T* dact = (const T*)t.ptrs[d.ptr0];
  const T* gate = (const T*)t.ptrs[d.ptr0 + 1];
  const T* up = (const T*)t.ptrs[d.ptr0 + 2];
  T* o = (T*)d.out;
  const int n = d.rows * d.cols;
  const int i0 = (blockIdx.x * 256 + threadIdx.x) * 8;
  if (i0 >= n) return;
  auto grad = [&](float da, float g, float u) {
    const float s = 1.f / (1.f + __expf(-g));
    return d.p.mode == 0 ? da * u * s * (1.f + g * (1.f - s)) : da * g * s;
  };
  if constexpr (sizeof(T) == 2) {
    if (i0 + 8 <= n) {  // 16-byte accesses
      uint4 va = *(const uint4*)(dact + i0), vg = *(const uint4*)(gate + i0), vu = *(const uint4*)(up + i0), vo;
      const bf16_t *pa = (const bf16_t*)&va, *pg = (const bf16_t*)&vg, *pu = (const bf16_t*)&vu;
      bf16_t* po = (bf16_t*)&vo;
#pragma unroll
      for (int k = 0; k < 8; ++k) po[k] = f2bf(grad(bf2f(pa[k]), bf2f(pg[k]), bf2f(pu[k])));
      *(uint4*)(o + i0) = vo;
      return;
    }
  }
  for (int i = i0; i < min(i0 + 8, n); ++i) st(o + i, grad(ld(dact + i), ld(gate + i), ld(up + i)));
}

// sum over the columns of a row block of dy * gain * x: one wavefront per row
template <typename T>
__global__ void __launch_bounds__(256) rms_bwd_stat_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= d.rows) return;
  const int nk = d.p.nk;
  float ss = 0.f;
  for (int j = 0; j < nk; ++j) {
    const int cols = t.aux[d.aux0 + j];
    const T* dy = (const T*)t.ptrs[d.ptr0 + j] + (size_t)row * cols;
    const T* x = (const T*)t.ptrs[d.ptr0 + nk + j] + (size_t)row * cols;
    const T* g = (const T*)t.ptrs[d.ptr0 + 2 * nk + j];
    if (sizeof(T) == 2 && (cols & 7) == 0) {  // 16-byte pieces
      for (int c = lane * 8; c < cols; c += 512) {
        const uint4 vd = *(const uint4*)(dy + c), vx = *(const uint4*)(x + c), vg = *(const uint4*)(g + c);
        const bf16_t *pd = (const bf16_t*)&vd, *px = (const bf16_t*)&vx, *pg = (const bf16_t*)&vg;
#pragma unroll
        for (int k = 0; k < 8; ++k) ss += bf2f(pd[k]) * bf2f(pg[k]) * bf2f(px[k]);
      }
    } else {
      for (int c = lane; c < cols; c += 64) ss += ld(dy + c) * ld(g + c) * ld(x + c);
    }
  }
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off, 64);
  if (lane == 0) ((float*)d.out)[row] = ss;
}

// gradient of x through y = x * stat * gain: stat * gain * dy - x * stat^3 * dot / d (+ residual gradient)
template <typename T>
__global__ void __launch_bounds__(256) rms_bwd_apply_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const T* dy = (const T*)t.ptrs[d.ptr0];
  const T* x = (const T*)t.ptrs[d.ptr0 + 1];
  const float* stat = (const float*)t.ptrs[d.ptr0 + 2];
  const float* dot = (const float*)t.ptrs[d.ptr0 + 3];
  const T* g = (const T*)t.ptrs[d.ptr0 + 4];
  const T* res = d.n_in == 6 ? (const T*)t.ptrs[d.ptr0 + 5] : nullptr;
  T* o = (T*)d.out;
  const int segs = (d.cols + 7) / 8;
  const int id = blockIdx.x * 256 + threadIdx.x;
  if (id >= d.rows * segs) return;
  const int row = id / segs, c0 = (id % segs) * 8;
  const float r = stat[row], k = r * r * r * dot[row] / (float)d.p.d;
  if constexpr (sizeof(T) == 2) {
    if ((d.cols & 7) == 0) {  // 16-byte pieces
      const size_t e = (size_t)row * d.cols + c0;
      const uint4 vd = *(const uint4*)(dy + e), vx = *(const uint4*)(x + e), vg = *(const uint4*)(g + c0);
      uint4 vr = make_uint4(0, 0, 0, 0), vo;
      if (res) vr = *(const uint4*)(res + e);
      const bf16_t *pd = (const bf16_t*)&vd, *px = (const bf16_t*)&vx, *pg = (const bf16_t*)&vg, *pr = (const bf16_t*)&vr;
      bf16_t* po = (bf16_t*)&vo;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        float v = r * bf2f(pg[q]) * bf2f(pd[q]) - bf2f(px[q]) * k;
        if (res) v += bf2f(pr[q]);
        po[q] = f2bf(v);
      }
      *(uint4*)(o + e) = vo;
      return;
    }
  }
  for (int c = c0; c < min(c0 + 8, d.cols); ++c) {
    const size_t e = (size_t)row * d.cols + c;
    float v = r * ld(g + c) * ld(dy + e) - ld(x + e) * k;
    if (res) v += ld(res + e);
    st(o + e, v);
  }
}

// out[c, r] = in[r, c]: 64x64 pieces through LDS, so that both the reads and the writes are row-wise
template <typename T>
__global__ void __launch_bounds__(256) transpose_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const int R = d.cols, C = d.rows;  // the operand is [R, C]; the output [C, R]
  const int tc = (C + 63) / 64;
  const int r0 = (blockIdx.x / tc) * 64, c0 = (blockIdx.x % tc) * 64;
  const T* x = (const T*)t.ptrs[d.ptr0];
  T* o = (T*)d.out;
  if constexpr (sizeof(T) == 2) {
    if ((R & 7) == 0 && (C & 7) == 0) {
      // 16-byte pieces both ways: a piece of 8 elements of an input row is scattered into the
      // transposed image in LDS, whose rows are then read back 8 elements at a time
      __shared__ __attribute__((aligned(16))) bf16_t tt[64][72];
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int s = threadIdx.x + 256 * k, i = s >> 3, c8 = (s & 7) * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r0 + i < R && c0 + c8 < C) v = *(const uint4*)(x + (size_t)(r0 + i) * C + c0 + c8);
        const bf16_t* pv = (const bf16_t*)&v;
#pragma unroll
        for (int e = 0; e < 8; ++e) tt[c8 + e][i] = pv[e];
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int s = threadIdx.x + 256 * k, j = s >> 3, r8 = (s & 7) * 8;
        if (c0 + j < C && r0 + r8 < R) *(uint4*)(o + (size_t)(c0 + j) * R + r0 + r8) = *(const uint4*)&tt[j][r8];
      }
      return;
    }
  }
  __shared__ T tile[64][65];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  for (int i = ty; i < 64; i += 4)
    if (r0 + i < R && c0 + tx < C) tile[i][tx] = x[(size_t)(r0 + i) * C + c0 + tx];
  __syncthreads();
  for (int i = ty; i < 64; i += 4)
    if (c0 + i < C && r0 + tx < R) o[(size_t)(c0 + i) * R + r0 + tx] = tile[tx][i];
}

// ---------------------------------------------------------------------------------------------
// generic GEMM on the vector ALUs (fp32 accumulate): 64x64 output tile per workgroup
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) gemm_generic_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  __shared__ float As[16][68];
  __shared__ float Bs[16][68];
  const int M = d.rows, N = d.cols, nk = d.p.nk;
  const int tn_ = (N + 63) / 64;
  const int m0 = (blockIdx.x / tn_) * 64, n0 = (blockIdx.x % tn_) * 64;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  float gate[4][4];  // mode 2: the first of the two products, while the second is formed
  for (int pass = 0; pass < (d.p.mode == 2 ? 2 : 1); ++pass) {
  if (pass == 1) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) { gate[i][j] = acc[i][j]; acc[i][j] = 0.f; }
  }
  for (int kt = 0; kt < nk; ++kt) {
    const T* A = (const T*)t.ptrs[d.ptr0 + kt];
    const T* B = (const T*)t.ptrs[d.ptr0 + (1 + pass) * nk + kt];
    const int K = t.aux[d.aux0 + kt];
    for (int k0 = 0; k0 < K; k0 += 16) {
      {
        const int r = threadIdx.x / 4, kk = (threadIdx.x % 4) * 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int gr = m0 + r, gk = k0 + kk + i;
          As[kk + i][r] = (gr < M && gk < K) ? ld(d.p.trans_a ? A + (size_t)gk * M + gr : A + (size_t)gr * K + gk) : 0.f;
        }
        if (d.trans_b) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int gc = n0 + r, gk = k0 + kk + i;
            Bs[kk + i][r] = (gc < N && gk < K) ? ld(B + (size_t)gc * K + gk) : 0.f;
          }
        } else {
          const int kr = threadIdx.x / 16, cc = (threadIdx.x % 16) * 4;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int gc = n0 + cc + i, gk = k0 + kr;
            Bs[kr][cc + i] = (gc < N && gk < K) ? ld(B + (size_t)gk * N + gc) : 0.f;
          }
        }
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < 16; ++k) {
        float a[4], bb[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; bb[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], bb[j], acc[i][j]);
      }
      __syncthreads();
    }
  }
  }
  T* Cp = (T*)d.out;
  const T* R = d.p.mode == 1 ? (const T*)t.ptrs[d.ptr0 + 2 * nk] : nullptr;  // the residual operand
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int r = m0 + ty * 4 + i, c = n0 + tx * 4 + j;
      if (r >= M || c >= N) continue;
      float v = acc[i][j];
      if (d.p.mode == 1) v += ld(R + (size_t)r * N + c);
      if (d.p.mode == 2) v = gate[i][j] / (1.f + __expf(-gate[i][j])) * v;
      st(d.p.trans_c ? Cp + (size_t)c * M + r : Cp + (size_t)r * N + c, v);
    }
}

// ---------------------------------------------------------------------------------------------
// MFMA bf16 GEMM, C[M,N] = sum_k A_k[M,K_k] * B_k[N,K_k]^T, fp32 accumulate, bf16 store.
// 128x128 output tile per workgroup of 4 wavefronts (2x2, 64x64 each = 2x2 MFMA 32x32 tiles),
// K step 64 staged through LDS.  Rows are padded by 8 elements so that the 16-byte fragment
// reads of the 32 lanes of a half-wave fall on different banks.
// ---------------------------------------------------------------------------------------------
// Writes a wavefront's TI x TJ grid of 32x32 accumulator tiles as bf16.  In an accumulator tile a
// lane holds column l32 and the rows 8*(r/4) + 4*g + r%4: four consecutive rows per group of four
// registers, which makes the transposed store (C^T, rows contiguous) an 8-byte store per group.
template <int TI, int TJ>
__device__ __forceinline__ void store_c_tiles(const f32x16 (&acc)[TI][TJ], bf16_t* Cp, int M, int N, int row0, int col0,
                                              int l32, int g, bool trans_c) {
  const bool wide = trans_c && (M & 3) == 0;
#pragma unroll
  for (int i = 0; i < TI; ++i) {
#pragma unroll
    for (int j = 0; j < TJ; ++j) {
      const int col = col0 + j * 32 + l32;
      const f32x16 c = acc[i][j];
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int row = row0 + i * 32 + 8 * a + 4 * g;
        const uint32_t h01 = f2bf2(c[4 * a], c[4 * a + 1]), h23 = f2bf2(c[4 * a + 2], c[4 * a + 3]);
        const bf16_t h0 = (bf16_t)h01, h1 = (bf16_t)(h01 >> 16), h2 = (bf16_t)h23, h3 = (bf16_t)(h23 >> 16);
        if (wide) {
          if (col < N && row < M) {
            uint2 v;
            v.x = h01;
            v.y = h23;
            *(uint2*)(Cp + (size_t)col * M + row) = v;
          }
        } else if (col < N) {
          const size_t sr = trans_c ? 1 : (size_t)N, sc = trans_c ? (size_t)M : 1;
          bf16_t* p = Cp + (size_t)row * sr + (size_t)col * sc;
          if (row < M) p[0] = h0;
          if (row + 1 < M) p[sr] = h1;
          if (row + 2 < M) p[2 * sr] = h2;
          if (row + 3 < M) p[3 * sr] = h3;
        }
      }
    }
  }
}

// Accumulator tiles formed with the operands exchanged (B fragments first): acc[i][j] is then the transpose
// of a 32x32 piece of C -- a lane holds row l32 of row group j and, per group of four registers, the four
// consecutive columns 8*(r/4) + 4*g + r%4 of column group i.  The wavefront's piece of C (32 TJ rows by
// 32 NT columns) goes through `stage`, LDS of its own (EpilogueStage<NT, TJ>::BYTES), as bf16 rows of a
// padded pitch -- 8-byte writes from this layout, 16-byte reads along the rows -- so that every global
// store instruction writes whole runs of 64 NT bytes.
// R: a [M, N] bf16 tensor added to the product before the rounding.
template <int NT, int TJ>
struct EpilogueStage {
  static constexpr int PITCH = 64 * NT + 16;  // bytes per row: the lanes of a half-wavefront write 32 rows at once
  static constexpr int BYTES = 32 * TJ * PITCH;
};
template <int NT, int TJ>
__device__ __forceinline__ void store_c_rows(const f32x16 (&acc)[NT][TJ], char* stage, bf16_t* Cp, int M, int N, int row0,
                                             int col0, int lane, const bf16_t* R) {
  constexpr int PITCH = EpilogueStage<NT, TJ>::PITCH;
  const int l32 = lane & 31, g = lane >> 5;
#pragma unroll
  for (int j = 0; j < TJ; ++j) {
    const int row = row0 + j * 32 + l32;
#pragma unroll
    for (int i = 0; i < NT; ++i) {
      const f32x16 c = acc[i][j];
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        const int cin = i * 32 + 8 * a + 4 * g;  // column inside the wavefront's piece
        float v[4] = {c[4 * a], c[4 * a + 1], c[4 * a + 2], c[4 * a + 3]};
        if (R != nullptr && row < M) {
          const size_t at = (size_t)row * N + col0 + cin;
          if ((N & 3) == 0 && col0 + cin + 3 < N) {
            const uint2 r = *(const uint2*)(R + at);
            v[0] += __uint_as_float(r.x << 16);
            v[1] += __uint_as_float(r.x & 0xFFFF0000u);
            v[2] += __uint_as_float(r.y << 16);
            v[3] += __uint_as_float(r.y & 0xFFFF0000u);
          } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
              if (col0 + cin + k < N) v[k] += bf2f(R[at + k]);
          }
        }
        uint2 o;
        o.x = f2bf2(v[0], v[1]);
        o.y = f2bf2(v[2], v[3]);
        *(uint2*)(stage + (j * 32 + l32) * PITCH + cin * 2) = o;
      }
    }
  }
  // rows of the piece, 16 bytes per lane: 4 NT lanes per row
  constexpr int LPR = 4 * NT, RPI = 64 / LPR;  // lanes per row, rows per instruction
  const int rin = lane / LPR, cin = (lane % LPR) * 8;
  const bool whole = (N & 7) == 0;  // rows of C are 16-byte aligned
#pragma unroll
  for (int q = 0; q < 32 * TJ / RPI; ++q) {
    const int r = q * RPI + rin, row = row0 + r, col = col0 + cin;
    const uint4 x = *(const uint4*)(stage + r * PITCH + cin * 2);
    if (row >= M || col >= N) continue;
    bf16_t* dst = Cp + (size_t)row * N + col;
    if (whole && col + 7 < N) {
      *(uint4*)dst = x;
    } else {
      const bf16_t* e = (const bf16_t*)&x;
#pragma unroll
      for (int k = 0; k < 8; ++k)
        if (col + k < N) dst[k] = e[k];
    }
  }
}

constexpr int GB_M = 128, GB_N = 128, GB_K = 64, GB_LD = GB_K + 8;

__global__ void __launch_bounds__(256) gemm_bf16_nt_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  __shared__ __attribute__((aligned(16))) bf16_t As[GB_M * GB_LD];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[GB_N * GB_LD];
  const int M = d.rows, N = d.cols, nk = d.p.nk;
  const int tn_ = (N + GB_N - 1) / GB_N;
  const int m0 = (blockIdx.x / tn_) * GB_M, n0 = (blockIdx.x % tn_) * GB_N;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, wm = w >> 1, wn = w & 1;
  const int l32 = lane & 31, g = lane >> 5;
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  for (int kt = 0; kt < nk; ++kt) {
    const bf16_t* A = (const bf16_t*)t.ptrs[d.ptr0 + kt];
    const bf16_t* B = (const bf16_t*)t.ptrs[d.ptr0 + nk + kt];
    const int K = t.aux[d.aux0 + kt];
    // 128 rows x 8 segments of 16 bytes per operand and K step; 4 segments per thread and operand.
    // The segments of the next step are fetched into registers while this step is multiplied.
    uint4 pa[4], pb[4];
    auto fetch = [&](int k0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int s = threadIdx.x + 256 * i, r = s >> 3, ks = (s & 7) * 8;
        pa[i] = make_uint4(0, 0, 0, 0);
        pb[i] = make_uint4(0, 0, 0, 0);
        if (m0 + r < M && k0 + ks < K) pa[i] = *(const uint4*)(A + (size_t)(m0 + r) * K + k0 + ks);
        if (n0 + r < N && k0 + ks < K) pb[i] = *(const uint4*)(B + (size_t)(n0 + r) * K + k0 + ks);
      }
    };
    fetch(0);
    for (int k0 = 0; k0 < K; k0 += GB_K) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int s = threadIdx.x + 256 * i, r = s >> 3, ks = (s & 7) * 8;
        *(uint4*)(As + r * GB_LD + ks) = pa[i];
        *(uint4*)(Bs + r * GB_LD + ks) = pb[i];
      }
      __syncthreads();
      if (k0 + GB_K < K) fetch(k0 + GB_K);
#pragma unroll
      for (int s = 0; s < GB_K / 16; ++s) {
        bf16x8 a[2], bb[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          a[i] = *(const bf16x8*)(As + (wm * 64 + i * 32 + l32) * GB_LD + s * 16 + g * 8);
          bb[i] = *(const bf16x8*)(Bs + (wn * 64 + i * 32 + l32) * GB_LD + s * 16 + g * 8);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bb[j], acc[i][j], 0, 0, 0);
      }
      __syncthreads();
    }
  }
  store_c_tiles<2, 2>(acc, (bf16_t*)d.out, M, N, m0 + wm * 64, n0 + wn * 64, l32, g, d.p.trans_c != 0);
}

// ---------------------------------------------------------------------------------------------
// MFMA bf16 GEMM for large tiles: 256x256 output tile per workgroup, 4 wavefronts in 2x2, each
// 128x128 = 4x4 MFMA 32x32x16 tiles (256 accumulator registers per lane).
//
// K advances in steps of 32 through a ring of four LDS stages that the global-to-LDS loads of
// gfx950 fill directly (no staging registers, no LDS store instructions).  The loads of step
// s+3 are issued while step s computes, so a load has three steps of MFMA work to land; one
// barrier per step both publishes stage s and frees the stage that step s-1 read.
//
// A direct load writes the 64 lanes' 16-byte chunks back to back, so the LDS image of a stage is
// unpadded: 256 rows x 4 chunks per operand.  Bank conflicts are avoided by choosing *which*
// chunk each lane fetches: logical chunk c of row r lives at position c ^ ((r >> 2) & 3).
// ---------------------------------------------------------------------------------------------
#ifndef TN_GEMM_WAVES
#define TN_GEMM_WAVES 8
#endif
constexpr int G2_K = 32, G2_STAGES = 4;
// LDS of a workgroup with a tile of bm rows and as many columns: per stage bm x 32 of A, then of B
constexpr int g2_lds_bytes(int bm) { return G2_STAGES * 2 * bm * G2_K * 2; }  // 128 KiB for 256, 64 KiB for 128

typedef __attribute__((address_space(3))) void* lptr_t;

// 16 bytes per lane from global memory straight into LDS at lds_addr + 16 * lane.  Issued as
// inline assembly so that the compiler does not track it: the kernel keeps several such loads
// in flight across barriers and waits for them with explicit vmcnt values.
__device__ __forceinline__ void load_lds16(const void* gsrc, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(gsrc), "s"(lds_addr) : "memory");
}
// The same with a wavefront-uniform base address and a 32-bit per-lane byte offset, which leaves
// the per-step address arithmetic to the scalar unit.
__device__ __forceinline__ void load_lds16_so(const void* sbase, uint32_t voff, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(voff), "s"(sbase), "s"(lds_addr) : "memory");
}
// Reads of the (read-only, wavefront-uniform) operand tables through the scalar unit, so that
// they are counted by lgkmcnt and never force a wait on the vector loads in flight.
__device__ __forceinline__ const void* sload_ptr(const void* const* addr) {
  const void* v;
  asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(addr) : "memory");
  return v;
}
__device__ __forceinline__ int sload_int(const int* addr) {
  int v;
  asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(addr) : "memory");
  return v;
}

// Workgroups are handed to the 8 XCDs round-robin in launch order, and each XCD has its own L2.
// This turns the launch position into a position in which each XCD gets a contiguous run of
// (vertex, tile) pairs, so that the workgroups sharing an L2 work on neighbouring tiles -- the
// tiles of one vertex and of vertices with the same A row block -- instead of every XCD
// streaming every operand.
__device__ __forceinline__ void xcd_remap(int& bx, int& by) {
  const int gx = gridDim.x, total = gx * gridDim.y;
  const int n = blockIdx.x + gx * blockIdx.y;
  const int xcd = n & 7, slot = n >> 3;
  const int q = total >> 3, r = total & 7;
  const int v = xcd * q + min(xcd, r) + slot;
  by = v / gx;
  bx = v - by * gx;
}

// The same idea for kernels whose workgroups of one vertex share operands (the query blocks of an
// attention head all read that head's keys and values): vertex by goes to XCD by % 8 as a whole,
// and vertices that differ in cost (blocks on and off the diagonal) stay spread over the XCDs.
__device__ __forceinline__ void xcd_remap_rows(int& bx, int& by) {
  const int gx = gridDim.x, full = (int)(gridDim.y / 8) * 8;
  bx = blockIdx.x;
  by = blockIdx.y;
  if (by >= full) return;  // the last, incomplete group of eight vertices stays as launched
  const int n = bx + gx * by;
  const int slot = n >> 3;
  const int grp = slot / gx;  // vertices 8 grp .. 8 grp + 7; which XCD takes which rotates with grp, so that a
  by = grp * 8 + ((n + grp) & 7);  // cost pattern with period 8 in the launch order does not pile up on one XCD
  bx = slot - grp * gx;
}

// NW = wavefronts per workgroup: 4 (2x2, 128x128 each, one per SIMD) or 8 (2x4, 128x64 each, two
// per SIMD, so that one wavefront's MFMAs fill the time the other spends issuing its loads).
// MFMA with the accumulator held in the accumulation registers.  Left to itself the compiler
// keeps the accumulators of this kernel in ordinary vector registers, where the matrix unit's
// result traffic competes with the fragment reads arriving from LDS.  The asm statements are
// volatile so that they, and the wait states that follow the last one, keep their order; the
// same accumulator is not touched again for at least seven other MFMAs.
#ifndef TN_MFMA_AGPR
#define TN_MFMA_AGPR 0
#endif
__device__ __forceinline__ void mfma_acc(f32x16& acc, const bf16x8& a, const bf16x8& b) {
#if TN_MFMA_AGPR
  asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
#else
  acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
#endif
}
__device__ __forceinline__ void mfma_acc_drain() {
#if TN_MFMA_AGPR
  asm volatile("s_nop 15\n\ts_nop 15\n\ts_nop 7" ::: "memory");  // the last results reach the registers
#endif
}

#ifndef TN_GEMM_STAGGER
#define TN_GEMM_STAGGER(w) (((w) >> 2) & 1)  // wavefronts w and w + 4 share a SIMD
#endif
// NW wavefronts in two rows; each holds TI x TJ accumulator tiles of 32x32, so the workgroup's output
// tile is 64 TI rows by as many columns: (8, 4) is the 256x256 tile, (4, 2) a 128x128 tile with half
// the LDS and a quarter of the registers, two workgroups per CU, for launches too small to give every
// CU a 256x256 tile.  Every output element sums its products in the same order of K in all forms (the
// same MFMA, the same sequence of 16-deep slabs), so the forms agree bit for bit.
template <int NW, int TI>
__global__ void __launch_bounds__(64 * NW, TI == 2 ? 2 : 1) gemm_bf16_nt256_kernel(DeviceTables t, Batch b) {
  constexpr int WNS = NW / 2;             // wavefronts along N
  constexpr int BM = 64 * TI, BN = BM;    // output tile of the workgroup
  constexpr int TJ = 2 * TI / WNS;        // 32-column MFMA tiles per wavefront
  constexpr int NLD = 4 * TI / NW;        // load instructions per thread, operand and step
  constexpr int OPER_BYTES = BM * G2_K * 2, STAGE_BYTES = 2 * OPER_BYTES;
  static_assert(TJ >= 1 && NLD >= 1 && BN == 32 * TJ * WNS, "tile shape");
  int bx, by;
  xcd_remap(bx, by);
  const OpDesc& d = t.descs[b.at(by)];
  const int M = d.rows, N = d.cols, nk = d.p.nk;
  // Mode 2 (gate and up products, silu(gate) * up): the workgroup's BN rows of B are half gate columns and
  // half up columns of the same BN / 2 output columns: 32 gate rows, then the 32 up rows of the same outputs,
  // and so on, so that a wavefront's two 32-column accumulator tiles are the gate and the up of one piece.
  const bool gated = d.p.mode == 2;
  static_assert(TJ == 2 && TI % 2 == 0, "the gated form pairs the two accumulator tiles of a wavefront; mode 1 stores in halves");
  const int bn_out = gated ? BN / 2 : BN;  // output columns per workgroup
  const int tn_ = (N + bn_out - 1) / bn_out;
  if (bx >= ((M + BM - 1) / BM) * tn_) return;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const void* const* ptrA = t.ptrs + d.ptr0;  // A_0.., then nk entries later B_0.. (and nk later again the up tiles)
  const int* ksz = t.aux + d.aux0;
  bf16_t* const Cp = (bf16_t*)d.out;
  const int m0 = (bx / tn_) * BM, n0 = (bx % tn_) * bn_out;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, wm = w / WNS, wn = w % WNS;
  const int l32 = lane & 31, g = lane >> 5;

  f32x16 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // loader: load instruction i of wavefront w fills chunks [(i*NW + w)*64, +64) of an operand;
  // this lane's chunk is row (i*NW + w)*16 + lane/4, logical chunk (lane & 3) ^ ((lane >> 4) & 3).
  // Rows past the edge of a ragged tile are clamped (their products are never stored).  A lane's
  // byte offset inside an operand tile changes only with the tile's K; the position along K is
  // added to the (scalar) tile address.
  const int lrow = w * 16 + (lane >> 2);
  const int lcol = ((lane & 3) ^ ((lane >> 4) & 3)) * 8;
  int rowA[NLD], rowB[NLD];
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    rowA[i] = min(m0 + lrow + i * 16 * NW, M - 1);
    const int rb = lrow + i * 16 * NW;  // row of the B operand in LDS; gated: columns (rb / 64) * 32 + rb % 32
    rowB[i] = min(n0 + (gated ? (rb >> 6) * 32 + (rb & 31) : rb), N - 1);
  }
  // gated: rows 32..63 of every 64 come from the up tiles; a wavefront's 16-row pieces lie all on one side
  const int bsel = __builtin_amdgcn_readfirstlane(gated ? nk * (1 + ((w >> 1) & 1)) : nk);
  int nsteps = 0;
  for (int k = 0; k < nk; ++k) nsteps += ksz[k] / G2_K;
  int kt = 0, k0 = 0, K = sload_int(ksz);
  const bf16_t* A = (const bf16_t*)sload_ptr(ptrA);
  const bf16_t* B = (const bf16_t*)sload_ptr(ptrA + bsel);
  uint32_t offA[NLD], offB[NLD];
  auto set_offsets = [&]() {
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      offA[i] = (uint32_t)(rowA[i] * K + lcol) * 2u;
      offB[i] = (uint32_t)(rowB[i] * K + lcol) * 2u;
    }
  };
  set_offsets();
  const uint32_t lds0 = (uint32_t)(size_t)(lptr_t)lds;
  const uint32_t ldsw = __builtin_amdgcn_readfirstlane(lds0 + w * 1024);
  auto issue = [&](int stage) {  // loads of the K step (kt, k0) into `stage`, then advance
    const uint32_t dstA = ldsw + stage * STAGE_BYTES;
    const bf16_t* a = A + k0;
    const bf16_t* bq = B + k0;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      load_lds16_so(a, offA[i], dstA + i * 1024 * NW);
      load_lds16_so(bq, offB[i], dstA + OPER_BYTES + i * 1024 * NW);
    }
    k0 += G2_K;
    if (k0 >= K && kt + 1 < nk) {
      ++kt;
      k0 = 0;
      const int Kn = sload_int(ksz + kt);
      A = (const bf16_t*)sload_ptr(ptrA + kt);
      B = (const bf16_t*)sload_ptr(ptrA + bsel + kt);
      if (Kn != K) {
        K = Kn;
        set_offsets();
      }
    }
  };

  // fragment addresses inside a stage: row-major chunks, swizzled as above
  const int sw = (l32 >> 2) & 3;
  // With a residual operand (mode 1) the product is formed with the operands exchanged: the first MFMA
  // operand (TI fragments, 32 TI rows of its region per wavefront row wm) comes from B and the second (TJ
  // fragments, wavefront column wn) from A, so an accumulator tile is a piece of C^T and a lane holds runs of
  // four consecutive columns of one row -- 8-byte pieces of the residual's rows instead of single elements
  // (see store_c_rows).  The sums are the same sums.  (For the plain product this form measures 2 % slower
  // than the stores straight from the registers below, so only mode 1 takes it.)
  const bool exch = d.p.mode == 1;
  const int fragA = (exch ? OPER_BYTES : 0) + ((wm * 32 * TI + l32) * 4) * 16;
  const int fragB = (exch ? 0 : OPER_BYTES) + ((wn * 32 * TJ + l32) * 4) * 16;
  const int c0 = ((0 + g) ^ sw) * 16, c1 = ((2 + g) ^ sw) * 16;

  for (int s = 0; s < G2_STAGES - 1 && s < nsteps; ++s) issue(s);
  // Each step covers two MFMA slabs of 16 along K, held in the register sets (xa, xb) and
  // (ya, yb).  While the MFMAs of one slab run, the fragments of the next slab are read,
  // one LDS read after each MFMA: a wavefront can issue a short instruction in the shadow of
  // its own MFMA, so the reads cost no matrix-unit time, and both register sets keep their role
  // from step to step (no copies).  The second slab of a step is multiplied after the barrier
  // of the next step.
  bf16x8 xa[TI], xb[TJ], ya[TI], yb[TJ];
  const bool loads_first = __builtin_amdgcn_readfirstlane(TN_GEMM_STAGGER(w)) != 0;
#define TN_READ_SLAB(DA, DB, COL)                                                                      \
  _Pragma("unroll") for (int i = 0; i < TI; ++i) DA[i] = *(const bf16x8*)(st_ + fragA + i * 2048 + COL); \
  _Pragma("unroll") for (int j = 0; j < TJ; ++j) DB[j] = *(const bf16x8*)(st_ + fragB + j * 2048 + COL);
#define TN_MFMA_SLAB(SA, SB)                                  \
  _Pragma("unroll") for (int i = 0; i < TI; ++i)              \
  _Pragma("unroll") for (int j = 0; j < TJ; ++j) mfma_acc(acc[i][j], SA[i], SB[j]);
  // one MFMA, then one LDS read, for as many reads as a slab has; the remaining MFMAs follow
#define TN_INTERLEAVE()                                                          \
  _Pragma("unroll") for (int q = 0; q < (TI + TJ < TI * TJ ? TI + TJ : TI * TJ); ++q) { \
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                           \
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                           \
  }                                                                              \
  if constexpr (TI * TJ > TI + TJ) __builtin_amdgcn_sched_group_barrier(0x008, TI * TJ - (TI + TJ), 0);
  // stage s must have landed: at most the loads of the next two steps may still be in flight
  // (2 NLD load instructions per thread and step)
  constexpr int W2 = NLD == 4 ? 0x4F70 : 0x0F78, W1 = NLD == 4 ? 0x0F78 : 0x0F74;  // vmcnt(16 | 8), vmcnt(8 | 4)
  static_assert(NLD == 2 || NLD == 4, "the wait counts above are written for 4 or 8 loads per step");
  for (int s = 0; s < nsteps; ++s) {
    if (s + 2 < nsteps) __builtin_amdgcn_s_waitcnt(W2);
    else if (s + 1 < nsteps) __builtin_amdgcn_s_waitcnt(W1);
    else __builtin_amdgcn_s_waitcnt(0x0F70);                                         // vmcnt(0)
    __syncthreads();
    const char* st_ = lds + (s % G2_STAGES) * STAGE_BYTES;
    const bool more = s + G2_STAGES - 1 < nsteps;
    // Issuing a load stalls a wavefront for as long as the address path is busy with the loads
    // of the others, so the two wavefronts of a SIMD issue theirs at different points of a step.
    if (loads_first && more) issue((s + G2_STAGES - 1) % G2_STAGES);
    __builtin_amdgcn_sched_barrier(0);
    if (s > 0) {
      TN_MFMA_SLAB(ya, yb)
      TN_READ_SLAB(xa, xb, c0)
      TN_INTERLEAVE()
    } else {
      TN_READ_SLAB(xa, xb, c0)
    }
    __builtin_amdgcn_sched_barrier(0);
    if (!loads_first && more) issue((s + G2_STAGES - 1) % G2_STAGES);
    __builtin_amdgcn_sched_barrier(0);
    TN_MFMA_SLAB(xa, xb)
    TN_READ_SLAB(ya, yb, c1)
    TN_INTERLEAVE()
    __builtin_amdgcn_sched_barrier(0);
  }
  if (nsteps > 0) {
    TN_MFMA_SLAB(ya, yb)
  }
#undef TN_READ_SLAB
#undef TN_MFMA_SLAB
#undef TN_INTERLEAVE
  mfma_acc_drain();

  if (gated) {
    f32x16 act[TI][1];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float gt = acc[i][0][r];
        act[i][0][r] = gt / (1.f + __expf(-gt)) * acc[i][1][r];
      }
    store_c_tiles<TI, 1>(act, Cp, M, N, m0 + wm * 32 * TI, n0 + wn * 32, l32, g, false);
    return;
  }
  if (!exch) {
    store_c_tiles<TI, TJ>(acc, Cp, M, N, m0 + wm * 32 * TI, n0 + wn * 32 * TJ, l32, g, d.p.trans_c != 0);
    return;
  }
  // exchanged: this wavefront holds rows m0 + 32 TJ wn .. and columns n0 + 32 TI wm ..; it stores them in
  // two halves of 16 TI columns through LDS of its own, once nobody reads the last stage any more
  static_assert(NW * EpilogueStage<TI / 2, TJ>::BYTES <= G2_STAGES * STAGE_BYTES, "the epilogue's rows fit the stages' LDS");
  __syncthreads();
  char* const ep = lds + w * EpilogueStage<TI / 2, TJ>::BYTES;
  const bf16_t* R = (const bf16_t*)sload_ptr(ptrA + 2 * nk);
#pragma unroll
  for (int hf = 0; hf < 2; ++hf) {
    f32x16 part[TI / 2][TJ];
#pragma unroll
    for (int i = 0; i < TI / 2; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j) part[i][j] = acc[hf * (TI / 2) + i][j];
    store_c_rows<TI / 2, TJ>(part, ep, Cp, M, N, m0 + wn * 32 * TJ, n0 + wm * 32 * TI + hf * 16 * TI, lane, R);
  }
}

// ---------------------------------------------------------------------------------------------
// attention block on the vector ALUs: one thread per (query row, head), online softmax over
// the key rows in ascending order.  Serves fp32 graphs and shapes the MFMA kernel does not take.
// aux: [rows per Q tile, rows per K/V tile, columns per tile, q rows, kv rows]
// ---------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ const T* tile_elem(void* const* tiles, int nc, int t_rows, int t_cols, int row, int col) {
  const int rt = row / t_rows, ct = col / t_cols;
  return (const T*)tiles[rt * nc + ct] + (size_t)(row - rt * t_rows) * t_cols + (col - ct * t_cols);
}

// The same for a grid of transposed tiles: tile (rt, ct) holds [its columns, its rows]; the last
// row tile may be shorter, which changes its pitch.
template <typename T>
__device__ __forceinline__ const T* tile_elem_t(void* const* tiles, int nc, int t_rows, int t_cols, int total_rows,
                                                int row, int col) {
  const int rt = row / t_rows, ct = col / t_cols;
  const int pitch = min(t_rows, total_rows - rt * t_rows);
  return (const T*)tiles[rt * nc + ct] + (size_t)(col - ct * t_cols) * pitch + (row - rt * t_rows);
}

template <typename T, int HD>
__global__ void __launch_bounds__(64) attn_generic_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const int* ax = t.aux + d.aux0;
  const int tq = ax[0], tk = ax[1], tc = ax[2], q_rows = ax[3], kv_rows = ax[4];
  const int nc = d.p.n_col_tiles, gw = nc * tc;
  const int hpg = gw / HD;
  const int qblocks = (q_rows + 63) / 64;
  const int h = blockIdx.x / qblocks, row = (blockIdx.x % qblocks) * 64 + threadIdx.x;
  if (row >= q_rows) return;
  void* const* Qt = t.ptrs + d.ptr0;
  void* const* Kt = Qt + d.p.n_q_tiles * nc;
  void* const* Vt = Kt + d.p.n_kv_tiles * nc;
  float q[HD], o[HD];
#pragma unroll
  for (int c = 0; c < HD; ++c) {
    q[c] = ld(tile_elem<T>(Qt, nc, tq, tc, row, h * HD + c)) * d.p.scale;
    o[c] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  const int qpos = d.p.q_pos0 + row;
  for (int j = 0; j < kv_rows; ++j) {
    if (d.p.causal && d.p.k_pos0 + j > qpos) break;
    float s = 0.f;
#pragma unroll
    for (int c = 0; c < HD; ++c) s = fmaf(q[c], ld(tile_elem<T>(Kt, nc, tk, tc, j, h * HD + c)), s);
    const float mn = fmaxf(m, s);
    const float alpha = __expf(m - mn), p = __expf(s - mn);
    l = l * alpha + p;
#pragma unroll
    for (int c = 0; c < HD; ++c) {
      const float v = d.p.v_trans ? ld(tile_elem_t<T>(Vt, nc, tk, tc, kv_rows, j, h * HD + c))
                                  : ld(tile_elem<T>(Vt, nc, tk, tc, j, h * HD + c));
      o[c] = o[c] * alpha + p * v;
    }
    m = mn;
  }
  float* out = (float*)d.out + (size_t)row * d.cols;
#pragma unroll
  for (int c = 0; c < HD; ++c) out[h * HD + c] = o[c];
  out[gw + h] = m;
  out[gw + hpg + h] = l;
}

// ---------------------------------------------------------------------------------------------
// attention backward on the vector ALUs.  Modes 0 (statistics) and 1 (dQ): one thread per (query
// row, head), keys ascending.  Modes 2 (dK) and 3 (dV): one thread per (key row, head), queries
// ascending.  Scores are recomputed from Q and K; p = exp(scale q.k - lse).
// aux: [rows per Q tile, rows per K/V tile, columns per tile, q rows, kv rows]
// ---------------------------------------------------------------------------------------------
template <typename T, int HD>
__global__ void __launch_bounds__(64) attn_bwd_kernel(DeviceTables t, Batch b) {
  const OpDesc& d = t.descs[b.at(blockIdx.y)];
  if ((int)blockIdx.x >= d.nblocks) return;
  const int* ax = t.aux + d.aux0;
  const int tq = ax[0], tk = ax[1], tc = ax[2], q_rows = ax[3], kv_rows = ax[4];
  const int nc = d.p.n_col_tiles, gw = nc * tc, hpg = gw / HD, mode = d.p.mode;
  const int nq = d.p.n_q_tiles, nkv = d.p.n_kv_tiles;
  void* const* Qt = t.ptrs + d.ptr0;
  void* const* Kt = Qt + nq * nc;
  void* const* Vt = Kt + nkv * nc;
  void* const* Dt = Vt + nkv * nc;   // dO tiles
  void* const* St = Dt + nq * nc;    // statistics, one tensor per Q row tile (modes 1..3)
  const int my_rows = mode <= 1 ? q_rows : kv_rows;
  const int rblocks = (my_rows + 63) / 64;
  const int h = blockIdx.x / rblocks, row = (blockIdx.x % rblocks) * 64 + threadIdx.x;
  if (row >= my_rows) return;
  const float scale = d.p.scale;
  auto vel = [&](int j, int c) -> float {  // V[j, h*HD + c]
    return d.p.v_trans ? ld(tile_elem_t<T>(Vt, nc, tk, tc, kv_rows, j, h * HD + c))
                       : ld(tile_elem<T>(Vt, nc, tk, tc, j, h * HD + c));
  };
  auto stat = [&](int r, int which) -> float {  // which 0: lse, 1: D
    const int rt = r / tq;
    const float* s = (const float*)St[rt];
    return s[(size_t)(r - rt * tq) * (2 * hpg) + which * hpg + h];
  };
  if (mode <= 1) {
    const int qpos = d.p.q_pos0 + row;
    float acc[HD];
#pragma unroll
    for (int c = 0; c < HD; ++c) acc[c] = 0.f;
    float m = -INFINITY, l = 0.f, dsum = 0.f;  // mode 0: running maximum, sum of exp, sum of exp * dp
    const float lse = mode == 1 ? stat(row, 0) : 0.f, D = mode == 1 ? stat(row, 1) : 0.f;
    for (int j = 0; j < kv_rows; ++j) {
      if (d.p.causal && d.p.k_pos0 + j > qpos) break;
      float s = 0.f, dp = 0.f;
#pragma unroll 8
      for (int c = 0; c < HD; ++c) {
        s = fmaf(ld(tile_elem<T>(Qt, nc, tq, tc, row, h * HD + c)), ld(tile_elem<T>(Kt, nc, tk, tc, j, h * HD + c)), s);
        dp = fmaf(ld(tile_elem<T>(Dt, nc, tq, tc, row, h * HD + c)), vel(j, c), dp);
      }
      s *= scale;
      if (mode == 0) {
        const float mn = fmaxf(m, s);
        const float alpha = __expf(m - mn), p = __expf(s - mn);
        l = l * alpha + p;
        dsum = dsum * alpha + p * dp;
        m = mn;
      } else {
        const float ds = __expf(s - lse) * (dp - D) * scale;
#pragma unroll 8
        for (int c = 0; c < HD; ++c) acc[c] = fmaf(ds, ld(tile_elem<T>(Kt, nc, tk, tc, j, h * HD + c)), acc[c]);
      }
    }
    if (mode == 0) {
      float* out = (float*)d.out + (size_t)row * (2 * hpg);
      out[h] = m + __logf(l);
      out[hpg + h] = dsum / l;
    } else {
      T* out = (T*)d.out + (size_t)row * gw + h * HD;
#pragma unroll 8
      for (int c = 0; c < HD; ++c) st(out + c, acc[c]);
    }
  } else {
    const int kpos = d.p.k_pos0 + row;
    float acc[HD];
#pragma unroll
    for (int c = 0; c < HD; ++c) acc[c] = 0.f;
    for (int r = 0; r < q_rows; ++r) {
      if (d.p.causal && kpos > d.p.q_pos0 + r) continue;
      float s = 0.f, dp = 0.f;
#pragma unroll 8
      for (int c = 0; c < HD; ++c) {
        s = fmaf(ld(tile_elem<T>(Qt, nc, tq, tc, r, h * HD + c)), ld(tile_elem<T>(Kt, nc, tk, tc, row, h * HD + c)), s);
        if (mode == 2) dp = fmaf(ld(tile_elem<T>(Dt, nc, tq, tc, r, h * HD + c)), vel(row, c), dp);
      }
      const float p = __expf(s * scale - stat(r, 0));
      if (mode == 2) {
        const float ds = p * (dp - stat(r, 1)) * scale;
#pragma unroll 8
        for (int c = 0; c < HD; ++c) acc[c] = fmaf(ds, ld(tile_elem<T>(Qt, nc, tq, tc, r, h * HD + c)), acc[c]);
      } else {
#pragma unroll 8
        for (int c = 0; c < HD; ++c) acc[c] = fmaf(p, ld(tile_elem<T>(Dt, nc, tq, tc, r, h * HD + c)), acc[c]);
      }
    }
    T* out = (T*)d.out + (size_t)row * gw + h * HD;
#pragma unroll 8
    for (int c = 0; c < HD; ++c) st(out + c, acc[c]);
  }
}

// ---------------------------------------------------------------------------------------------
// MFMA attention backward (bf16 storage, V given as plain [keys, columns] tiles).
//
// Modes 0 (statistics) and 1 (dQ): one workgroup = one head x 128 queries, a wavefront owns 32
// queries and a lane one of them (its MFMA column), exactly as in the forward kernel: per 32 keys
// it forms S^T = K Q^T and dP^T = V dO^T with the key rows fed in the permuted order that leaves a
// lane with 8 consecutive keys per 16-key slab, so that dS^T is directly the B operand of
// dQ^T += K^T dS^T; the A operand is a 16-byte read of a row of a K^T tile.
// Modes 2 (dK) and 3 (dV): one workgroup = one head x 128 keys, a lane owns a key; per 32 queries
// S = Q K^T and dP = dO V^T with the query rows permuted likewise, and dK^T += Q^T dS,
// dV^T += dO^T P read rows of Q^T / dO^T tiles.
// The eight wavefronts of a workgroup need the same rows of the other side: the workgroup brings
// them in 64 rows at a time through two LDS stages filled by direct global-to-LDS loads (the next
// chunk arrives while the current one is multiplied), together with the statistics of those rows.
// Probabilities and dS enter the MFMA as single bf16.
// aux: [rows per Q tile, rows per K/V tile, columns per tile, q rows, kv rows]
// ---------------------------------------------------------------------------------------------
// two floats rounded to bf16 (nearest even), the first in the low half
__device__ __forceinline__ uint32_t pack_bf16_pair(float a, float b) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  return __builtin_bit_cast(uint32_t, __builtin_convertvector((f32x2_t){a, b}, bf16x2_t));
}

constexpr int kAttnBwdThreads = 512, kAttnBwdRows = 256;  // eight wavefronts of 32 rows
constexpr int kAttnBwdChunk = 64;                          // rows of the other side staged per round
constexpr int attn_bwd_lds(int hd) { return 2 * 3 * kAttnBwdChunk * hd * 2 + 2 * 2 * kAttnBwdChunk * 4; }
template <int HD, int mode>
__global__ void __launch_bounds__(kAttnBwdThreads) attn_bwd_bf16_kernel(DeviceTables t, Batch b) {
  int bx, by;
  xcd_remap_rows(bx, by);
  const OpDesc& d = t.descs[b.at(by)];
  if (bx >= d.nblocks) return;
  constexpr int CH = kAttnBwdChunk;  // rows of the other side per round
  constexpr int CPR = HD / 8;        // 16-byte pieces per row of a [CH][HD] chunk
  constexpr int ABYTES = CH * HD * 2, STAGE = 3 * ABYTES;  // K | V | K^T (or Q | dO | Q^T or dO^T): equal sizes
  // two stages, then the statistics (lse * log2(e), D) of the queries of both stages
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  float* const bufS = (float*)(lds + 2 * STAGE);
  const int* ax = t.aux + d.aux0;
  const int tq = ax[0], tk = ax[1], tc = ax[2], q_rows = ax[3], kv_rows = ax[4];
  const int nc = d.p.n_col_tiles, gw = nc * tc, hpg = gw / HD;  // mode (template) == d.p.mode: its own launch class
  const int nq = d.p.n_q_tiles, nkv = d.p.n_kv_tiles;
  void* const* Qt = t.ptrs + d.ptr0;
  void* const* Kt = Qt + nq * nc;
  void* const* Vt = Kt + nkv * nc;
  void* const* Dt = Vt + nkv * nc;  // dO tiles
  void* const* St = Dt + nq * nc;   // statistics per Q row tile (modes 1..3)
  void* const* Tt = St + nq;        // transposed grid (modes 1..3)
  const int my_rows = mode <= 1 ? q_rows : kv_rows;
  const int rblocks = (my_rows + kAttnBwdRows - 1) / kAttnBwdRows;
  const int h = bx / rblocks, rb = bx % rblocks;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, l32 = lane & 31, g = lane >> 5;
  const int myrow = rb * kAttnBwdRows + w * 32 + l32;  // this lane's query (modes 0, 1) or key (modes 2, 3)
  const bool valid = myrow < my_rows;
  constexpr float LOG2E = 1.44269504088896340736f, LN2 = 0.69314718055994530942f;
  const float scale = d.p.scale, scale2 = scale * LOG2E;
  const int causal = d.p.causal;
  const int a_ = l32 >> 3, b_ = l32 & 3, g_ = (l32 >> 2) & 1;
  const int perm = 16 * (a_ >> 1) + 8 * g_ + 4 * (a_ & 1) + b_;  // row i of an MFMA tile is fed row perm(i)
  auto frag = [&](void* const* grid, int t_rows, int row, int col) -> bf16x8 {
    uint4 v = *(const uint4*)tile_elem<bf16_t>(grid, nc, t_rows, tc, row, col);
    return *(bf16x8*)&v;
  };
  auto stat = [&](int r, int which) -> float {
    const int rt = r / tq;
    return ((const float*)St[rt])[(size_t)(r - rt * tq) * (2 * hpg) + which * hpg + h];
  };
  // the other side: keys for modes 0 and 1, queries for modes 2 and 3
  void* const* gridA = mode <= 1 ? Kt : Qt;
  void* const* gridB = mode <= 1 ? Vt : Dt;
  const int o_trows = mode <= 1 ? tk : tq, o_rows = mode <= 1 ? kv_rows : q_rows;
  // Rows [row0, row0 + CH) of the other side go to LDS stage `stg` by direct global-to-LDS loads:
  // piece p = i*512 + tid of an operand lands at byte 16 p.  [CH][HD] chunks: row p / CPR, and the
  // piece stored at p % CPR is piece (p % CPR) ^ swizzle(row) of that row; the transposed [HD][CH]
  // chunk: row p / 8, stored piece p % 8 is piece (p % 8) ^ ((row >> 1) & 7).  The swizzles keep
  // the fragment reads below free of bank conflicts without padding, which these loads cannot do.
  // A head's columns lie inside one column tile and a chunk inside one row tile (the executor
  // checks both), so the tile pointers are wavefront-uniform and change rarely.
  const uint32_t lds0 = (uint32_t)(size_t)(lptr_t)lds;
  const int ct = (h * HD) / tc, cin0 = (h * HD) % tc;
  int rt = -1, trows = 0;
  const bf16_t* At = nullptr;
  const bf16_t* Bt = nullptr;
  const bf16_t* Tp = nullptr;
  auto issue = [&](int row0, int stg) {
    const int nrt = row0 / o_trows;
    if (nrt != rt) {
      rt = nrt;
      At = (const bf16_t*)sload_ptr((const void* const*)(gridA + rt * nc + ct));
      if (mode != 3) Bt = (const bf16_t*)sload_ptr((const void* const*)(gridB + rt * nc + ct));
      if (mode >= 1) Tp = (const bf16_t*)sload_ptr((const void* const*)(Tt + rt * nc + ct));
      trows = min(o_trows, o_rows - rt * o_trows);
    }
    const int rin = row0 - rt * o_trows;
    const uint32_t dst = __builtin_amdgcn_readfirstlane(lds0 + stg * STAGE + w * 1024);
#pragma unroll
    for (int i = 0; i < CH * CPR / kAttnBwdThreads; ++i) {
      const int p = i * kAttnBwdThreads + threadIdx.x, r = p / CPR;
      const int col = cin0 + (((p % CPR) ^ (CPR == 16 ? (r & 15) : ((r >> 1) & 7))) * 8);
      const int gr = min(rin + r, trows - 1);  // rows past the end: any valid row, their weights are zero
      load_lds16(At + (size_t)gr * tc + col, dst + i * (kAttnBwdThreads * 16));
      if (mode != 3) load_lds16(Bt + (size_t)gr * tc + col, dst + ABYTES + i * (kAttnBwdThreads * 16));
    }
    if (mode >= 1) {
#pragma unroll
      for (int i = 0; i < HD * (CH / 8) / kAttnBwdThreads; ++i) {
        const int p = i * kAttnBwdThreads + threadIdx.x, dd = p / 8;
        const int r8 = min(rin + ((p % 8) ^ ((dd >> 1) & 7)) * 8, trows - 8);  // 8 rows at once
        load_lds16(Tp + (size_t)(cin0 + dd) * trows + r8, dst + 2 * ABYTES + i * (kAttnBwdThreads * 16));
      }
    }
  };
  // the statistics of a chunk's queries (modes 2, 3) travel through a register of the first 2 CH lanes
  auto load_stat = [&](int row0) -> float {
    if (mode < 2 || threadIdx.x >= 2 * CH) return 0.f;
    const int r = threadIdx.x >> 1, which = threadIdx.x & 1;
    const float v = stat(min(row0 + r, q_rows - 1), which);
    return which ? v : v * LOG2E;
  };
  f32x16 acc[HD / 32];
#pragma unroll
  for (int i = 0; i < HD / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;

  bf16x8 mine[HD / 16], mine2[HD / 16];  // this lane's own row: Q and dO (modes 0, 1) or K and V (modes 2, 3)
  {
    const int r = min(myrow, my_rows - 1);
#pragma unroll
    for (int s = 0; s < HD / 16; ++s) {
      mine[s] = frag(mode <= 1 ? Qt : Kt, mode <= 1 ? tq : tk, r, h * HD + s * 16 + g * 8);
      mine2[s] = frag(mode <= 1 ? Dt : Vt, mode <= 1 ? tq : tk, r, h * HD + s * 16 + g * 8);
    }
  }
  const int mypos = (mode <= 1 ? d.p.q_pos0 : d.p.k_pos0) + myrow;
  float lse2 = 0.f, Dq = 0.f, m = -INFINITY, l = 0.f, dsum = 0.f;
  if (mode == 1) {
    lse2 = stat(min(myrow, q_rows - 1), 0) * LOG2E;
    Dq = stat(min(myrow, q_rows - 1), 1);
  }
  // range of the other side that this workgroup can see at all
  int begin = 0, end = o_rows;
  if (causal && mode <= 1) end = min(kv_rows, d.p.q_pos0 + rb * kAttnBwdRows + kAttnBwdRows - d.p.k_pos0);
  if (causal && mode >= 2) begin = max(0, d.p.k_pos0 + rb * kAttnBwdRows - d.p.q_pos0) & ~(CH - 1);

  // fragment addresses inside a stage (see the layouts above)
  const int kx0 = (g ^ (CPR == 16 ? (perm & 15) : ((perm >> 1) & 7))) * 16;
  const int vsw = (l32 >> 1) & 7;
  float snext = 0.f;
  if (begin < end) {
    issue(begin, 0);
    snext = load_stat(begin);
  }
  int stg = 0;
  for (int row0 = begin; row0 < end; row0 += CH, stg ^= 1) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this chunk and its statistics have arrived
    float* const sbuf = bufS + stg * (2 * CH);
    if (mode >= 2 && threadIdx.x < 2 * CH) sbuf[threadIdx.x] = snext;
    __syncthreads();  // ... for everybody, and everybody is done with the chunk before
    if (row0 + CH < end) {
      issue(row0 + CH, stg ^ 1);
      snext = load_stat(row0 + CH);
    }
    const char* const bufA = lds + stg * STAGE;
#pragma unroll 1
    for (int sub = 0; sub < CH / 32; ++sub) {
      const int base = row0 + sub * 32;
      if (base >= end) break;
      int kx = kx0;
      asm volatile("" : "+v"(kx));  // formed where it is used, not kept ready for every s
      const char* ra = bufA + (sub * 32 + perm) * (CPR * 16);
      f32x16 sc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sc[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int s = 0; s < HD / 16; ++s) {
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)(ra + (kx ^ (32 * s))), mine[s], sc, 0, 0, 0);
        if (mode != 3) dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)(ra + ABYTES + (kx ^ (32 * s))), mine2[s], dp, 0, 0, 0);
      }
      // register r of this lane: row base + 16*(r>>3) + 8*g + (r&7) of the other side
      if (mode == 0) {
        // the maximum is taken over the raw products (a positive scale commutes with it); a slab
        // inside the matrix and wholly visible to every query of the wavefront needs no mask
        const int wq0 = d.p.q_pos0 + rb * kAttnBwdRows + w * 32;
        float mx = -INFINITY;
        if (base + 32 > kv_rows || (causal && d.p.k_pos0 + base + 31 > wq0)) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kv = base + 16 * (r >> 3) + 8 * g + (r & 7);
            const bool ok = kv < kv_rows && !(causal && d.p.k_pos0 + kv > mypos);
            sc[r] = ok ? sc[r] : -INFINITY;
            mx = fmaxf(mx, sc[r]);
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[r]);
        }
        const float mn = fmaxf(m, mx * scale2);
        if (mn != -INFINITY) {
          const float alpha = __builtin_amdgcn_exp2f(m - mn);
          float ls = 0.f, ds = 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[r], scale2, -mn));
            ls += p;
            ds = fmaf(p, dp[r], ds);
          }
          l = l * alpha + ls;
          dsum = dsum * alpha + ds;
          m = mn;
        }
        continue;
      }
      // Weights of the 32 x 32 pairs of this slab: p (mode 3) or p (dp - D) (modes 1, 2; the factor
      // `scale` of dS is applied to the finished sums).  A slab that lies wholly inside the matrix and
      // on the visible side of the diagonal for every row of the wavefront needs no mask.
      const int wrow0 = rb * kAttnBwdRows + w * 32;  // first row of this wavefront
      bool need_mask;
      if (mode == 1) {
        need_mask = base + 32 > kv_rows || (causal && d.p.k_pos0 + base + 31 > d.p.q_pos0 + wrow0);
      } else {
        need_mask = wrow0 + 32 > my_rows || base + 32 > q_rows || (causal && d.p.k_pos0 + wrow0 + 31 > d.p.q_pos0 + base);
      }
      float pr[16];
      if (need_mask) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int lr = sub * 32 + 16 * (r >> 3) + 8 * g + (r & 7), o = row0 + lr;
          bool ok;
          if (mode == 1) ok = o < kv_rows && !(causal && d.p.k_pos0 + o > mypos);
          else ok = valid && o < q_rows && !(causal && mypos > d.p.q_pos0 + o);
          float p;
          if (mode == 1) p = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[r], scale2, -lse2)) * (dp[r] - Dq);
          else p = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[r], scale2, -sbuf[lr * 2]));
          if (mode == 2) p *= dp[r] - sbuf[lr * 2 + 1];
          pr[r] = ok ? p : 0.f;
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int lr = sub * 32 + 16 * (r >> 3) + 8 * g + (r & 7);
          float p;
          if (mode == 1) p = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[r], scale2, -lse2)) * (dp[r] - Dq);
          else p = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[r], scale2, -sbuf[lr * 2]));
          if (mode == 2) p *= dp[r] - sbuf[lr * 2 + 1];
          pr[r] = p;
        }
      }
      union { uint32_t u[4]; bf16x8 v; } s0u, s1u;
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const uint32_t pk = pack_bf16_pair(pr[r], pr[r + 1]);
        if (r < 8) s0u.u[r >> 1] = pk; else s1u.u[(r - 8) >> 1] = pk;
      }
      const bf16x8 s0 = s0u.v, s1 = s1u.v;
#pragma unroll
      for (int i = 0; i < HD / 32; ++i) {
        const char* tr = bufA + 2 * ABYTES + (i * 32 + l32) * 128;  // i * 32 leaves the swizzle of the row alone
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)(tr + ((sub * 4 + g) ^ vsw) * 16), s0, acc[i], 0, 0, 0);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)(tr + ((sub * 4 + 2 + g) ^ vsw) * 16), s1, acc[i], 0, 0, 0);
      }
    }
  }
  if (mode == 0) {
    // the two halves of the wavefront saw different keys of the same query: merge their states
    const float m2 = __shfl_xor(m, 32, 64), l2 = __shfl_xor(l, 32, 64), d2 = __shfl_xor(dsum, 32, 64);
    const float mn = fmaxf(m, m2);
    const float w1 = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - mn), w2 = m2 == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m2 - mn);
    const float lt = l * w1 + l2 * w2, dt = dsum * w1 + d2 * w2;
    if (valid && g == 0) {
      float* out = (float*)d.out + (size_t)myrow * (2 * hpg);
      out[h] = (mn + __builtin_amdgcn_logf(lt)) * LN2;
      out[hpg + h] = dt / lt;
    }
    return;
  }
  if (!valid) return;
  // accumulator tile i: this lane holds column myrow and rows (= head columns) 8a + 4g + k of it
  bf16_t* out = (bf16_t*)d.out + (size_t)myrow * gw + h * HD;
  const float oscale = mode == 3 ? 1.f : scale;  // dS = scale * p (dp - D): the factor left out above
#pragma unroll
  for (int i = 0; i < HD / 32; ++i)
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      uint2 v;
      v.x = (uint32_t)f2bf(acc[i][4 * a] * oscale) | ((uint32_t)f2bf(acc[i][4 * a + 1] * oscale) << 16);
      v.y = (uint32_t)f2bf(acc[i][4 * a + 2] * oscale) | ((uint32_t)f2bf(acc[i][4 * a + 3] * oscale) << 16);
      *(uint2*)(out + i * 32 + 8 * a + 4 * g) = v;
    }
}

// ---------------------------------------------------------------------------------------------
// MFMA attention block (bf16 storage, V given as V^T tiles).  One workgroup = one head x 128 query
// rows; each of its 4 wavefronts owns 32 query rows; two workgroups share a compute unit.
//
// Per 32 keys a wavefront forms the *transposed* score tile S^T = K Q^T, so that a lane owns one
// query (its column) and the softmax statistics are per-lane scalars.  The rows of S^T are fed
// with the keys in a permuted order, pi(i) = 16*(a>>1) + 8*g + 4*(a&1) + b for i = 8a + 4g + b,
// chosen so that the 8 probabilities a lane holds per 16-key slab belong to 8 consecutive keys:
// P^T is then already the B operand of O^T += V^T P^T, and the A operand is a plain 16-byte read
// of a V^T row.  K and V^T chunks of 64 keys are double-buffered in LDS and filled by direct
// global-to-LDS loads; conflicts are avoided by swizzling which chunk each lane fetches.
// ---------------------------------------------------------------------------------------------
// two weights as a pair of bf16 (hi) and the bf16 of what that rounding left over (lo), packed
__device__ __forceinline__ void split_bf16_pair(float a, float b, uint32_t& hi, uint32_t& lo) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const bf16x2_t h = __builtin_convertvector((f32x2_t){a, b}, bf16x2_t);
  hi = __builtin_bit_cast(uint32_t, h);
  const float ha = __uint_as_float(hi << 16), hb = __uint_as_float(hi & 0xFFFF0000u);
  const bf16x2_t r = __builtin_convertvector((f32x2_t){a - ha, b - hb}, bf16x2_t);
  lo = __builtin_bit_cast(uint32_t, r);
}

constexpr float kLazy = 8.f;  // see the rescaling step of attn_bf16_kernel

template <int HD>
__global__ void __launch_bounds__(256, 2) attn_bf16_kernel(DeviceTables t, Batch b) {
  int bx, by;
  xcd_remap_rows(bx, by);
  const OpDesc& d = t.descs[b.at(by)];
  if (bx >= d.nblocks) return;
  constexpr int KC = 64;                   // keys per iteration
  constexpr int CPR = HD / 8;              // 16-byte chunks per K row
  constexpr int KBYTES = KC * HD * 2, BUF = 2 * KBYTES;  // K chunk, then V^T chunk [HD][KC]
  constexpr int NLD = KC * CPR / 256;      // wave-instructions per thread and operand
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int* ax = t.aux + d.aux0;
  const int tq = ax[0], tk = ax[1], tc = ax[2], q_rows = ax[3], kv_rows = ax[4];
  const int nc = d.p.n_col_tiles, gw = nc * tc, hpg = gw / HD;
  const int qblocks = (q_rows + 127) / 128;
  const int h = bx / qblocks, qb = bx % qblocks;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, l32 = lane & 31, g = lane >> 5;
  void* const* Qp = t.ptrs + d.ptr0;
  void* const* Kp = Qp + d.p.n_q_tiles * nc;
  void* const* Vp = Kp + d.p.n_kv_tiles * nc;
  const int qrow = qb * 128 + w * 32 + l32;
  const bool qvalid = qrow < q_rows;
  const float scale = d.p.scale;
  const int causal = d.p.causal, k_pos0 = d.p.k_pos0;
  const int qpos = d.p.q_pos0 + qrow;
  float* const outp = (float*)d.out;
  const int ldo = d.cols;

  bf16x8 qf[HD / 16];
#pragma unroll
  for (int s = 0; s < HD / 16; ++s) {
    uint4 v = *(const uint4*)tile_elem<bf16_t>(Qp, nc, tq, tc, min(qrow, q_rows - 1), h * HD + s * 16 + g * 8);
    qf[s] = *(bf16x8*)&v;
  }
  f32x16 ot[HD / 32];
#pragma unroll
  for (int i = 0; i < HD / 32; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) ot[i][r] = 0.f;
  float m = -INFINITY, l = 0.f;
  int kv_end = kv_rows;  // keys above the diagonal of this workgroup's rows contribute nothing
  if (causal) kv_end = min(kv_rows, d.p.q_pos0 + qb * 128 + 128 - k_pos0);
  const int niter = (kv_end + KC - 1) / KC;

  // loader: operand chunk p = i*256 + tid.  K: row p / CPR, stored chunk p % CPR holds logical
  // chunk (p % CPR) ^ swizzle(row).  V^T: row (= head column) p / 8, stored chunk p % 8.
  // A head's columns lie inside one column tile and a chunk of 64 keys inside one row tile (the
  // executor checks both), so the tile pointers are wavefront-uniform and change rarely.
  const uint32_t lds0 = (uint32_t)(size_t)(lptr_t)lds;
  const int ct = (h * HD) / tc, cin0 = (h * HD) % tc;
  int kr_[NLD], kcol_[NLD], vrow_[NLD], vkv_[NLD];
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    const int p = i * 256 + threadIdx.x;
    const int kr = p / CPR;
    kr_[i] = kr;
    kcol_[i] = cin0 + (((p % CPR) ^ (CPR == 16 ? (kr & 15) : ((kr >> 1) & 7))) * 8);
    const int vr = p / 8;
    vrow_[i] = cin0 + vr;
    vkv_[i] = ((p % 8) ^ ((vr >> 1) & 7)) * 8;
  }
  int rt = -1;                 // row tile the current chunk lies in
  const bf16_t* Kt = nullptr;  // its K tile and V^T tile
  const bf16_t* Vt = nullptr;
  int trows = 0;               // rows of that tile
  auto issue = [&](int it, int buf) {
    const int kv0 = it * KC;
    const int nrt = kv0 / tk;
    if (nrt != rt) {
      rt = nrt;
      Kt = (const bf16_t*)sload_ptr((const void* const*)(Kp + rt * nc + ct));
      Vt = (const bf16_t*)sload_ptr((const void* const*)(Vp + rt * nc + ct));
      trows = min(tk, kv_rows - rt * tk);
    }
    const int kin = kv0 - rt * tk;
    const uint32_t dst = __builtin_amdgcn_readfirstlane(lds0 + buf * BUF + w * 1024);
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int krow = min(kin + kr_[i], trows - 1);  // rows past the end: any valid row, masked later
      load_lds16(Kt + (size_t)krow * tc + kcol_[i], dst + i * 4096);
      int kv = kin + vkv_[i];
      if (kv >= trows) kv = 0;  // multiplied by zero probabilities; any valid data will do
      load_lds16(Vt + (size_t)vrow_[i] * trows + kv, dst + KBYTES + i * 4096);
    }
  };

  constexpr float LOG2E = 1.44269504088896340736f;
  const float scale2 = scale * LOG2E;  // scores are kept in units of log2: exp(x) = exp2(x * log2 e)
  // first query row of this wavefront: a chunk whose last key is not after it needs no mask
  const int qpos_w0 = d.p.q_pos0 + qb * 128 + w * 32;
  const int a_ = l32 >> 3, b_ = l32 & 3, g_ = (l32 >> 2) & 1;
  const int kperm = 16 * (a_ >> 1) + 8 * g_ + 4 * (a_ & 1) + b_;

  if (niter > 0) issue(0, 0);
  for (int it = 0; it < niter; ++it) {
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this iteration's chunk has landed
    __syncthreads();                     // ... for everybody, and the other buffer is free
    if (it + 1 < niter) issue(it + 1, (it + 1) & 1);
    const char* kb = lds + (it & 1) * BUF;
    const char* vb = kb + KBYTES;
#pragma unroll
    for (int sub = 0; sub < 2; ++sub) {
      // S^T: row i of the MFMA tile is key pi(i)
      const int krow = sub * 32 + kperm;
      const int ksw = CPR == 16 ? (krow & 15) : ((krow >> 1) & 7);
      f32x16 sT;
#pragma unroll
      for (int r = 0; r < 16; ++r) sT[r] = 0.f;
#pragma unroll
      for (int s = 0; s < HD / 16; ++s) {
        bf16x8 a = *(const bf16x8*)(kb + (krow * CPR + ((2 * s + g) ^ ksw)) * 16);
        sT = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[s], sT, 0, 0, 0);
      }
      // register r = 4a + b of this lane is the score of key 16*(a>>1) + 8g + 4*(a&1) + b
      const int kvs = it * KC + sub * 32;
      const bool need_mask = kvs + 32 > kv_rows || (causal && k_pos0 + kvs + 31 > qpos_w0);
      // the maximum is taken over the raw products: scaling by a positive factor commutes with it
      float mx = -INFINITY;
      if (need_mask) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = kvs + 16 * (r >> 3) + 8 * g + (r & 7);
          const bool ok = kv < kv_rows && !(causal && k_pos0 + kv > qpos);
          sT[r] = ok ? sT[r] : -INFINITY;
          mx = fmaxf(mx, sT[r]);
        }
      } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sT[r]);
      }
      mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * scale2;
      const float mn = fmaxf(m, mx);
      // What is summed so far is rescaled only when the maximum of some query of the wavefront has
      // grown by more than kLazy (in units of log2): until then probabilities are taken relative to
      // the older maximum and stay below 2^kLazy, which costs fp32 and the bf16 pair nothing.
      if (__any(mn > m + kLazy)) {
        const float alpha = mn == -INFINITY ? 1.f : __builtin_amdgcn_exp2f(m - mn);
        l *= alpha;
#pragma unroll
        for (int i = 0; i < HD / 32; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) ot[i][r] *= alpha;
        m = mn;
      }
      const float msub = m == -INFINITY ? 0.f : m;  // nothing visible yet: every probability is exp2(-inf) = 0
      // Probabilities enter the MFMA as bf16.  A single bf16 would carry 8 bits of each weight;
      // the remainder p - bf16(p) is fed through a second MFMA, so that the product sees 16 bits
      // and the block's result does not depend on where the running maximum stood.
      union { uint32_t u[4]; bf16x8 v; } p0, p1, q0, q1;
      float ls = 0.f;
#pragma unroll
      for (int r = 0; r < 16; r += 2) {
        const float pa = __builtin_amdgcn_exp2f(__builtin_fmaf(sT[r], scale2, -msub));
        const float pb = __builtin_amdgcn_exp2f(__builtin_fmaf(sT[r + 1], scale2, -msub));
        ls += pa + pb;
        uint32_t hi, lo;
        split_bf16_pair(pa, pb, hi, lo);
        if (r < 8) { p0.u[r >> 1] = hi; q0.u[r >> 1] = lo; } else { p1.u[(r - 8) >> 1] = hi; q1.u[(r - 8) >> 1] = lo; }
      }
      l += ls;
      // O^T[d, q] += sum over the slab's 16 keys of V^T[d, key] P^T[key, q]
#pragma unroll
      for (int i = 0; i < HD / 32; ++i) {
        const int dr = i * 32 + l32, vsw = (dr >> 1) & 7;
        bf16x8 a0 = *(const bf16x8*)(vb + (dr * 8 + ((sub * 4 + g) ^ vsw)) * 16);
        bf16x8 a1 = *(const bf16x8*)(vb + (dr * 8 + ((sub * 4 + 2 + g) ^ vsw)) * 16);
        ot[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, q0.v, ot[i], 0, 0, 0);
        ot[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, q1.v, ot[i], 0, 0, 0);
        ot[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, p0.v, ot[i], 0, 0, 0);
        ot[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, p1.v, ot[i], 0, 0, 0);
      }
    }
  }
  m *= 0.69314718055994530942f;  // back to natural-log units for the combine step
  l += __shfl_xor(l, 32, 64);
  if (!qvalid) return;
  float* out = outp + (size_t)qrow * ldo;
#pragma unroll
  for (int i = 0; i < HD / 32; ++i)
#pragma unroll
    for (int a = 0; a < 4; ++a) {
      float* o4 = out + h * HD + i * 32 + 8 * a + 4 * g;
      if ((ldo & 3) == 0) {  // rows of the partial are 16-byte aligned
        *(float4*)o4 = make_float4(ot[i][4 * a], ot[i][4 * a + 1], ot[i][4 * a + 2], ot[i][4 * a + 3]);
      } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) o4[k] = ot[i][4 * a + k];
      }
    }
  if (g == 0) {
    out[gw + h] = m;
    out[gw + hpg + h] = l;
  }
}

// ---------------------------------------------------------------------------------------------
// grouped tensor copy (see kernels.h).  The copies of a group are cut into 32 KiB pieces; a
// small, fixed number of 1024-lane workgroups walks over them, two 16-byte loads in flight per
// lane.  What keeps the host link busy is the number of waves with a load outstanding, not the
// loads per wave (measured: 8 such workgroups reach 56 GB/s, the rate of the copy engines).
// The large GEMM kernel needs a whole compute unit for one workgroup, so every compute unit
// that holds a copy workgroup is lost to it (see `held` below): hence few, wide workgroups.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kCopyThreads) copy_kernel(CopyBatch b) {
  // What a lane has loaded waits in LDS, each lane in a place of its own (no barrier): 32 KiB per workgroup, which is
  // what keeps a copy workgroup off a compute unit that holds a workgroup of the 256x256 tile product (128 KiB
  // of the 160) or two of the attention kernel.  Sharing a unit with those costs them far more than the unit is
  // worth to the copy (measured with the data held in registers instead: tile products 970 -> 610 TFLOP/s on the
  // 80-layer workload); reserving 96 KiB instead costs the compute-bound workloads 5-13 %.
  __shared__ uint4 held[kCopyLoads][kCopyThreads];
  int item = 0;
  for (uint32_t g = blockIdx.x; g < (uint32_t)b.total_blocks; g += gridDim.x) {
    while (item + 1 < b.n && g >= b.it[item + 1].first_block) ++item;
    const CopyItem it = b.it[item];
    const uint32_t off = (g - it.first_block) * kCopyBlockBytes;
    const uint32_t len = min(kCopyBlockBytes, it.bytes - off);
    const char* src = (const char*)it.src + off;
    char* dst = (char*)it.dst + off;
    const uint32_t vec = len / 16;  // whole 16-byte pieces (tensor locations are 256-byte aligned)
#pragma unroll
    for (int k = 0; k < kCopyLoads; ++k) {
      const uint32_t i = threadIdx.x + kCopyThreads * k;
      if (i < vec) held[k][threadIdx.x] = ((const uint4*)src)[i];
    }
#pragma unroll
    for (int k = 0; k < kCopyLoads; ++k) {
      const uint32_t i = threadIdx.x + kCopyThreads * k;
      if (i < vec) ((uint4*)dst)[i] = held[k][threadIdx.x];
    }
    const uint32_t tail = vec * 16 + threadIdx.x;
    if (tail < len) dst[tail] = src[tail];
  }
}

}  // namespace

// ---------------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------------
static inline int32_t cdiv(int64_t a, int64_t b) { return (int32_t)((a + b - 1) / b); }

int32_t blocks_for(int cls, const OpDesc& d, const int32_t* aux) {
  switch (cls) {
    case LC_GEMM_F32: return cdiv(d.rows, 64) * cdiv(d.cols, 64);
    case LC_GEMM_BF16_NT: return cdiv(d.rows, GB_M) * cdiv(d.cols, GB_N);
    case LC_GEMM_BF16_NT256: return cdiv(d.rows, 256) * cdiv(d.cols, d.p.mode == 2 ? 128 : 256);
    case LC_RMS_STAT: return cdiv(d.rows, 4);
    case LC_RMS_APPLY: return cdiv((int64_t)d.rows * cdiv(d.cols, 8), 256);
    case LC_ROPE:
      return rope_whole_heads(d) ? cdiv((int64_t)d.rows * (d.p.head_dim / 8), 256) : cdiv((int64_t)d.rows * (d.cols / 2), 256);
    case LC_ATTN_F32: {
      const int gw = d.p.n_col_tiles * aux[d.aux0 + 2];
      return (gw / d.p.head_dim) * cdiv(aux[d.aux0 + 3], 64);
    }
    case LC_ATTN_BF16: {
      const int gw = d.p.n_col_tiles * aux[d.aux0 + 2];
      return (gw / d.p.head_dim) * cdiv(aux[d.aux0 + 3], 128);
    }
    case LC_ATTN_COMBINE: return cdiv((int64_t)d.rows * d.cols / (combine_by_four(d) ? 4 : 1), 256);
    case LC_SILU_MUL:
    case LC_ADD:
    case LC_SILU_BWD: return cdiv((int64_t)d.rows * d.cols, 256 * 8);
    case LC_TRANSPOSE: return cdiv(d.rows, 64) * cdiv(d.cols, 64);
    case LC_ZERO: return cdiv((int64_t)d.rows * d.cols * (d.dtype == TN_BF16 ? 2 : 4), 256 * 16);
    case LC_SOFTMAX_STAT: return cdiv(d.rows, 4);
    case LC_SOFTMAX_APPLY: return cdiv((int64_t)d.rows * cdiv(d.cols, 8), 256);
    case LC_RMS_BWD_STAT: return cdiv(d.rows, 4);
    case LC_RMS_BWD_APPLY: return cdiv((int64_t)d.rows * cdiv(d.cols, 8), 256);
    case LC_ATTN_BWD: {
      const int gw = d.p.n_col_tiles * aux[d.aux0 + 2];
      return (gw / d.p.head_dim) * cdiv(aux[d.aux0 + (d.p.mode <= 1 ? 3 : 4)], 64);
    }
    case LC_ATTN_BWD_BF16:
    case LC_ATTN_BWD_BF16_DQ:
    case LC_ATTN_BWD_BF16_DK:
    case LC_ATTN_BWD_BF16_DV: {
      const int gw = d.p.n_col_tiles * aux[d.aux0 + 2];
      return (gw / d.p.head_dim) * cdiv(aux[d.aux0 + (d.p.mode <= 1 ? 3 : 4)], kAttnBwdRows);
    }
    default: return 0;
  }
}

// The static table region (kernels.h).  In host code the array's name is only a handle for
// hipGetSymbolAddress; every use of the memory goes through the address that call returns.
static __device__ __align__(256) unsigned char scratch[kStaticTableBytes];

hipError_t static_table_region(void** ptr) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* region_of[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!region_of[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    region_of[dev] = p;
  }
  *ptr = region_of[dev];
  return hipSuccess;
}

hipError_t launch_copies(const CopyBatch& b, int max_workgroups, hipStream_t s) {
  if (b.n <= 0 || b.total_blocks <= 0) return hipSuccess;
  const int wgs = std::min(b.total_blocks, max_workgroups > 0 ? max_workgroups : kDefaultCopyWorkgroups);
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)wgs), dim3(kCopyThreads), 0, s, b);
  return hipGetLastError();
}

hipError_t launch_batch(int cls, int dtype, int head_dim, const DeviceTables& t, const Batch& b,
                        int32_t max_blocks, hipStream_t s) {
  if (b.n <= 0 || max_blocks <= 0) return hipSuccess;
  const dim3 grid((unsigned)max_blocks, (unsigned)b.n), wg(256);
  const bool bf = dtype == TN_BF16;
#define TN_LAUNCH_T(kernel)                                                     \
  do {                                                                          \
    if (bf) hipLaunchKernelGGL(kernel<bf16_t>, grid, wg, 0, s, t, b);           \
    else hipLaunchKernelGGL(kernel<float>, grid, wg, 0, s, t, b);               \
  } while (0)
  switch (cls) {
    case LC_GEMM_F32: TN_LAUNCH_T(gemm_generic_kernel); break;
    case LC_GEMM_BF16_NT: hipLaunchKernelGGL(gemm_bf16_nt_kernel, grid, wg, 0, s, t, b); break;
    case LC_GEMM_BF16_NT256: {
      static const hipError_t attr = hipFuncSetAttribute((const void*)gemm_bf16_nt256_kernel<TN_GEMM_WAVES, 4>,
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, g2_lds_bytes(256));
      if (attr != hipSuccess) return attr;
      hipLaunchKernelGGL((gemm_bf16_nt256_kernel<TN_GEMM_WAVES, 4>), grid, dim3(64 * TN_GEMM_WAVES), g2_lds_bytes(256), s, t, b);
      break;
    }
    case LC_GEMM_BF16_NT256_SMALL: {
      static const hipError_t attr = hipFuncSetAttribute((const void*)gemm_bf16_nt256_kernel<4, 2>,
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, g2_lds_bytes(128));
      if (attr != hipSuccess) return attr;
      hipLaunchKernelGGL((gemm_bf16_nt256_kernel<4, 2>), grid, dim3(256), g2_lds_bytes(128), s, t, b);
      break;
    }
    case LC_RMS_STAT: TN_LAUNCH_T(rms_stat_kernel); break;
    case LC_RMS_APPLY: TN_LAUNCH_T(rms_apply_kernel); break;
    case LC_ROPE: TN_LAUNCH_T(rope_kernel); break;
    case LC_ATTN_COMBINE: TN_LAUNCH_T(attn_combine_kernel); break;
    case LC_SILU_MUL:
      if (bf) hipLaunchKernelGGL((ewise2_kernel<bf16_t, true>), grid, wg, 0, s, t, b);
      else hipLaunchKernelGGL((ewise2_kernel<float, true>), grid, wg, 0, s, t, b);
      break;
    case LC_ADD:
      if (bf) hipLaunchKernelGGL((ewise2_kernel<bf16_t, false>), grid, wg, 0, s, t, b);
      else hipLaunchKernelGGL((ewise2_kernel<float, false>), grid, wg, 0, s, t, b);
      break;
    case LC_TRANSPOSE: TN_LAUNCH_T(transpose_kernel); break;
    case LC_ZERO: TN_LAUNCH_T(zero_kernel); break;
    case LC_SOFTMAX_STAT: TN_LAUNCH_T(softmax_stat_kernel); break;
    case LC_SOFTMAX_APPLY: TN_LAUNCH_T(softmax_apply_kernel); break;
    case LC_SILU_BWD: TN_LAUNCH_T(silu_bwd_kernel); break;
    case LC_RMS_BWD_STAT: TN_LAUNCH_T(rms_bwd_stat_kernel); break;
    case LC_RMS_BWD_APPLY: TN_LAUNCH_T(rms_bwd_apply_kernel); break;
#define TN_LAUNCH_ATTN_BWD(MODE)                                                                                  \
  do {                                                                                                            \
    if (head_dim == 64) {                                                                                         \
      hipLaunchKernelGGL((attn_bwd_bf16_kernel<64, MODE>), grid, dim3(kAttnBwdThreads), attn_bwd_lds(64), s, t, b); \
    } else if (head_dim == 128) {                                                                                 \
      static const hipError_t attr = hipFuncSetAttribute((const void*)attn_bwd_bf16_kernel<128, MODE>,            \
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, attn_bwd_lds(128)); \
      if (attr != hipSuccess) return attr;                                                                        \
      hipLaunchKernelGGL((attn_bwd_bf16_kernel<128, MODE>), grid, dim3(kAttnBwdThreads), attn_bwd_lds(128), s, t, b); \
    } else {                                                                                                      \
      return hipErrorInvalidValue;                                                                                \
    }                                                                                                             \
  } while (0)
    case LC_ATTN_BWD_BF16: TN_LAUNCH_ATTN_BWD(0); break;
    case LC_ATTN_BWD_BF16_DQ: TN_LAUNCH_ATTN_BWD(1); break;
    case LC_ATTN_BWD_BF16_DK: TN_LAUNCH_ATTN_BWD(2); break;
    case LC_ATTN_BWD_BF16_DV: TN_LAUNCH_ATTN_BWD(3); break;
#undef TN_LAUNCH_ATTN_BWD
    case LC_ATTN_BWD:
      if (head_dim == 64) {
        if (bf) hipLaunchKernelGGL((attn_bwd_kernel<bf16_t, 64>), grid, dim3(64), 0, s, t, b);
        else hipLaunchKernelGGL((attn_bwd_kernel<float, 64>), grid, dim3(64), 0, s, t, b);
      } else if (head_dim == 128) {
        if (bf) hipLaunchKernelGGL((attn_bwd_kernel<bf16_t, 128>), grid, dim3(64), 0, s, t, b);
        else hipLaunchKernelGGL((attn_bwd_kernel<float, 128>), grid, dim3(64), 0, s, t, b);
      } else {
        return hipErrorInvalidValue;
      }
      break;
    case LC_ATTN_F32:
      if (head_dim == 64) {
        if (bf) hipLaunchKernelGGL((attn_generic_kernel<bf16_t, 64>), grid, dim3(64), 0, s, t, b);
        else hipLaunchKernelGGL((attn_generic_kernel<float, 64>), grid, dim3(64), 0, s, t, b);
      } else if (head_dim == 128) {
        if (bf) hipLaunchKernelGGL((attn_generic_kernel<bf16_t, 128>), grid, dim3(64), 0, s, t, b);
        else hipLaunchKernelGGL((attn_generic_kernel<float, 128>), grid, dim3(64), 0, s, t, b);
      } else {
        return hipErrorInvalidValue;
      }
      break;
    case LC_ATTN_BF16:
      if (head_dim == 64) {
        hipLaunchKernelGGL(attn_bf16_kernel<64>, grid, wg, 4 * 64 * 64 * 2, s, t, b);
      } else if (head_dim == 128) {
        static const hipError_t attr = hipFuncSetAttribute((const void*)attn_bf16_kernel<128>,
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, 4 * 64 * 128 * 2);
        if (attr != hipSuccess) return attr;
        hipLaunchKernelGGL(attn_bf16_kernel<128>, grid, wg, 4 * 64 * 128 * 2, s, t, b);
      } else {
        return hipErrorInvalidValue;
      }
      break;
    default: return hipErrorInvalidValue;
  }
#undef TN_LAUNCH_T
  return hipGetLastError();
}

}  // namespace tn
