// Generic kernels of libfreqattn: plain fp32 arithmetic for any shape (the fp32 configuration and every shape the
// MFMA kernels do not cover), plus the small helper kernels both paths share (pooling, summaries, band energy).
#include <hip/hip_runtime.h>

#include <algorithm>

#include "ctx.h"

namespace fa {

__device__ __forceinline__ float bf16_to_f32(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float load_as_f32(const void* p, int64_t i, int kind) {
  if (kind == 0) return ((const float*)p)[i];
  if (kind == 1) return bf16_to_f32(((const uint16_t*)p)[i]);
  return (float)((const half_t*)p)[i];
}
__device__ __forceinline__ void store_from_f32(void* p, int64_t i, float v, int kind) {
  if (kind == 0) ((float*)p)[i] = v;
  else if (kind == 1) ((uint16_t*)p)[i] = f32_to_bf16(v);
  else ((half_t*)p)[i] = (half_t)v;
}

// One 1-D transform along one grid axis (section 3.2 / 3.7): out[s, k, i] = sum_j M[k][j] in[s, j, i].
// One thread per output element.  With perm_in / perm_out the rows of the W-axis pass are looked up in the
// band-major order (section 3.3), and with masks set the row's source buffer is chosen per band (section 3.7:
// bands that were not processed contribute V~ unchanged).
__global__ void k_axis_pass(AxisPassArgs a, int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int64_t i = idx % a.inner;
  const int64_t r = idx / a.inner;
  const int k = (int)(r % a.n_out);
  const int64_t s = r / a.n_out;
  const int64_t slice = s / a.outer;
  const int64_t o = s % a.outer;
  const float* Mrow = a.M + (int64_t)k * a.n;
  float acc = 0.f;
  for (int j = 0; j < a.n; ++j) {
    int64_t e;
    const void* src = a.in;
    if (a.perm_in) {
      const int32_t row = a.perm_in[o * a.n + j];
      if (a.masks) {
        const int band = row < a.band_off1 ? 0 : (row < a.band_off2 ? 1 : (row < a.band_off3 ? 2 : 3));
        if (!((a.masks[slice % a.slice_mod] >> band) & 1)) src = a.in_alt;
      }
      e = (slice * a.Ntok + row) * a.inner + i;
    } else {
      e = (s * a.n + j) * a.inner + i;
    }
    acc = fmaf(Mrow[j], load_as_f32(src, e, a.in_kind), acc);
  }
  int64_t eo;
  if (a.perm_out) eo = (slice * a.Ntok + a.perm_out[o * a.n_out + k]) * a.inner + i;
  else eo = (s * a.n_out + k) * a.inner + i;
  store_from_f32(a.out, eo, acc, a.out_kind);
}

hipError_t launch_generic_axis_pass(const AxisPassArgs& a, hipStream_t st) {
  const int64_t total = a.nslab * a.n_out * a.inner;
  if (total == 0) return hipSuccess;
  const int bs = 256;
  const int64_t nb = (total + bs - 1) / bs;
  hipLaunchKernelGGL(k_axis_pass, dim3((unsigned)nb), dim3(bs), 0, st, a, total);
  return hipGetLastError();
}

// Attention of one query row per wave over a list of contiguous key ranges (sections 3.4.1-3.4.3, 3.6).
// Lanes first take one key each (dot product over the channels), the wave does the running softmax, then lanes
// take channels for the weighted sum of values.
#define GATT_MAXC 4  // channels per lane: head_dim <= 256
__global__ void __launch_bounds__(64) k_generic_attn(GenericAttnArgs a) {
  __shared__ float qs[64 * GATT_MAXC];
  const int lane = threadIdx.x;
  const int64_t i = blockIdx.x;  // query row
  const int slice = a.slice_list ? a.slice_list[blockIdx.y] : (int)blockIdx.y;
  const float* Q = a.Q + (int64_t)slice * a.slice_stride;
  const float* K = a.K + (int64_t)slice * a.kv_slice_stride;
  const float* V = a.V + (int64_t)slice * a.kv_slice_stride;
  float* O = a.O + (int64_t)slice * a.slice_stride;
  const int d = a.d;
  for (int c = lane; c < d; c += 64) qs[c] = Q[i * d + c];
  __syncthreads();

  float acc[GATT_MAXC];
#pragma unroll
  for (int u = 0; u < GATT_MAXC; ++u) acc[u] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;

  int n_ranges = 1, e0 = 0;
  if (a.mode == 1) {
    const int I = (int)(i / a.block);
    e0 = a.row_ptr[I];
    n_ranges = a.row_ptr[I + 1] - e0;
  }
  for (int rg = 0; rg < n_ranges; ++rg) {
    int64_t k0, k1;
    if (a.mode == 0) { k0 = 0; k1 = a.nk; }
    else if (a.mode == 1) {
      const int64_t J = a.col_idx[e0 + rg];
      k0 = J * a.block;
      k1 = k0 + a.block < a.nk ? k0 + a.block : a.nk;
    } else {
      k0 = i - a.window > 0 ? i - a.window : 0;
      k1 = (i + a.window + 1 < a.nk) ? i + a.window + 1 : a.nk;
    }
    for (int64_t kb = k0; kb < k1; kb += 64) {
      const int64_t key = kb + lane;
      const bool valid = key < k1;
      float s = -INFINITY;
      if (valid) {
        const float* kr = K + key * d;
        float dot = 0.f;
        for (int c = 0; c < d; ++c) dot = fmaf(qs[c], kr[c], dot);
        s = dot * a.scale;
      }
      float mx = s;
      for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
      const float m_new = fmaxf(m_run, mx);
      const float p = valid ? expf(s - m_new) : 0.f;
      float ps = p;
      for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off);
      const float alpha = (m_run == -INFINITY) ? 0.f : expf(m_run - m_new);
      l_run = l_run * alpha + ps;
      m_run = m_new;
#pragma unroll
      for (int u = 0; u < GATT_MAXC; ++u) acc[u] *= alpha;
      const int cnt = (int)((k1 - kb) < 64 ? (k1 - kb) : 64);
      for (int j = 0; j < cnt; ++j) {
        const float pj = __shfl(p, j);
        const float* vr = V + (kb + j) * d;
#pragma unroll
        for (int u = 0; u < GATT_MAXC; ++u) {
          const int c = lane + 64 * u;
          if (c < d) acc[u] = fmaf(pj, vr[c], acc[u]);
        }
      }
    }
  }
  const float inv = 1.f / l_run;
#pragma unroll
  for (int u = 0; u < GATT_MAXC; ++u) {
    const int c = lane + 64 * u;
    if (c < d) {
      float r = acc[u] * inv;
      if (a.residual) r += qs[c];
      O[i * d + c] = r;
    }
  }
}

hipError_t launch_generic_attn(const GenericAttnArgs& a, hipStream_t st) {
  if (a.nq <= 0 || a.n_slices <= 0 || a.nk <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_generic_attn, dim3((unsigned)a.nq, (unsigned)a.n_slices), dim3(64), 0, st, a);
  return hipGetLastError();
}

// Low-band compression (section 3.3): mean of c consecutive band rows.  T is float or fp16.
template <typename T>
__global__ void k_pool_low(const T* spec, T* low, const int32_t* slice_list, int64_t N, int d, int64_t n_low,
                           int64_t nbar, int c, int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int ch = (int)(idx % d);
  const int64_t j = (idx / d) % nbar;
  const int li = (int)(idx / ((int64_t)d * nbar));
  const int slice = slice_list[li];
  const int64_t r0 = j * c;
  const int64_t r1 = r0 + c < n_low ? r0 + c : n_low;
  float s = 0.f;
  for (int64_t r = r0; r < r1; ++r) s += (float)spec[((int64_t)slice * N + r) * d + ch];
  low[((int64_t)slice * nbar + j) * d + ch] = (T)(s / (float)(r1 - r0));
}

hipError_t launch_pool_low(const void* spec, void* low, const int32_t* slice_list, int n_slices, int64_t N, int d,
                           int64_t n_low, int64_t nbar, int c, int is_half, hipStream_t st) {
  const int64_t total = (int64_t)n_slices * nbar * d;
  if (total == 0) return hipSuccess;
  const unsigned nb = (unsigned)((total + 255) / 256);
  if (is_half)
    hipLaunchKernelGGL(k_pool_low<half_t>, dim3(nb), dim3(256), 0, st, (const half_t*)spec, (half_t*)low, slice_list, N,
                       d, n_low, nbar, c, total);
  else
    hipLaunchKernelGGL(k_pool_low<float>, dim3(nb), dim3(256), 0, st, (const float*)spec, (float*)low, slice_list, N, d,
                       n_low, nbar, c, total);
  return hipGetLastError();
}

// Every low-band position takes the output of its group (section 3.4.1 reading: Y_i = Ybar_{floor(i/c)}).
template <typename T>
__global__ void k_expand_low(const T* lowY, T* Y, const int32_t* slice_list, int64_t N, int d, int64_t n_low,
                             int64_t nbar, int c, int64_t total) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= total) return;
  const int ch = (int)(idx % d);
  const int64_t i = (idx / d) % n_low;
  const int li = (int)(idx / ((int64_t)d * n_low));
  const int slice = slice_list[li];
  Y[((int64_t)slice * N + i) * d + ch] = lowY[((int64_t)slice * nbar + i / c) * d + ch];
}

hipError_t launch_expand_low(const void* lowY, void* Y, const int32_t* slice_list, int n_slices, int64_t N, int d,
                             int64_t n_low, int64_t nbar, int c, int is_half, hipStream_t st) {
  const int64_t total = (int64_t)n_slices * n_low * d;
  if (total == 0) return hipSuccess;
  const unsigned nb = (unsigned)((total + 255) / 256);
  if (is_half)
    hipLaunchKernelGGL(k_expand_low<half_t>, dim3(nb), dim3(256), 0, st, (const half_t*)lowY, (half_t*)Y, slice_list, N,
                       d, n_low, nbar, c, total);
  else
    hipLaunchKernelGGL(k_expand_low<float>, dim3(nb), dim3(256), 0, st, (const float*)lowY, (float*)Y, slice_list, N, d,
                       n_low, nbar, c, total);
  return hipGetLastError();
}

// Summary tokens (section 3.6, U = I): chunk u of band l covers band rows [floor(u n / m), floor((u+1) n / m)).
// One workgroup per (slice, band, chunk); threads split the chunk's rows 256/d ways and the partial sums are added in
// a fixed order, so the result does not depend on scheduling.  The mean is written to the C rows of the other
// bands (band l sees the summaries of the other bands, ascending band index).
struct SkipBits { uint64_t w[NBMAX][4]; };   // per band: slices whose summaries of that band are not pooled here (unused, or summed from the untransformed V)
struct BandGeom { int64_t off[NBMAX], n[NBMAX]; int m[NBMAX]; int nb; };   // first row, rows and summary tokens per band; nb bands

// row of band `band`'s token u among the tokens band b != band looks at
__device__ __forceinline__ int summary_pos(const BandGeom& g, int band, int b, int u) {
  int pos = u;
  for (int o = 0; o < band; ++o)
    if (o != b) pos += g.m[o];
  return pos;
}

template <typename T>
__global__ void __launch_bounds__(256) k_summaries(const T* Y, const T* V, T* C, const int32_t* masks, int64_t N, int d,
                                                   BandGeom g, int m2rows, SkipBits skip) {
  __shared__ float part[256];
  const int slice = blockIdx.z, band = blockIdx.y, u = blockIdx.x;
  if (slice < 256 && ((skip.w[band][slice >> 6] >> (slice & 63)) & 1)) return;
  const int64_t off = g.off[band], n = g.n[band];
  const int me = g.m[band];
  if (u >= me) return;
  const T* src = ((masks[slice] >> band) & 1) ? Y : V;
  const int64_t r0 = ((int64_t)u * n) / me, r1 = ((int64_t)(u + 1) * n) / me;
  const int groups = 256 / d;  // head_dim <= 256
  const int tid = threadIdx.x;
  const int ch = tid % d, grp = tid / d;
  float s = 0.f;
  if (grp < groups)
    for (int64_t r = r0 + grp; r < r1; r += groups) s += (float)src[((int64_t)slice * N + off + r) * d + ch];
  part[tid] = s;
  __syncthreads();
  if (grp == 0) {
    float t = 0.f;
    for (int g2 = 0; g2 < groups; ++g2) t += part[g2 * d + ch];
    const T mean = (T)(t / (float)(r1 - r0));
    for (int b = 0; b < g.nb; ++b) {
      if (b == band) continue;
      C[(((int64_t)slice * g.nb + b) * m2rows + summary_pos(g, band, b, u)) * d + ch] = mean;
    }
  }
}

// fp16 variant with 16-byte loads: a thread owns 8 adjacent channels, 256 / (d/8) row groups per workgroup, sixteen
// rows in flight per thread.  Same chunk rule, same fixed summation order per (row group, then groups ascending).
__global__ void __launch_bounds__(256) k_summaries_h8(const half_t* Y, const half_t* V, half_t* C, const int32_t* masks,
                                                      int64_t N, int d, BandGeom g, int m2rows, SkipBits skip, int nsplit,
                                                      float* split_part) {
  typedef _Float16 h8 __attribute__((ext_vector_type(8)));
  __shared__ float part[256 * 8];
  const int slice = blockIdx.z, band = blockIdx.y, u = blockIdx.x / nsplit, sp = blockIdx.x % nsplit;
  if (slice < 256 && ((skip.w[band][slice >> 6] >> (slice & 63)) & 1)) return;
  const int64_t off = g.off[band], n = g.n[band];
  const int me = g.m[band];
  if (u >= me) return;
  const half_t* src = (((masks[slice] >> band) & 1) ? Y : V) + ((int64_t)slice * N + off) * d;
  const int64_t c0 = ((int64_t)u * n) / me, c1 = ((int64_t)(u + 1) * n) / me;   // the chunk
  // with few chunks (small m) a chunk is cut into nsplit row ranges, one workgroup each; their sums meet in
  // k_summaries_finish in a fixed order
  const int64_t r0 = c0 + ((c1 - c0) * sp) / nsplit, r1 = c0 + ((c1 - c0) * (sp + 1)) / nsplit;
  const int tpr = d / 8;               // threads per row
  const int groups = 256 / tpr;        // rows per workgroup step
  const int tid = threadIdx.x;
  const int c8 = tid % tpr, grp = tid / tpr;
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (grp < groups) {
    int64_t r = r0 + grp;
    constexpr int INF = 16;   // rows in flight per thread: few workgroups may be left with all the work (see skip)
    for (; r + (INF - 1) * (int64_t)groups < r1; r += INF * (int64_t)groups) {
      h8 x[INF];
#pragma unroll
      for (int k = 0; k < INF; ++k) x[k] = *(const h8*)(src + (r + (int64_t)k * groups) * d + c8 * 8);
#pragma unroll
      for (int k = 0; k < INF; ++k)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += (float)x[k][j];
    }
    for (; r < r1; r += groups) {
      const h8 x = *(const h8*)(src + r * d + c8 * 8);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += (float)x[j];
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) part[tid * 8 + j] = acc[j];
  __syncthreads();
  if (grp == 0) {
    const float inv = 1.f / (float)(c1 - c0);
    h8 mean;
    float sum[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float t = 0.f;
      for (int g2 = 0; g2 < groups; ++g2) t += part[(g2 * tpr + c8) * 8 + j];
      sum[j] = t;
      mean[j] = (_Float16)(t * inv);
    }
    if (nsplit > 1) {   // [slice][band][u][split][d]
      float* dst = split_part + ((((int64_t)slice * g.nb + band) * gridDim.x + blockIdx.x) * d) + c8 * 8;
#pragma unroll
      for (int j = 0; j < 8; ++j) dst[j] = sum[j];
      return;
    }
    for (int b = 0; b < g.nb; ++b) {
      if (b == band) continue;
      *(h8*)(C + (((int64_t)slice * g.nb + b) * m2rows + summary_pos(g, band, b, u)) * d + c8 * 8) = mean;
    }
  }
}

// Second stage of the split pooling: adds the nsplit partial sums of a chunk in order and writes the mean rows.
__global__ void __launch_bounds__(256) k_summaries_finish(const float* split_part, half_t* C, int d, BandGeom g, int m2rows,
                                                          SkipBits skip, int nsplit, int mmax) {
  const int slice = blockIdx.z, band = blockIdx.y, u = blockIdx.x, ch = threadIdx.x;
  if (slice < 256 && ((skip.w[band][slice >> 6] >> (slice & 63)) & 1)) return;
  const int64_t n = g.n[band];
  const int me = g.m[band];
  if (u >= me || ch >= d) return;
  const int64_t c0 = ((int64_t)u * n) / me, c1 = ((int64_t)(u + 1) * n) / me;
  const float* src = split_part + ((((int64_t)slice * g.nb + band) * (mmax * nsplit) + (int64_t)u * nsplit) * d) + ch;
  float t = 0.f;
  for (int sp = 0; sp < nsplit; ++sp) t += src[(int64_t)sp * d];
  const half_t mean = (half_t)(t / (float)(c1 - c0));
  for (int b = 0; b < g.nb; ++b) {
    if (b == band) continue;
    C[(((int64_t)slice * g.nb + b) * m2rows + summary_pos(g, band, b, u)) * d + ch] = mean;
  }
}

hipError_t launch_summaries(const void* Y, const void* V, void* C, const int32_t* masks, int slices, int64_t N, int d,
                            int nb, const int64_t band_off[NBMAX], const int64_t band_n[NBMAX], const int m_eff[NBMAX], int m2rows,
                            int is_half, const uint64_t* skip_bits /*[NBMAX][4] or NULL*/, float* split_part, hipStream_t st) {
  SkipBits skip;
  BandGeom g;
  g.nb = nb;
  int mmax = 0;
  for (int l = 0; l < NBMAX; ++l) {
    for (int i = 0; i < 4; ++i) skip.w[l][i] = skip_bits ? skip_bits[l * 4 + i] : 0;
    g.off[l] = band_off[l]; g.n[l] = l < nb ? band_n[l] : 0; g.m[l] = l < nb ? m_eff[l] : 0;
    if (g.m[l] > mmax) mmax = g.m[l];
  }
  if (mmax == 0 || slices == 0) return hipSuccess;
  dim3 grid((unsigned)mmax, (unsigned)nb, (unsigned)slices);
  if (is_half && d % 8 == 0 && 256 % (d / 8) == 0) {
    // at least 64 workgroups per (slice, band): with few chunks each is cut into row ranges (scratch: 128 rows per pair)
    const int nsplit = (split_part && mmax < 64) ? (64 + mmax - 1) / mmax : 1;
    hipLaunchKernelGGL(k_summaries_h8, dim3((unsigned)(mmax * nsplit), (unsigned)nb, (unsigned)slices), dim3(256), 0, st, (const half_t*)Y,
                       (const half_t*)V, (half_t*)C, masks, N, d, g, m2rows, skip, nsplit, split_part);
    if (nsplit > 1)
      hipLaunchKernelGGL(k_summaries_finish, grid, dim3(256), 0, st, split_part, (half_t*)C, d, g, m2rows, skip, nsplit, mmax);
  } else if (is_half)
    hipLaunchKernelGGL(k_summaries<half_t>, grid, dim3(256), 0, st, (const half_t*)Y, (const half_t*)V, (half_t*)C,
                       masks, N, d, g, m2rows, skip);
  else
    hipLaunchKernelGGL(k_summaries<float>, grid, dim3(256), 0, st, (const float*)Y, (const float*)V, (float*)C, masks, N,
                       d, g, m2rows, skip);
  return hipGetLastError();
}

// Summary tokens of the projected forward (sections 3.1 + 3.6): the mean over a chunk of band rows commutes with the
// value projection, so the rows of the transformed model-width input X~ are pooled once per batch entry -
// P[b][band][u][:] = mean of X~ rows of chunk u (the chunk rule of the kernels above) - and every head's summary tokens
// of a band it passes through are P times its W_V.  Workgroup = (chunk, band, batch entry) x a block of 256 columns:
// 32 threads across the columns (8 each), 8 row phases, eight rows in flight per thread; fixed summation order.
__global__ void __launch_bounds__(256) k_pool_wide(const half_t* __restrict__ X, half_t* __restrict__ P, int64_t N, int dm,
                                                   BandGeom g, int mrows) {
  typedef _Float16 h8 __attribute__((ext_vector_type(8)));
  __shared__ float part[8][32][8];
  const int u = blockIdx.x, band = blockIdx.y % g.nb, b = blockIdx.y / g.nb, cb = blockIdx.z;
  const int64_t off = g.off[band];
  const int64_t n = g.n[band];
  const int me = g.m[band];
  const int tid = threadIdx.x, cg = tid & 31, ph = tid >> 5;
  const int col = cb * 256 + cg * 8;
  half_t* dst = P + (((int64_t)b * g.nb + band) * mrows + u) * dm + col;
  const bool live = col < dm;   // (dm is a multiple of 8: a thread's 8 columns are all inside or all outside)
  float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  int64_t c0 = 0, c1 = 0;
  if (u < me && live) {
    c0 = ((int64_t)u * n) / me; c1 = ((int64_t)(u + 1) * n) / me;
    const half_t* src = X + ((int64_t)b * N + off) * dm + col;
    int64_t r = c0 + ph;
    constexpr int INF = 8;
    for (; r + (INF - 1) * 8 < c1; r += INF * 8) {
      h8 x[INF];
#pragma unroll
      for (int k = 0; k < INF; ++k) x[k] = *(const h8*)(src + (r + k * 8) * dm);
#pragma unroll
      for (int k = 0; k < INF; ++k)
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += (float)x[k][j];
    }
    for (; r < c1; r += 8) {
      const h8 x = *(const h8*)(src + r * dm);
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += (float)x[j];
    }
  }
#pragma unroll
  for (int j = 0; j < 8; ++j) part[ph][cg][j] = acc[j];
  __syncthreads();
  if (ph == 0 && live) {
    const float inv = c1 > c0 ? 1.f / (float)(c1 - c0) : 0.f;   // rows beyond the band's chunk count are zero
    h8 mean;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      float t = 0.f;
      for (int q = 0; q < 8; ++q) t += part[q][cg][j];
      mean[j] = (_Float16)(t * inv);
    }
    *(h8*)dst = mean;
  }
}
static BandGeom band_geom(int nb, const int64_t band_off[NBMAX], const int64_t band_n[NBMAX], const int m_eff[NBMAX]) {
  BandGeom g;
  g.nb = nb;
  for (int l = 0; l < NBMAX; ++l) {
    g.off[l] = band_off[l]; g.n[l] = l < nb ? band_n[l] : 0; g.m[l] = l < nb ? m_eff[l] : 0;
  }
  return g;
}
hipError_t launch_pool_wide(const void* X, void* P, int batch, int64_t N, int dm, int nb, const int64_t band_off[NBMAX],
                            const int64_t band_n[NBMAX], const int m_eff[NBMAX], int mrows, hipStream_t st) {
  if (mrows <= 0 || batch <= 0) return hipSuccess;
  if (dm % 8 != 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_pool_wide, dim3((unsigned)mrows, (unsigned)(nb * batch), (unsigned)((dm + 255) / 256)), dim3(256), 0, st,
                     (const half_t*)X, (half_t*)P, N, dm, band_geom(nb, band_off, band_n, m_eff), mrows);
  return hipGetLastError();
}

// T[slice][band][u][:] (the projected pooled rows, mrows per band) -> the slots of C where the other bands of the slice
// look for band `band`'s summary tokens, for every band the slice passes through while it runs another one.
__global__ void __launch_bounds__(256) k_place_summaries(const half_t* __restrict__ T, half_t* __restrict__ C,
                                                         const int32_t* __restrict__ masks, int d, BandGeom g,
                                                         int mrows, int m2rows) {
  const int u = blockIdx.x, band = blockIdx.y, slice = blockIdx.z;
  const int me = g.m[band];
  const int mask = masks[slice] & ((1 << g.nb) - 1);
  if (u >= me || ((mask >> band) & 1) || (mask & ~(1 << band)) == 0) return;
  const half_t* src = T + (((int64_t)slice * g.nb + band) * mrows + u) * d;
  for (int b = 0; b < g.nb; ++b) {
    if (b == band) continue;
    const int pos = summary_pos(g, band, b, u);
    half_t* dst = C + (((int64_t)slice * g.nb + b) * m2rows + pos) * d;
    for (int ch = threadIdx.x; ch < d; ch += 256) dst[ch] = src[ch];
  }
}
hipError_t launch_place_summaries(const void* T, void* C, const int32_t* masks, int slices, int d, int nb, const int m_eff[NBMAX],
                                  int mrows, int m2rows, hipStream_t st) {
  if (mrows <= 0 || slices <= 0) return hipSuccess;
  const int64_t none[NBMAX] = {0, 0, 0, 0};
  hipLaunchKernelGGL(k_place_summaries, dim3((unsigned)mrows, (unsigned)nb, (unsigned)slices), dim3(256), 0, st, (const half_t*)T,
                     (half_t*)C, masks, d, band_geom(nb, none, none, m_eff), mrows, m2rows);
  return hipGetLastError();
}

// Router statistics (section 3.5): per band and channel, the sum of squared coefficients over all slices and the
// three spectral tensors.  Workgroup (chunk, band) adds its rows in a fixed order into part[chunk][band][d]; the
// second kernel adds the chunks in order.  No floating-point atomics, so the result is reproducible.
#define BE_CHUNKS 64
template <typename T>
__global__ void __launch_bounds__(256) k_band_energy(const T* sq, const T* sk, const T* sv, float* part, int slices,
                                                     int64_t N, int d, int64_t off0, int64_t off1, int64_t off2,
                                                     int64_t n0, int64_t n1, int64_t n2) {
  __shared__ float red[256];
  const int chunk = blockIdx.x, band = blockIdx.y;
  const int64_t off = band == 0 ? off0 : band == 1 ? off1 : off2;
  const int64_t n = band == 0 ? n0 : band == 1 ? n1 : n2;
  const int64_t rows = n * slices;  // virtual row index: slice-major
  const int64_t r0 = (chunk * rows) / BE_CHUNKS, r1 = ((chunk + 1) * rows) / BE_CHUNKS;
  const int tid = threadIdx.x;
  const int groups = 256 / d, ch = tid % d, grp = tid / d;
  float s = 0.f;
  if (grp < groups)
    for (int64_t r = r0 + grp; r < r1; r += groups) {
      const int64_t slice = r / n, row = r % n;
      const int64_t e = ((int64_t)slice * N + off + row) * d + ch;
      const float a = (float)sq[e], b = (float)sk[e], c = (float)sv[e];
      s += a * a + b * b + c * c;
    }
  red[tid] = s;
  __syncthreads();
  if (grp == 0) {
    float t = 0.f;
    for (int g2 = 0; g2 < groups; ++g2) t += red[g2 * d + ch];
    part[((int64_t)chunk * 3 + band) * d + ch] = t;
  }
}
__global__ void k_band_energy_final(const float* part, float* stats, int d) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= 3 * d) return;
  float t = 0.f;
  for (int c = 0; c < BE_CHUNKS; ++c) t += part[(int64_t)c * 3 * d + idx];
  stats[idx] = t;
}

hipError_t launch_band_energy(const void* sq, const void* sk, const void* sv, float* stats, int slices, int64_t N, int d,
                              const int64_t band_off[3], const int64_t band_n[3], int is_half, hipStream_t st) {
  // stats holds [3][d] results followed by BE_CHUNKS*3*d partial sums
  float* part = stats + 3 * d;
  dim3 grid(BE_CHUNKS, 3);
  if (is_half)
    hipLaunchKernelGGL(k_band_energy<half_t>, grid, dim3(256), 0, st, (const half_t*)sq, (const half_t*)sk,
                       (const half_t*)sv, part, slices, N, d, band_off[0], band_off[1], band_off[2], band_n[0],
                       band_n[1], band_n[2]);
  else
    hipLaunchKernelGGL(k_band_energy<float>, grid, dim3(256), 0, st, (const float*)sq, (const float*)sk,
                       (const float*)sv, part, slices, N, d, band_off[0], band_off[1], band_off[2], band_n[0], band_n[1],
                       band_n[2]);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(k_band_energy_final, dim3((3 * d + 255) / 256), dim3(256), 0, st, part, stats, d);
  return hipGetLastError();
}

__global__ void k_fill_zero(float* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0.f;
}
hipError_t launch_fill_zero(float* p, int64_t n, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_fill_zero, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n);
  return hipGetLastError();
}

// Plain streaming copy, 16 bytes per thread and step: the machine's achievable HBM read+write rate, measured next
// to the transform passes (which are read-once / write-once kernels of the same kind).
__global__ void __launch_bounds__(256) k_probe_copy(const uint4* __restrict__ in, uint4* __restrict__ out, int64_t n) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) out[i] = in[i];
}
hipError_t launch_probe_copy(const void* in, void* out, int64_t bytes, int num_cu, hipStream_t st) {
  if (bytes < 16) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_probe_copy, dim3((unsigned)(num_cu * 16)), dim3(256), 0, st, (const uint4*)in, (uint4*)out, bytes / 16);
  return hipGetLastError();
}

__global__ void k_copy_slices(const uint4* in, uint4* out, const int32_t* slice_list, int64_t vec_per_slice) {
  const int64_t base = (int64_t)slice_list[blockIdx.y] * vec_per_slice;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < vec_per_slice; i += (int64_t)gridDim.x * blockDim.x)
    out[base + i] = in[base + i];
}
hipError_t launch_copy_slices(const void* in, void* out, const int32_t* slice_list, int n_slices, int64_t slice_bytes,
                              hipStream_t st) {
  if (n_slices <= 0 || slice_bytes <= 0) return hipSuccess;
  if (slice_bytes % 16) return hipErrorInvalidValue;
  const int64_t vec = slice_bytes / 16;
  const unsigned gx = (unsigned)std::min<int64_t>((vec + 255) / 256, 2048);
  hipLaunchKernelGGL(k_copy_slices, dim3(gx, (unsigned)n_slices), dim3(256), 0, st, (const uint4*)in, (uint4*)out,
                     slice_list, vec);
  return hipGetLastError();
}

// Element-wise conversions between the caller's bf16 tensors and fp16 scratch (n a multiple of 8): the dense comparison
// runs the attention kernel's direct-to-LDS path, which needs its operands in fp16 in memory.
__global__ void k_bf16_to_f16(const uint4* in, uint4* out, int64_t nvec) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * blockDim.x) {
    const uint4 v = in[i];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const half_t lo = (half_t)__uint_as_float(w[j] << 16), hi = (half_t)__uint_as_float(w[j] & 0xffff0000u);
      o[j] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
    }
    out[i] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}
__global__ void k_f16_to_bf16(const uint4* in, uint4* out, int64_t nvec) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * blockDim.x) {
    const uint4 v = in[i];
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t o[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint32_t r[2];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const float f = (float)__builtin_bit_cast(half_t, (uint16_t)(h ? (w[j] >> 16) : (w[j] & 0xffffu)));
        uint32_t u = __float_as_uint(f);
        u = (u & 0x7f800000u) == 0x7f800000u ? u : u + 0x7fffu + ((u >> 16) & 1u);   // round to nearest even
        r[h] = u >> 16;
      }
      o[j] = r[0] | (r[1] << 16);
    }
    out[i] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}
hipError_t launch_convert_16(const void* in, void* out, int64_t n, int to_bf16, hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (n % 8) return hipErrorInvalidValue;
  const int64_t nvec = n / 8;
  const unsigned gx = (unsigned)std::min<int64_t>((nvec + 255) / 256, 8192);
  if (to_bf16) hipLaunchKernelGGL(k_f16_to_bf16, dim3(gx), dim3(256), 0, st, (const uint4*)in, (uint4*)out, nvec);
  else hipLaunchKernelGGL(k_bf16_to_f16, dim3(gx), dim3(256), 0, st, (const uint4*)in, (uint4*)out, nvec);
  return hipGetLastError();
}

// Fixed-order sum of the per-wave partial statistics written by the fused forward passes of Q, K and V.
// Wave w of a launch worked on column chunk w % (d/64) only, and left [3 bands][64 columns] floats behind (768 bytes).
// Two stages.  Stage 1: d workgroups of 4 x 192 threads (thread = band, column); workgroup b takes the waves w = b, b + d,
// ... of every slot (d is a multiple of d/64, so all of them belong to chunk b % (d/64)) and reads their 768 bytes
// whole.  Stage 2: one thread per (band, channel) adds the stage-1 sums of its chunk in ascending workgroup order.
// With tot_part set, the tensors in slots 0..2 were only computed on the low+mid box: their high-band energy is the
// energy of the input (Parseval, the transform is orthonormal) minus their low and mid energies.
__global__ void __launch_bounds__(768) k_energy_reduce1(const float* __restrict__ part, const float* __restrict__ tot_part,
                                                        float* __restrict__ part1 /*[d][3][64]*/, int d, EnergyWaves nw) {
  // four groups of 192 threads share a workgroup's waves (group q takes every fourth of them), four loads in flight each
  __shared__ float red[4][192];
  const int b = blockIdx.x, q = threadIdx.x / 192, tid = threadIdx.x % 192, band = tid >> 6, col = tid & 63;
  const bool parseval = tot_part != nullptr && band == 2;
  const int first = b + q * d, step = 4 * d;
  float t[4] = {0.f, 0.f, 0.f, 0.f};
  for (int tensor = 0; tensor < 6; ++tensor) {   // slots: Q, K, V on the box (Parseval for the high band), Q, K, V on the whole grid
    const float* base = part + (size_t)tensor * DCT_MAX_WAVES * 192;
    const int n = nw.en[tensor];
    if (parseval && tensor < 3) {
      for (int w = first; w < n; w += 4 * step)
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (w + u * step < n) t[u] -= base[(size_t)(w + u * step) * 192 + col] + base[(size_t)(w + u * step) * 192 + 64 + col];
    } else {
      for (int w = first; w < n; w += 4 * step)
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (w + u * step < n) t[u] += base[(size_t)(w + u * step) * 192 + tid];
    }
  }
  if (parseval)
    for (int tensor = 0; tensor < 3; ++tensor) {
      const int n = nw.tot[tensor];
      for (int w = first; w < n; w += 4 * step)
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (w + u * step < n) t[u] += tot_part[((size_t)tensor * DCT_MAX_WAVES + w + u * step) * 64 + col];
    }
  red[q][tid] = (t[0] + t[1]) + (t[2] + t[3]);
  __syncthreads();
  if (q == 0) part1[(size_t)b * 192 + tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
}

__global__ void __launch_bounds__(384) k_energy_reduce2(const float* __restrict__ part1, float* __restrict__ stats, int d, int parseval) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= 3 * d) return;
  const int band = idx / d, ch = idx % d;
  const int chunks = d / 64, chunk = ch / 64, col = ch % 64;
  float t = 0.f;
  for (int b = chunk; b < d; b += chunks) t += part1[(size_t)b * 192 + band * 64 + col];
  // The Parseval difference of a band that holds (almost) no energy can come out slightly negative (the low and mid
  // sums carry the rounding of the fp16 transform): an energy is never below zero.
  stats[idx] = (parseval && band == 2 && t < 0.f) ? 0.f : t;   // (a NaN stays a NaN: the host reports it)
}

// stats: [3][d] results followed by at least 3 * d * 64 floats of scratch (the stage-1 sums)
hipError_t launch_energy_reduce(const float* energy_part, const float* tot_part, float* stats, int d, const EnergyWaves& nw,
                                hipStream_t st) {
  if (d % 64 != 0 || d <= 0) return hipErrorInvalidValue;
  float* part1 = stats + 3 * d;
  hipLaunchKernelGGL(k_energy_reduce1, dim3(d), dim3(768), 0, st, energy_part, tot_part, part1, d, nw);
  hipLaunchKernelGGL(k_energy_reduce2, dim3((3 * d + 383) / 384), dim3(384), 0, st, part1, stats, d, tot_part != nullptr ? 1 : 0);
  return hipGetLastError();
}

}  // namespace fa
