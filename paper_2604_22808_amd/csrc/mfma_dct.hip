// One axis of the separable DCT (paper sections 3.2, 3.7) as a batched small-matrix contraction on the gfx950
// matrix cores:  out[s, k, i] = sum_j M[k][j] * in[s, j, i],  s = slab, j/k = position/frequency along the axis,
// i = everything that is contiguous behind the axis (trailing grid axes times head_dim).
//
// Work decomposition: a wave owns a tile of all n rows x 64 contiguous columns.  Rows arrive as coalesced 128-byte
// segments, are parked row-major in a wave-private LDS buffer 32 rows at a time, and are read back column-wise as
// the B operand of v_mfma_f32_32x32x16_f16 (lane = column, 8 consecutive j per lane); the A operand is the fp16
// transform matrix, staged once per workgroup in LDS.  The next 32 rows are fetched while the current 32 are
// multiplied.  Accumulators are fp32; results go back through the same LDS buffer so that global stores are again
// full 128-byte rows.  The kernel is bandwidth-bound by design: every element is read once and written once.
#include <hip/hip_runtime.h>

#include "ctx.h"

namespace fa {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

#define DCT_WAVES 4
#define DCT_XS_STRIDE 72  // halfs per staged row: 64 columns + 8 pad (144 bytes keeps 16-byte alignment)

__device__ __forceinline__ uint16_t dct_f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// eight bf16 (as four dwords) -> eight fp16 (exact for every bf16 value inside the fp16 range)
__device__ __forceinline__ uint4v bf16x8_to_f16x8(uint4v v) {
  uint4v r;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = __uint_as_float(v[i] << 16);
    const float hi = __uint_as_float(v[i] & 0xffff0000u);
    const _Float16 hl = (_Float16)lo, hh = (_Float16)hi;
    r[i] = (uint32_t)__builtin_bit_cast(uint16_t, hl) | ((uint32_t)__builtin_bit_cast(uint16_t, hh) << 16);
  }
  return r;
}

template <int N>
__global__ void __launch_bounds__(64 * DCT_WAVES) k_dct_pass(DctPassArgs a, int64_t n_tiles, int chunks_per_slab) {
  constexpr int MT = (N + 31) / 32;        // 32-row tiles of output frequencies
  constexpr int RC = (N % 32 == 0) ? 32 : 16;  // rows staged per step
  constexpr int NCH = N / RC;              // staging steps per tile
  constexpr int FS = N + 8;                // row stride of the matrix in LDS (halfs)
  constexpr int LPC = RC / 8;              // 16-byte loads per lane per staging step
  __shared__ __attribute__((aligned(16))) half_t Fs[32 * MT * FS];
  __shared__ __attribute__((aligned(16))) half_t Xs_all[DCT_WAVES][32 * DCT_XS_STRIDE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int nn = lane & 31, g = lane >> 5;
  // transform matrix -> LDS, rows beyond N zero
  for (int e = tid; e < 32 * MT * (N / 8); e += 64 * DCT_WAVES) {
    const int row = e / (N / 8), c8 = e % (N / 8);
    uint4v v = {0u, 0u, 0u, 0u};
    if (row < N) v = *(const uint4v*)(a.M + (size_t)row * N + c8 * 8);
    *(uint4v*)(Fs + row * FS + c8 * 8) = v;
  }
  __syncthreads();

  half_t* Xs = Xs_all[wave];
  const int lrow = lane >> 3, lcol = (lane & 7) * 8;  // this lane's row (within 8) and first column of a row segment

  for (int64_t tile = (int64_t)blockIdx.x * DCT_WAVES + wave; tile < n_tiles; tile += (int64_t)gridDim.x * DCT_WAVES) {
    const int64_t s = tile / chunks_per_slab;
    const int64_t col0 = (tile % chunks_per_slab) * 64;
    const int64_t slice = s / a.outer, o = s % a.outer;

    auto row_ptr_in = [&](int j) -> const uint16_t* {
      if (a.perm_in) {
        const int32_t row = a.perm_in[o * N + j];
        const void* src = a.in;
        if (a.masks) {
          const int band = row < a.band_off1 ? 0 : (row < a.band_off2 ? 1 : 2);
          if (!((a.masks[slice % a.slice_mod] >> band) & 1)) src = a.in_alt;
        }
        return (const uint16_t*)src + ((slice * a.Ntok + row) * a.inner + col0);
      }
      return (const uint16_t*)a.in + ((s * N + j) * a.inner + col0);
    };

    float16v acc[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.f;

    uint4v R[LPC];
#pragma unroll
    for (int it = 0; it < LPC; ++it) R[it] = *(const uint4v*)(row_ptr_in(it * 8 + lrow) + lcol);

#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int it = 0; it < LPC; ++it) {
        uint4v v = R[it];
        if (a.in_bf16) v = bf16x8_to_f16x8(v);
        *(uint4v*)(Xs + (it * 8 + lrow) * DCT_XS_STRIDE + lcol) = v;
      }
      if (ch + 1 < NCH) {
#pragma unroll
        for (int it = 0; it < LPC; ++it) R[it] = *(const uint4v*)(row_ptr_in((ch + 1) * RC + it * 8 + lrow) + lcol);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int ks = 0; ks < RC / 16; ++ks) {
        half8 B[2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int jj = 0; jj < 8; ++jj) B[nt][jj] = Xs[(ks * 16 + g * 8 + jj) * DCT_XS_STRIDE + nt * 32 + nn];
        const int kglob = ch * RC + ks * 16 + g * 8;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
          const half8 A = *(const half8*)(Fs + (mt * 32 + nn) * FS + kglob);
#pragma unroll
          for (int nt = 0; nt < 2; ++nt)
            acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(A, B[nt], acc[mt][nt], 0, 0, 0);
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    }

    // epilogue: 32 output rows at a time through the staging buffer
    uint16_t* Xo = (uint16_t*)Xs;
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = 8 * (r >> 2) + 4 * g + (r & 3);
          const float val = acc[mt][nt][r];
          uint16_t bits;
          if (a.out_bf16) bits = dct_f32_to_bf16(val);
          else { const _Float16 hv = (_Float16)val; bits = __builtin_bit_cast(uint16_t, hv); }
          Xo[row * DCT_XS_STRIDE + nt * 32 + nn] = bits;
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int k = mt * 32 + it * 8 + lrow;
        if (k < N) {
          const uint4v v = *(const uint4v*)(Xo + (it * 8 + lrow) * DCT_XS_STRIDE + lcol);
          uint16_t* dst;
          if (a.perm_out) dst = (uint16_t*)a.out + ((slice * a.Ntok + a.perm_out[o * N + k]) * a.inner + col0);
          else dst = (uint16_t*)a.out + ((s * N + k) * a.inner + col0);
          *(uint4v*)(dst + lcol) = v;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    }
  }
}

template <int N>
static hipError_t launch_n(const DctPassArgs& a, int num_cu, hipStream_t st) {
  const int chunks = (int)(a.inner / 64);
  const int64_t n_tiles = a.nslab * chunks;
  if (n_tiles == 0) return hipSuccess;
  int64_t blocks = (n_tiles + DCT_WAVES - 1) / DCT_WAVES;
  const int64_t cap = (int64_t)num_cu * 2;
  if (blocks > cap) blocks = cap;
  hipLaunchKernelGGL(k_dct_pass<N>, dim3((unsigned)blocks), dim3(64 * DCT_WAVES), 0, st, a, n_tiles, chunks);
  return hipGetLastError();
}

hipError_t launch_mfma_dct_pass(const DctPassArgs& a, int num_cu, hipStream_t st) {
  if (a.inner % 64 != 0 || a.n % 16 != 0 || a.n < 16 || a.n > 128) return hipErrorInvalidValue;
  switch (a.n) {
    case 16: return launch_n<16>(a, num_cu, st);
    case 32: return launch_n<32>(a, num_cu, st);
    case 48: return launch_n<48>(a, num_cu, st);
    case 64: return launch_n<64>(a, num_cu, st);
    case 80: return launch_n<80>(a, num_cu, st);
    case 96: return launch_n<96>(a, num_cu, st);
    case 112: return launch_n<112>(a, num_cu, st);
    case 128: return launch_n<128>(a, num_cu, st);
  }
  return hipErrorInvalidValue;
}

}  // namespace fa
