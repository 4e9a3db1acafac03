// One axis of the separable DCT (paper sections 3.2, 3.7) as a batched small-matrix contraction on the gfx950
// matrix cores:  out[s, k, i] = sum_j M[k][j] * in[s, j, i],  s = slab, j/k = position/frequency along the axis,
// i = everything that is contiguous behind the axis (trailing grid axes times head_dim).
//
// Work decomposition: a wave owns a tile of all n rows x 64 contiguous columns.  Rows arrive as coalesced 128-byte
// segments, are parked row-major in a wave-private LDS buffer 32 rows at a time, and are read back column-wise as
// the B operand of v_mfma_f32_32x32x16_f16 (lane = column, 8 consecutive j per lane); the A operand is the fp16
// transform matrix, staged once per workgroup in LDS.  The next 32 rows (of this tile or of the wave's next tile)
// are fetched while the current 32 are multiplied.  Accumulators are fp32; results go back through the same LDS
// buffer so that global stores are again full 128-byte rows.  The kernel is bandwidth-bound by design: every element
// is read once and written once per axis.
//
// The pass that touches the band-major spectral buffers (section 3.3) looks rows up through the coefficient ->
// band-row permutation: on output for the forward transform (scatter), on input for the inverse (gather, with the
// source buffer chosen per band, section 3.7).  The same forward pass can add up the router's band statistics
// (section 3.5) from its fp32 results.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>

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

template <int N, bool ENERGY>
__global__ void __launch_bounds__(64 * DCT_WAVES) __attribute__((amdgpu_waves_per_eu(2))) k_dct_pass(DctPassArgs a, int64_t n_tiles, int chunks_per_slab) {
  constexpr int MT = (N + 31) / 32;            // 32-row tiles of output frequencies
  constexpr int RC = (N % 32 == 0) ? 32 : 16;  // rows staged per step
  constexpr int NCH = N / RC;                  // staging steps per tile
  constexpr int FS = N + 8;                    // row stride of the matrix in LDS (halfs)
  constexpr int LPC = RC / 8;                  // 16-byte loads per lane per staging step
  __shared__ __attribute__((aligned(16))) half_t Fs[32 * MT * FS];
  __shared__ __attribute__((aligned(16))) half_t Xs_all[DCT_WAVES][32 * DCT_XS_STRIDE];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: tile addressing stays in scalar registers
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
  float en[3][2] = {{0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}};  // band x column tile, this lane's rows only

  // Per-tile addressing, computed once per tile: rows of a tile are `stride` elements apart from `base`, except on the
  // band-major side where every row is looked up through the permutation.
  struct TileAddr {
    const uint16_t* in_base; int64_t in_stride;   // regular / swapped input
    uint16_t* out_base; int64_t out_stride;       // regular / swapped output
    int64_t bm_off;                               // band-major side: slice*Ntok (rows), and
    int32_t pidx, dcol, o, mask;                  // o*perm_o + col0/d, col0 % d, slab within slice, band mask of slice
  };
  auto tile_addr = [&](uint32_t tile) -> TileAddr {
    TileAddr t;
    const uint32_t s = tile / (uint32_t)chunks_per_slab;
    const int32_t col0 = (int32_t)(tile % (uint32_t)chunks_per_slab) * 64;
    const uint32_t slice = s / (uint32_t)a.outer;
    t.o = (int32_t)(s % (uint32_t)a.outer);
    const int32_t ctok = col0 / a.d;
    t.dcol = col0 - ctok * a.d;
    t.pidx = t.o * (int32_t)a.perm_o + ctok;
    t.bm_off = (int64_t)slice * a.Ntok;
    t.mask = a.masks ? a.masks[slice] : 7;
    if (a.in_swap) {
      const uint32_t sa = s / (uint32_t)a.sw, sb = s % (uint32_t)a.sw;
      t.in_base = (const uint16_t*)a.in + (((int64_t)sa * N * a.sw_total + sb + a.sw_off) * a.inner + col0);
      t.in_stride = (int64_t)a.sw_total * a.inner;
    } else {
      t.in_base = (const uint16_t*)a.in + ((int64_t)s * N * a.inner + col0);
      t.in_stride = a.inner;
    }
    if (a.out_swap) {
      const uint32_t sa = s / (uint32_t)a.sw, sb = s % (uint32_t)a.sw;
      t.out_base = (uint16_t*)a.out + (((int64_t)sa * N * a.sw_total + sb + a.sw_off) * a.inner + col0);
      t.out_stride = (int64_t)a.sw_total * a.inner;
    } else {
      t.out_base = (uint16_t*)a.out + ((int64_t)s * N * a.inner + col0);
      t.out_stride = a.inner;
    }
    return t;
  };
  // this lane's 16-byte piece of input row j
  auto src_ptr = [&](const TileAddr& t, int j) -> const uint16_t* {
    if (a.perm_in) {
      const int32_t row = a.perm_in[(int64_t)j * a.perm_k + t.pidx];
      const int band = row < a.band_off1 ? 0 : (row < a.band_off2 ? 1 : 2);
      const void* src = ((t.mask >> band) & 1) ? a.in : a.in_alt;
      return (const uint16_t*)src + ((t.bm_off + row) * a.d + t.dcol) + lcol;
    }
    return t.in_base + (int64_t)j * t.in_stride + lcol;
  };

  const uint32_t tile_step = gridDim.x * DCT_WAVES;
  uint32_t tile = blockIdx.x * DCT_WAVES + wave;
  const uint32_t n_tiles32 = (uint32_t)n_tiles;
  // staging steps requested ahead of their use (of this tile, then of the next); step c lives in R[c % PD], which
  // carries over to the next tile only when PD divides NCH
  constexpr int PD = (NCH % 2 == 0) ? 2 : 1;
  uint4v R[PD][LPC];
  TileAddr cur, nxt;
  if (tile < n_tiles32) {
    cur = tile_addr(tile);
#pragma unroll
    for (int ch = 0; ch < PD; ++ch)
#pragma unroll
      for (int it = 0; it < LPC; ++it) R[ch][it] = *(const uint4v*)src_ptr(cur, ch * RC + it * 8 + lrow);
  }

  for (; tile < n_tiles32; tile += tile_step) {
    const bool has_next = tile + tile_step < n_tiles32;
    if (has_next) nxt = tile_addr(tile + tile_step);

    float16v acc[MT][2];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.f;

#pragma unroll
    for (int ch = 0; ch < NCH; ++ch) {
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int it = 0; it < LPC; ++it) {
        uint4v v = R[ch % PD][it];
        if (a.in_bf16) v = bf16x8_to_f16x8(v);
        *(uint4v*)(Xs + (it * 8 + lrow) * DCT_XS_STRIDE + lcol) = v;
      }
      if (ch + PD < NCH) {
#pragma unroll
        for (int it = 0; it < LPC; ++it)
          R[ch % PD][it] = *(const uint4v*)src_ptr(cur, (ch + PD) * RC + it * 8 + lrow);
      } else if (has_next) {
#pragma unroll
        for (int it = 0; it < LPC; ++it)
          R[ch % PD][it] = *(const uint4v*)src_ptr(nxt, (ch + PD - NCH) * RC + it * 8 + lrow);
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

    if (ENERGY) {
      // flat index over the two axes the pass does not transform (perm_o == en_omul on this pass)
      const int32_t other = cur.pidx;
      const int u = other / a.en_div, v = other % a.en_div;
      const int t1 = (u < a.low_u && v < a.low_v) ? a.low_a : 0;
      const int t2 = (u < a.mid_u && v < a.mid_v) ? a.mid_a : 0;
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int row = mt * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
            const float v2 = acc[mt][nt][r] * acc[mt][nt][r];   // rows >= N hold exact zeros
            en[0][nt] += row < t1 ? v2 : 0.f;
            en[1][nt] += (row >= t1 && row < t2) ? v2 : 0.f;
            en[2][nt] += row >= t2 ? v2 : 0.f;
          }
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
          if (a.perm_out)
            dst = (uint16_t*)a.out + ((cur.bm_off + a.perm_out[(int64_t)k * a.perm_k + cur.pidx]) * a.d + cur.dcol);
          else
            dst = cur.out_base + (int64_t)k * cur.out_stride;
          *(uint4v*)(dst + lcol) = v;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    }
    cur = nxt;
  }
  if (ENERGY) {
    const int gwave = blockIdx.x * DCT_WAVES + wave;
#pragma unroll
    for (int b = 0; b < 3; ++b)
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const float tot = en[b][nt] + __shfl_xor(en[b][nt], 32);
        float* slot = a.energy_part + ((size_t)gwave * 3 + b) * 64 + nt * 32 + nn;
        if (g == 0) *slot = *slot + tot;   // launches on one stream are ordered: no other writer of this slot
      }
  }
}

template <int N>
static hipError_t launch_n(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out) {
  const int chunks = (int)(a.inner / 64);
  const int64_t n_tiles = a.nslab * chunks;
  if (n_tiles == 0) return hipSuccess;
  // workgroups per CU: bounded by the 160 KB of LDS of a gfx950 CU (the runtime's occupancy query assumes 64 KB)
  constexpr int lds_bytes = (32 * ((N + 31) / 32) * (N + 8) + DCT_WAVES * 32 * DCT_XS_STRIDE) * 2;
  static int occ = 0;
  if (occ == 0) {
    const char* e = getenv("FREQATTN_DCT_OCC");
    occ = (e && atoi(e) > 0) ? atoi(e) : std::min(4, (160 * 1024) / lds_bytes);
  }
  int64_t blocks = (n_tiles + DCT_WAVES - 1) / DCT_WAVES;
  int64_t cap = (int64_t)num_cu * occ;
  if (cap * DCT_WAVES > DCT_MAX_WAVES) cap = DCT_MAX_WAVES / DCT_WAVES;
  if (blocks > cap) blocks = cap;
  if (a.energy_part) {
    // every wave must keep one column chunk for all its tiles: the tile stride has to be a multiple of the chunks
    // per head_dim (columns of a token).  Slots of energy_part are accumulated into; the caller zeroes them first.
    const int cpt = a.d / 64;
    if ((blocks * DCT_WAVES) % cpt != 0 || !a.perm_out || !waves_out) return hipErrorInvalidValue;
    if ((int)(blocks * DCT_WAVES) > *waves_out) *waves_out = (int)(blocks * DCT_WAVES);
    hipLaunchKernelGGL((k_dct_pass<N, true>), dim3((unsigned)blocks), dim3(64 * DCT_WAVES), 0, st, a, n_tiles, chunks);
  } else {
    hipLaunchKernelGGL((k_dct_pass<N, false>), dim3((unsigned)blocks), dim3(64 * DCT_WAVES), 0, st, a, n_tiles, chunks);
  }
  return hipGetLastError();
}

hipError_t launch_mfma_dct_pass(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out) {
  if (a.inner % 64 != 0 || a.n % 16 != 0 || a.n < 16 || a.n > 128 || a.inner % a.d != 0) return hipErrorInvalidValue;
  switch (a.n) {
    case 16: return launch_n<16>(a, num_cu, st, waves_out);
    case 32: return launch_n<32>(a, num_cu, st, waves_out);
    case 48: return launch_n<48>(a, num_cu, st, waves_out);
    case 64: return launch_n<64>(a, num_cu, st, waves_out);
    case 80: return launch_n<80>(a, num_cu, st, waves_out);
    case 96: return launch_n<96>(a, num_cu, st, waves_out);
    case 112: return launch_n<112>(a, num_cu, st, waves_out);
    case 128: return launch_n<128>(a, num_cu, st, waves_out);
  }
  return hipErrorInvalidValue;
}

}  // namespace fa
