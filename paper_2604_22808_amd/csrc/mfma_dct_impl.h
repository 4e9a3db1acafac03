#pragma once
// One axis of the separable DCT (paper sections 3.2, 3.7) as a batched small-matrix contraction on the gfx950
// matrix cores:  out[s, k, i] = sum_j M[k][j] * in[s, j, i],  s = slab, j/k = position/frequency along the axis,
// i = everything that is contiguous behind the axis (trailing grid axes times head_dim).
//
// Work decomposition: a wave owns a tile of all n rows x 64 contiguous columns.  Rows arrive as coalesced 128-byte
// segments, are parked row-major in a wave-private LDS buffer 32 rows at a time, and are read back column-wise as
// the B operand of v_mfma_f32_32x32x16_f16 (lane = column, 8 consecutive j per lane: two transposing LDS reads of
// four rows each); the A operand is the fp16 transform matrix, staged once per workgroup in LDS.  The next 32 rows (of this tile or of the wave's next tile)
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
namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));
typedef __fp16 fp16x4 __attribute__((__vector_size__(4 * sizeof(__fp16))));

#define DCT_WAVES 4
#define DCT_XS_STRIDE 96  // halfs per staged input row: 64 columns + 32 pad.  192 bytes = 3/4 of the 256 bytes the LDS banks
                          // span, so the four rows x two 32-byte column groups that half a wave's transposing read touches
                          // fall on all banks once
#define DCT_XO_STRIDE 72  // halfs per staged output row (144 bytes: the two lane halves, four rows apart, hit different banks)

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

// MODE selects what the pass touches besides plain row-major tensors, so that each variant carries only its own
// addressing in registers: 0 plain, 1 plain + sum of squares of the input, 2 scatter into the band-major buffer,
// 3 scatter + router statistics, 4 gather from the band-major buffers.
enum { DCT_PLAIN = 0, DCT_PLAIN_TOT = 1, DCT_SCATTER = 2, DCT_SCATTER_EN = 3, DCT_GATHER = 4 };

// Waves per SIMD the register allocation aims at: three (168 registers) for the variants with at most 64 accumulator
// registers, whose tiles are small enough that a third wave's loads in flight matter more than spare registers.
template <int NI, int MT, int MODE> constexpr int dct_min_waves() {
  int w = MT <= 2 ? 3 : 2;
  if (MODE == 4 && NI > 64 && w > 2) --w;   // the gather pass also holds the looked-up rows of two tiles
  return w;
}

template <int NI, int MT, int MODE>
__global__ void __launch_bounds__(64 * DCT_WAVES) __attribute__((amdgpu_waves_per_eu(dct_min_waves<NI, MT, MODE>())))
k_dct_pass(DctPassArgs a, int64_t n_tiles, int chunks_per_slab) {
  // NI input rows are contracted into up to 32*MT output rows, of which the first a.n_out are stored.
  constexpr int RC = (NI % 32 == 0) ? 32 : 16;  // rows staged per step
  constexpr int NCH = NI / RC;                  // staging steps per tile
  constexpr int FS = NI + 8;                    // row stride of the matrix in LDS (halfs)
  constexpr int LPC = RC / 8;                   // 16-byte loads per lane per staging step
  __shared__ __attribute__((aligned(16))) half_t Fs[32 * MT * FS];
  __shared__ __attribute__((aligned(16))) half_t Xs_all[DCT_WAVES][32 * DCT_XS_STRIDE];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform: tile addressing stays in scalar registers
  const int nn = lane & 31, g = lane >> 5;
  constexpr bool PERM_IN = MODE == DCT_GATHER, PERM_OUT = MODE == DCT_SCATTER || MODE == DCT_SCATTER_EN;
  constexpr bool ENERGY = MODE == DCT_SCATTER_EN, TOT = MODE == DCT_PLAIN_TOT;
  const int NO = a.n_out;
  const int pscale = a.perm_scale > 1 ? a.perm_scale : 1;
  // transform matrix -> LDS, rows beyond n_out zero
  for (int e = tid; e < 32 * MT * (NI / 8); e += 64 * DCT_WAVES) {
    const int row = e / (NI / 8), c8 = e % (NI / 8);
    uint4v v = {0u, 0u, 0u, 0u};
    if (row < NO) v = *(const uint4v*)(a.M + (size_t)row * a.ldm + c8 * 8);
    *(uint4v*)(Fs + row * FS + c8 * 8) = v;
  }
  __syncthreads();

  half_t* Xs = Xs_all[wave];
  const int lrow = lane >> 3, lcol = (lane & 7) * 8;  // this lane's row (within 8) and first column of a row segment
  // Transposing LDS read (ds_read_b64_tr_b16): lane i of a group of 16 receives, for k = 0..3, element i % 4 of the 8-byte
  // piece that lane 4 k + i / 4 of the group names.  With lane j naming row j / 4, columns 4 (j % 4) .. + 3, lane i ends up
  // with column i of four consecutive rows.  The two groups of a wave half take columns 0-15 and 16-31, the upper half
  // of the wave the rows eight further down.
  const int boff = (((lane & 15) >> 2) + 8 * g) * DCT_XS_STRIDE + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
  float en[3][2] = {{0.f, 0.f}, {0.f, 0.f}, {0.f, 0.f}};  // band x column tile, this lane's rows only
  float te[2] = {0.f, 0.f};  // sum of squares of the input: column tile x this lane's rows
  bool out_of_range = false;   // scatter passes: a spectral coefficient that fp16 cannot hold (or a non-finite one)

  // Addressing.  Everything that depends on the tile is wave-uniform and lives in scalar registers; a lane adds one
  // 32-bit offset of its own (its row within a group of 8 and its 16-byte piece of the row segment), fixed for the whole
  // launch.  Rows of a tile are `stride` elements apart from the tile's base, except on the band-major side, where every
  // row is looked up through the permutation.  (The host side checks that the per-lane offsets fit 32 bits.)
  const int64_t in_stride = a.in_swap ? (int64_t)a.sw_total * a.inner : a.inner;
  const int64_t out_stride = a.out_swap ? (int64_t)a.sw_total * a.inner : a.inner;
  const uint32_t lane_in = (uint32_t)(lrow * in_stride + lcol) * 2u;     // bytes
  const uint32_t lane_out = (uint32_t)(lrow * out_stride + lcol) * 2u;   // bytes
  const uint32_t lane_perm = (uint32_t)(lrow * a.perm_k) * 4u;           // bytes into the permutation table
  struct TileAddr {
    const char* in_base;                          // regular / swapped input: first row of the tile, column col0
    int64_t out_off;                              // regular / swapped output (element offset into out / resid)
    int64_t bm_off;                               // band-major side: (slice*Ntok*d + col0 % d) elements, and
    int32_t pidx, mask;                           // o*perm_o + col0/d, band mask of the slice
  };
  auto tile_addr = [&](uint32_t tile) -> TileAddr {
    TileAddr t;
    const uint32_t s = tile / (uint32_t)chunks_per_slab;
    const int32_t col0 = (int32_t)(tile % (uint32_t)chunks_per_slab) * 64;
    const uint32_t sl = s / (uint32_t)a.outer;              // slice within this launch
    const int32_t o = (int32_t)(s % (uint32_t)a.outer);     // slab within the slice
    const int64_t slice = a.slice_list ? a.slice_list[sl] : (int64_t)sl;   // slice of the caller's tensors
    t.pidx = 0; t.bm_off = 0; t.mask = 7; t.in_base = nullptr; t.out_off = 0;
    if (PERM_IN || PERM_OUT) {
      const int32_t ctok = col0 / a.d;
      t.pidx = o * (int32_t)a.perm_o + ctok;
      t.bm_off = slice * a.Ntok * a.d + (col0 - ctok * a.d);
      if (PERM_IN) t.mask = a.masks[slice];
    }
    if (PERM_IN) {
    } else if (a.in_swap) {
      const uint32_t sa = s / (uint32_t)a.sw, sb = s % (uint32_t)a.sw;
      t.in_base = (const char*)((const uint16_t*)a.in + (((int64_t)sa * NI * a.sw_total + sb + a.sw_off) * a.inner + col0));
    } else if (a.list_in) {
      t.in_base = (const char*)((const uint16_t*)a.in + (slice * a.slice_elems + (int64_t)o * NI * a.inner + col0));
    } else {
      t.in_base = (const char*)((const uint16_t*)a.in + ((int64_t)s * NI * a.inner + col0));
    }
    if (PERM_OUT) {
    } else if (a.out_swap) {
      const uint32_t sa = s / (uint32_t)a.sw, sb = s % (uint32_t)a.sw;
      t.out_off = ((int64_t)sa * NO * a.sw_total + sb + a.sw_off) * a.inner + col0;
    } else if (a.list_out) {
      t.out_off = slice * a.slice_elems + (int64_t)o * NO * a.inner + col0;
    } else {
      t.out_off = (int64_t)s * NO * a.inner + col0;
    }
    return t;
  };
  // this lane's 16-byte piece of input row j0 + lrow (j0 a multiple of 8)
  // (gather: `row` is the band-major row of that input row, looked up one tile ahead by perm_rows)
  auto load_piece = [&](const TileAddr& t, int j0, int32_t row) -> uint4v {
    if (PERM_IN) {
      const int band = row < a.band_off1 ? 0 : (row < a.band_off2 ? 1 : (row < a.band_off3 ? 2 : 3));
      const bool active = (t.mask >> band) & 1;
      const uint64_t lane_off = ((uint64_t)(uint32_t)row * (uint32_t)a.d + (uint32_t)lcol) * 2u;   // bytes within the slice
      if (a.delta) {   // change of the active bands against V~ (zero elsewhere)
        uint4v r = {0u, 0u, 0u, 0u};
        if (active) {
          const half8 y = *(const half8*)((const char*)((const uint16_t*)a.in + t.bm_off) + lane_off);
          const half8 v = *(const half8*)((const char*)((const uint16_t*)a.in_alt + t.bm_off) + lane_off);
          r = __builtin_bit_cast(uint4v, y - v);
        }
        return r;
      }
      return *(const uint4v*)((const char*)((const uint16_t*)(active ? a.in : a.in_alt) + t.bm_off) + lane_off);
    }
    return *(const uint4v*)(t.in_base + (int64_t)j0 * in_stride * 2 + lane_in);
  };

  // A wave strides over the tile list by the size of the grid: at any time the resident waves work on one narrow,
  // advancing range of tiles.
  const uint32_t tile_step = gridDim.x * DCT_WAVES;
  uint32_t tile = blockIdx.x * DCT_WAVES + wave;
  const uint32_t n_tiles32 = (uint32_t)n_tiles;
  // staging steps requested ahead of their use (of this tile, then of the next); step c lives in R[c % PD], which
  // carries over to the next tile only when PD divides NCH
  constexpr int PD = (NCH % 2 == 0) ? 2 : 1;
  uint4v R[PD][LPC];
  TileAddr cur, nxt;
  // gather: band-major rows of this lane's NCH*LPC input rows, of the current tile and (requested at the start of the
  // current tile, so that the data loads at its end do not wait for them) of the next one
  constexpr int NPR = PERM_IN ? NCH * LPC : 1;
  int32_t pcur[NPR], pnxt[NPR];
  auto perm_rows = [&](const TileAddr& t, int32_t (&pr)[NPR]) {
    if (PERM_IN) {
#pragma unroll
      for (int i = 0; i < NPR; ++i)
        pr[i] = *(const int32_t*)((const char*)(a.perm_in + ((int64_t)((i / LPC) * RC + (i % LPC) * 8) * a.perm_k + (int64_t)t.pidx * pscale)) + lane_perm);
    }
  };
  if (tile < n_tiles32) {
    cur = tile_addr(tile);
    perm_rows(cur, pcur);
#pragma unroll
    for (int ch = 0; ch < PD; ++ch)
#pragma unroll
      for (int it = 0; it < LPC; ++it) R[ch][it] = load_piece(cur, ch * RC + it * 8, pcur[PERM_IN ? ch * LPC + it : 0]);
  }

  for (; tile < n_tiles32; tile += tile_step) {
    const bool has_next = tile + tile_step < n_tiles32;
    if (has_next) { nxt = tile_addr(tile + tile_step); perm_rows(nxt, pnxt); }

    // band-major rows of this lane's output rows, requested now so that the stores of the epilogue do not wait for them
    // (the row index goes through an empty asm once per tile so that what depends on it - the "row exists" tests of every
    // group of 8 rows - is recomputed where it is used instead of being kept in registers for the whole launch)
    int lrow_t = lrow;
    asm volatile("" : "+v"(lrow_t));
    int32_t prow[MT][4];
    if (PERM_OUT) {
#pragma unroll
      for (int mt = 0; mt < MT; ++mt)
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int k0 = mt * 32 + it * 8;
          prow[mt][it] = k0 + lrow_t < NO
              ? *(const int32_t*)((const char*)(a.perm_out + ((int64_t)k0 * a.perm_k + (int64_t)cur.pidx * pscale)) + lane_perm) : 0;
        }
    }
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
          R[ch % PD][it] = load_piece(cur, (ch + PD) * RC + it * 8, pcur[PERM_IN ? (ch + PD) * LPC + it : 0]);
      } else if (has_next) {
#pragma unroll
        for (int it = 0; it < LPC; ++it)
          R[ch % PD][it] = load_piece(nxt, (ch + PD - NCH) * RC + it * 8, pnxt[PERM_IN ? (ch + PD - NCH) * LPC + it : 0]);
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int ks = 0; ks < RC / 16; ++ks) {
        // B operand (lane = column nn, rows 16 ks + 8 g + 0..7) out of the row-major staging buffer by two transposing
        // reads of four rows each
        half8 B[2];
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          uint4v b4;
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            const half_t* ptr = Xs + boff + (ks * 16 + 4 * h) * DCT_XS_STRIDE + nt * 32;
            const fp16x4 t4 = __builtin_amdgcn_ds_read_tr16_b64_v4f16((fp16x4 __attribute__((address_space(3)))*)ptr);
            const uint2v u2 = __builtin_bit_cast(uint2v, t4);
            b4[2 * h] = u2[0]; b4[2 * h + 1] = u2[1];
          }
          B[nt] = __builtin_bit_cast(half8, b4);
          if (TOT) {   // squares of the input, summed in fp32: this lane's column, its 8 rows of the step
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const half2v h2 = {B[nt][2 * q], B[nt][2 * q + 1]};
              te[nt] = __builtin_amdgcn_fdot2(h2, h2, te[nt], false);
            }
            asm volatile("" : "+v"(te[nt]));   // take the sum here: left to itself the compiler postpones all of a tile's
                                               // sums to its end and keeps every operand alive until then
          }
        }
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

    // Router statistics (ENERGY): en[0] collects the squares of rows below t1, en[1] of rows below t2, en[2] of all rows;
    // the bands are differences of these.  The sums are taken inside the epilogue below, group of 32 rows by group, where
    // each accumulator register is read anyway and dies right after.
    float f1 = 0.f, f2 = 0.f;
    if (ENERGY) {
      // flat index over the two axes the pass does not transform (perm_o == tokens per slab row on this pass)
      const int32_t other = cur.pidx;
      const int u = other / a.en_div, v = other % a.en_div;
      const int t1 = (u < a.low_u && v < a.low_v) ? a.low_a : 0;
      const int t2 = (u < a.mid_u && v < a.mid_v) ? a.mid_a : 0;
      f1 = (float)(t1 - 4 * g); f2 = (float)(t2 - 4 * g);
    }

    // epilogue: 32 output rows at a time through the staging buffer
    uint16_t* Xo = (uint16_t*)Xs;
    const bool stage_bf16 = a.out_bf16 && (PERM_OUT || !a.resid);
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
      if (mt * 32 >= NO) break;
      // the residual rows of this group of 32 are requested before the trip through the staging buffer
      uint4v rsd[4];
      if (!PERM_OUT && a.resid) {
#pragma unroll
        for (int it = 0; it < 4; ++it) {
          const int k0 = mt * 32 + it * 8;
          if (k0 + lrow_t < NO) rsd[it] = *(const uint4v*)((const char*)((const uint16_t*)a.resid + cur.out_off + (int64_t)k0 * out_stride) + lane_out);
        }
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int nt = 0; nt < 2; ++nt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = 8 * (r >> 2) + 4 * g + (r & 3);
          const float val = acc[mt][nt][r];
          if (ENERGY) {
            // row = rc + 4*g; row < t  <=>  clamp(t - row, 0, 1) == 1 for integers (kept in floats: no lane masks to hold);
            // rows >= n_out hold exact zeros
            const float rc = (float)(mt * 32 + 8 * (r >> 2) + (r & 3));
            const float w1 = __builtin_amdgcn_fmed3f(f1 - rc, 0.f, 1.f), w2 = __builtin_amdgcn_fmed3f(f2 - rc, 0.f, 1.f);
            const float v2 = val * val;
            en[0][nt] = fmaf(v2, w1, en[0][nt]);
            en[1][nt] = fmaf(v2, w2, en[1][nt]);
            en[2][nt] += v2;
          }
          if (PERM_OUT) out_of_range = out_of_range || !(__builtin_fabsf(val) <= 65504.f);
          uint16_t bits;
          if (stage_bf16) bits = dct_f32_to_bf16(val);
          else { const _Float16 hv = (_Float16)val; bits = __builtin_bit_cast(uint16_t, hv); }
          Xo[row * DCT_XO_STRIDE + nt * 32 + nn] = bits;
        }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
      __builtin_amdgcn_wave_barrier();
      __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
      for (int it = 0; it < 4; ++it) {
        const int k0 = mt * 32 + it * 8;
        if (k0 + lrow_t < NO) {
          uint4v v = *(const uint4v*)(Xo + (it * 8 + lrow) * DCT_XO_STRIDE + lcol);
          char* dst;   // wave-uniform base plus this lane's 32-bit offset
          if (PERM_OUT) dst = (char*)((uint16_t*)a.out + cur.bm_off) + ((uint64_t)(uint32_t)prow[mt][it] * (uint32_t)a.d + (uint32_t)lcol) * 2u;
          else dst = (char*)((uint16_t*)a.out + cur.out_off + (int64_t)k0 * out_stride) + lane_out;
          if (!PERM_OUT && a.resid) {   // out = resid + result, both bf16 in memory, the sum formed in fp32
            const uint4v rs = rsd[it];
            const half8 h = __builtin_bit_cast(half8, v);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              const float lo = __uint_as_float(rs[i] << 16) + (float)h[2 * i];
              const float hi = __uint_as_float(rs[i] & 0xffff0000u) + (float)h[2 * i + 1];
              v[i] = (uint32_t)dct_f32_to_bf16(lo) | ((uint32_t)dct_f32_to_bf16(hi) << 16);
            }
          }
          *(uint4v*)dst = v;
        }
      }
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    }
    cur = nxt;
#pragma unroll
    for (int i = 0; i < NPR; ++i) pcur[i] = pnxt[i];
  }
  if (PERM_OUT && a.range_flag && out_of_range) *a.range_flag = 1;   // (every writer stores the same value)
  if (ENERGY || TOT) {
    const int gwave = blockIdx.x * DCT_WAVES + wave;
    if (ENERGY) {
#pragma unroll
      for (int b = 0; b < 3; ++b)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
          // band sums from the prefix sums: low = below t1, mid = below t2 minus below t1, high = all minus below t2
          const float mine = b == 0 ? en[0][nt] : b == 1 ? en[1][nt] - en[0][nt] : en[2][nt] - en[1][nt];
          const float tot = mine + __shfl_xor(mine, 32);
          float* slot = a.energy_part + ((size_t)gwave * 3 + b) * 64 + nt * 32 + nn;
          if (g == 0) *slot = tot;   // this wave is the only writer of the slot (waves without a tile store zeros)
        }
    }
    if (TOT) {
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const float tot = te[nt] + __shfl_xor(te[nt], 32);   // the two lane halves hold different rows of the same column
        float* slot = a.tot_part + (size_t)gwave * 64 + nt * 32 + nn;
        if (g == 0) *slot = tot;
      }
    }
  }
}

template <int NI, int MT, int MODE>
static hipError_t launch_n(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out) {
  const int chunks = (int)(a.inner / 64);
  const int64_t n_tiles = a.nslab * chunks;
  if (n_tiles == 0) return hipSuccess;
  if (n_tiles > 0x7fffffff) return hipErrorInvalidValue;
  {
    // the kernel adds per-lane byte offsets as unsigned 32-bit numbers: 8 rows of the larger row stride, 8 rows of the
    // permutation table (band-major rows times the row width are formed in 64 bits)
    const int64_t stride = (a.in_swap || a.out_swap) ? (int64_t)a.sw_total * a.inner : a.inner;
    if (stride * 8 * 2 + 128 > 0xffffffffLL) return hipErrorInvalidValue;
    if ((a.perm_in || a.perm_out) && (a.Ntok > 0x7fffffffLL || a.perm_k * 8 * 4 > 0xffffffffLL)) return hipErrorInvalidValue;
  }
  // workgroups per CU: bounded by the 160 KB of LDS of a gfx950 CU (the runtime's occupancy query assumes 64 KB)
  constexpr int lds_bytes = (32 * MT * (NI + 8) + DCT_WAVES * 32 * DCT_XS_STRIDE) * 2;
  static int occ = 0;
  if (occ == 0) {
    const char* e = getenv("FREQATTN_DCT_OCC");
    occ = (e && atoi(e) > 0) ? atoi(e) : std::min(4, (160 * 1024) / lds_bytes);
  }
  int64_t blocks = (n_tiles + DCT_WAVES - 1) / DCT_WAVES;
  int64_t cap = (int64_t)num_cu * occ;
  if (cap * DCT_WAVES > DCT_MAX_WAVES) cap = DCT_MAX_WAVES / DCT_WAVES;
  // Grid size: not the resident capacity but about two tiles per wave.  A wave still strides over the tile list by the
  // size of the grid, so the waves in flight work on one narrow, advancing range of tiles, and with fresh workgroups
  // arriving all the time the loads of new tiles do not queue behind the stores of finished ones (measured: 7.9 instead of
  // 8.5 ms for the forward transforms of the 1M-token workload; one tile per wave loses the prefetch across tiles,
  // contiguous runs of tiles per workgroup are slower than either).  FREQATTN_DCT_TPW overrides; 0 = resident grid.
  static int tpw_env = -1;
  if (tpw_env < 0) { const char* e = getenv("FREQATTN_DCT_TPW"); tpw_env = e ? atoi(e) : 2; }
  int tpw = tpw_env;
  if (tpw > 0) {
    // statistics modes keep one partial-sum slot per wave: the grid must fit DCT_MAX_WAVES
    if (MODE == DCT_SCATTER || MODE == DCT_GATHER) {
      static int tpw_perm = -1;
      if (tpw_perm < 0) { const char* e = getenv("FREQATTN_DCT_TPW_PERM"); tpw_perm = e ? atoi(e) : tpw; }
      tpw = tpw_perm;
    }
    if (MODE == DCT_SCATTER_EN || MODE == DCT_PLAIN_TOT) {
      static int tpw_stats = -1;
      if (tpw_stats < 0) { const char* e = getenv("FREQATTN_DCT_TPW_STATS"); tpw_stats = e ? atoi(e) : 16; }   // (these passes measured best with longer-lived waves)
      tpw = std::max(tpw, tpw_stats);
      tpw = (int)std::max<int64_t>(tpw, (n_tiles + DCT_MAX_WAVES - 1) / DCT_MAX_WAVES);
    }
    blocks = std::max<int64_t>(1, (n_tiles + (int64_t)tpw * DCT_WAVES - 1) / ((int64_t)tpw * DCT_WAVES));
    if (blocks < cap) blocks = std::min<int64_t>(cap, (n_tiles + DCT_WAVES - 1) / DCT_WAVES);   // small launches: fill the machine first
  } else if (blocks > cap) {
    blocks = cap;
  }
  if (MODE == DCT_SCATTER_EN || MODE == DCT_PLAIN_TOT) {
    // every wave must keep one column chunk for all its tiles: the tile stride has to be a multiple of the chunks
    // per head_dim (columns of a token).  Every wave of the grid stores its partial sums into its own slots; the caller
    // gets the number of waves back and sums exactly those.
    const int cpt = a.d / 64;
    if ((blocks * DCT_WAVES) % cpt != 0 || !waves_out || (a.energy_part && !a.perm_out) || (a.tot_part && a.inner != a.d))
      return hipErrorInvalidValue;
    *waves_out = (int)(blocks * DCT_WAVES);
  }
  // Workgroups per compute unit.  The passes over 64 rows and fewer run best with all the waves their registers allow
  // (three or four per SIMD: a tile is 8 KB, and the loads in flight are what keeps the memory system busy); the passes
  // over 128 rows measured 3 % faster held to two workgroups per unit, which is enforced by asking for LDS the kernel does
  // not use.  FREQATTN_DCT_WGS / FREQATTN_DCT_WGS_128 override (0 = no limit).
  static int dyn_lds = -1;
  if (dyn_lds < 0) {
    const char* e = getenv(NI >= 128 ? "FREQATTN_DCT_WGS_128" : "FREQATTN_DCT_WGS");
    const int wgs = e ? atoi(e) : (NI >= 128 ? 2 : 0);
    dyn_lds = 0;
    if (wgs > 0) {
      const int per = (160 * 1024 / wgs) / 1024 * 1024;
      if (per > lds_bytes) dyn_lds = per - lds_bytes;
      if (dyn_lds > 0) {
        const hipError_t e2 = hipFuncSetAttribute((const void*)k_dct_pass<NI, MT, MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, dyn_lds);
        if (e2 != hipSuccess) { dyn_lds = -1; return e2; }
      }
    }
  }
  hipLaunchKernelGGL((k_dct_pass<NI, MT, MODE>), dim3((unsigned)blocks), dim3(64 * DCT_WAVES), (size_t)dyn_lds, st, a, n_tiles, chunks);
  return hipGetLastError();
}


// Size dispatch of one mode; every translation unit that includes this file instantiates one mode.
template <int MODE>
static hipError_t dispatch_mode(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out) {
  int mt = (a.n_out + 31) / 32;
  if (mt == 3 && (a.n == 16 || a.n == 32 || a.n == 64 || a.n == 128)) mt = 4;
#define FA_DCT_CASE(NI_, MT_) if (a.n == NI_ && mt == MT_) return launch_n<NI_, MT_, MODE>(a, num_cu, st, waves_out);
  FA_DCT_CASE(16, 1) FA_DCT_CASE(16, 2) FA_DCT_CASE(16, 4)
  FA_DCT_CASE(32, 1) FA_DCT_CASE(32, 2) FA_DCT_CASE(32, 4)
  FA_DCT_CASE(64, 1) FA_DCT_CASE(64, 2) FA_DCT_CASE(64, 4)
  FA_DCT_CASE(128, 1) FA_DCT_CASE(128, 2) FA_DCT_CASE(128, 4)
  FA_DCT_CASE(48, 2) FA_DCT_CASE(80, 3) FA_DCT_CASE(96, 3) FA_DCT_CASE(112, 4)
#undef FA_DCT_CASE
  return hipErrorInvalidValue;
}

}  // namespace
}  // namespace fa
