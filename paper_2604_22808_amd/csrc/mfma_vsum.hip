// Summary tokens of the high band straight from the untransformed V (gfx950).
//
// Section 3.6 (U = I) takes, per band, the mean of the band's spectral rows over m contiguous chunks.  For a band that
// a slice does not run, those rows are rows of V~ = B V (B the orthonormal 3-D transform matrix), so the mean over
// chunk u is a linear functional of the input:
//     mean_u = (1 / |chunk u|) * sum_n Wsum[u][n] V[n],      Wsum[u][n] = sum_{k in chunk u} B[k][n].
// Wsum depends on the band layout only and is built once per context (host, from the same rounded axis matrices the
// transform kernels use).  With it, a slice that does not run the high band needs V~ on the low+mid box only - an
// eighth of the grid for the usual thresholds - instead of on the whole grid, and the only other consumer of its
// high-band rows, the summary pooling, is served by this kernel: one pass over V (bf16, as the caller gave it).
//
// k_vsum: C^T[ch][u] += V^T[ch][n] Wsum^T[n][u] on the matrix cores (v_mfma_f32_32x32x16_bf16).  A workgroup owns one
// slice and a contiguous range of tokens; tiles of 64 tokens go straight into LDS (global_load_lds_dwordx4, row-major,
// 16-byte chunks permuted through the source address so that the transposing LDS reads that form the V^T operand are
// conflict-free), three tiles deep (two in flight while one is used).  Wave w owns 32 channels and all 64 chunk
// columns.  The weights are stored tile by tile ([N/64][64 chunks][64 tokens], 8 KB contiguous per tile) and take the
// same road into LDS; the workgroups of all slices that share a token range run side by side, so they hit in L2.
// Partial sums over the token ranges go to a scratch buffer and are added in a fixed order by k_vsum_reduce, which
// also scales by 1 / |chunk| and writes the fp16 summary rows where the exchange looks for them.
#include "ctx.h"

namespace fa {

typedef float float16v __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __fp16 fp16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

// lane l's 16 bytes land at dst + 16 l (dst wave-uniform); issued as assembly so that the compiler does not order the
// LDS reads of the tile in use behind it.  The kernel waits for these copies itself, with vmcnt(0) before the barrier.
__device__ __forceinline__ void vs_lds_dma16(const void* src, const uint16_t* dst) {
  const unsigned base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(const __attribute__((address_space(3))) uint16_t*)dst);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(base) : "memory", "m0");
}

// index of the j-th set bit of the 256-bit set (j < popcount)
__device__ __forceinline__ int nth_set_bit(const uint64_t bits[4], int j) {
  for (int w = 0; w < 4; ++w) {
    const int c = __popcll(bits[w]);
    if (j < c) {
      uint64_t b = bits[w];
      for (int i = 0; i < j; ++i) b &= b - 1;
      return w * 64 + __ffsll((unsigned long long)b) - 1;
    }
    j -= c;
  }
  return 0;
}

struct VsumBits { uint64_t w[4]; };

template <int D>
__global__ void __launch_bounds__(256, 2) k_vsum(const uint16_t* __restrict__ V, const uint16_t* __restrict__ Wsum,
                                                 float* __restrict__ part, VsumBits sel, int nsel, int64_t N,
                                                 int tiles_per_split, int nsplit) {
  constexpr int KT = 64;            // tokens per tile
  constexpr int DT = D / 32;        // 32-channel tiles
  constexpr int SUBS = 4 / DT;      // waves per channel tile: they split the tile's four 16-token steps
  constexpr int KSPW = 4 / SUBS;    // 16-token steps per wave and tile
  constexpr int CPR = D / 8;        // 16-byte chunks per V row
  constexpr int RPI = 64 / CPR;     // V rows per copy instruction
  constexpr int NIW = KT / (RPI * 4);   // V copy instructions per wave and tile
  constexpr int PW = NIW + 2;       // copy instructions per wave and tile: V rows, then two of the weight tile's eight
  constexpr int NB = 3;             // tiles in LDS: one in use, two on their way
  __shared__ __attribute__((aligned(16))) uint16_t Vt3[NB][KT * D];
  __shared__ __attribute__((aligned(16))) uint16_t Wt3[NB][64 * KT];   // [chunk u][64 tokens], 16-byte pieces at c ^ (u & 7)
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nn = lane & 31, g = lane >> 5;
  const int jsel = blockIdx.x % nsel, split = blockIdx.x / nsel;
  const int slice = nth_set_bit(sel.w, jsel);
  const int dt = wave % DT, sub = wave / DT;
  auto fV = [](int r) -> int { return D == 128 ? ((r & 3) << 2) : (((r >> 1) & 1) << 2); };
  // V^T operand (channels 32 dt + nn, 8 tokens): two transposing reads of 4 consecutive tokens each,
  // tokens 16 ks + 8 h + 4 g + 0..3 for read h (the weight rows are stored in that order)
  const int sl = lane & 15, g1 = (lane >> 4) & 1;
  const int voff = (4 * g + (sl >> 2)) * D + (sl & 1) * 4 + (((4 * dt + 2 * g1 + ((sl & 3) >> 1)) ^ fV(sl >> 2)) << 3);
  const int64_t ntiles = N / KT;
  const int64_t t_lo = (int64_t)split * tiles_per_split;
  int64_t t_hi = t_lo + tiles_per_split;
  if (t_hi > ntiles) t_hi = ntiles;
  const uint16_t* Vs = V + (int64_t)slice * N * D;
  auto dma_tile = [&](int64_t tile, int buf) {
    const int lr = lane / CPR, c = lane % CPR;
#pragma unroll
    for (int j = 0; j < NIW; ++j) {
      const int rowbase = (wave * NIW + j) * RPI;
      const int r = rowbase + lr;
      vs_lds_dma16(Vs + (tile * KT + r) * D + ((c ^ fV(r)) << 3), Vt3[buf] + rowbase * D);
    }
#pragma unroll
    for (int j = 0; j < 2; ++j) {   // weight tile: 8 rows of 128 bytes per instruction
      const int rowbase = (wave * 2 + j) * 8;
      const int u = rowbase + (lane >> 3), c = lane & 7;
      vs_lds_dma16(Wsum + tile * (64 * KT) + u * KT + ((c ^ (u & 7)) << 3), Wt3[buf] + rowbase * KT);
    }
  };
  float16v acc[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  // the copies of a wave complete in the order they were issued: waiting until at most PW are outstanding leaves only
  // the youngest tile's in flight
  if (t_lo < t_hi) dma_tile(t_lo, 0);
  if (t_lo + 1 < t_hi) {
    dma_tile(t_lo + 1, 1);
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PW) : "memory");
  } else {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  }
  __syncthreads();
  for (int64_t tile = t_lo; tile < t_hi; ++tile) {
    const int i = (int)(tile - t_lo);
    const int buf = i % NB;
    const bool more = tile + 2 < t_hi;
    if (more) dma_tile(tile + 2, (i + 2) % NB);   // that copy was last read before the barrier that ended the previous iteration
    const uint16_t* Vt = Vt3[buf];
    const uint16_t* Wt = Wt3[buf];
#pragma unroll
    for (int k = 0; k < KSPW; ++k) {
      const int ks = sub * KSPW + k;
      uint4v a4;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const uint16_t* ptr = Vt + (ks * 16 + 8 * h) * D + voff;
        const fp16x4 t4 = __builtin_amdgcn_ds_read_tr16_b64_v4f16((fp16x4 __attribute__((address_space(3)))*)ptr);
        const uint2v u2 = __builtin_bit_cast(uint2v, t4);
        a4[2 * h] = u2[0]; a4[2 * h + 1] = u2[1];
      }
      const bf16x8 A = __builtin_bit_cast(bf16x8, a4);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int u = 32 * j + nn;
        const uint4v b4 = *(const uint4v*)(Wt + u * KT + (((2 * ks + g) ^ (u & 7)) << 3));
        acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A, __builtin_bit_cast(bf16x8, b4), acc[j], 0, 0, 0);
      }
    }
    if (more) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(PW) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }
  // partial sums: part[jsel][split * SUBS + sub][ch][u]
  float* dst = part + ((int64_t)(jsel * nsplit * SUBS + split * SUBS + sub) * D) * 64;
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int ch = 32 * dt + 8 * (r >> 2) + 4 * g + (r & 3);
      dst[ch * 64 + 32 * j + nn] = acc[j][r];
    }
}

// C rows of the high band's summaries for the selected slices: fixed-order sum of the partial sums, times 1 / |chunk|.
// The high band's summaries sit behind the other band's in the C block of band b (b = 0: after mid's, b = 1: after low's).
__global__ void __launch_bounds__(256) k_vsum_reduce(const float* __restrict__ part, half_t* __restrict__ C, VsumBits sel,
                                                     int nparts, int d, int64_t n_high, int m_high, int m0, int m1,
                                                     int m2rows) {
  const int jsel = blockIdx.y;
  const int slice = nth_set_bit(sel.w, jsel);
  const int idx = blockIdx.x * 256 + threadIdx.x;   // (channel, chunk) pair, d * 64 of them
  const int ch = idx >> 6, u = idx & 63;
  if (ch >= d || u >= m_high) return;
  const float* src = part + ((int64_t)jsel * nparts * d) * 64 + idx;
  const int64_t stride = (int64_t)d * 64;
  float t4[4] = {0.f, 0.f, 0.f, 0.f};   // four interleaved running sums: loads of independent terms overlap, order fixed
  int p = 0;
  for (; p + 3 < nparts; p += 4) {
#pragma unroll
    for (int k = 0; k < 4; ++k) t4[k] += src[(p + k) * stride];
  }
  for (; p < nparts; ++p) t4[0] += src[p * stride];
  const float t = (t4[0] + t4[1]) + (t4[2] + t4[3]);
  const int64_t r0 = ((int64_t)u * n_high) / m_high, r1 = ((int64_t)(u + 1) * n_high) / m_high;
  const half_t mean = (half_t)(t / (float)(r1 - r0));
  C[(((int64_t)slice * 3 + 0) * m2rows + m1 + u) * d + ch] = mean;
  C[(((int64_t)slice * 3 + 1) * m2rows + m0 + u) * d + ch] = mean;
}

hipError_t launch_vsum(const void* V, const void* Wsum, float* part, void* C, const uint64_t sel[4], int nsel, int64_t N,
                       int d, int nsplit, int64_t n_high, const int m_eff[3], int m2rows, hipStream_t st) {
  if (nsel <= 0) return hipSuccess;
  if ((d != 64 && d != 128) || N % 64 != 0 || m_eff[2] > 64 || m_eff[2] < 1) return hipErrorInvalidValue;
  VsumBits b;
  for (int i = 0; i < 4; ++i) b.w[i] = sel[i];
  const int64_t ntiles = N / 64;
  const int tps = (int)((ntiles + nsplit - 1) / nsplit);   // (the caller sized `part` for nsel * nsplit token ranges)
  const dim3 grid((unsigned)(nsel * nsplit));
  if (d == 128)
    hipLaunchKernelGGL(k_vsum<128>, grid, dim3(256), 0, st, (const uint16_t*)V, (const uint16_t*)Wsum, part, b, nsel, N, tps, nsplit);
  else
    hipLaunchKernelGGL(k_vsum<64>, grid, dim3(256), 0, st, (const uint16_t*)V, (const uint16_t*)Wsum, part, b, nsel, N, tps, nsplit);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int nparts = nsplit * (d == 128 ? 1 : 2);
  hipLaunchKernelGGL(k_vsum_reduce, dim3((unsigned)(d * 64 / 256), (unsigned)nsel), dim3(256), 0, st, part, (half_t*)C, b, nparts, d, n_high, m_eff[2],
                     m_eff[0], m_eff[1], m2rows);
  return hipGetLastError();
}

}  // namespace fa
