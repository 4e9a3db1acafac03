// Channel-mixing products around the spectral transform (paper sections 3.1 and 3.7: Q = X W_Q, K = X W_K, V = X W_V,
// concatenated heads times W_O).  The transform acts on the token axes and the projections on the channel axis, so
// they commute: F(X W) = F(X) W.  This file holds the matrix-core kernel those products run on once X itself has been
// transformed:
//
//   C[i][j] = sum over segments s, sum over k < K_s:  A_s[i][k] * B_s[j][k]
//
// with every operand K-contiguous (A_s [m][K_s], row stride lda; B_s [n][K_s], row stride ldb), fp16 in, fp32
// accumulation, fp16 out.  Segments let one product take its K range from several tensors (the output projection sums
// over heads whose rows live in per-head buffers, and picks per head the band output or the passed-through V~).
//
// Tile: 128 rows of C x 128 columns per workgroup of four waves, K in steps of 64.  Both operand tiles are copied from
// global memory straight into LDS (16 bytes per lane, rows of 128 bytes, the 16-byte chunks of a row permuted through
// the source address so that the 16-byte operand reads of 16 consecutive rows hit 16 different bank groups), double
// buffered, one barrier per step.  A wave owns 32 rows and all 128 columns: C^T = B A^T, so that a lane owns one row
// of C and its accumulator registers run over columns - the same register layout as the attention kernel's output.
#include <hip/hip_runtime.h>

#include <cstdlib>

#include "ctx.h"

namespace fa {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));

namespace {

__device__ __forceinline__ void gemm_dma16(const void* src, const half_t* dst) {
  // one wave-wide copy of 16 bytes per lane into LDS at dst + 16 * lane (dst wave-uniform); issued as assembly so that the
  // compiler does not order every later LDS read behind it - the kernel waits for its copies itself
  const unsigned base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(const __attribute__((address_space(3))) half_t*)dst);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(base) : "memory", "m0");
}
__device__ __forceinline__ uint32_t gemm_pack_h2(float a, float b) {
  const _Float16 ha = (_Float16)a, hb = (_Float16)b;
  return (uint32_t)__builtin_bit_cast(uint16_t, ha) | ((uint32_t)__builtin_bit_cast(uint16_t, hb) << 16);
}

constexpr int GM = 128, GN = 128, GK = 64;   // tile of C and K step

// A launch runs `per` problems that share m, n and - in the callers here - their A rows (the same spectral rows
// projected with different heads' weights).  Workgroups are dealt to the 8 XCDs round-robin by blockIdx and each XCD has
// its own L2: XCD x takes the row tiles x, x + 8, ... and walks, for each of them, all column tiles of all problems
// back to back, so that a row tile of A is fetched into one L2 once and reused tiles_n * per times.
__global__ void __launch_bounds__(256, 2) k_gemm_nt(const GemmProblem* __restrict__ probs, const GemmSeg* __restrict__ segs,
                                                    int per, int tiles_m, int tiles_n) {
  __shared__ __attribute__((aligned(16))) half_t As[2][GM * GK];
  __shared__ __attribute__((aligned(16))) half_t Bs[2][GN * GK];
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int inner_n = tiles_n * per;
  const int mt = (seq / inner_n) * 8 + xcd, inner = seq % inner_n;
  if (mt >= tiles_m) return;   // (uniform over the workgroup: the grid is padded to whole rounds of 8 row tiles)
  const GemmProblem pr = probs[inner / tiles_n];
  const int m0 = mt * GM, n0 = (inner % tiles_n) * GN;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nn = lane & 31, g = lane >> 5;
  auto fK = [](int r) -> int { return (r >> 1) & 7; };

  // this lane's rows of the copies: instruction i of this wave moves rows (wave*4 + i)*8 + lane/8, chunk lane%8
  const int lr = lane >> 3, lc = lane & 7;
  int a_row[4], b_row[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = (wave * 4 + i) * 8 + lr;
    a_row[i] = m0 + r < pr.m ? m0 + r : pr.m - 1;   // rows past the end repeat the last row; their results are not stored
    b_row[i] = n0 + r < pr.n ? n0 + r : pr.n - 1;
  }
  auto stage = [&](const GemmSeg& sg, int k0, int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = (wave * 4 + i) * 8 + lr;
      const int chunk = (lc ^ fK(r)) << 3;
      gemm_dma16(sg.A + (int64_t)a_row[i] * sg.lda + k0 + chunk, As[buf] + (wave * 4 + i) * 8 * GK);
      gemm_dma16(sg.B + (int64_t)b_row[i] * sg.ldb + k0 + chunk, Bs[buf] + (wave * 4 + i) * 8 * GK);
    }
  };

  float16v acc[4];
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[nt][r] = 0.f;

  // flattened (segment, k) iteration; the copy of step i+1 is in flight while step i is multiplied
  int seg_i = 0, k_i = 0;               // position of the step being staged next
  GemmSeg sg = segs[pr.seg0];
  int total_steps = 0;
  for (int s = 0; s < pr.nseg; ++s) total_steps += segs[pr.seg0 + s].K / GK;
  auto advance = [&]() {
    k_i += GK;
    if (k_i >= sg.K) {
      k_i = 0;
      ++seg_i;
      if (seg_i < pr.nseg) sg = segs[pr.seg0 + seg_i];
    }
  };
  if (total_steps > 0) { stage(sg, k_i, 0); advance(); }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  for (int step = 0; step < total_steps; ++step) {
    const int buf = step & 1;
    if (step + 1 < total_steps) { stage(sg, k_i, buf ^ 1); advance(); }
    const half_t* Ab = As[buf] + (32 * wave + nn) * GK;
    const half_t* Bb = Bs[buf] + nn * GK;
#pragma unroll
    for (int ks = 0; ks < GK / 16; ++ks) {
      const int pos = ((2 * ks + g) ^ fK(nn)) << 3;        // fK(32 w + nn) = fK(32 t + nn) = fK(nn)
      const half8 rows = *(const half8*)(Ab + pos);
#pragma unroll
      for (int nt = 0; nt < 4; ++nt) {
        const half8 cols = *(const half8*)(Bb + nt * 32 * GK + pos);
        acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(cols, rows, acc[nt], 0, 0, 0);
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  }

  // store: lane = row of C, registers = columns; a register swap with the partner lane (lane ^ 32, same row) leaves
  // every lane with 8 consecutive columns, i.e. 16-byte stores
  const int row = m0 + 32 * wave + nn;
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      float o[8];   // columns nt*32 + j*16 + g*8 + 0..7
#pragma unroll
      for (int b = 0; b < 4; ++b) {
        const uint32_t lo = __float_as_uint(acc[nt][(2 * j) * 4 + b]);
        const uint32_t hi = __float_as_uint(acc[nt][(2 * j + 1) * 4 + b]);
        const auto sw = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
        o[b] = __uint_as_float(sw[0]);
        o[4 + b] = __uint_as_float(sw[1]);
      }
      const int col = n0 + nt * 32 + j * 16 + g * 8;
      if (row < pr.m && col < pr.n) {   // (n is a multiple of 8)
        uint4v st4;
#pragma unroll
        for (int b = 0; b < 4; ++b) st4[b] = gemm_pack_h2(o[2 * b], o[2 * b + 1]);
        *(uint4v*)(pr.C + (int64_t)row * pr.ldc + col) = st4;
      }
    }
}

// The same product with a 256 x 256 tile per workgroup of eight waves (a wave owns 64 rows x 128 columns: per K step of 16
// it reads 2 + 4 operands from LDS for 8 MFMAs, and the tile brings half the bytes per flop into LDS that the 128 x 128
// tile above does).  One workgroup per compute unit; K advances in steps of 64 through two LDS buffers of 64 KB (a
// variant with steps of 32 through four buffers - three steps in flight - measured 6 % slower, and so did touching the
// lines of later steps ahead of time to have them in L2, and so did spreading a step's copies between its MFMAs: the
// copies' latency is not what holds this kernel back; its LDS reads and copy writes together keep the LDS about as busy
// as the MFMAs keep the matrix cores).
// The columns of a launch run over all its problems back to back (problem p owns columns [p n, (p + 1) n), n a
// multiple of 32), so that a tile can span several narrow problems - the per-head projections are 64 or 128 columns
// wide.  All problems of a launch must have the same A segments (pointers, strides and K); B and C are the problem's own.
constexpr int WM = 256, WN = 256, WK = 64, WST = 2;

__global__ void __launch_bounds__(512, 1) k_gemm_nt_wide(const GemmProblem* __restrict__ probs, const GemmSeg* __restrict__ segs,
                                                         int per, int n, int tiles_m, int tiles_n) {
  static_assert((WM + WN) * WK * 2 * WST <= 160 * 1024, "LDS budget");
  __shared__ __attribute__((aligned(16))) half_t As[WST][WM * WK];
  __shared__ __attribute__((aligned(16))) half_t Bs[WST][WN * WK];
  const int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  const int mt = (seq / tiles_n) * 8 + xcd;
  if (mt >= tiles_m) return;   // (uniform over the workgroup: the grid is padded to whole rounds of 8 row tiles)
  const int m0 = mt * WM, gc0 = (seq % tiles_n) * WN;   // first row / first column (over all problems) of the tile
  const int n_total = per * n;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nn = lane & 31, g = lane >> 5;
  const int wm = wave & 3, wn = wave >> 2;              // this wave's 64 rows and 128 columns of the tile
  // Rows are WK halfs in LDS; the 16-byte chunks of row r are permuted through the source address so that the operand
  // reads of 16 consecutive rows fall on 16 different 16-byte bank groups
  constexpr int CPR = WK / 8;                           // chunks per row
  constexpr int RPI = 64 / CPR;                         // rows per copy instruction (64 lanes x 16 bytes)
  constexpr int IPW = 32 / RPI;                         // copy instructions per wave, step and matrix
  auto fK = [](int r) -> int { return (r >> 1) & 7; };
  const int lr = lane / CPR, lc = lane % CPR;

  // the copies: wave w moves rows [32 w, 32 w + 32) of the A tile and of the B tile
  const int bcol0 = gc0 + 32 * wave;                                    // first B row (= column of C) this wave copies
  const int pb = min(bcol0, n_total - 1) / n;                           // its problem (n % 32 == 0: one problem per wave)
  const GemmProblem prb = probs[pb];
  const int m = prb.m;
  int a_row[IPW], b_row[IPW];   // row within the tile's A rows / within the problem's B rows, clamped to what exists
#pragma unroll
  for (int i = 0; i < IPW; ++i) {
    const int r = 32 * wave + RPI * i + lr;
    a_row[i] = min(m0 + r, m - 1) - m0;
    b_row[i] = min(bcol0 + RPI * i + lr, n_total - 1) - pb * n;
  }
  auto stage = [&](const GemmSeg& sg, int k0, int buf) {
    const half_t* abase = sg.A + (int64_t)m0 * sg.lda + k0;   // wave-uniform
    const half_t* bbase = sg.B + k0;
#pragma unroll
    for (int i = 0; i < IPW; ++i) {
      const int r = 32 * wave + RPI * i + lr;
      const int chunk = (lc ^ fK(r)) << 3;
      gemm_dma16(abase + (uint32_t)(a_row[i] * sg.lda + chunk), As[buf] + (32 * wave + RPI * i) * WK);
      gemm_dma16(bbase + (uint32_t)(b_row[i] * sg.ldb + chunk), Bs[buf] + (32 * wave + RPI * i) * WK);
    }
  };

  float16v acc[4][2];   // [column tile][row tile]
#pragma unroll
  for (int ct = 0; ct < 4; ++ct)
#pragma unroll
    for (int rt = 0; rt < 2; ++rt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[ct][rt][r] = 0.f;

  int seg_i = 0, k_i = 0;   // position of the step that is copied next
  GemmSeg sg = segs[prb.seg0];
  int total_steps = 0;
  for (int s2 = 0; s2 < prb.nseg; ++s2) total_steps += segs[prb.seg0 + s2].K / WK;
  auto advance = [&]() {
    k_i += WK;
    if (k_i >= sg.K) {
      k_i = 0;
      ++seg_i;
      if (seg_i < prb.nseg) sg = segs[prb.seg0 + seg_i];
    }
  };
  if (total_steps > 0) { stage(sg, k_i, 0); advance(); }
  for (int step = 0; step < total_steps; ++step) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of step `step` has landed
    __syncthreads();   // step `step` is in LDS for every wave, and nobody reads the buffer of step - 1 any more
    if (step + 1 < total_steps) { stage(sg, k_i, (step + 1) % WST); advance(); }
    const int buf = step % WST;
    const half_t* Ab = As[buf] + (64 * wm + nn) * WK;
    const half_t* Bb = Bs[buf] + (128 * wn + nn) * WK;
    constexpr int NKS = WK / 16;
    half8 rows[2][2], cols[2][4];
    auto operands = [&](int ks, int set) {
      const int pos = ((2 * ks + g) ^ fK(nn)) << 3;        // fK(32 t + nn) = fK(nn)
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) rows[set][rt] = *(const half8*)(Ab + rt * 32 * WK + pos);
#pragma unroll
      for (int ct = 0; ct < 4; ++ct) cols[set][ct] = *(const half8*)(Bb + ct * 32 * WK + pos);
    };
    operands(0, 0);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      if (ks + 1 < NKS) operands(ks + 1, (ks + 1) & 1);
#pragma unroll
      for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt)
          acc[ct][rt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(cols[ks & 1][ct], rows[ks & 1][rt], acc[ct][rt], 0, 0, 0);
    }
  }

  // store: lane = row of C, registers = columns; a register swap with the partner lane (lane ^ 32, same row) leaves
  // every lane with 8 consecutive columns, i.e. 16-byte stores.  Every 32-column tile looks up its own problem.
#pragma unroll
  for (int ct = 0; ct < 4; ++ct) {
    const int gc = gc0 + 128 * wn + 32 * ct;
    if (gc >= n_total) break;
    const int pc = gc / n;
    const GemmProblem pr = probs[pc];
    const int col0 = gc - pc * n;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
      const int row = m0 + 64 * wm + 32 * rt + nn;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        float o[8];   // columns col0 + j*16 + g*8 + 0..7
#pragma unroll
        for (int b = 0; b < 4; ++b) {
          const uint32_t lo = __float_as_uint(acc[ct][rt][(2 * j) * 4 + b]);
          const uint32_t hi = __float_as_uint(acc[ct][rt][(2 * j + 1) * 4 + b]);
          const auto sw = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
          o[b] = __uint_as_float(sw[0]);
          o[4 + b] = __uint_as_float(sw[1]);
        }
        if (row < pr.m) {
          uint4v st4;
#pragma unroll
          for (int b = 0; b < 4; ++b) st4[b] = gemm_pack_h2(o[2 * b], o[2 * b + 1]);
          *(uint4v*)(pr.C + (int64_t)row * pr.ldc + col0 + j * 16 + g * 8) = st4;
        }
      }
    }
  }
}

// out[c][r] = (fp16) in[r][c] for a bf16 matrix [R][Cc]: the weights arrive [k][n] (n contiguous) and the product wants
// them K-contiguous.  32 x 32 tiles through LDS.
__global__ void __launch_bounds__(256) k_transpose_bf16_to_f16(const uint16_t* __restrict__ in, half_t* __restrict__ out, int R, int Cc) {
  __shared__ half_t tile[32][33];
  const int c0 = blockIdx.x * 32, r0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  for (int i = ty; i < 32; i += 8) {
    const int r = r0 + i, c = c0 + tx;
    float v = 0.f;
    if (r < R && c < Cc) v = __uint_as_float((uint32_t)in[(int64_t)r * Cc + c] << 16);
    tile[i][tx] = (half_t)v;
  }
  __syncthreads();
  for (int i = ty; i < 32; i += 8) {
    const int c = c0 + i, r = r0 + tx;
    if (r < R && c < Cc) out[(int64_t)c * R + r] = tile[tx][i];
  }
}

}  // namespace

// `per` problems d_probs[0 .. per) of identical m and n (host-checked by the caller).
hipError_t launch_gemm_nt(const GemmProblem* d_probs, const GemmSeg* d_segs, int per, int m, int n, hipStream_t st) {
  if (per <= 0 || m <= 0 || n <= 0) return hipSuccess;
  static int wide = -1;
  if (wide < 0) { const char* e = getenv("FREQATTN_GEMM_WIDE"); wide = e ? atoi(e) : 1; }
  if (wide && n % 32 == 0 && m >= WM && (int64_t)per * n >= WN) {
    // (the callers' launches share their A segments between problems, which the wide kernel relies on)
    const int tiles_m = (m + WM - 1) / WM, tiles_n = (int)(((int64_t)per * n + WN - 1) / WN);
    const int64_t blocks = (int64_t)((tiles_m + 7) / 8) * 8 * tiles_n;
    if (blocks > 0x7fffffff) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_gemm_nt_wide, dim3((unsigned)blocks), dim3(512), 0, st, d_probs, d_segs, per, n, tiles_m, tiles_n);
    return hipGetLastError();
  }
  const int tiles_m = (m + GM - 1) / GM, tiles_n = (n + GN - 1) / GN;
  const int64_t blocks = (int64_t)((tiles_m + 7) / 8) * 8 * tiles_n * per;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(k_gemm_nt, dim3((unsigned)blocks), dim3(256), 0, st, d_probs, d_segs, per, tiles_m, tiles_n);
  return hipGetLastError();
}

hipError_t launch_transpose_bf16_to_f16(const void* in, void* out, int R, int Cc, hipStream_t st) {
  if (R <= 0 || Cc <= 0) return hipSuccess;
  hipLaunchKernelGGL(k_transpose_bf16_to_f16, dim3((unsigned)((Cc + 31) / 32), (unsigned)((R + 31) / 32)), dim3(256), 0, st,
                     (const uint16_t*)in, (half_t*)out, R, Cc);
  return hipGetLastError();
}

}  // namespace fa
