// Band attention on the gfx950 matrix cores (paper sections 3.4.1-3.4.3, 3.6, 6.2).
//
// One kernel serves every branch.  A work item is a tile of 32*NW query rows of one branch of one (batch, head)
// slice; the branches differ only in which 64-key tiles the item visits and how scores are masked:
//   low   all tiles of the compressed low band            (dense global attention)
//   mid   the tiles of the key blocks listed for the query block (block-sparse pattern)
//   high  the tiles overlapping [q - w, q + w]            (sliding window, element mask on the edge tiles)
//   exchange  the <= 2m summary tokens of the other bands, result added to the query row (residual)
//   dense all tiles of the untransformed sequence         (comparison baseline)
// The launch is persistent: workgroups stride over the item list (branch by branch, long items first), so the
// three branches are co-scheduled in one launch.
//
// Per 64-key tile, with S^T = K Q^T kept transposed so that a lane owns one query column:
//   K tile   -> LDS row-major, A operand of v_mfma_f32_32x32x16_f16 (lane = key, 8 consecutive channels)
//   Q        -> registers, B operand (lane = query, 8 consecutive channels), loaded once per item
//   softmax  -> running max / sum per lane (one query per lane; the two lane halves hold different keys)
//   V tile   -> V^T operand (A) in the key order of the S^T accumulator, so that the accumulator registers,
//               converted to fp16, are the B operand of O^T += V^T P^T directly.
// Staging: K and V rows are copied straight from global memory into LDS, row-major; V^T comes out of transposing LDS
// reads.  All tensors are fp16 (the dense comparison converts its bf16 tensors into fp16 scratch first).
#include <hip/hip_runtime.h>

#include "ctx.h"

namespace fa {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef __fp16 fp16x4 __attribute__((__vector_size__(4 * sizeof(__fp16))));
typedef float float16v __attribute__((ext_vector_type(16)));
typedef unsigned int uint4v __attribute__((ext_vector_type(4)));
typedef unsigned int uint2v __attribute__((ext_vector_type(2)));

#define KT 64  // keys per tile

__device__ __forceinline__ uint32_t pack_h2(float a, float b) {
  const _Float16 ha = (_Float16)a, hb = (_Float16)b;
  return (uint32_t)__builtin_bit_cast(uint16_t, ha) | ((uint32_t)__builtin_bit_cast(uint16_t, hb) << 16);
}

// One wave-wide 16-byte-per-lane copy from global memory straight into LDS: lane l's 16 bytes land at dst + 16 l,
// dst wave-uniform.  Issued as assembly on purpose: the compiler orders every LDS read behind a pending copy of this
// kind that it knows of (it cannot tell the two LDS tile copies apart), which would put the whole latency of the next
// tile's fetch in front of the current tile's arithmetic.  The kernel waits for these copies itself (vmcnt(0) in front
// of the barrier that publishes the tile); the compiler's own waits for its global loads only become stricter.
__device__ __forceinline__ void lds_dma16(const void* src, const half_t* dst) {
  const unsigned base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)(const __attribute__((address_space(3))) half_t*)dst);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src), "s"(base) : "memory", "m0");
}

template <int D, int NW>
__global__ void __launch_bounds__(64 * NW, (D == 64 || NW == 4) ? 2 : 1) k_attn(AttnParams p, const AttnItem* __restrict__ items, int n_items) {
  constexpr int DT = D / 32;    // 32-channel tiles of the output
  constexpr int DK = D / 16;    // MFMA steps over the channels for S
  constexpr int NT = 64 * NW;
  constexpr int ROWS = 32 * NW;  // query rows per item
  constexpr int WROWS = 32;      // query rows per wave
  // two copies of the K / V tiles: tile i+1 is written while tile i is still being read, one barrier per tile
  __shared__ __attribute__((aligned(16))) half_t Ks2[2][KT * D];
  __shared__ __attribute__((aligned(16))) half_t Vt2[2][KT * D];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nn = lane & 31, g = lane >> 5;
  // K and V tiles are row-major in LDS, rows of D halfs without padding, loaded by
  // global_load_lds_dwordx4 (lane l of a wave instruction fills bytes 16 l .. 16 l + 15 behind a wave-uniform LDS base,
  // whatever global address the lane names).  Bank conflicts are avoided by permuting the 16-byte chunks inside a row
  // through the global address: chunk c of row r sits at position c ^ fK(r) (K, read as 16-byte A operands by 16
  // consecutive rows) or c ^ fV(r) (V, read through ds_read_b64_tr_b16, which hands lane i of a 16-lane group, for
  // k = 0..3, element i % 4 of the 8-byte piece named by lane 4 k + i / 4: four rows of 32 bytes per group).
  constexpr int CPR = D / 8;                       // 16-byte chunks per row
  auto fK = [](int r) -> int { return D == 128 ? (r & 15) : ((r >> 1) & 7); };
  auto fV = [](int r) -> int { return D == 128 ? ((r & 3) << 2) : (((r >> 1) & 1) << 2); };
  // per-lane parts of the operand addresses of the DMA layout (halfs), fixed for the whole kernel:
  //   K operand (t2, ks):  Ks + t2*32*D + koff_row + kx[ks]         row nn, chunk (2 ks + g) ^ fK(nn)
  //   V operand (dt, ts, h): Vt + (16 ts + 8 h)*D + voff_row + vx[dt]  row 4 g + sl/4 (+ 16 ts + 8 h), chunk (4 dt + 2 g1 + (sl & 3)/2) ^ fV(row)
  int kx[D / 16], vx[D / 32];
  int koff_row, voff_row;
  {
    const int sl = lane & 15, g1 = (lane >> 4) & 1;
    koff_row = nn * D;
    voff_row = (4 * g + (sl >> 2)) * D + (sl & 1) * 4;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) kx[ks] = ((2 * ks + g) ^ fK(nn)) << 3;
#pragma unroll
    for (int dt = 0; dt < D / 32; ++dt) vx[dt] = ((4 * dt + 2 * g1 + ((sl & 3) >> 1)) ^ fV(sl >> 2)) << 3;
  }
  const float c2 = p.scale * 1.4426950408889634f;  // folded into Q: scores come out of the MFMA in units of log2

  // Workgroups are dealt to the 8 XCDs round-robin by blockIdx, and each XCD has its own L2.  Consecutive items are
  // neighbouring query tiles of one slice, which visit largely the same K/V tiles (all of them in the dense branches,
  // most of the window in the high band): each round of gridDim.x items is cut into 8 contiguous runs, one per XCD,
  // so that those tiles are fetched into one L2 once instead of into all eight.
  int it_first = blockIdx.x;
  if ((gridDim.x & 7) == 0) it_first = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
  int lds_holds = -1;   // (slice, band) whose summary tiles the LDS copies hold, -1: something else
  // the next item's descriptor is fetched while the current item runs (its fields start a chain of dependent loads)
  AttnItem item_nx = items[it_first < n_items ? it_first : 0];
  for (int it = it_first; it < n_items; it += gridDim.x) {
    const AttnItem item = item_nx;
    if (it + (int)gridDim.x < n_items) item_nx = items[it + gridDim.x];
    const int kind = item.kind_band & 0xff, band = (item.kind_band >> 8) & 0xff;   // bit 16: exchange in the item (phase 1)
    const int64_t slice = item.slice;
    const int q0 = item.q0;
    const uint16_t *Qp, *Kp, *Vp;
    uint16_t* Op;
    int nq, nk;
    if (kind == 0) {
      const int64_t o = slice * p.nbar * D;
      Qp = (const uint16_t*)p.lowQ + o; Kp = (const uint16_t*)p.lowK + o; Vp = (const uint16_t*)p.lowV + o;
      Op = (uint16_t*)p.lowY + o; nq = nk = p.nbar;
    } else if (kind == 1 || kind == 2) {
      const int64_t o = (slice * p.N + p.band_off[band]) * D;
      Qp = (const uint16_t*)p.specQ + o; Kp = (const uint16_t*)p.specK + o; Vp = (const uint16_t*)p.specV + o;
      Op = (uint16_t*)p.Y + o; nq = nk = p.band_n[band];
    } else if (kind == 3) {
      const int64_t o = (slice * p.N + p.band_off[band]) * D;
      Qp = (const uint16_t*)p.Y + o; Op = (uint16_t*)p.Y + o; nq = p.band_n[band];
      Kp = Vp = (const uint16_t*)p.C + ((slice * p.nb + band) * p.m2) * (int64_t)D; nk = p.n_c[band];
    } else {
      const int64_t o = slice * p.N * D;
      Qp = (const uint16_t*)p.denseQ + o; Kp = (const uint16_t*)p.denseK + o; Vp = (const uint16_t*)p.denseV + o;
      Op = (uint16_t*)p.denseO + o; nq = nk = p.N;
    }
    const int w = p.high_window;
    const int r0 = q0 + WROWS * wave;   // first query row of this wave

    // Q operand: lane holds channels 16*ks + 8*g .. +8 of its query row, pre-scaled
    half8 Qr[DK];
    {
      const int row = r0 + nn;
#pragma unroll
      for (int ks = 0; ks < DK; ++ks) {
        uint4v v = {0u, 0u, 0u, 0u};
        if (row < nq) v = *(const uint4v*)(Qp + (int64_t)row * D + ks * 16 + g * 8);
        half8 h = __builtin_bit_cast(half8, v);
#pragma unroll
        for (int j = 0; j < 8; ++j) h[j] = (_Float16)((float)h[j] * c2);
        Qr[ks] = h;
      }
    }

    float16v O[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) O[dt][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    // C operand that starts a score accumulation: minus the lane's reference maximum in every register, so that the
    // matrix core delivers the scores already shifted (0 while the row has seen no valid key): in the common case (no new
    // reference) they go into exp2 without a subtraction, and no accumulator is initialised per tile
    float16v Minit;
#pragma unroll
    for (int r = 0; r < 16; ++r) Minit[r] = 0.f;

    // Staging: this wave's share of a tile is RPI rows per instruction, NIW instructions per tensor; rows past the
    // end of the key range are clamped to its last row (their scores are masked, and V rows of real data times zero are zero)
    constexpr int RPI = 64 / CPR, NIW = KT / (RPI * NW);
    // piece pi of a tile: K rows (pi even) or V rows (pi odd) of instruction pi / 2 of this wave's share
    auto dma_piece = [&](const uint16_t* Ksrc, const uint16_t* Vsrc, int nkeys, int key0, int buf, int pi) {
      const int lr = lane / CPR, c = lane % CPR;
      const int rowbase = (wave * NIW + pi / 2) * RPI;      // wave-uniform
      const int r = rowbase + lr;
      int key = key0 + r;
      if (key > nkeys - 1) key = nkeys - 1;
      if ((pi & 1) == 0) lds_dma16(Ksrc + (int64_t)key * D + ((c ^ fK(r)) << 3), Ks2[buf] + rowbase * D);
      else lds_dma16(Vsrc + (int64_t)key * D + ((c ^ fV(r)) << 3), Vt2[buf] + rowbase * D);
    };

    // An item runs one or two phases over the same query rows.  Phase 0 is the band operator.  Phase 1 (items marked
    // for it: every other band of the slice passes V~ through, so the summary tokens this band attends to were pooled
    // before the launch) is the cross-band exchange of section 3.6, with the phase-0 result - rounded to fp16 exactly as
    // it would have been stored - as the query and as the residual, and the <= 2m summary tokens as keys and values.
    const int n_phases = 1 + (item.kind_band >> 16 & 1);
    const uint16_t* Cp = (const uint16_t*)p.C + ((slice * p.nb + band) * p.m2) * (int64_t)D;
    int tile_base = 0;   // tiles staged so far in this item: tile i of the item lives in LDS copy i & 1
    bool staged = false; // the first tile of the coming phase is already in its LDS copy
    for (int phase = 0; phase < n_phases; ++phase) {
      const int kind_p = phase ? 0 : kind;
      const uint16_t* Kq = phase ? Cp : Kp;
      const uint16_t* Vq = phase ? Cp : Vp;
      const int nkp = phase ? p.n_c[band] : nk;
      if (phase) {
        // phase-0 output -> fp16 (what the band operator alone would store) -> query operand and residual
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            uint4v y4;
            half8 qh;
            float o[8];
#pragma unroll
            for (int b = 0; b < 4; ++b) {
              const uint32_t lo = __float_as_uint(O[dt][(2 * j) * 4 + b] * inv);
              const uint32_t hi = __float_as_uint(O[dt][(2 * j + 1) * 4 + b] * inv);
              const auto sw = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
              o[b] = __uint_as_float(sw[0]);
              o[4 + b] = __uint_as_float(sw[1]);
            }
#pragma unroll
            for (int b = 0; b < 4; ++b) y4[b] = pack_h2(o[2 * b], o[2 * b + 1]);
            const half8 yh = __builtin_bit_cast(half8, y4);
#pragma unroll
            for (int b = 0; b < 8; ++b) qh[b] = (_Float16)((float)yh[b] * c2);
            // The rows are parked in the output tensor - exactly what the band operator alone would have stored - and
            // come back as the residual in the epilogue (same lane, same address: no other reader in this launch).
            if (r0 + nn < nq) *(uint4v*)(Op + (int64_t)(r0 + nn) * D + dt * 32 + j * 16 + g * 8) = y4;
            Qr[dt * 2 + j] = qh;
          }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) O[dt][r] = 0.f;
        m_run = -INFINITY; l_run = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) Minit[r] = 0.f;
      }

      // tile iteration space of the phase
      int n_outer = 1, e0 = 0, sub_n = 1, t_lo = 0, t_hi = 0;
      if (kind_p == 1) {
        const int I = q0 / p.mid_block;
        const int32_t* rp = band == MID2 ? p.mid2_row_ptr : p.mid_row_ptr;   // each block-sparse band has its own list
        e0 = rp[I];
        n_outer = rp[I + 1] - e0;
        sub_n = p.mid_block / KT;
      } else if (kind_p == 2) {
        const int klo = q0 - w > 0 ? q0 - w : 0;
        int khi = q0 + ROWS - 1 + w;
        if (khi > nkp - 1) khi = nkp - 1;
        t_lo = klo / KT; t_hi = khi / KT;
        n_outer = t_hi - t_lo + 1;
      } else {
        n_outer = (nkp + KT - 1) / KT;
      }
      const int n_tt = n_outer * sub_n;
      // The key blocks of a block-sparse item are read once, 64 at a time, one per lane (a wave-wide load in the tile
      // loop would put a trip through the memory hierarchy in front of every tile's copies); key0_of picks its entry
      // out of the register.
      const int32_t* cidx = (band == MID2 ? p.mid2_col_idx : p.mid_col_idx) + e0;
      int colv = 0, cbase = 0;
      auto load_cols = [&](int base) {
        cbase = base;
        colv = (kind_p == 1 && base + lane < n_outer) ? cidx[base + lane] : 0;
      };
      load_cols(0);
      auto key0_of = [&](int idx) -> int {
        if (kind_p == 1) {
          const int blk = idx / sub_n;
          if (blk < cbase || blk >= cbase + 64) load_cols(blk & ~63);   // (uniform; only items with more than 64 key blocks)
          return (__builtin_amdgcn_readlane(colv, blk - cbase) * sub_n + (idx - blk * sub_n)) * KT;
        }
        return (t_lo + idx) * KT;
      };
      // Exchange items of one (slice, band) all see the same <= 2 tiles of summary tokens: a workgroup that has them in
      // its two LDS copies from its previous item keeps them (no loads, no stores for this item).
      const int lds_key = (kind == 3 && n_tt <= 2) ? (int)(slice * 4 + band) : -1;
      const bool reuse = lds_key >= 0 && lds_key == lds_holds;
      lds_holds = lds_key;
      if (!staged) {
        if (n_tt > 0 && !reuse) {
#pragma unroll
          for (int pi = 0; pi < 2 * NIW; ++pi) dma_piece(Kq, Vq, nkp, key0_of(0), tile_base & 1, pi);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
      }
      staged = false;
      for (int idx = 0; idx < n_tt; ++idx, __builtin_amdgcn_s_waitcnt(0x0070), __syncthreads()) {
        const int key0 = key0_of(idx);
        const int buf = (tile_base + idx) & 1;
        const half_t* Ks = Ks2[buf];
        const half_t* Vt = Vt2[buf];
        // The next tile goes straight into the other LDS copy (free since the barrier that ended the previous iteration);
        // the wait for it sits in front of the barrier that ends this iteration.  Its copy instructions are spread over the
        // score MFMAs below (a wave issues in order, and a burst of them right behind the barrier holds every wave of the
        // CU in the memory pipeline's queue); an iteration that skips the MFMAs issues them at once.  The last tile of
        // phase 0 fetches the first summary tile of phase 1 the same way.
        const bool next_in_phase = idx + 1 < n_tt;
        const bool next_phase = !next_in_phase && phase + 1 < n_phases;
        const bool dma_next = (next_in_phase && !reuse) || next_phase;
        const uint16_t* Kn = next_phase ? Cp : Kq;
        const uint16_t* Vn = next_phase ? Cp : Vq;
        const int nkn = next_phase ? p.n_c[band] : nkp;
        const int key0_next = next_in_phase ? key0_of(idx + 1) : 0;
        if (next_phase) staged = true;
        auto stage = [&]() {
          if (dma_next) {
#pragma unroll
            for (int pi = 0; pi < 2 * NIW; ++pi) dma_piece(Kn, Vn, nkn, key0_next, buf ^ 1, pi);
          }
        };
        if (key0 >= nkp) {  // block tail beyond the band (uniform over the workgroup)
          stage();
          continue;
        }

        // ---- does this wave need the tile at all (window), and does it need the element mask
        const int key_hi = key0 + KT - 1;
        bool need = true, need_mask = key_hi >= nkp;
        if (kind_p == 2) {
          need = !(key_hi < r0 - w || key0 > r0 + WROWS - 1 + w);
          need_mask = need_mask || (key0 < r0 + WROWS - 1 - w) || (key_hi > r0 + w);
        }
        if (!need) {  // uniform per wave; the tile's barrier sits in the loop increment, which `continue` still runs
          stage();
          continue;
        }

        // ---- S^T = K Q^T for the two 32-key halves of the tile
        float16v S[2];   // (each starts from Minit)
        // K operands are requested PF steps ahead of the MFMA that consumes them, so LDS latency overlaps the matrix core
        // The wave takes the higher issue priority for the score stage (its operand reads, its MFMAs and the next tile's
        // copies spread between them) and gives it back for the softmax: with two waves per SIMD the one that starts a
        // tile gets its copies and reads under way while the other is in its vector work (measured: block-sparse branch
        // 6 % faster, window branch 2 %; priority in the other stages instead, or in all MFMA stages, gains less).
        __builtin_amdgcn_s_setprio(1);
        constexpr int PF = 8;
        {
          constexpr int NS = 2 * DK;
          auto kptr = [&](int i) -> const half8* {
            return (const half8*)(Ks + (i / DK) * 32 * D + koff_row + kx[i % DK]);   // fK(t2*32 + nn) = fK(nn)
          };
          half8 Abuf[PF];
#pragma unroll
          for (int i = 0; i < PF; ++i) Abuf[i] = *kptr(i);
#pragma unroll
          for (int i = 0; i < NS; ++i) {
            const int t2 = i / DK, ks = i % DK;
            const half8 A = Abuf[i % PF];
            if (i + PF < NS)
              Abuf[i % PF] = *kptr(i + PF);
            S[t2] = __builtin_amdgcn_mfma_f32_32x32x16_f16(A, Qr[ks], ks == 0 ? Minit : S[t2], 0, 0, 0);
            if (dma_next) {
#pragma unroll
              for (int pi = i * (2 * NIW) / NS; pi < (i + 1) * (2 * NIW) / NS; ++pi) dma_piece(Kn, Vn, nkn, key0_next, buf ^ 1, pi);
            }
          }
          // pin the order: PF reads up front, then one read per MFMA
          __builtin_amdgcn_sched_group_barrier(0x100, PF, 0);
#pragma unroll
          for (int i = 0; i < NS - PF; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          }
          __builtin_amdgcn_sched_group_barrier(0x008, PF, 0);
        }
        __builtin_amdgcn_s_setprio(0);
        // ---- mask, running softmax (lane = query row; registers = keys).  m_run is a reference maximum, not the exact
        // one: it moves only when a score exceeds it by more than 2^kBump (or when the row sees its first valid key), so
        // probabilities stay within [0, 2^kBump] - exact in the ratio P / sum(P) - and the rescale is rare.
        constexpr float kBump = 8.f;
        half8 P[2][2];
        if (need_mask) {
          // valid keys of this lane's row form one interval [lo, hi]; relative to the lane's first key of the tile,
          // register r holds key offset c_r (a compile-time constant), valid iff (unsigned)(c_r - lo') <= (unsigned)(hi' - lo')
          const int row = r0 + nn;
          int lo = 0, hi = nkp - 1;
          if (kind_p == 2) { lo = row - w > 0 ? row - w : 0; hi = row + w < nkp - 1 ? row + w : nkp - 1; }
          const int base = key0 + 4 * g;
          int dlo = lo - base, dhi = hi - base;
          dlo = dlo < -1 ? -1 : (dlo > 65 ? 65 : dlo);    // clamped: only the range of c_r matters
          dhi = dhi < -1 ? -1 : (dhi > 65 ? 65 : dhi);
          unsigned range = (unsigned)(dhi - dlo);
          if (dhi < dlo) { dlo = 1000; range = 0u; }      // empty interval: no c_r passes
          const unsigned ndlo = (unsigned)(-dlo);
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const unsigned cr = (unsigned)(t2 * 32 + 8 * (r >> 2) + (r & 3));
              S[t2][r] = (cr + ndlo <= range) ? S[t2][r] : -INFINITY;
            }
        }
        // row maximum: four independent chains (short dependency depth), then the other lane half through a register
        // swap (v_permlane32_swap leaves [lo, lo] / [hi, hi] in the two registers; no trip through the LDS pipe)
        float mc[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
          for (int r = 0; r < 16; r += 2)
            mc[(r >> 1) & 3] = __builtin_fmaxf(__builtin_fmaxf(mc[(r >> 1) & 3], S[t2][r]), S[t2][r + 1]);
        float mx = fmaxf(fmaxf(mc[0], mc[1]), fmaxf(mc[2], mc[3]));
        {
          const uint32_t mb = __float_as_uint(mx);
          const auto sw = __builtin_amdgcn_permlane32_swap(mb, mb, false, false);
          mx = fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
        }
        const bool bump = (m_run == -INFINITY) ? (mx > -INFINITY) : (mx > kBump);
        // Probabilities, two per register, rounded toward zero; the row sum is taken over the rounded values (the ones
        // the matrix core multiplies), so the rounding direction cancels in P / sum(P).  They are formed before the
        // (rare) reference bump is known, so that the exponentials overlap the maximum's dependency chain.
        auto probabilities = [&]() -> float {
          float ps[4] = {0.f, 0.f, 0.f, 0.f};
          const half2v ones = {(_Float16)1.f, (_Float16)1.f};
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
              uint4v pk;
#pragma unroll
              for (int j = 0; j < 4; ++j) {
                const half2v h2 = __builtin_bit_cast(half2v, __builtin_amdgcn_cvt_pkrtz(
                    __builtin_amdgcn_exp2f(S[t2][s2 * 8 + 2 * j]), __builtin_amdgcn_exp2f(S[t2][s2 * 8 + 2 * j + 1])));
                ps[j] = __builtin_amdgcn_fdot2(h2, ones, ps[j], false);
                pk[j] = __builtin_bit_cast(uint32_t, h2);
              }
              P[t2][s2] = __builtin_bit_cast(half8, pk);
            }
          return (ps[0] + ps[1]) + (ps[2] + ps[3]);
        };
        float psum = probabilities();
        if (__builtin_amdgcn_ballot_w64(bump) != 0) {
          const bool fresh = m_run == -INFINITY;
          const float delta = bump ? mx : 0.f;
          const float alpha = (bump && !fresh) ? __builtin_amdgcn_exp2f(-delta) : 1.f;
          if (bump) m_run = fresh ? delta : m_run + delta;
          l_run *= alpha;
          {
            const float mi = (m_run == -INFINITY) ? 0.f : -m_run;
#pragma unroll
            for (int r = 0; r < 16; ++r) Minit[r] = mi;
            asm volatile("" : "+v"(Minit));   // (sixteen registers on purpose, not one value spread again per tile)
          }
#pragma unroll
          for (int t2 = 0; t2 < 2; ++t2)
#pragma unroll
            for (int r = 0; r < 16; ++r) S[t2][r] -= delta;
#pragma unroll
          for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) O[dt][r] *= alpha;
          psum = probabilities();   // again, against the moved reference
        }
        l_run += psum;
        // ---- O^T += V^T P^T
        {
          constexpr int NS = 4 * DT;   // (t2, s2, dt) flattened, dt fastest
          // V is row-major in LDS; the operand (lane = channel, 8 keys in the order of P's registers) comes from two
          // transposing reads, each delivering 4 consecutive keys: keys 16 ts + 8 h + 4 g + 0..3 for read h
          auto vread = [&](int i) -> half8 {
            const int dt = i % DT, ts = i / DT;   // ts = t2 * 2 + s2
            uint4v r4;
#pragma unroll
            for (int h = 0; h < 2; ++h) {
              const half_t* ptr = Vt + (ts * 16 + 8 * h) * D + voff_row + vx[dt];   // fV only sees row & 3 = sl / 4
              const fp16x4 t4 = __builtin_amdgcn_ds_read_tr16_b64_v4f16((fp16x4 __attribute__((address_space(3)))*)ptr);
              const uint2v u2 = __builtin_bit_cast(uint2v, t4);
              r4[2 * h] = u2[0]; r4[2 * h + 1] = u2[1];
            }
            return __builtin_bit_cast(half8, r4);
          };
          half8 Abuf[PF];
#pragma unroll
          for (int i = 0; i < PF; ++i) Abuf[i] = vread(i);
#pragma unroll
          for (int i = 0; i < NS; ++i) {
            const int dt = i % DT, ts = i / DT;
            const half8 A = Abuf[i % PF];
            if (i + PF < NS) Abuf[i % PF] = vread(i + PF);
            O[dt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(A, P[ts >> 1][ts & 1], O[dt], 0, 0, 0);
          }
        }
      }
      tile_base += n_tt;
    }

    // ---- epilogue: normalise, optional residual, store.  A lane holds, per 16 channels, two groups of four that
    // interleave with its partner lane's (lane ^ 32, same query): swapping one group each (v_permlane32_swap) leaves
    // every lane with 8 consecutive channels, i.e. 16-byte stores (and 16-byte residual loads) of whole 32-byte sectors.
    {
      const int row = r0 + nn;
      const float l_tot = l_run + __shfl_xor(l_run, 32);
      const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
#pragma unroll
      for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          float o[8];   // after the swap: channels dt*32 + j*16 + g*8 + 0..7
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            const uint32_t lo = __float_as_uint(O[dt][(2 * j) * 4 + b] * inv);       // channels 16j + 4g + b
            const uint32_t hi = __float_as_uint(O[dt][(2 * j + 1) * 4 + b] * inv);   // channels 16j + 8 + 4g + b
            const auto sw = __builtin_amdgcn_permlane32_swap(lo, hi, false, false);
            o[b] = __uint_as_float(sw[0]);
            o[4 + b] = __uint_as_float(sw[1]);
          }
          if (row < nq) {
            const int dd = dt * 32 + j * 16 + g * 8;
            uint16_t* dst = Op + (int64_t)row * D + dd;
            if (kind == 3 || n_phases == 2) {   // residual: the exchange's query rows (parked in the output by phase 1's start)
              const uint4v y = *(const volatile uint4v*)((kind == 3 ? Qp : (const uint16_t*)Op) + (int64_t)row * D + dd);
              const half8 yh = __builtin_bit_cast(half8, y);
#pragma unroll
              for (int b = 0; b < 8; ++b) o[b] += (float)yh[b];
            }
            uint4v st4;
#pragma unroll
            for (int b = 0; b < 4; ++b) st4[b] = pack_h2(o[2 * b], o[2 * b + 1]);
            *(uint4v*)dst = st4;
          }
        }
    }
  }
}

// Loop of independent v_mfma_f32_32x32x16_f16 (four accumulators per wave, two waves per SIMD): the matrix-core rate
// the machine sustains for this instruction, measured next to the attention kernel.
__global__ void __launch_bounds__(256, 2) k_probe_mfma(float* out, int iters) {
  half8 a, b;
#pragma unroll
  for (int j = 0; j < 8; ++j) { a[j] = (_Float16)(0.001f * (threadIdx.x & 63) + j); b[j] = (_Float16)(0.5f * j - 0.002f * (threadIdx.x & 63)); }
  float16v c0, c1, c2, c3;
#pragma unroll
  for (int r = 0; r < 16; ++r) c0[r] = c1[r] = c2[r] = c3[r] = 0.f;
  for (int i = 0; i < iters; ++i) {
    c0 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c0, 0, 0, 0);
    c1 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c1, 0, 0, 0);
    c2 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c2, 0, 0, 0);
    c3 = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c3, 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int r = 0; r < 16; ++r) s += c0[r] + c1[r] + c2[r] + c3[r];
  out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}
// flops of one launch: blocks * 4 waves * iters * 4 MFMAs * 32*32*16*2; out needs blocks*256 floats
hipError_t launch_probe_mfma(float* out, int blocks, int iters, hipStream_t st) {
  hipLaunchKernelGGL(k_probe_mfma, dim3((unsigned)blocks), dim3(256), 0, st, out, iters);
  return hipGetLastError();
}

template <int D, int NW>
static hipError_t launch_dn(const AttnParams& p, const AttnItem* items, int n_items, int num_cu, hipStream_t st) {
  // resident workgroups per CU: register-limited waves per SIMD, 4 SIMDs per CU (matches the kernel's launch bounds)
  const int waves_per_simd = (D == 64 || NW == 4) ? 2 : 1;
  int occ = waves_per_simd * 4 / NW;
  if (occ < 1) occ = 1;
  int64_t blocks = (int64_t)num_cu * occ;
  if (blocks > n_items) blocks = n_items;
  if (blocks > 8) blocks -= blocks % 8;   // whole runs per XCD (see the kernel's item mapping)
  hipLaunchKernelGGL((k_attn<D, NW>), dim3((unsigned)blocks), dim3(64 * NW), 0, st, p, items, n_items);
  return hipGetLastError();
}

hipError_t launch_mfma_attn(const AttnParams& p, const AttnItem* items, int n_items, int rows_per_item, int num_cu,
                            hipStream_t st) {
  if (n_items <= 0) return hipSuccess;
#define FA_ATTN_CASE(D_, R_, NW_) \
  if (p.d == D_ && rows_per_item == R_) return launch_dn<D_, NW_>(p, items, n_items, num_cu, st);
  FA_ATTN_CASE(64, 64, 2) FA_ATTN_CASE(64, 128, 4) FA_ATTN_CASE(128, 64, 2) FA_ATTN_CASE(128, 128, 4)
#undef FA_ATTN_CASE
  return hipErrorInvalidValue;
}

}  // namespace fa
