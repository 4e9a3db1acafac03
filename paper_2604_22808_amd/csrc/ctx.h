// Internal definitions shared by the host side and the kernel launchers of libfreqattn.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string>
#include <vector>

#include "freqattn.h"

namespace fa {

typedef _Float16 half_t;

enum { LOW = 0, MID = 1, HIGH = 2, MID2 = 3 };   // MID2: the second block-sparse band of a four-band layout (its rows follow the high band's)
enum { NBMAX = 4 };

// Work item of the attention kernels: a tile of query rows of one branch of one (batch*heads) slice.
// kind: 0 low (compressed tokens), 1 mid (block list), 2 high (window), 3 exchange on band `band`, 4 dense baseline.
struct AttnItem {
  int32_t kind_band;  // kind | band << 8
  int32_t slice;      // batch*heads index
  int32_t q0;         // first query row of the tile, in band order
  int32_t cost;       // key tiles the item visits (used for ordering only)
};

// Everything the attention kernels need besides the item list (device pointers into context-owned memory).
struct AttnParams {
  const void* specQ;  // [slices][N][d] band-major, band l starts at row band_off[l]
  const void* specK;
  const void* specV;
  void* Y;            // [slices][N][d] band-major band outputs
  const void* lowQ;   // [slices][nbar][d] compressed low band
  const void* lowK;
  const void* lowV;
  void* lowY;
  const void* C;      // [slices][nb][(nb-1) m][d] summary tokens seen by band l
  const int32_t* mid_row_ptr;
  const int32_t* mid_col_idx;
  const int32_t* mid2_row_ptr;   // block list of band MID2
  const int32_t* mid2_col_idx;
  int32_t band_off[NBMAX];
  int32_t band_n[NBMAX];
  int32_t n_c[NBMAX]; // valid rows of C per band
  int32_t nb;         // bands: 3 or 4
  int32_t N, d, nbar, m2;  // m2 = (nb-1) m = rows reserved per band in C
  int32_t mid_block, high_window;
  float scale;
  // dense baseline
  const void* denseQ; const void* denseK; const void* denseV; void* denseO;   // fp16
};

// Matrix products of the projected forward (mfma_gemm.hip): C[i][j] = sum_s sum_k A_s[i][k] B_s[j][k], fp16, K-contiguous.
struct GemmSeg { const half_t* A; const half_t* B; int32_t lda, ldb, K, pad; };
struct GemmProblem { half_t* C; int32_t ldc, m, n, seg0, nseg, pad; };

struct Ctx {
  freqattn_shape shape;
  freqattn_band_cfg cfg;
  int path;         // resolved freqattn_path
  int launch_mode;
  int exchange_fusion = 1;   // band items of single-band slices carry the exchange (section 3.6) themselves
  int slices;       // batch*heads
  int64_t N;
  int d;
  int nb = 3;       // bands: 3, or 4 with cfg.mid2_num > 0
  int64_t band_n[NBMAX] = {0, 0, 0, 0}, band_off[NBMAX] = {0, 0, 0, 0};
  int64_t nbar, nb_mid, nb_mid2 = 0;
  int m_eff[NBMAX] = {0, 0, 0, 0}, n_c[NBMAX] = {0, 0, 0, 0};
  std::string err;

  // host tables
  std::vector<int32_t> h_band_index[NBMAX];
  std::vector<int32_t> h_perm;       // flat coefficient index -> band-major row
  std::vector<int32_t> h_row_ptr, h_col_idx;
  std::vector<int32_t> h_row_ptr2, h_col_idx2;   // block list of band MID2
  std::vector<double> h_F[3];        // per-axis DCT matrices as rounded for the device, [n][n]
  std::vector<int32_t> h_alloc;      // last head_alloc seen (size heads), empty before the first forward
  bool alloc_valid = false;

  // device tables
  int32_t* d_perm = nullptr;
  int32_t* d_perm_t = nullptr;   // the same map stored [kh*W + kw][kt]: the 64..128 rows a T-axis tile looks up are adjacent (MFMA path)
  int32_t* d_row_ptr = nullptr;
  int32_t* d_col_idx = nullptr;
  int32_t* d_row_ptr2 = nullptr;
  int32_t* d_col_idx2 = nullptr;
  float* d_F32[3] = {nullptr, nullptr, nullptr};    // F  [n][n] fp32 (generic path)
  float* d_Ft32[3] = {nullptr, nullptr, nullptr};   // F^T
  half_t* d_F16[3] = {nullptr, nullptr, nullptr};   // F  fp16 (MFMA path)
  half_t* d_Ft16[3] = {nullptr, nullptr, nullptr};  // F^T fp16

  // device scratch (element type float on the generic path, fp16 on the MFMA path)
  void* specQ = nullptr; void* specK = nullptr; void* specV = nullptr; void* Y = nullptr;
  void* tmp0 = nullptr; void* tmp1 = nullptr;     // transform ping-pong, 3*slices*N*d
  void* lowQ = nullptr; void* lowK = nullptr; void* lowV = nullptr; void* lowY = nullptr;
  void* Cbuf = nullptr;
  int32_t* d_range_flag = nullptr;                // set by the scattering transform passes when a coefficient leaves the fp16 range (sticky)
  float* d_stats = nullptr;                       // router statistics [3][d] (+ partial sums of the generic kernel)
  float* d_energy_part = nullptr;                 // per-wave partial sums of the fused statistics (MFMA path)
  float* d_tot_part = nullptr;                    // per-wave partial sums of the inputs' squares (Q, K), MFMA path
  int tot_waves[3] = {0, 0, 0};                   // waves that stored sums of squares in the last W-axis pass, per statistics slot
  bool qk_on_mid_box = false;                     // the last routed transforms left Q~, K~ on the low+mid box only
  int energy_waves[6] = {0, 0, 0, 0, 0, 0};       // waves that stored band statistics in the last T-axis pass, per statistics slot
  int low_box[3] = {0, 0, 0}, mid_box[3] = {0, 0, 0};  // extent of the low / low+mid box per axis
  float* h_stats = nullptr;                       // pinned mirror

  // per-forward lists (device + pinned host mirror)
  int32_t* d_lists = nullptr; int32_t* h_lists = nullptr; size_t lists_bytes = 0;
  // layout inside lists (int32 units)
  size_t off_masks = 0;               // [slices] band mask per slice
  size_t off_list[NBMAX] = {0, 0, 0, 0};     // [slices] slices with band l active
  int n_list[NBMAX] = {0, 0, 0, 0};
  size_t off_cls[4] = {0, 0, 0, 0};   // [slices] slices by class: 0 low only, 1 mid (no high, no second mid band), 2 high or second mid band, 3 nothing active
  int n_cls[4] = {0, 0, 0, 0};
  size_t off_nonhigh = 0;             // [slices] classes 0, 1 and 3 together (every slice that does not run the high band)
  int n_nonhigh = 0;
  size_t off_fix = 0;                 // [slices] routed forward: slices whose Q~/K~ have to be completed after routing
  int predict_alloc = 1;              // routed forward: transform Q/K of the last allocation's high slices in full at once
  std::vector<char> qk_full;          // routed forward: slices whose Q~/K~ (and V~) the first phase computed on the whole grid
  // V~ on the low+mid box only for slices that do not run the high band (MFMA path): their high-band summary tokens
  // come from the untransformed V through the weights d_wsum (mfma_vsum.hip)
  bool v_box_ok = false;              // the context can do it: summary weights built, or no summaries configured
  uint16_t* d_wsum = nullptr;         // bf16 [N/64][64][64]
  float* d_vsum_part = nullptr;       // [slices][vsum_parts][d][64] partial sums
  float* d_pool_part = nullptr;       // [slices][3][128][d]: partial sums of the pooling when chunks are cut into row ranges (m < 64)
  int vsum_nsplit = 0;
  std::vector<char> v_full;           // per slice: the current forward computed V~ on the whole grid
  size_t off_items = 0;               // AttnItem array (fused order: all branches), then exchange items
  int n_items_branch = 0;             // low+mid+high items in cost order
  int n_items_kind[3] = {0, 0, 0};    // per-branch sub-lists follow at off_items_kind
  size_t off_items_kind[3] = {0, 0, 0};
  size_t off_items_xchg = 0; int n_items_xchg = 0;
  size_t off_items_dense = 0; int n_items_dense = 0;
  size_t cap_items_kind = 0, cap_items_xchg = 0;   // AttnItem capacity of each branch / fused region and of the exchange / dense regions
  int attn_rows = 0;                  // query rows per attention item on the MFMA path
  int num_cu = 256;

  // stage timing
  bool timing = false;
  static const int MAX_STAGES = 16;
  static const int MAX_TIMED = 64;                // forwards whose events are kept (ring)
  hipEvent_t ev[MAX_TIMED][MAX_STAGES + 1];
  const char* stage_name[MAX_STAGES];
  int n_stages = 0;                               // stages of the last timed forward
  int64_t timed_steps = 0;                        // timed forwards since timing was switched on
  bool ev_created = false;

  // Projected forward (freqattn_forward_projected): buffers allocated at its first call for a model width
  int proj_d_model = 0;
  void* projX = nullptr; void* projZ = nullptr;           // X~ and the projected spectral output, [batch][N][d_model] fp16, band-major rows
  half_t* projWq = nullptr; half_t* projWk = nullptr; half_t* projWv = nullptr;   // [heads*d][d_model]: W^T, K-contiguous
  half_t* projWo = nullptr;                               // [d_model][heads*d]: W_O^T
  // Pass-through folding: on a band a head does not run, its V~ only feeds the output projection and the summary
  // tokens; both are taken from X~ directly (X~ (W_V,h W_O,h) summed over the passing heads; pooled X~ times W_V,h)
  bool proj_fold = false;                                 // this call's tables use the folding (decided per call)
  half_t* projWvN = nullptr;                              // [d_model][heads*d]: W_V as given, fp16
  half_t* projM = nullptr;                                // [3][d_model][d_model]: (sum over passing heads of W_V,h W_O,h)^T per band
  half_t* projPool = nullptr;                             // [batch][3][m][d_model]: chunk means of X~
  half_t* projCtmp = nullptr;                             // [slices][3][m][d]: the same projected with every head's W_V
  int32_t* proj_ones = nullptr;                           // [batch] band masks "every band from the first source" of the wide inverse
  GemmProblem* d_gemm_prob = nullptr; GemmProblem* h_gemm_prob = nullptr;   // device table + pinned mirror
  GemmSeg* d_gemm_seg = nullptr; GemmSeg* h_gemm_seg = nullptr;
  int gemm_cap_prob = 0, gemm_cap_seg = 0;
  struct GemmGroup { int first, per, m, n, stage; };       // one launch: problems [first, first + per) of equal m, n and A rows
  std::vector<GemmGroup> gemm_groups;                     // stage 0: Q~/K~ and V~ projections, stage 1: output projection
  bool gemm_tables_valid = false;                         // built for the current allocation (h_alloc)

  int64_t dev_bytes = 0;
  uint64_t uid = 0;                 // distinct for every context of the process
  // A context whose device memory is carved out of a caller-provided arena instead of hipMalloc (static scratch)
  char* arena_base = nullptr; size_t arena_cap = 0, arena_need = 0;
};

// ---- host tables (tables.cpp) --------------------------------------------------------------------------------
void build_dct_matrix(int n, std::vector<double>& F);  // [n][n], row = frequency
void build_haar_matrix(int n, std::vector<double>& F); // [n][n], row = scale (coarse to fine), n a power of two
void build_bands(Ctx& c);
void build_mid_blocks(Ctx& c);   // both block-sparse bands
void build_summary_weights(const Ctx& c, int band, std::vector<float>& out);   // [m_eff[band]][N]
void pack_vsum_weights(const std::vector<float>& w, int m, int64_t N, std::vector<uint16_t>& out);  // bf16 [N/64][64][64], see mfma_vsum.hip

// ---- generic fp32 kernels (generic_kernels.hip) -----------------------------------------------------------------
struct AxisPassArgs {
  const void* in; void* out;
  const float* M;           // [n_out][n]: out[k] = sum_j M[k][j] in[j]
  int n, n_out;
  int64_t inner, outer;     // element index ((s*n + j)*inner + i), s in [0, nslab), slab s belongs to slice s/outer
  int64_t nslab;
  const int32_t* perm_in;   // when set (axis W only, inner == d): input row of token (s%outer)*n + j is perm[token]
  const int32_t* perm_out;  // same for output rows
  int64_t Ntok;
  // input source selection per band for the first inverse pass (perm_in set): rows of band l of slice hb come from
  // `in` when bit l of masks[hb] is set, else from `in_alt`.
  const void* in_alt; const int32_t* masks; int32_t band_off1, band_off2, band_off3;   // first rows of bands 1, 2, 3 (band_off3 = Ntok without a fourth band)
  int in_kind, out_kind;    // 0 float, 1 bf16, 2 fp16
  int slice_mod;            // number of slices the masks array covers (slab slice index is taken modulo this)
};
hipError_t launch_generic_axis_pass(const AxisPassArgs& a, hipStream_t st);

struct GenericAttnArgs {
  const float* Q; const float* K; const float* V; float* O;
  const int32_t* slice_list; int n_slices;
  int64_t slice_stride;     // elements between slices for Q/K/V/O
  int64_t kv_slice_stride;  // elements between slices for K/V (differs from Q for the exchange)
  int nq, nk, d;
  int mode;                 // 0 dense, 1 block list, 2 window
  const int32_t* row_ptr; const int32_t* col_idx; int block; int window;
  int residual;             // O = Q + attention (exchange)
  float scale;
};
hipError_t launch_generic_attn(const GenericAttnArgs& a, hipStream_t st);

hipError_t launch_pool_low(const void* spec, void* low, const int32_t* slice_list, int n_slices, int64_t N, int d,
                           int64_t n_low, int64_t nbar, int c, int is_half, hipStream_t st);
hipError_t launch_expand_low(const void* lowY, void* Y, const int32_t* slice_list, int n_slices, int64_t N, int d,
                             int64_t n_low, int64_t nbar, int c, int is_half, hipStream_t st);
// Summary tokens of all bands of all slices, written into the C slots of the two other bands.
// skip_bits[l][..]: bit s set = band l of slice s is not pooled here (no active band of the slice looks at it, or - high
// band only - its V~ rows do not exist and launch_vsum supplies it).
hipError_t launch_summaries(const void* Y, const void* V, void* C, const int32_t* masks, int slices, int64_t N, int d,
                            int nb, const int64_t band_off[NBMAX], const int64_t band_n[NBMAX], const int m_eff[NBMAX], int m2, int is_half,
                            const uint64_t* skip_bits /*[NBMAX][4] or NULL*/, float* split_part /*[slices][nb][128][d] or NULL*/, hipStream_t st);
// High-band summary tokens of the slices in `sel` (bit set, nsel of them) from the untransformed bf16 V.
hipError_t launch_vsum(const void* V, const void* Wsum, float* part, void* C, const uint64_t sel[4], int nsel, int64_t N,
                       int d, int nsplit, int64_t n_high, const int m_eff[NBMAX], int m2rows, hipStream_t st);   // (three-band contexts only)
// Projected forward: P[batch][nb][mrows][dm] = per-chunk means of the band rows of X~ [batch][N][dm] (fp16), and the
// placement of the projected pooled rows T[slices][nb][mrows][d] into the C slots of the bands a slice passes through.
hipError_t launch_pool_wide(const void* X, void* P, int batch, int64_t N, int dm, int nb, const int64_t band_off[NBMAX],
                            const int64_t band_n[NBMAX], const int m_eff[NBMAX], int mrows, hipStream_t st);
hipError_t launch_place_summaries(const void* T, void* C, const int32_t* masks, int slices, int d, int nb, const int m_eff[NBMAX],
                                  int mrows, int m2rows, hipStream_t st);
// Router statistics: per band and channel, sum of squares over slices and the three spectral buffers.
hipError_t launch_band_energy(const void* sq, const void* sk, const void* sv, float* stats /*[3][d], zeroed inside*/,
                              int slices, int64_t N, int d, const int64_t band_off[3], const int64_t band_n[3],
                              int is_half, hipStream_t st);
hipError_t launch_fill_zero(float* p, int64_t n, hipStream_t st);
hipError_t launch_probe_copy(const void* in, void* out, int64_t bytes, int num_cu, hipStream_t st);
hipError_t launch_probe_mfma(float* out, int blocks, int iters, hipStream_t st);
// out[slice] = in[slice] for the listed slices (slice_bytes each, a multiple of 16).
// out[i] = in[i] converted bf16 -> fp16 (to_bf16 = 0) or fp16 -> bf16 (round to nearest even), n elements, n % 8 == 0.
hipError_t launch_convert_16(const void* in, void* out, int64_t n, int to_bf16, hipStream_t st);
hipError_t launch_copy_slices(const void* in, void* out, const int32_t* slice_list, int n_slices, int64_t slice_bytes,
                              hipStream_t st);
struct EnergyWaves { int en[6]; int tot[3]; };   // waves whose slots hold this forward's partial sums, per statistics slot
hipError_t launch_energy_reduce(const float* energy_part /*[6][DCT_MAX_WAVES][3][64]: Q, K, V (box), Q, K, V (whole grid)*/,
                                const float* tot_part /*[3][DCT_MAX_WAVES][64] or NULL*/, float* stats /*[3][d] + 3*d*64 floats of scratch*/, int d,
                                const EnergyWaves& nw, hipStream_t st);

// ---- MFMA kernels (mfma_dct.hip, mfma_attn.hip) -------------------------------------------------------------------
struct DctPassArgs {
  const void* in; void* out;
  const half_t* M;          // fp16, row stride ldm: out[k] = sum_{j < n} M[k*ldm + j] in[j], k < n_out
  int n, n_out, ldm;        // rows contracted (multiple of 16, <= 128), rows produced (<= 128)
  // Slices of the caller's tensors: with slice_list set, slice sl of this launch is slice_list[sl] of q/k/v/out, of the
  // band-major buffers and of masks; list_in / list_out make the regular-layout input / output use it too
  // (element offset slice*slice_elems + slab_in_slice*rows*inner), otherwise those are compact scratch.
  const int32_t* slice_list; int list_in, list_out; int64_t slice_elems;
  int delta;                // gather side: read (in - in_alt) on active bands and zero elsewhere instead of selecting
  const void* resid;        // bf16, addressed like out: out = resid + result (the sum is formed in fp32)
  float* tot_part;          // [global wave][64]: sum of squares of the input per column (pass with inner == d only)
  int64_t inner, outer, nslab;
  // Band-major side (section 3.3): with perm_in / perm_out set, row j (k) of the tile at slab s = slice*outer + o and
  // first column col0 is the band-major row perm[j*perm_k + o*perm_o + col0/d] of slice `slice`.
  const int32_t* perm_in; const int32_t* perm_out; int64_t Ntok, perm_k, perm_o;
  int32_t perm_scale;       // 0/1: index = k*perm_k + tile index; otherwise k*perm_k + tile index*perm_scale (transposed table)
  const void* in_alt; const int32_t* masks; int32_t band_off1, band_off2, band_off3;
  int in_bf16, out_bf16;    // element type of in / out: bf16 when set, else fp16
  int d;
  // Swapped scratch layout: with out_swap (in_swap) set, slab s = a*sw + b writes (reads) row k at
  // (((a*n + k)*sw_total) + b + sw_off)*inner instead of (s*n + k)*inner, i.e. the slab index b becomes the inner of the
  // two row indices.  The H-axis pass uses it to leave [h][t] order behind so that the T-axis pass finds its rows
  // W*d elements apart instead of H*W*d.
  int in_swap, out_swap, sw, sw_total, sw_off;
  // Router statistics fused into the forward pass that scatters into the band-major buffer (perm_out set): every
  // wave adds the squares of its fp32 results per band and column to energy_part[global wave][3][64].  With (u, v) the
  // coordinates of the tile on the two axes the pass does not transform (flat index = u*en_div + v), rows [0, t1) are
  // low, [t1, t2) mid and the rest high, t1 = low_a if u < low_u and v < low_v else 0, t2 likewise from the mid box.
  float* energy_part;
  // Scatter passes (perm_out set): a lane whose result leaves the fp16 range (or is not finite) stores 1 here.
  int32_t* range_flag;
  int en_omul, en_div, low_u, low_v, low_a, mid_u, mid_v, mid_a;  // flat index of the tile = o*en_omul + col0/d
};
#define DCT_MAX_WAVES 65536   // upper bound of waves in one launch of the DCT pass (sizes energy_part)
hipError_t launch_mfma_dct_pass(const DctPassArgs& a, int num_cu, hipStream_t st, int* waves_out = nullptr);
bool mfma_dct_supported(int n_in, int n_out);
hipError_t launch_gemm_nt(const GemmProblem* d_probs, const GemmSeg* d_segs, int per, int m, int n, hipStream_t st);
hipError_t launch_transpose_bf16_to_f16(const void* in /*[R][Cc] bf16*/, void* out /*[Cc][R] fp16*/, int R, int Cc, hipStream_t st);
hipError_t launch_mfma_attn(const AttnParams& p, const AttnItem* items, int n_items, int rows_per_item, int num_cu,
                            hipStream_t st);

}  // namespace fa
