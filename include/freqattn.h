/*
 * freqattn -- FreqFormer's per-head frequency-domain heterogeneous attention on one AMD Instinct MI355X (gfx950).
 *
 * The library computes, for every (batch, head) independently (paper section 3.1):
 *   section 3.2  X~ = F(X) for X in {Q, K, V}, F = F_t (x) F_h (x) F_w, orthonormal DCT-II per token-grid axis
 *   section 3.3  split of the coefficient grid into low / mid / high bands, compression of the low band
 *   section 3.4  dense attention on the compressed low band, block-sparse attention on the mid band,
 *                sliding-window attention on the high band (in band order = ascending flat coefficient index)
 *   section 3.6  m summary tokens per band, every active band attends to the other bands' summaries (residual)
 *   section 3.7  scatter of the bands back to the grid (disjoint supports) and inverse transform
 * and, as a stand-in for the router of section 3.5, a fixed or small-MLP head allocator.
 *
 * All entry points are plain C.  Pointers are marked HOST or DEVICE.  Nothing here allocates on behalf of the
 * caller except freqattn_create (tables and scratch, owned by the context, released by freqattn_destroy).
 * Errors are returned as codes; freqattn_last_error gives the text of the last failure on a context.
 * A context must be used from one host thread at a time and with one stream at a time.
 *
 * Environment switches (diagnostics and A/B runs; results agree within rounding either way):
 *   FREQATTN_V_BOX=0|1     read at freqattn_create: never / always compute V~ of slices without the high band on the
 *                          low+mid box only (default: from 64K tokens on; see freqattn_get_v_box)
 *   FREQATTN_DCT_OCC=n     read at the first transform launch of each pass shape: resident workgroups per compute unit
 *                          of the transform passes (default: what 160 KB of LDS allow, at most 4)
 *   FREQATTN_DCT_TPW=n     read at the first transform launch of each pass shape: tiles per wave that size the grids of
 *                          the transform passes (default 2; 0 = a resident grid of FREQATTN_DCT_OCC workgroups per unit)
 *   FREQATTN_DCT_TPW_PERM=n   the same for the passes that scatter into / gather from band-major rows (default: as above)
 *   FREQATTN_DCT_TPW_STATS=n  the same for the passes that add up router statistics (default 16)
 *   FREQATTN_DCT_WGS=n, FREQATTN_DCT_WGS_128=n   read at the first launch of each pass shape: most workgroups of a transform
 *                          pass per compute unit, for passes over fewer than 128 rows / over 128 rows (0 = whatever fits;
 *                          defaults 0 and 2)
 *   FREQATTN_GEMM_WIDE=0|1  read at the first product launch of freqattn_forward_projected: 0 keeps every product on the
 *                          128 x 128-tile kernel (default 1: 256 x 256 tiles where a launch has that many rows and columns)
 */
#ifndef FREQATTN_H
#define FREQATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct freqattn_ctx freqattn_ctx; /* opaque, library-owned */

typedef enum {
  FREQATTN_OK = 0,
  FREQATTN_EINVAL = 1,       /* bad argument; nothing was launched */
  FREQATTN_ENOMEM = 2,       /* host or device allocation failed in freqattn_create */
  FREQATTN_EHIP = 3,         /* a HIP runtime call failed */
  FREQATTN_EUNSUPPORTED = 4, /* valid request that this build has no kernel for */
  FREQATTN_ERANGE = 5        /* non-finite values met: inputs outside the range contract of freqattn_forward */
} freqattn_status;

typedef enum { FREQATTN_F32 = 0, FREQATTN_BF16 = 1 } freqattn_dtype;

/* Problem shape (section 3.1): q, k, v, out are [batch, heads, N, head_dim] with N = T*H*W and token index
 * n = (t*H + h)*W + w; head_dim is contiguous.  dtype is the type of q, k, v and out. */
typedef struct {
  int32_t batch, heads, head_dim, T, H, W;
  int32_t dtype; /* freqattn_dtype */
} freqattn_shape;

/* Band operators (sections 3.3, 3.4, 3.6).  Band edges are rationals so that membership is decided with integer
 * compares: a coefficient (kt, kh, kw) is in the low band iff k*low_den < low_num*n on all three axes, in low or mid
 * iff the same holds with (mid_num, mid_den), and in the high band otherwise. */
typedef struct {
  int32_t low_num, low_den, mid_num, mid_den;
  int32_t low_compress; /* c >= 1: c consecutive low-band tokens are averaged into one (section 3.3 uses 4)          */
  int32_t mid_block;    /* B: block edge of the mid-band pattern                                                   */
  int32_t mid_diag;     /* query block I sees key block J if |I-J| <= mid_diag ...                                  */
  int32_t mid_stride;   /* ... or (I-J) mod mid_stride == 0 ...                                                     */
  int32_t mid_block0;   /* ... or (mid_block0 != 0 and J == 0)                                                      */
  int32_t high_window;  /* w_h: query i sees keys i-w_h .. i+w_h of the high band (clipped, two-sided)              */
  int32_t n_summary;    /* m summary tokens per band; 0 switches the cross-band exchange off                        */
  float softmax_scale;  /* <= 0 selects 1/sqrt(head_dim)                                                            */
  int32_t transform;    /* freqattn_transform: the 1-D transform applied along each grid axis (section 3.2)         */
  int32_t mid2_num, mid2_den; /* four bands (the L = 4 of section 8's ablation list) when mid2_num > 0: a third edge,
                           mid <= mid2 <= 1.  The paper names no fourth operator; here the coefficients between the
                           mid edge and this edge form a second block-sparse band (band 3, mask bit 8: same block
                           pattern parameters, inside its own band order) and the high band is what lies outside.
                           mid2_num <= 0: three bands.                                                               */
} freqattn_band_cfg;

/* Per-axis transform of section 3.2: the reference design's orthonormal DCT-II, or the orthonormal Haar wavelet (the
 * alternative the section names; needs T, H, W to be powers of two).  Haar rows run from coarse to fine - row 0 the
 * mean, row 2^j + i the level-j wavelet at position i - and the band edges cut the row index like a frequency. */
typedef enum { FREQATTN_TRANSFORM_DCT = 0, FREQATTN_TRANSFORM_HAAR = 1 } freqattn_transform;

/* How the three band branches are launched (paper section 6.2: one launch for all branches vs one per branch). */
typedef enum { FREQATTN_LAUNCH_FUSED = 0, FREQATTN_LAUNCH_SEPARATE = 1 } freqattn_launch_mode;
/* Which kernels run: AUTO picks the MFMA kernels when dtype is BF16 and the shape allows them (T, H, W multiples
 * of 16 and at most 128, head_dim 64 or 128, mid_block a multiple of 64), otherwise the generic fp32 kernels. */
typedef enum {
  FREQATTN_PATH_AUTO = 0,
  FREQATTN_PATH_GENERIC = 1,
  FREQATTN_PATH_MFMA = 2,
  FREQATTN_PATH_TABLES_ONLY = 3 /* host tables only: no device is touched, only the introspection calls work */
} freqattn_path;

/* Builds the per-axis DCT matrices, band index lists, block list of the mid band and summary chunk bounds (host,
 * then uploaded) and allocates all device scratch on the current HIP device.  `path` is a freqattn_path.
 * Band count (the L of the ablation list in section 8): three bands is the reference design; mid edge == low edge leaves
 * the mid band empty, i.e. two bands (compressed dense low band, windowed high band); mid edge == 1 leaves the high
 * band empty (low + block-sparse rest); mid2_num > 0 adds a second block-sparse band between the mid band and the high
 * band (four bands: band indices and mask bits 0 low, 1 mid, 2 high, 3 second mid band).  Four-band contexts take
 * freqattn_forward, freqattn_forward_static, freqattn_forward_projected and the introspection calls; the router entry
 * points (section 3.5 is written for three bands) return FREQATTN_EUNSUPPORTED on them.
 * Returns EINVAL for non-positive dimensions, edges not satisfying 0 < low <= mid (<= mid2) <= 1, low_compress < 1,
 * mid_block < 1, mid_stride < 1, mid_diag < 0, high_window < 0, n_summary < 0, unknown dtype or NULL pointers;
 * EUNSUPPORTED if FREQATTN_PATH_MFMA is forced on a shape it cannot run; ENOMEM / EHIP on allocation failure. */
freqattn_status freqattn_create(const freqattn_shape* shape /*HOST*/, const freqattn_band_cfg* cfg /*HOST*/,
                                int32_t path, freqattn_ctx** out_ctx /*HOST*/);

/* Whole hot path (sections 3.2-3.7) for all batches and heads.
 *   q, k, v   DEVICE, contiguous [batch, heads, N, head_dim] of shape.dtype, read only
 *   band_cfg  HOST; must equal the configuration given to freqattn_create in every field except softmax_scale
 *   head_alloc HOST [heads]; bit 0 / 1 / 2 of entry h switch the low / mid / high operator of head h on (bit 3 the second
 *             mid band of a four-band context).  A band whose bit is clear passes V~ through unchanged on that band
 *             (it still contributes summary tokens).
 *   out       DEVICE, same shape and type as q; must not overlap q, k, v
 *   stream    hipStream_t (NULL = default stream)
 * Range contract of BF16 contexts on the matrix-core path: spectral coefficients are kept in fp16, and an orthonormal
 * transform can concentrate sqrt(N) * max|x| in one coefficient (the mean of a channel lands in one place), so the
 * inputs must satisfy sqrt(N) * max|x| < 65504 (|x| < 64 at 2^20 tokens).  A violation is detected on the device -
 * freqattn_check_range reports it, freqattn_forward_routed and freqattn_route_mlp return FREQATTN_ERANGE by themselves -
 * and the output of such a forward is not defined.  FREQATTN_F32 contexts and FREQATTN_PATH_GENERIC have no such limit.
 * Asynchronous: work is enqueued on `stream` and the call returns.  The one exception is a call whose head_alloc
 * differs from the previous call's on this context: it first waits for `stream` so that the work lists of earlier
 * calls are no longer in use.  Allocates nothing.  To capture the call into a HIP graph, run it once eagerly with the
 * same head_alloc first: the first launch of a kernel variant reads the environment switches and sets its launch
 * attributes, and a changed head_alloc waits for the stream - neither belongs under capture.  EINVAL: NULL pointer,
 * head_alloc entry outside 0..7 (0..15 on a four-band context), band_cfg mismatch.  EHIP: a launch failed. */
freqattn_status freqattn_forward(freqattn_ctx* ctx, const void* q, const void* k, const void* v,
                                 const freqattn_band_cfg* band_cfg, const int32_t* head_alloc, void* out, void* stream);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): freqattn_forward with every device buffer the library needs - transform matrices, band and block
 * tables, spectral scratch, work lists - laid out inside one static device array of 128 MiB (each GPU the library runs
 * on holds its copy until the process ends).  Calls no hipMalloc, hipFree, hipHostMalloc or event creation.  `ctx` may be
 * any context, including a FREQATTN_PATH_TABLES_ONLY one, whose freqattn_create touches no device either; a
 * tables-only context runs on the path FREQATTN_PATH_AUTO would pick.  Arguments, results and error codes as in
 * freqattn_forward, plus FREQATTN_ENOMEM when the shape needs more than the array holds (the message names the bytes).
 * The first call for a context (and the first after a call for another context on the same GPU) waits for `stream`,
 * copies the tables into the array through `stream` and waits again; later calls for the same context only launch
 * kernels (and, when head_alloc changes, wait for `stream` and upload the new work lists like freqattn_forward).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU - different streams or host
 * threads - race, and stage timing and freqattn_read_spectral do not apply to these calls. */
freqattn_status freqattn_forward_static(freqattn_ctx* ctx, const void* q, const void* k, const void* v,
                                        const freqattn_band_cfg* band_cfg, const int32_t* head_alloc, void* out,
                                        void* stream);

/* Releases everything the context owns.  freqattn_destroy(NULL) is a no-op.  The caller must have synchronised. */
void freqattn_destroy(freqattn_ctx* ctx);

/* Text of the last error on this context (or of the last failed freqattn_create when ctx is NULL). Never NULL. */
const char* freqattn_last_error(const freqattn_ctx* ctx);

/* FREQATTN_LAUNCH_FUSED (default): low, mid and high work items run in one persistent launch (section 6.2).
 * FREQATTN_LAUNCH_SEPARATE: one launch per branch (the unfused comparison of section 6.6). */
freqattn_status freqattn_set_launch_mode(freqattn_ctx* ctx, int32_t mode);
/* Cross-band exchange (section 3.6) inside the band items (default, enabled = 1): a slice that runs a single band gets
 * its summary tokens from the passed-through V~ of the other bands, which exist before the band operators run, so the
 * item that computes a tile of the band's output goes on to attend to them and adds the residual without the output
 * leaving the registers; slices that run several bands use the separate exchange launch.  enabled = 0: the separate
 * launch for every slice.  Results are bit-identical either way.  MFMA path; ignored on the generic path. */
freqattn_status freqattn_set_exchange_fusion(freqattn_ctx* ctx, int32_t enabled);
/* Returns the path the context resolved to (FREQATTN_PATH_GENERIC or FREQATTN_PATH_MFMA). */
int32_t freqattn_get_path(const freqattn_ctx* ctx);
/* 1 when the context computes V~ of a slice that does not run the high band on the low+mid box only (MFMA path, grids
 * of 64K tokens and more unless FREQATTN_V_BOX says otherwise; see freqattn_summary_weights), else 0. */
int32_t freqattn_get_v_box(const freqattn_ctx* ctx);

/* ---- introspection of the integer tables (section 3.3 band lists, section 3.4.2 block pattern) ---------------- */
/* n[l] = number of coefficients in band l (0 low, 1 mid, 2 high, 3 second mid band: 0 on a three-band context); HOST
 * out, four entries. */
freqattn_status freqattn_band_sizes(const freqattn_ctx* ctx, int64_t n[4]);
/* Flat coefficient indices (kt*H + kh)*W + kw of band `band`, ascending; host_out HOST [n[band]]. */
freqattn_status freqattn_band_index(const freqattn_ctx* ctx, int32_t band, int32_t* host_out);
/* Block list of the mid band in CSR form, columns ascending in a row.  *nnz is always written; row_ptr (HOST
 * [nb+1], nb = ceil(n_mid / mid_block)) and col_idx (HOST [nnz]) are filled when not NULL. */
freqattn_status freqattn_mid_blocks(const freqattn_ctx* ctx, int32_t* row_ptr, int32_t* col_idx, int64_t* nnz);
/* The same for the second mid band of a four-band context (nb = ceil(n[3] / mid_block); nnz = 0 otherwise). */
freqattn_status freqattn_mid2_blocks(const freqattn_ctx* ctx, int32_t* row_ptr, int32_t* col_idx, int64_t* nnz);
/* Section 3.6 with U = I, read through the transform's linearity: summary token u of band `band` of a tensor whose
 * coefficients pass through unchanged is (1 / |chunk u|) * sum_n w[u][n] x[n], with w[u][n] the sum of the transform's
 * rows of chunk u (band rows [floor(u n_l / m), floor((u+1) n_l / m)), m = min(n_summary, n_l)).  host_out HOST
 * [m][T*H*W], token order (t*H + h)*W + w.  The MFMA path sums the high band's summaries of slices that do not run the
 * high band with these weights, from the untransformed V.  Host only; works on tables-only contexts. */
freqattn_status freqattn_summary_weights(const freqattn_ctx* ctx, int32_t band, float* host_out);
/* Per-axis transform matrix as used on the device, widened to double: axis 0/1/2 = T/H/W, HOST out [n*n] row-major
 * (row = frequency for the DCT, scale for the Haar transform; the entry point keeps its name for both). */
freqattn_status freqattn_dct_matrix(const freqattn_ctx* ctx, int32_t axis, double* host_out);

/* ---- intermediate results of the last forward, for stage-wise checks ------------------------------------------
 * Copies one band of one (batch*heads + head) slice of a spectral buffer to HOST as float [n[band], head_dim],
 * after synchronising `stream`.  which: 0 = Q~, 1 = K~, 2 = V~ (section 3.2/3.3, band-major),
 * 3 = band outputs after the exchange, Y^ (section 3.6).  Rows follow freqattn_band_index.  Q~ and K~ of a band
 * that is inactive for the slice are not defined (they are not computed when not needed). */
freqattn_status freqattn_read_spectral(freqattn_ctx* ctx, int32_t which, int32_t slice, int32_t band, float* host_out,
                                       void* stream);

/* ---- head allocation (section 3.5 stand-in) -------------------------------------------------------------------- */
/* Fixed allocation: the first n_low heads get mask 1, the next n_mid mask 2, the last n_high mask 4.  HOST out. */
freqattn_status freqattn_route_fixed(int32_t heads, int32_t n_low, int32_t n_mid, int32_t n_high, int32_t* head_alloc);
/* Router: band statistics g (per band, 64 channel groups: log(1e-6 + mean squared coefficient over batch, heads,
 * band and Q~/K~/V~), centred by the mean of the 192 values), sinusoidal timestep embedding of width 64, two-layer ReLU
 * MLP with the given weights (HOST float: w1 [256, hidden] row-major, b1 [hidden], w2 [hidden, 3], b2 [3]), the
 * prior 1.5*(2t-1)*(+1, 0, -1) on the logits, softmax -> pi[3]; heads per band = 1 + largest-remainder share of
 * (heads-3) (plain largest remainder if heads < 3), handed out contiguously low, mid, high.
 * q, k, v DEVICE as in freqattn_forward.  Synchronous: transforms Q, K, V on `stream`, waits, then runs the MLP on
 * the host.  head_alloc HOST [heads] and pi HOST [3] are outputs; stats_out HOST [192] may be NULL. */
freqattn_status freqattn_route_mlp(freqattn_ctx* ctx, const void* q, const void* k, const void* v, float t,
                                   int32_t hidden, const float* w1, const float* b1, const float* w2, const float* b2,
                                   int32_t* head_alloc, float pi[3], float* stats_out, void* stream);

/* The path with the projections of sections 3.1 and 3.7 folded around it: Q = X W_Q, K = X W_K, V = X W_V per head, the
 * per-head path, then concat(heads) W_O.  The transform acts on the token axes and the projections on channels, so they
 * commute: X is transformed once instead of Q, K and V, the projections run on spectral rows (Q~, K~ and V~ only on
 * the rows of the bands a head runs), W_O is applied to the band outputs and one inverse transform of model width
 * follows.  On a band a head passes through, its V~ only reaches the output projection and the summary tokens: the
 * first as X~ times the sum over the passing heads of W_V,h W_O,h (one more K segment of the band's output product), the
 * second as chunk means of X~ rows times W_V,h.  (With more than 256 slices, or FREQATTN_PROJ_FOLD=0 - read at every
 * call - V~ is projected on every row instead.)
 *   x, out   DEVICE, contiguous [batch, N, d_model] bf16; out must not overlap x
 *   wq, wk, wv  DEVICE bf16 [d_model, heads * head_dim] row-major (head h owns columns h*head_dim ..)
 *   wo       DEVICE bf16 [heads * head_dim, d_model] row-major
 *   d_model  multiple of 64, at most heads * head_dim
 * BF16 contexts on the matrix-core path only (FREQATTN_EUNSUPPORTED otherwise).  The first call for a d_model allocates
 * the model-width buffers (two of batch * N * d_model fp16, the transposed weights, 3 * d_model^2 for the pass-through
 * weights) and synchronises; later calls allocate nothing.  Asynchronous otherwise, like freqattn_forward; the range contract stated there applies to x. */
freqattn_status freqattn_forward_projected(freqattn_ctx* ctx, const void* x, int32_t d_model, const void* wq,
                                           const void* wk, const void* wv, const void* wo,
                                           const freqattn_band_cfg* band_cfg, const int32_t* head_alloc, void* out,
                                           void* stream);

/* Load-balancing term of section 3.5: lambda * sum over the three bands of (mean over heads of pi[h][l] - 1/3)^2.
 * pi_heads HOST [heads][3] (a router with one distribution for all heads repeats it; a hard allocation passes one-hot
 * rows); *out HOST.  Host only, needs no context.  EINVAL: NULL pointer or heads < 1. */
freqattn_status freqattn_load_balance(const float* pi_heads, int32_t heads, float lambda, float* out);

/* Whole hot path with the router in the loop (sections 3.2-3.7 including 3.5): transforms Q, K, V once, reduces the
 * band statistics on the device, waits for them (the single host synchronisation of the call), evaluates the MLP
 * and the apportionment on the host exactly as freqattn_route_mlp does, then runs the band operators, the exchange
 * and the inverse transform with that allocation.  Arguments as in freqattn_forward and freqattn_route_mlp;
 * head_alloc_out HOST [heads] and pi_out HOST [3] receive the allocation that was used. */
freqattn_status freqattn_forward_routed(freqattn_ctx* ctx, const void* q, const void* k, const void* v,
                                        const freqattn_band_cfg* band_cfg, float t, int32_t hidden, const float* w1,
                                        const float* b1, const float* w2, const float* b2, void* out,
                                        int32_t* head_alloc_out, float pi_out[3], void* stream);

/* ---- dense comparison (section 4: N^2 pairs per head) ----------------------------------------------------------
 * Plain softmax(scale * Q K^T) V over all N tokens of every head with the library's own flash-style MFMA kernel;
 * BF16 contexts on the MFMA path only.  Same pointer conventions as freqattn_forward.  Asynchronous.  Uses the
 * context's scratch (fp16 copies of q, k, v and of the result): freqattn_read_spectral is meaningless afterwards until
 * the next forward. */
freqattn_status freqattn_dense_forward(freqattn_ctx* ctx, const void* q, const void* k, const void* v, void* out,
                                       void* stream);

/* ---- per-stage timing of the forward ---------------------------------------------------------------------------
 * When enabled, every forward records HIP events on its stream around each stage (the last 64 forwards are kept).
 * freqattn_stage_times waits for the last forward's events and returns, for stage s < *n_stages, its name and the
 * milliseconds between its events averaged over the kept forwards since timing was enabled.  names_out HOST
 * [max_stages] receives pointers to static strings; ms_out HOST [max_stages]. */
freqattn_status freqattn_set_stage_timing(freqattn_ctx* ctx, int32_t enabled);
freqattn_status freqattn_stage_times(freqattn_ctx* ctx, int32_t max_stages, const char** names_out, float* ms_out,
                                     int32_t* n_stages);

/* freqattn_forward_routed has to transform Q and K (and V, see freqattn_get_v_box) before it knows which heads run the
 * high band (the only ones that need them on the whole grid).  With prediction on (the default) it assumes the heads that ran the high band in
 * the context's last forward will do so again - allocations move slowly along a sampling trajectory (section 3.5) - and
 * transforms them in full at once; heads that are newly high after routing are completed then, as all of them are
 * without prediction.  Outputs do not depend on the setting (statistics agree to fp32 rounding). */
freqattn_status freqattn_set_alloc_prediction(freqattn_ctx* ctx, int32_t enabled);

/* Machine rates for the rooflines (section 6 discusses both bounds), measured with the context's own scratch on
 * `stream`; the call synchronises.  *copy_bytes_per_s HOST: bytes read plus bytes written per second by a plain
 * streaming copy of one scratch tensor into another (up to 4 GiB; meaningful when the scratch is much larger than the
 * 256 MB last-level cache).  *mfma_flops_per_s HOST: flops per second of a loop of independent
 * v_mfma_f32_32x32x16_f16 on every SIMD.  Either pointer may be NULL.  MFMA path only (FREQATTN_EUNSUPPORTED else). */
freqattn_status freqattn_measure_peaks(freqattn_ctx* ctx, double* copy_bytes_per_s, double* mfma_flops_per_s, void* stream);

/* Waits for `stream`, then reports whether a forward on this context since the last call met spectral coefficients
 * outside the fp16 range (see the range contract at freqattn_forward): *out_of_range HOST is set to 1 and
 * FREQATTN_ERANGE returned if so (the mark is cleared), else 0 and FREQATTN_OK. */
freqattn_status freqattn_check_range(freqattn_ctx* ctx, int32_t* out_of_range, void* stream);

/* Device bytes owned by the context (tables + scratch). */
int64_t freqattn_workspace_bytes(const freqattn_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* FREQATTN_H */
