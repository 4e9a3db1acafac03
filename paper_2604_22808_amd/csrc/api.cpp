// C-ABI entry points of libfreqattn and the host-side orchestration of the hot path.
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "ctx.h"

using namespace fa;

struct freqattn_ctx : public fa::Ctx {};

static thread_local std::string g_create_error;

static freqattn_status fail(freqattn_ctx* c, freqattn_status s, const std::string& msg) {
  if (c) c->err = msg; else g_create_error = msg;
  return s;
}

#define HIP_TRY(ctx, expr)                                                                         \
  do {                                                                                             \
    hipError_t e__ = (expr);                                                                       \
    if (e__ != hipSuccess)                                                                         \
      return fail(ctx, FREQATTN_EHIP, std::string(#expr) + ": " + hipGetErrorString(e__));        \
  } while (0)

// No exception may cross the C boundary: entry points whose bodies can allocate on the host run inside this.
template <class F>
static freqattn_status guarded(freqattn_ctx* c, const char* who, F&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return fail(c, FREQATTN_ENOMEM, std::string(who) + ": host allocation failed");
  } catch (...) {
    return fail(c, FREQATTN_EHIP, std::string(who) + ": unexpected exception");
  }
}

static size_t esize(const Ctx& c) { return c.path == FREQATTN_PATH_MFMA ? sizeof(half_t) : sizeof(float); }
static int io_kind(const Ctx& c) { return c.shape.dtype == FREQATTN_BF16 ? 1 : 0; }

static bool mfma_shape_ok(const freqattn_shape& s, const freqattn_band_cfg& g) {
  auto ax = [](int n) { return n % 16 == 0 && n >= 16 && n <= 128; };
  return s.dtype == FREQATTN_BF16 && ax(s.T) && ax(s.H) && ax(s.W) && (s.head_dim == 64 || s.head_dim == 128) &&
         g.mid_block % 64 == 0;
}

// Device memory of a context: hipMalloc, or - for a context that lives in a caller-provided arena (the static scratch
// of freqattn_forward_static) - the next 256-byte-aligned piece of that arena.  arena_need keeps counting past the end,
// so that a failed set-up can say how much it would have taken.
static hipError_t dev_alloc_bytes(Ctx& c, void** p, size_t bytes) {
  *p = nullptr;
  if (bytes == 0) bytes = 16;
  if (c.arena_base) {
    const size_t at = (c.arena_need + 255) & ~(size_t)255;
    c.arena_need = at + bytes;
    if (c.arena_need > c.arena_cap) return hipErrorOutOfMemory;
    *p = c.arena_base + at;
    c.dev_bytes += (int64_t)bytes;
    return hipSuccess;
  }
  hipError_t e = hipMalloc(p, bytes);
  if (e == hipSuccess) c.dev_bytes += (int64_t)bytes;
  return e;
}
template <typename T>
static hipError_t dev_alloc(Ctx& c, T** p, size_t count) {
  return dev_alloc_bytes(c, (void**)p, (count == 0 ? 1 : count) * sizeof(T));
}

static void free_all(Ctx* c) {
  if (c->arena_base) {   // nothing was allocated on the device, and the host mirrors are plain memory
    delete[] c->h_lists;
    delete[] c->h_stats;
    return;
  }
  auto F = [](void* p) { if (p) (void)hipFree(p); };
  F(c->d_perm); F(c->d_perm_t); F(c->d_row_ptr); F(c->d_col_idx); F(c->d_row_ptr2); F(c->d_col_idx2);
  for (int a = 0; a < 3; ++a) { F(c->d_F32[a]); F(c->d_Ft32[a]); F(c->d_F16[a]); F(c->d_Ft16[a]); }
  F(c->specQ); F(c->specK); F(c->specV); F(c->Y); F(c->tmp0); F(c->tmp1);
  F(c->lowQ); F(c->lowK); F(c->lowV); F(c->lowY); F(c->Cbuf); F(c->d_stats); F(c->d_range_flag); F(c->d_lists); F(c->d_energy_part);
  F(c->d_tot_part); F(c->d_wsum); F(c->d_vsum_part); F(c->d_pool_part);
  F(c->projX); F(c->projZ); F(c->projWq); F(c->projWk); F(c->projWv); F(c->projWo); F(c->proj_ones);
  F(c->projWvN); F(c->projM); F(c->projPool); F(c->projCtmp);
  F(c->d_gemm_prob); F(c->d_gemm_seg);
  if (c->h_gemm_prob) (void)hipHostFree(c->h_gemm_prob);
  if (c->h_gemm_seg) (void)hipHostFree(c->h_gemm_seg);
  if (c->h_lists) (void)hipHostFree(c->h_lists);
  if (c->h_stats) (void)hipHostFree(c->h_stats);
  if (c->ev_created)
    for (int t = 0; t < Ctx::MAX_TIMED; ++t)
      for (int i = 0; i <= Ctx::MAX_STAGES; ++i) (void)hipEventDestroy(c->ev[t][i]);
}

static int items_per_slice_max(const Ctx& c, int rows) {
  auto cd = [](int64_t a, int64_t b) { return (int)((a + b - 1) / b); };
  return cd(c.nbar, rows) + cd(c.band_n[MID], rows) + cd(c.band_n[HIGH], rows) + cd(c.band_n[MID2], rows) + 4;
}

static int keep_rows(int box, int n);

static std::atomic<uint64_t> g_next_uid{1};

// Host half of freqattn_create: argument checks, path resolution and every host table.  No device is touched.
static freqattn_status host_setup(const freqattn_shape* shape, const freqattn_band_cfg* cfg, int32_t path,
                                  freqattn_ctx** out_ctx) {
  *out_ctx = nullptr;
  const freqattn_shape& s = *shape;
  const freqattn_band_cfg& g = *cfg;
  if (s.batch < 1 || s.heads < 1 || s.head_dim < 1 || s.T < 1 || s.H < 1 || s.W < 1)
    return fail(nullptr, FREQATTN_EINVAL, "freqattn_create: dimensions must be positive");
  if (s.head_dim > 256) return fail(nullptr, FREQATTN_EUNSUPPORTED, "freqattn_create: head_dim > 256");
  if (s.dtype != FREQATTN_F32 && s.dtype != FREQATTN_BF16)
    return fail(nullptr, FREQATTN_EINVAL, "freqattn_create: unknown dtype");
  if ((int64_t)s.T * s.H * s.W > (int64_t)1 << 30 ||
      (int64_t)s.batch * s.heads * s.T * s.H * s.W > (int64_t)2000000000)
    return fail(nullptr, FREQATTN_EUNSUPPORTED, "freqattn_create: token count too large for 32-bit row indices");
  if (g.low_num < 1 || g.low_den < 1 || g.mid_num < 1 || g.mid_den < 1 ||
      !((int64_t)g.low_num * g.mid_den <= (int64_t)g.mid_num * g.low_den) || g.mid_num > g.mid_den)
    return fail(nullptr, FREQATTN_EINVAL, "freqattn_create: band edges must satisfy 0 < low <= mid <= 1");
  if (g.mid2_num > 0 && (g.mid2_den < 1 || g.mid2_num > g.mid2_den ||
                         !((int64_t)g.mid_num * g.mid2_den <= (int64_t)g.mid2_num * g.mid_den)))
    return fail(nullptr, FREQATTN_EINVAL, "freqattn_create: the third band edge must satisfy mid <= mid2 <= 1");
  if (g.low_compress < 1 || g.mid_block < 1 || g.mid_stride < 1 || g.mid_diag < 0 || g.high_window < 0 ||
      g.n_summary < 0)
    return fail(nullptr, FREQATTN_EINVAL, "freqattn_create: band operator parameter out of range");
  if (g.transform != FREQATTN_TRANSFORM_DCT && g.transform != FREQATTN_TRANSFORM_HAAR)
    return fail(nullptr, FREQATTN_EINVAL, "freqattn_create: unknown transform");
  auto pow2 = [](int n) { return (n & (n - 1)) == 0; };
  if (g.transform == FREQATTN_TRANSFORM_HAAR && !(pow2(s.T) && pow2(s.H) && pow2(s.W)))
    return fail(nullptr, FREQATTN_EINVAL, "freqattn_create: the Haar transform needs T, H and W to be powers of two");
  if (path != FREQATTN_PATH_AUTO && path != FREQATTN_PATH_GENERIC && path != FREQATTN_PATH_MFMA &&
      path != FREQATTN_PATH_TABLES_ONLY)
    return fail(nullptr, FREQATTN_EINVAL, "freqattn_create: unknown path");
  const bool mfma_ok = mfma_shape_ok(s, g);
  if (path == FREQATTN_PATH_MFMA && !mfma_ok)
    return fail(nullptr, FREQATTN_EUNSUPPORTED,
                "freqattn_create: MFMA path needs bf16, T/H/W multiples of 16 in [16,128], head_dim 64 or 128, "
                "mid_block multiple of 64");

  freqattn_ctx* c = new (std::nothrow) freqattn_ctx();
  if (!c) return fail(nullptr, FREQATTN_ENOMEM, "freqattn_create: host allocation failed");
  c->shape = s;
  c->cfg = g;
  c->path = (path == FREQATTN_PATH_AUTO) ? (mfma_ok ? FREQATTN_PATH_MFMA : FREQATTN_PATH_GENERIC) : path;
  c->launch_mode = FREQATTN_LAUNCH_FUSED;
  c->slices = s.batch * s.heads;
  c->N = (int64_t)s.T * s.H * s.W;
  c->d = s.head_dim;

  try {
    build_bands(*c);
    build_mid_blocks(*c);
    const int dims[3] = {s.T, s.H, s.W};
    for (int a = 0; a < 3; ++a) {
      if (g.transform == FREQATTN_TRANSFORM_HAAR) build_haar_matrix(dims[a], c->h_F[a]);
      else build_dct_matrix(dims[a], c->h_F[a]);
    }
  } catch (const std::bad_alloc&) {
    delete c;
    return fail(nullptr, FREQATTN_ENOMEM, "freqattn_create: host allocation failed");
  }
  c->nbar = (c->band_n[LOW] + g.low_compress - 1) / g.low_compress;
  for (int l = 0; l < NBMAX; ++l) c->m_eff[l] = c->n_c[l] = 0;
  for (int l = 0; l < c->nb; ++l) c->m_eff[l] = (int)std::min<int64_t>(g.n_summary, c->band_n[l]);
  for (int l = 0; l < c->nb; ++l) {
    c->n_c[l] = 0;
    for (int o = 0; o < c->nb; ++o)
      if (o != l) c->n_c[l] += c->m_eff[o];
  }
  if (c->path == FREQATTN_PATH_MFMA && (c->nb - 1) * g.n_summary > 1024) {
    delete c;
    return fail(nullptr, FREQATTN_EUNSUPPORTED, "freqattn_create: (bands - 1) * n_summary > 1024 on the MFMA path");
  }
  c->attn_rows = (g.mid_block % 128 == 0) ? 128 : 64;
  c->uid = g_next_uid.fetch_add(1);
  *out_ctx = c;
  return FREQATTN_OK;
}

// Device half of freqattn_create: uploads the tables and carves out the scratch, with hipMalloc or - when the context
// has an arena - from that arena, in which case the uploads go through `st` (each one waited for, the sources are
// temporaries) and nothing is allocated, neither pinned host memory nor events (such a context cannot time its stages).
// On failure the caller releases the context (free_all + delete).
static hipError_t device_setup(freqattn_ctx* c, hipStream_t st) {
  const freqattn_shape& s = c->shape;
  const freqattn_band_cfg& g = c->cfg;
  const bool mf = c->path == FREQATTN_PATH_MFMA;
  const bool arena = c->arena_base != nullptr;
  hipDeviceProp_t prop;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return hipErrorNoDevice;
  c->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

  // ---- device tables
  hipError_t e = hipSuccess;
  auto up = [&](void* dst, const void* src, size_t bytes) {
    if (e != hipSuccess || !bytes) return;
    if (arena) {
      e = hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, st);
      if (e == hipSuccess) e = hipStreamSynchronize(st);
    } else {
      e = hipMemcpy(dst, src, bytes, hipMemcpyHostToDevice);
    }
  };
  auto A = [&](hipError_t r) { if (e == hipSuccess) e = r; };
  A(dev_alloc(*c, &c->d_perm, (size_t)c->N));
  up(c->d_perm, c->h_perm.data(), (size_t)c->N * 4);
  if (mf) {   // [kh*W + kw][kt] copy for the T-axis passes of the MFMA path
    std::vector<int32_t> pt((size_t)c->N);
    const int64_t hw = (int64_t)s.H * s.W;
    for (int64_t kt = 0; kt < s.T; ++kt)
      for (int64_t r = 0; r < hw; ++r) pt[(size_t)(r * s.T + kt)] = c->h_perm[(size_t)(kt * hw + r)];
    A(dev_alloc(*c, &c->d_perm_t, (size_t)c->N));
    up(c->d_perm_t, pt.data(), (size_t)c->N * 4);
  }
  A(dev_alloc(*c, &c->d_row_ptr, c->h_row_ptr.size()));
  up(c->d_row_ptr, c->h_row_ptr.data(), c->h_row_ptr.size() * 4);
  A(dev_alloc(*c, &c->d_col_idx, c->h_col_idx.size()));
  up(c->d_col_idx, c->h_col_idx.data(), c->h_col_idx.size() * 4);
  A(dev_alloc(*c, &c->d_row_ptr2, c->h_row_ptr2.size()));
  up(c->d_row_ptr2, c->h_row_ptr2.data(), c->h_row_ptr2.size() * 4);
  A(dev_alloc(*c, &c->d_col_idx2, c->h_col_idx2.size()));
  up(c->d_col_idx2, c->h_col_idx2.data(), c->h_col_idx2.size() * 4);
  {
    const int dims[3] = {s.T, s.H, s.W};
    for (int a = 0; a < 3 && e == hipSuccess; ++a) {
      const int n = dims[a];
      std::vector<double>& F = c->h_F[a];
      if (mf) {
        std::vector<half_t> f16((size_t)n * n), ft16((size_t)n * n);
        for (int k = 0; k < n; ++k)
          for (int j = 0; j < n; ++j) {
            const half_t hv = (half_t)F[(size_t)k * n + j];
            f16[(size_t)k * n + j] = hv;
            ft16[(size_t)j * n + k] = hv;
            F[(size_t)k * n + j] = (double)hv;  // what the device really multiplies with
          }
        A(dev_alloc(*c, &c->d_F16[a], (size_t)n * n));
        up(c->d_F16[a], f16.data(), (size_t)n * n * sizeof(half_t));
        A(dev_alloc(*c, &c->d_Ft16[a], (size_t)n * n));
        up(c->d_Ft16[a], ft16.data(), (size_t)n * n * sizeof(half_t));
      } else {
        std::vector<float> f32((size_t)n * n), ft32((size_t)n * n);
        for (int k = 0; k < n; ++k)
          for (int j = 0; j < n; ++j) {
            const float fv = (float)F[(size_t)k * n + j];
            f32[(size_t)k * n + j] = fv;
            ft32[(size_t)j * n + k] = fv;
            F[(size_t)k * n + j] = (double)fv;
          }
        A(dev_alloc(*c, &c->d_F32[a], (size_t)n * n));
        up(c->d_F32[a], f32.data(), (size_t)n * n * 4);
        A(dev_alloc(*c, &c->d_Ft32[a], (size_t)n * n));
        up(c->d_Ft32[a], ft32.data(), (size_t)n * n * 4);
      }
    }
  }
  // ---- scratch
  const size_t es = esize(*c);
  const size_t slab = (size_t)c->slices * (size_t)c->N * (size_t)c->d * es;
  const size_t lowb = (size_t)c->slices * (size_t)std::max<int64_t>(c->nbar, 1) * (size_t)c->d * es;
  A(dev_alloc_bytes(*c, &c->specQ, slab));
  A(dev_alloc_bytes(*c, &c->specK, slab));
  A(dev_alloc_bytes(*c, &c->specV, slab));
  A(dev_alloc_bytes(*c, &c->Y, slab));
  A(dev_alloc_bytes(*c, &c->tmp0, slab));
  A(dev_alloc_bytes(*c, &c->tmp1, slab));
  A(dev_alloc_bytes(*c, &c->lowQ, lowb));
  A(dev_alloc_bytes(*c, &c->lowK, lowb));
  A(dev_alloc_bytes(*c, &c->lowV, lowb));
  A(dev_alloc_bytes(*c, &c->lowY, lowb));
  A(dev_alloc_bytes(*c, &c->Cbuf, (size_t)c->slices * c->nb * (c->nb - 1) * (size_t)std::max(g.n_summary, 1) * c->d * es));
  const size_t stats_floats = (size_t)3 * c->d * (1 + 64);
  A(dev_alloc(*c, &c->d_stats, stats_floats));
  A(dev_alloc(*c, &c->d_range_flag, 64));
  if (e == hipSuccess) e = launch_fill_zero((float*)c->d_range_flag, 64, st);   // (a zero float is a zero int)
  if (mf && g.n_summary > 0 && g.n_summary < 64) A(dev_alloc(*c, &c->d_pool_part, (size_t)c->slices * c->nb * 128 * c->d));
  // (partial sums of the router statistics: the routed entry points do not run on an arena context)
  if (mf && !arena) A(dev_alloc(*c, &c->d_energy_part, (size_t)6 * DCT_MAX_WAVES * 3 * 64));
  if (mf && !arena) A(dev_alloc(*c, &c->d_tot_part, (size_t)3 * DCT_MAX_WAVES * 64));
  {
    auto box = [](int64_t num, int64_t den, int n) { return (int)((num * n + den - 1) / den); };  // #k with k*den < num*n
    const int dims[3] = {s.T, s.H, s.W};
    for (int a = 0; a < 3; ++a) {
      c->low_box[a] = std::min(dims[a], box(g.low_num, g.low_den, dims[a]));
      c->mid_box[a] = std::min(dims[a], box(g.mid_num, g.mid_den, dims[a]));
    }
  }
  // Slices that do not run the high band get V~ on the low+mid box only (see mfma_vsum.hip) when that box is smaller
  // than the grid and the high band's summary tokens (at most 64) can come from the untransformed V instead.
  {
    const int dims[3] = {s.T, s.H, s.W};
    bool smaller = false;
    for (int a = 0; a < 3; ++a) smaller = smaller || keep_rows(c->mid_box[a], dims[a]) < dims[a];
    // (FREQATTN_V_BOX = 0 / 1 switches it off / on whatever the size; by default grids below 64K tokens keep the
    // whole-grid V~: the extra launches cost more there than the smaller passes save)
    const char* env = getenv("FREQATTN_V_BOX");
    const bool wanted = env ? atoi(env) != 0 : c->N >= 65536;
    // (three bands only: with a second mid band outside the box its summary tokens would need the same treatment)
    c->v_box_ok = mf && smaller && c->N % 64 == 0 && c->slices <= 256 && c->band_n[HIGH] > 0 && c->nb == 3 &&
                  (g.n_summary == 0 || c->m_eff[HIGH] <= 64) && wanted;
    if (c->v_box_ok && g.n_summary > 0 && e == hipSuccess) {
      try {
        std::vector<uint16_t> w;
        {
          std::vector<float> wf;
          build_summary_weights(*c, HIGH, wf);
          pack_vsum_weights(wf, c->m_eff[HIGH], c->N, w);
        }
        A(dev_alloc_bytes(*c, (void**)&c->d_wsum, w.size() * sizeof(uint16_t)));
        up(c->d_wsum, w.data(), w.size() * sizeof(uint16_t));
      } catch (const std::bad_alloc&) {
        e = hipErrorOutOfMemory;
      }
      // token ranges per slice: about two workgroups per CU in one launch (the kernel's LDS footprint allows two)
      c->vsum_nsplit = 2 * c->num_cu;
      A(dev_alloc(*c, &c->d_vsum_part, (size_t)(2 * c->num_cu + c->slices) * 2 * c->d * 64));
    }
    c->v_full.assign((size_t)c->slices, 1);
  }
  if (e == hipSuccess) {
    if (arena) { c->h_stats = new (std::nothrow) float[(size_t)3 * c->d + 1]; if (!c->h_stats) e = hipErrorOutOfMemory; }
    else e = hipHostMalloc((void**)&c->h_stats, (3 * c->d + 1) * sizeof(float), hipHostMallocDefault);
  }

  // ---- per-forward lists
  {
    const int rows = c->attn_rows;
    const size_t per_slice = (size_t)items_per_slice_max(*c, rows);
    const size_t xchg_per_slice = (size_t)((c->N + rows - 1) / rows + NBMAX);
    size_t ints = 0;
    c->off_masks = ints; ints += (size_t)c->slices;
    for (int l = 0; l < NBMAX; ++l) { c->off_list[l] = ints; ints += (size_t)c->slices; }
    for (int k = 0; k < 4; ++k) { c->off_cls[k] = ints; ints += (size_t)c->slices; }
    c->off_nonhigh = ints; ints += (size_t)c->slices;
    c->off_fix = ints; ints += (size_t)c->slices;
    ints = (ints + 3) & ~(size_t)3;
    c->cap_items_kind = mf ? per_slice * c->slices : 0;      // the generic kernels read no item lists
    c->cap_items_xchg = mf ? xchg_per_slice * c->slices : 0;
    c->off_items = ints; ints += 4 * c->cap_items_kind;
    for (int l = 0; l < 3; ++l) { c->off_items_kind[l] = ints; ints += 4 * c->cap_items_kind; }
    c->off_items_xchg = ints; ints += 4 * c->cap_items_xchg;
    c->off_items_dense = ints; ints += 4 * c->cap_items_xchg;
    c->lists_bytes = ints * 4;
    A(dev_alloc_bytes(*c, (void**)&c->d_lists, c->lists_bytes));
    if (e == hipSuccess) {
      if (arena) { c->h_lists = new (std::nothrow) int32_t[ints]; if (!c->h_lists) e = hipErrorOutOfMemory; }
      else e = hipHostMalloc((void**)&c->h_lists, c->lists_bytes, hipHostMallocDefault);
    }
  }
  if (e == hipSuccess && !arena) {
    bool all = true;
    for (int t = 0; t < Ctx::MAX_TIMED; ++t)
      for (int i = 0; i <= Ctx::MAX_STAGES; ++i) {
        if (e == hipSuccess) e = hipEventCreate(&c->ev[t][i]);
        if (e != hipSuccess && all) {  // destroy what exists, leave the rest untouched
          all = false;
          for (int t2 = 0; t2 <= t; ++t2)
            for (int i2 = 0; i2 <= Ctx::MAX_STAGES && (t2 < t || i2 < i); ++i2) (void)hipEventDestroy(c->ev[t2][i2]);
        }
      }
    c->ev_created = all;
  }
  return e;
}

extern "C" freqattn_status freqattn_create(const freqattn_shape* shape, const freqattn_band_cfg* cfg, int32_t path,
                                           freqattn_ctx** out_ctx) {
  if (!shape || !cfg || !out_ctx) return fail(nullptr, FREQATTN_EINVAL, "freqattn_create: NULL argument");
  freqattn_ctx* c = nullptr;
  freqattn_status fs = host_setup(shape, cfg, path, &c);
  if (fs != FREQATTN_OK || c->path == FREQATTN_PATH_TABLES_ONLY) {
    *out_ctx = c;
    return fs;
  }
  const hipError_t e = device_setup(c, nullptr);
  if (e != hipSuccess) {
    const bool oom = (e == hipErrorOutOfMemory);
    std::string msg = std::string("freqattn_create: ") + hipGetErrorString(e);
    free_all(c);
    delete c;
    (void)hipGetLastError();
    *out_ctx = nullptr;
    return fail(nullptr, oom ? FREQATTN_ENOMEM : FREQATTN_EHIP, msg);
  }
  *out_ctx = c;
  return FREQATTN_OK;
}

extern "C" void freqattn_destroy(freqattn_ctx* c) {
  if (!c) return;
  free_all(c);
  delete c;
}

extern "C" const char* freqattn_last_error(const freqattn_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

extern "C" freqattn_status freqattn_set_launch_mode(freqattn_ctx* c, int32_t mode) {
  if (!c) return FREQATTN_EINVAL;
  if (mode != FREQATTN_LAUNCH_FUSED && mode != FREQATTN_LAUNCH_SEPARATE)
    return fail(c, FREQATTN_EINVAL, "freqattn_set_launch_mode: unknown mode");
  c->launch_mode = mode;
  return FREQATTN_OK;
}
extern "C" freqattn_status freqattn_set_exchange_fusion(freqattn_ctx* c, int32_t enabled) {
  if (!c) return FREQATTN_EINVAL;
  if (c->exchange_fusion != (enabled ? 1 : 0)) {
    c->exchange_fusion = enabled ? 1 : 0;
    c->alloc_valid = false;   // the work lists carry the choice
  }
  return FREQATTN_OK;
}
extern "C" freqattn_status freqattn_set_alloc_prediction(freqattn_ctx* c, int32_t enabled) {
  if (!c) return FREQATTN_EINVAL;
  c->predict_alloc = enabled ? 1 : 0;
  return FREQATTN_OK;
}
extern "C" int32_t freqattn_get_path(const freqattn_ctx* c) { return c ? c->path : -1; }
extern "C" freqattn_status freqattn_measure_peaks(freqattn_ctx* c, double* copy_bytes_per_s, double* mfma_flops_per_s,
                                                  void* stream) {
  if (!c) return FREQATTN_EINVAL;
  if (c->path != FREQATTN_PATH_MFMA) return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_measure_peaks: MFMA path only");
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t e0, e1;
  HIP_TRY(c, hipEventCreate(&e0));
  HIP_TRY(c, hipEventCreate(&e1));
  auto timed = [&](auto&& launch, int reps, float* ms) -> hipError_t {
    hipError_t e;
    if ((e = launch()) != hipSuccess) return e;                      // warm-up
    if ((e = hipEventRecord(e0, st)) != hipSuccess) return e;
    for (int i = 0; i < reps; ++i)
      if ((e = launch()) != hipSuccess) return e;
    if ((e = hipEventRecord(e1, st)) != hipSuccess) return e;
    if ((e = hipEventSynchronize(e1)) != hipSuccess) return e;
    return hipEventElapsedTime(ms, e0, e1);
  };
  hipError_t err = hipSuccess;
  if (copy_bytes_per_s) {
    const int64_t bytes = std::min<int64_t>((int64_t)c->slices * c->N * c->d * (int64_t)sizeof(half_t), (int64_t)4 << 30) / 16 * 16;
    float ms = 0.f;
    err = timed([&] { return launch_probe_copy(c->tmp0, c->tmp1, bytes, c->num_cu, st); }, 3, &ms);
    if (err == hipSuccess) *copy_bytes_per_s = 2.0 * (double)bytes * 3 / (ms * 1e-3);
  }
  if (err == hipSuccess && mfma_flops_per_s) {
    const int blocks = c->num_cu * 2, iters = 20000;   // needs blocks*256 floats of scratch: tmp0 is far larger
    if ((int64_t)blocks * 256 * 4 > (int64_t)c->slices * c->N * c->d * (int64_t)sizeof(half_t)) err = hipErrorInvalidValue;
    float ms = 0.f;
    if (err == hipSuccess) err = timed([&] { return launch_probe_mfma((float*)c->tmp0, blocks, iters, st); }, 2, &ms);
    if (err == hipSuccess) *mfma_flops_per_s = (double)blocks * 4 * iters * 4 * 32768.0 * 2 / (ms * 1e-3);
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (err != hipSuccess) return fail(c, FREQATTN_EHIP, std::string("freqattn_measure_peaks: ") + hipGetErrorString(err));
  return FREQATTN_OK;
}

extern "C" freqattn_status freqattn_check_range(freqattn_ctx* c, int32_t* out_of_range, void* stream) {
  if (!c || !out_of_range) return FREQATTN_EINVAL;
  *out_of_range = 0;
  if (c->path == FREQATTN_PATH_TABLES_ONLY) return FREQATTN_OK;
  hipStream_t st = (hipStream_t)stream;
  int32_t flag = 0;
  HIP_TRY(c, hipStreamSynchronize(st));
  HIP_TRY(c, hipMemcpy(&flag, c->d_range_flag, sizeof(flag), hipMemcpyDeviceToHost));
  if (flag == 0) return FREQATTN_OK;
  *out_of_range = 1;
  HIP_TRY(c, launch_fill_zero((float*)c->d_range_flag, 1, st));
  HIP_TRY(c, hipStreamSynchronize(st));
  return fail(c, FREQATTN_ERANGE, "spectral coefficients left the fp16 range of the matrix-core path in a forward since the "
                                  "last check: the inputs must satisfy sqrt(N) * max|x| < 65504 (or use the fp32 path)");
}

extern "C" int64_t freqattn_workspace_bytes(const freqattn_ctx* c) { return c ? c->dev_bytes : 0; }

extern "C" freqattn_status freqattn_band_sizes(const freqattn_ctx* c, int64_t n[4]) {
  if (!c || !n) return FREQATTN_EINVAL;
  for (int l = 0; l < NBMAX; ++l) n[l] = l < c->nb ? c->band_n[l] : 0;
  return FREQATTN_OK;
}
extern "C" freqattn_status freqattn_band_index(const freqattn_ctx* c, int32_t band, int32_t* host_out) {
  if (!c || !host_out || band < 0 || band >= c->nb) return FREQATTN_EINVAL;
  std::memcpy(host_out, c->h_band_index[band].data(), c->h_band_index[band].size() * sizeof(int32_t));
  return FREQATTN_OK;
}
extern "C" int32_t freqattn_get_v_box(const freqattn_ctx* c) { return (c && c->v_box_ok) ? 1 : 0; }

extern "C" freqattn_status freqattn_summary_weights(const freqattn_ctx* c, int32_t band, float* host_out) {
  if (!c || !host_out || band < 0 || band >= c->nb) return FREQATTN_EINVAL;
  try {
    std::vector<float> w;
    build_summary_weights(*c, band, w);
    if (!w.empty()) std::memcpy(host_out, w.data(), w.size() * sizeof(float));
  } catch (const std::bad_alloc&) {
    return FREQATTN_ENOMEM;
  }
  return FREQATTN_OK;
}

extern "C" freqattn_status freqattn_mid_blocks(const freqattn_ctx* c, int32_t* row_ptr, int32_t* col_idx, int64_t* nnz) {
  if (!c || !nnz) return FREQATTN_EINVAL;
  *nnz = (int64_t)c->h_col_idx.size();
  if (row_ptr) std::memcpy(row_ptr, c->h_row_ptr.data(), c->h_row_ptr.size() * sizeof(int32_t));
  if (col_idx) std::memcpy(col_idx, c->h_col_idx.data(), c->h_col_idx.size() * sizeof(int32_t));
  return FREQATTN_OK;
}
extern "C" freqattn_status freqattn_mid2_blocks(const freqattn_ctx* c, int32_t* row_ptr, int32_t* col_idx, int64_t* nnz) {
  if (!c || !nnz) return FREQATTN_EINVAL;
  *nnz = (int64_t)c->h_col_idx2.size();
  if (row_ptr) std::memcpy(row_ptr, c->h_row_ptr2.data(), c->h_row_ptr2.size() * sizeof(int32_t));
  if (col_idx) std::memcpy(col_idx, c->h_col_idx2.data(), c->h_col_idx2.size() * sizeof(int32_t));
  return FREQATTN_OK;
}
extern "C" freqattn_status freqattn_dct_matrix(const freqattn_ctx* c, int32_t axis, double* host_out) {
  if (!c || !host_out || axis < 0 || axis > 2) return FREQATTN_EINVAL;
  std::memcpy(host_out, c->h_F[axis].data(), c->h_F[axis].size() * sizeof(double));
  return FREQATTN_OK;
}

extern "C" freqattn_status freqattn_route_fixed(int32_t heads, int32_t n_low, int32_t n_mid, int32_t n_high,
                                                int32_t* head_alloc) {
  if (!head_alloc || heads < 1 || n_low < 0 || n_mid < 0 || n_high < 0 || n_low + n_mid + n_high != heads)
    return FREQATTN_EINVAL;
  int h = 0;
  for (int i = 0; i < n_low; ++i) head_alloc[h++] = 1;
  for (int i = 0; i < n_mid; ++i) head_alloc[h++] = 2;
  for (int i = 0; i < n_high; ++i) head_alloc[h++] = 4;
  return FREQATTN_OK;
}

extern "C" freqattn_status freqattn_load_balance(const float* pi_heads, int32_t heads, float lambda, float* out) {
  if (!pi_heads || !out || heads < 1) return FREQATTN_EINVAL;
  double loss = 0.0;
  for (int l = 0; l < 3; ++l) {
    double mean = 0.0;
    for (int h = 0; h < heads; ++h) mean += (double)pi_heads[(size_t)h * 3 + l];
    mean /= heads;
    loss += (mean - 1.0 / 3.0) * (mean - 1.0 / 3.0);
  }
  *out = (float)((double)lambda * loss);
  return FREQATTN_OK;
}

// ------------------------------------------------------------------------------------------------ work lists
static bool same_cfg(const freqattn_band_cfg& a, const freqattn_band_cfg& b) {
  return a.low_num == b.low_num && a.low_den == b.low_den && a.mid_num == b.mid_num && a.mid_den == b.mid_den &&
         a.low_compress == b.low_compress && a.mid_block == b.mid_block && a.mid_diag == b.mid_diag &&
         a.mid_stride == b.mid_stride && (a.mid_block0 != 0) == (b.mid_block0 != 0) &&
         a.high_window == b.high_window && a.n_summary == b.n_summary && a.transform == b.transform &&
         std::max(a.mid2_num, 0) == std::max(b.mid2_num, 0) && (a.mid2_num <= 0 || a.mid2_den == b.mid2_den);
}

// Fills the pinned host mirror of the per-forward lists.  The item lists are only read by the MFMA attention kernel;
// the generic path gets the slice lists alone.  Nothing here allocates; every item region is written through a
// capacity check, and the function returns false (lists unusable) if a region would overflow.
static bool build_lists(Ctx& c, const int32_t* head_alloc) {
  int32_t* L = c.h_lists;
  const int heads = c.shape.heads;
  for (int l = 0; l < NBMAX; ++l) c.n_list[l] = 0;
  for (int k = 0; k < 4; ++k) c.n_cls[k] = 0;
  c.n_nonhigh = 0;
  for (int s = 0; s < c.slices; ++s) {
    const int mask = head_alloc[s % heads];
    L[c.off_masks + s] = mask;
    int eff = 0;   // bands that really run (a band without coefficients runs nothing)
    for (int l = 0; l < c.nb; ++l)
      if (((mask >> l) & 1) && c.band_n[l] > 0) eff |= 1 << l;
    // (the second mid band lies outside the low+mid box, like the high band: its slices take the whole-grid transforms)
    const int cls = (eff & (4 | 8)) ? 2 : (eff & 2) ? 1 : (eff & 1) ? 0 : 3;
    L[c.off_cls[cls] + c.n_cls[cls]++] = s;
    if (cls != 2) L[c.off_nonhigh + c.n_nonhigh++] = s;
    for (int l = 0; l < c.nb; ++l)
      if (((mask >> l) & 1) && c.band_n[l] > 0) L[c.off_list[l] + c.n_list[l]++] = s;
  }
  c.n_items_branch = 0;
  for (int k = 0; k < 3; ++k) c.n_items_kind[k] = 0;
  c.n_items_xchg = 0;
  c.n_items_dense = 0;
  if (c.path != FREQATTN_PATH_MFMA) return true;

  const int rows = c.attn_rows;
  const int KT = 64;  // key tile of the MFMA attention kernel
  bool ok = true;
  // A band item also carries the band's exchange (section 3.6) when every other band of the slice passes V~ through:
  // the summary tokens it attends to are then pooled from V~ before the band operators run (bit 16 of kind_band).
  const bool fusion = c.exchange_fusion && c.cfg.n_summary > 0 && c.slices <= 256;
  auto fused_xchg = [&](int mask, int l) -> bool {
    if (!fusion || c.n_c[l] <= 0) return false;
    int eff = 0;
    for (int o = 0; o < c.nb; ++o)
      if (((mask >> o) & 1) && c.band_n[o] > 0) eff |= 1 << o;
    return eff == (1 << l);
  };
  auto push = [&](size_t off, int& n, size_t cap, AttnItem it) {
    if ((size_t)n >= cap) { ok = false; return; }
    std::memcpy(L + off + (size_t)4 * n, &it, sizeof(AttnItem));
    ++n;
  };
  auto cd = [](int64_t a, int64_t b) { return (a + b - 1) / b; };
  const size_t cap_kind = c.cap_items_kind, cap_x = c.cap_items_xchg;
  for (int s = 0; s < c.slices; ++s) {
    const int mask = L[c.off_masks + s];
    if ((mask & 1) && c.band_n[LOW] > 0)
      for (int64_t q0 = 0; q0 < c.nbar; q0 += rows)
        push(c.off_items_kind[0], c.n_items_kind[0], cap_kind, {0 | (LOW << 8) | (fused_xchg(mask, LOW) ? 1 << 16 : 0), s, (int32_t)q0, (int32_t)cd(c.nbar, KT)});
    for (int l = MID; l < c.nb; l += MID2 - MID) {   // the block-sparse bands: mid, and the second mid band if there is one
      if (!((mask >> l) & 1) || c.band_n[l] <= 0) continue;
      // Query blocks I with the same I mod stride share all their strided key blocks (J = I mod stride): they are listed
      // together, so that workgroups running at the same time fetch those K/V tiles into their L2 once.
      const std::vector<int32_t>& row_ptr = l == MID ? c.h_row_ptr : c.h_row_ptr2;
      const int64_t tiles_per_block = std::max<int64_t>(1, c.cfg.mid_block / rows);   // items per query block
      const int64_t nblocks = (c.band_n[l] + c.cfg.mid_block - 1) / c.cfg.mid_block;
      const int64_t stride = std::min<int64_t>(c.cfg.mid_stride, nblocks);
      for (int64_t r = 0; r < stride; ++r)
        for (int64_t I = r; I < nblocks; I += stride)
          for (int64_t u = 0; u < tiles_per_block; ++u) {
            const int64_t q0 = I * c.cfg.mid_block + u * rows;
            if (q0 >= c.band_n[l]) break;
            const int nblk = row_ptr[I + 1] - row_ptr[I];
            push(c.off_items_kind[1], c.n_items_kind[1], cap_kind, {1 | (l << 8) | (fused_xchg(mask, l) ? 1 << 16 : 0), s, (int32_t)q0, (int32_t)(nblk * cd(c.cfg.mid_block, KT))});
          }
    }
    if ((mask & 4) && c.band_n[HIGH] > 0)
      for (int64_t q0 = 0; q0 < c.band_n[HIGH]; q0 += rows) {
        const int64_t k0 = std::max<int64_t>(0, q0 - c.cfg.high_window);
        const int64_t k1 = std::min<int64_t>(c.band_n[HIGH] - 1, q0 + rows - 1 + (int64_t)c.cfg.high_window);
        push(c.off_items_kind[2], c.n_items_kind[2], cap_kind, {2 | (HIGH << 8) | (fused_xchg(mask, HIGH) ? 1 << 16 : 0), s, (int32_t)q0, (int32_t)(k1 / KT - k0 / KT + 1)});
      }
    if (c.cfg.n_summary > 0)
      for (int l = 0; l < c.nb; ++l)
        if (((mask >> l) & 1) && c.band_n[l] > 0 && c.n_c[l] > 0 && !fused_xchg(mask, l))
          for (int64_t q0 = 0; q0 < c.band_n[l]; q0 += rows)
            push(c.off_items_xchg, c.n_items_xchg, cap_x, {3 | (l << 8), s, (int32_t)q0, (int32_t)cd(c.n_c[l], KT)});
  }
  // One list for the fused launch: the branches one after the other (long low and mid items first, the many short
  // window items last, which keeps the tail of the launch short), inside a branch by slice and query tile, so that
  // workgroups running at the same time work on neighbouring query tiles and share their K/V tiles in the L2.  (Sorting
  // the whole list by cost scatters the mid band's query tiles and measured 3 % slower.)
  for (int k = 0; k < 3; ++k) {
    if ((size_t)(c.n_items_branch + c.n_items_kind[k]) > cap_kind) { ok = false; break; }
    if (c.n_items_kind[k] > 0)
      std::memcpy(L + c.off_items + (size_t)4 * c.n_items_branch, L + c.off_items_kind[k], (size_t)c.n_items_kind[k] * sizeof(AttnItem));
    c.n_items_branch += c.n_items_kind[k];
  }
  // dense baseline items (do not depend on the allocation)
  for (int s = 0; s < c.slices; ++s)
    for (int64_t q0 = 0; q0 < c.N; q0 += rows) push(c.off_items_dense, c.n_items_dense, cap_x, {4, s, (int32_t)q0, (int32_t)cd(c.N, KT)});
  return ok;
}

static freqattn_status ensure_lists(freqattn_ctx* c, const int32_t* head_alloc, hipStream_t st) {
  const int heads = c->shape.heads;
  if (c->alloc_valid && std::memcmp(c->h_alloc.data(), head_alloc, heads * sizeof(int32_t)) == 0) return FREQATTN_OK;
  HIP_TRY(c, hipStreamSynchronize(st));  // earlier forwards may still read the lists
  if (!build_lists(*c, head_alloc)) {
    c->alloc_valid = false;
    return fail(c, FREQATTN_EINVAL, "work lists: item count exceeds the capacity sized at freqattn_create");
  }
  // upload what the new allocation uses: the slice lists, the used part of each item list, and the dense comparison's
  // list (independent of the allocation) the first time only
  auto up = [&](size_t off_ints, size_t n_ints) -> hipError_t {
    if (n_ints == 0) return hipSuccess;
    return hipMemcpyAsync(c->d_lists + off_ints, c->h_lists + off_ints, n_ints * sizeof(int32_t), hipMemcpyHostToDevice, st);
  };
  HIP_TRY(c, up(0, c->off_items));
  HIP_TRY(c, up(c->off_items, (size_t)4 * c->n_items_branch));
  for (int kd = 0; kd < 3; ++kd) HIP_TRY(c, up(c->off_items_kind[kd], (size_t)4 * c->n_items_kind[kd]));
  HIP_TRY(c, up(c->off_items_xchg, (size_t)4 * c->n_items_xchg));
  if (!c->alloc_valid) HIP_TRY(c, up(c->off_items_dense, (size_t)4 * c->n_items_dense));
  c->h_alloc.assign(head_alloc, head_alloc + heads);
  c->alloc_valid = true;
  c->gemm_tables_valid = false;
  return FREQATTN_OK;
}

// ------------------------------------------------------------------------------------------------ transforms
// Forward transform of one [slices, N, d] tensor into a band-major spectral buffer (sections 3.2, 3.3).
// Coefficients kept per axis when only the box [0, box) of an axis is needed: rounded up to the kernel's granularity,
// or the full axis when the rectangular pass is not available for that pair of sizes.
static int keep_rows(int box, int n) {
  const int r = std::min(n, (box + 15) / 16 * 16);
  return (r < n && mfma_dct_supported(n, r) && mfma_dct_supported(r, n)) ? r : n;
}

// MFMA path, forward, for `ns` slices (slice_list on the device, NULL = slices 0..ns-1): W axis (tmp0), H axis (tmp1,
// left in [h][t] order so that the rows of the T pass are W*d elements apart), T axis, which scatters into the
// band-major spectral buffer.  keep[] = coefficients computed per axis (T, H, W): a head that only runs the low (low
// and mid) band needs Q~ and K~ on that box only, and every pass after the first then moves a fraction of the tensor.
// energy_slot >= 0 adds up the router's band statistics in the T pass, tot_slot >= 0 the input's sum of squares in
// the W pass.
// `width` > 0 transforms a tensor of that many channels per token instead of head_dim (the projected forward transforms X,
// [batch][N][d_model], as `ns` = batch slices).
static hipError_t forward_transform_mfma(Ctx& c, const void* x, void* spec, hipStream_t st, const int32_t* slice_list,
                                         int ns, const int keep[3], int energy_slot, int tot_slot, int width = 0) {
  if (ns <= 0) return hipSuccess;
  const int T = c.shape.T, H = c.shape.H, W = c.shape.W, d = width > 0 ? width : c.d;
  const int kt = keep[0], kh = keep[1], kw = keep[2];
  hipError_t e;
  DctPassArgs a{};
  a.d = d; a.Ntok = c.N; a.slice_elems = c.N * d;
  a.in = x; a.slice_list = slice_list; a.list_in = 1; a.out = c.tmp0; a.M = c.d_F16[2]; a.ldm = W; a.n = W; a.n_out = kw;
  a.inner = d; a.outer = (int64_t)T * H; a.nslab = (int64_t)ns * T * H; a.in_bf16 = 1;
  if (tot_slot >= 0) a.tot_part = c.d_tot_part + (size_t)tot_slot * DCT_MAX_WAVES * 64;
  int w_dummy = 0;
  if ((e = launch_mfma_dct_pass(a, c.num_cu, st, tot_slot >= 0 ? &c.tot_waves[tot_slot] : &w_dummy)) != hipSuccess) return e;

  DctPassArgs b{};
  b.d = d; b.Ntok = c.N;
  b.in = c.tmp0; b.out = c.tmp1; b.M = c.d_F16[1]; b.ldm = H; b.n = H; b.n_out = kh; b.inner = (int64_t)kw * d;
  b.nslab = (int64_t)ns * T; b.outer = b.nslab; b.out_swap = 1; b.sw = T; b.sw_total = T; b.sw_off = 0;
  if ((e = launch_mfma_dct_pass(b, c.num_cu, st)) != hipSuccess) return e;

  DctPassArgs t{};
  t.d = d; t.Ntok = c.N;
  t.in = c.tmp1; t.out = spec; t.M = c.d_F16[0]; t.ldm = T; t.n = T; t.n_out = kt; t.inner = (int64_t)kw * d;
  t.nslab = (int64_t)ns * kh; t.outer = kh; t.slice_list = slice_list;
  t.perm_out = c.d_perm_t; t.perm_k = 1; t.perm_o = W; t.perm_scale = T;
  t.range_flag = c.d_range_flag;
  if (energy_slot >= 0) {
    t.energy_part = c.d_energy_part + (size_t)energy_slot * DCT_MAX_WAVES * 3 * 64;
    t.en_omul = W; t.en_div = W;  // the tile's other coordinates are (kh, kw)
    t.low_u = c.low_box[1]; t.low_v = c.low_box[2]; t.low_a = c.low_box[0];
    t.mid_u = c.mid_box[1]; t.mid_v = c.mid_box[2]; t.mid_a = c.mid_box[0];
  }
  return launch_mfma_dct_pass(t, c.num_cu, st, energy_slot >= 0 ? &c.energy_waves[energy_slot] : &w_dummy);
}

// MFMA path, inverse (section 3.7) for `ns` slices: the T axis pass gathers band-major rows into tmp1 in [h][t]
// order, then H axis (tmp1 -> tmp0) and W axis (tmp0 -> out, bf16).  Two forms:
//   select (delta = false): rows come from Y where the band is active for the slice, else from V~;
//   delta  (delta = true):  rows are Y - V~ on the active bands and zero elsewhere, restricted to the box keep[] that
//                           contains the active bands, and the last pass adds the input V:  out = V + F^-1(Y^ - V~),
//                           which is the same sum because F^-1(V~) = V.
// `wide` != nullptr: the same three passes on one band-major tensor of `width` channels per token ([ns][N][width], every
// band read from it; `wide_masks` device [ns], all 7).
static hipError_t inverse_transform_mfma(Ctx& c, void* out, const void* v_in, hipStream_t st, const int32_t* slice_list,
                                         int ns, const int keep[3], bool delta, const void* wide = nullptr, int width = 0,
                                         const int32_t* wide_masks = nullptr) {
  if (ns <= 0) return hipSuccess;
  const int T = c.shape.T, H = c.shape.H, W = c.shape.W, d = wide ? width : c.d;
  const int kt = keep[0], kh = keep[1], kw = keep[2];
  hipError_t e;
  DctPassArgs a{};
  a.d = d; a.Ntok = c.N;
  a.in = wide ? wide : c.Y; a.in_alt = wide ? wide : c.specV; a.masks = wide ? wide_masks : c.d_lists + c.off_masks;
  a.slice_list = slice_list; a.delta = delta ? 1 : 0;
  a.band_off1 = (int32_t)c.band_off[1]; a.band_off2 = (int32_t)c.band_off[2];
  a.band_off3 = (int32_t)(c.nb > 3 ? c.band_off[3] : c.N);
  a.perm_in = c.d_perm_t; a.perm_k = 1; a.perm_o = W; a.perm_scale = T;
  a.out = c.tmp1; a.M = c.d_Ft16[0]; a.ldm = T; a.n = kt; a.n_out = T; a.inner = (int64_t)kw * d;
  a.nslab = (int64_t)ns * kh; a.outer = kh;
  if ((e = launch_mfma_dct_pass(a, c.num_cu, st)) != hipSuccess) return e;

  DctPassArgs b{};
  b.d = d; b.Ntok = c.N;
  b.in = c.tmp1; b.out = c.tmp0; b.M = c.d_Ft16[1]; b.ldm = H; b.n = kh; b.n_out = H; b.inner = (int64_t)kw * d;
  b.nslab = (int64_t)ns * T; b.outer = b.nslab; b.in_swap = 1; b.sw = T; b.sw_total = T; b.sw_off = 0;
  if ((e = launch_mfma_dct_pass(b, c.num_cu, st)) != hipSuccess) return e;

  DctPassArgs w{};
  w.d = d; w.Ntok = c.N; w.slice_elems = c.N * d;
  w.in = c.tmp0; w.out = out; w.M = c.d_Ft16[2]; w.ldm = W; w.n = kw; w.n_out = W; w.inner = d;
  w.nslab = (int64_t)ns * T * H; w.outer = (int64_t)T * H; w.slice_list = slice_list; w.list_out = 1; w.out_bf16 = 1;
  w.resid = delta ? v_in : nullptr;
  return launch_mfma_dct_pass(w, c.num_cu, st);
}

// Forward transform of one [slices, N, d] tensor into a band-major spectral buffer (sections 3.2, 3.3).
static hipError_t forward_transform(Ctx& c, const void* x, void* spec, hipStream_t st, int energy_slot = -1) {
  const int T = c.shape.T, H = c.shape.H, W = c.shape.W, d = c.d;
  hipError_t e;
  if (c.path == FREQATTN_PATH_MFMA) {
    const int full[3] = {T, H, W};
    return forward_transform_mfma(c, x, spec, st, nullptr, c.slices, full, energy_slot, -1);
  }
  AxisPassArgs a{};
  a.Ntok = c.N; a.slice_mod = c.slices;
  a.in = x; a.out = c.tmp0; a.M = c.d_F32[0]; a.n = a.n_out = T; a.inner = (int64_t)H * W * d; a.outer = 1;
  a.nslab = c.slices; a.in_kind = io_kind(c); a.out_kind = 0;
  if ((e = launch_generic_axis_pass(a, st)) != hipSuccess) return e;
  a.in = c.tmp0; a.out = c.tmp1; a.M = c.d_F32[1]; a.n = a.n_out = H; a.inner = (int64_t)W * d; a.outer = T;
  a.nslab = (int64_t)c.slices * T; a.in_kind = 0;
  if ((e = launch_generic_axis_pass(a, st)) != hipSuccess) return e;
  a.in = c.tmp1; a.out = spec; a.M = c.d_F32[2]; a.n = a.n_out = W; a.inner = d; a.outer = (int64_t)T * H;
  a.nslab = (int64_t)c.slices * T * H; a.perm_out = c.d_perm;
  return launch_generic_axis_pass(a, st);
}

// Inverse transform (section 3.7): rows of band l of slice s are read from Y when the band is active for s, else
// from V~; W axis first (it reads the band-major rows), then H, then T, which writes `out` in the I/O type.
static hipError_t inverse_transform(Ctx& c, void* out, const void* v_in, hipStream_t st) {
  const int T = c.shape.T, H = c.shape.H, W = c.shape.W, d = c.d;
  const int32_t* masks = c.d_lists + c.off_masks;
  hipError_t e;
  if (c.path == FREQATTN_PATH_MFMA) {
    // slices grouped by what they ran: low only / low+mid -> delta form on the box, high -> select form on the whole
    // grid, nothing -> the output is V itself
    const int full[3] = {T, H, W};
    int low[3], mid[3];
    for (int a = 0; a < 3; ++a) { low[a] = keep_rows(c.low_box[a], full[a]); mid[a] = keep_rows(c.mid_box[a], full[a]); }
    const int32_t* L = c.d_lists;
    // (a box that is the whole grid saves nothing, and out = V + F^-1(Y^ - V~) would then cancel most of V against its own
    // round trip through the fp16 transform: such a class takes the select form)
    auto boxed = [&](const int* keep) { return keep[0] < T || keep[1] < H || keep[2] < W; };
    if ((e = inverse_transform_mfma(c, out, v_in, st, L + c.off_cls[0], c.n_cls[0], low, boxed(low))) != hipSuccess) return e;
    if ((e = inverse_transform_mfma(c, out, v_in, st, L + c.off_cls[1], c.n_cls[1], mid, boxed(mid))) != hipSuccess) return e;
    if ((e = inverse_transform_mfma(c, out, v_in, st, L + c.off_cls[2], c.n_cls[2], full, false)) != hipSuccess) return e;
    return launch_copy_slices(v_in, out, L + c.off_cls[3], c.n_cls[3], c.N * c.d * 2, st);
  }
  AxisPassArgs a{};
  a.Ntok = c.N; a.slice_mod = c.slices;
  a.in = c.Y; a.in_alt = c.specV; a.masks = masks; a.band_off1 = (int32_t)c.band_off[1];
  a.band_off2 = (int32_t)c.band_off[2]; a.band_off3 = (int32_t)(c.nb > 3 ? c.band_off[3] : c.N); a.perm_in = c.d_perm;
  a.out = c.tmp0; a.M = c.d_Ft32[2]; a.n = a.n_out = W; a.inner = d; a.outer = (int64_t)T * H;
  a.nslab = (int64_t)c.slices * T * H; a.in_kind = 0; a.out_kind = 0;
  if ((e = launch_generic_axis_pass(a, st)) != hipSuccess) return e;
  a.perm_in = nullptr; a.masks = nullptr; a.in_alt = nullptr;
  a.in = c.tmp0; a.out = c.tmp1; a.M = c.d_Ft32[1]; a.n = a.n_out = H; a.inner = (int64_t)W * d; a.outer = T;
  a.nslab = (int64_t)c.slices * T;
  if ((e = launch_generic_axis_pass(a, st)) != hipSuccess) return e;
  a.in = c.tmp1; a.out = out; a.M = c.d_Ft32[0]; a.n = a.n_out = T; a.inner = (int64_t)H * W * d; a.outer = 1;
  a.nslab = c.slices; a.out_kind = io_kind(c);
  return launch_generic_axis_pass(a, st);
}

static void fill_attn_params(const Ctx& c, AttnParams& p, float scale) {
  std::memset(&p, 0, sizeof(p));
  p.specQ = c.specQ; p.specK = c.specK; p.specV = c.specV; p.Y = c.Y;
  p.lowQ = c.lowQ; p.lowK = c.lowK; p.lowV = c.lowV; p.lowY = c.lowY; p.C = c.Cbuf;
  p.mid_row_ptr = c.d_row_ptr; p.mid_col_idx = c.d_col_idx;
  p.mid2_row_ptr = c.d_row_ptr2; p.mid2_col_idx = c.d_col_idx2;
  p.nb = c.nb;
  for (int l = 0; l < c.nb; ++l) {
    p.band_off[l] = (int32_t)c.band_off[l];
    p.band_n[l] = (int32_t)c.band_n[l];
    p.n_c[l] = c.n_c[l];
  }
  p.N = (int32_t)c.N; p.d = c.d; p.nbar = (int32_t)c.nbar; p.m2 = (c.nb - 1) * std::max(c.cfg.n_summary, 1);
  p.mid_block = c.cfg.mid_block; p.high_window = c.cfg.high_window; p.scale = scale;
}

struct StageTimer {
  Ctx& c; hipStream_t st; bool on; int slot;
  StageTimer(Ctx& c_, hipStream_t s) : c(c_), st(s), on(c_.timing), slot(0) {
    if (on) {
      slot = (int)(c.timed_steps % Ctx::MAX_TIMED);
      c.n_stages = 0;
      (void)hipEventRecord(c.ev[slot][0], st);
    }
  }
  void done(const char* name) {
    if (on && c.n_stages < Ctx::MAX_STAGES) {
      c.stage_name[c.n_stages] = name;
      (void)hipEventRecord(c.ev[slot][c.n_stages + 1], st);
      ++c.n_stages;
    }
  }
  ~StageTimer() { if (on) ++c.timed_steps; }
};

// sections 3.2 / 3.3: spectral transform of Q, K, V into band-major buffers; with_stats also leaves the router's
// band statistics (section 3.5) in d_stats.
static freqattn_status transforms_phase(freqattn_ctx* c, const void* q, const void* k, const void* v, hipStream_t st,
                                        bool with_stats, bool predict = false, bool whole_grid = false) {
  const bool fused_stats = with_stats && c->path == FREQATTN_PATH_MFMA;
  if (fused_stats) {
    // Router in the loop: the allocation is not known yet.  Q~ and K~ - and V~ where the context keeps it on the box
    // for slices without the high band (v_box_ok; otherwise V~ is computed everywhere) - are computed on the low+mid
    // box only, which gives their low and mid statistics exactly and their high-band energy by Parseval; slices that
    // turn out to run the high band get them completed afterwards (complete_qk_for_high).
    // With `predict`, the slices that ran the high band under the context's last allocation (allocations move
    // slowly along a sampling trajectory) get the whole-grid transform straight away, with all three statistics
    // taken directly; whatever the router then decides, only slices that are newly high need the completion.
    const int full[3] = {c->shape.T, c->shape.H, c->shape.W};
    int mid[3];
    bool pruned = false;
    for (int a = 0; a < 3; ++a) { mid[a] = keep_rows(c->mid_box[a], full[a]); pruned = pruned || mid[a] < full[a]; }
    if (whole_grid) pruned = false;   // every statistic taken directly from whole-grid transforms
    for (int i = 0; i < 6; ++i) c->energy_waves[i] = 0;
    for (int i = 0; i < 3; ++i) c->tot_waves[i] = 0;
    c->qk_on_mid_box = pruned;
    c->qk_full.assign((size_t)c->slices, pruned ? 0 : 1);
    // statistics slots: 0..2 = Q, K, V on the box (high band by Parseval when pruned), 3..5 = the same on the whole grid
    const bool vbox = pruned && c->v_box_ok;
    c->v_full.assign((size_t)c->slices, vbox ? 0 : 1);
    if (pruned && predict && c->alloc_valid && c->n_cls[2] > 0) {
      const int32_t* L = c->d_lists;
      const int32_t* hl = c->h_lists + c->off_cls[2];
      for (int i = 0; i < c->n_cls[2]; ++i) c->qk_full[(size_t)hl[i]] = c->v_full[(size_t)hl[i]] = 1;
      HIP_TRY(c, forward_transform_mfma(*c, q, c->specQ, st, L + c->off_nonhigh, c->n_nonhigh, mid, 0, 0));
      HIP_TRY(c, forward_transform_mfma(*c, k, c->specK, st, L + c->off_nonhigh, c->n_nonhigh, mid, 1, 1));
      if (vbox) HIP_TRY(c, forward_transform_mfma(*c, v, c->specV, st, L + c->off_nonhigh, c->n_nonhigh, mid, 2, 2));
      HIP_TRY(c, forward_transform_mfma(*c, q, c->specQ, st, L + c->off_cls[2], c->n_cls[2], full, 3, -1));
      HIP_TRY(c, forward_transform_mfma(*c, k, c->specK, st, L + c->off_cls[2], c->n_cls[2], full, 4, -1));
      if (vbox) HIP_TRY(c, forward_transform_mfma(*c, v, c->specV, st, L + c->off_cls[2], c->n_cls[2], full, 5, -1));
    } else {
      HIP_TRY(c, forward_transform_mfma(*c, q, c->specQ, st, nullptr, c->slices, pruned ? mid : full, 0, pruned ? 0 : -1));
      HIP_TRY(c, forward_transform_mfma(*c, k, c->specK, st, nullptr, c->slices, pruned ? mid : full, 1, pruned ? 1 : -1));
      if (vbox) HIP_TRY(c, forward_transform_mfma(*c, v, c->specV, st, nullptr, c->slices, mid, 2, 2));
    }
    if (!vbox) HIP_TRY(c, forward_transform_mfma(*c, v, c->specV, st, nullptr, c->slices, full, pruned ? 5 : 2, -1));
    EnergyWaves nw;
    for (int i = 0; i < 6; ++i) nw.en[i] = c->energy_waves[i];
    for (int i = 0; i < 3; ++i) nw.tot[i] = c->tot_waves[i];
    HIP_TRY(c, launch_energy_reduce(c->d_energy_part, pruned ? c->d_tot_part : nullptr, c->d_stats, c->d, nw, st));
    return FREQATTN_OK;
  }
  if (c->path == FREQATTN_PATH_MFMA && !with_stats) {
    // allocation known: Q~ and K~ are only needed on the bands a slice runs (none at all for an idle slice)
    const int full[3] = {c->shape.T, c->shape.H, c->shape.W};
    int low[3], mid[3];
    for (int a = 0; a < 3; ++a) { low[a] = keep_rows(c->low_box[a], full[a]); mid[a] = keep_rows(c->mid_box[a], full[a]); }
    const int32_t* L = c->d_lists;
    const void* xs[2] = {q, k};
    void* sp[2] = {c->specQ, c->specK};
    for (int i = 0; i < 2; ++i) {
      HIP_TRY(c, forward_transform_mfma(*c, xs[i], sp[i], st, L + c->off_cls[0], c->n_cls[0], low, -1, -1));
      HIP_TRY(c, forward_transform_mfma(*c, xs[i], sp[i], st, L + c->off_cls[1], c->n_cls[1], mid, -1, -1));
      HIP_TRY(c, forward_transform_mfma(*c, xs[i], sp[i], st, L + c->off_cls[2], c->n_cls[2], full, -1, -1));
    }
    if (c->v_box_ok) {   // V~ of a slice without the high band: the low+mid box (its high summaries come from V itself)
      c->v_full.assign((size_t)c->slices, 0);
      const int32_t* hl = c->h_lists + c->off_cls[2];
      for (int i = 0; i < c->n_cls[2]; ++i) c->v_full[(size_t)hl[i]] = 1;
      HIP_TRY(c, forward_transform_mfma(*c, v, c->specV, st, L + c->off_nonhigh, c->n_nonhigh, mid, -1, -1));
      HIP_TRY(c, forward_transform_mfma(*c, v, c->specV, st, L + c->off_cls[2], c->n_cls[2], full, -1, -1));
    } else {
      c->v_full.assign((size_t)c->slices, 1);
      HIP_TRY(c, forward_transform_mfma(*c, v, c->specV, st, nullptr, c->slices, full, -1, -1));
    }
    return FREQATTN_OK;
  }
  c->v_full.assign((size_t)c->slices, 1);
  HIP_TRY(c, forward_transform(*c, q, c->specQ, st));
  HIP_TRY(c, forward_transform(*c, k, c->specK, st));
  HIP_TRY(c, forward_transform(*c, v, c->specV, st));
  if (with_stats)
    HIP_TRY(c, launch_band_energy(c->specQ, c->specK, c->specV, c->d_stats, c->slices, c->N, c->d, c->band_off, c->band_n,
                                  0, st));
  return FREQATTN_OK;
}

// After routing with Q~ and K~ (and V~) on the low+mid box only: the slices that run the high band get the full transforms.
// (The caller has synchronised the stream since the first phase was queued - the router reads the statistics back -
// so the fix list's region of the pinned host buffer is not the source of a copy still in flight.)
static freqattn_status complete_qk_for_high(freqattn_ctx* c, const void* q, const void* k, const void* v, hipStream_t st) {
  if (c->path != FREQATTN_PATH_MFMA || !c->qk_on_mid_box || c->n_cls[2] == 0) return FREQATTN_OK;
  const int full[3] = {c->shape.T, c->shape.H, c->shape.W};
  int32_t* fix = c->h_lists + c->off_fix;
  const int32_t* high = c->h_lists + c->off_cls[2];
  int n_fix = 0;
  for (int i = 0; i < c->n_cls[2]; ++i)
    if (!c->qk_full[(size_t)high[i]]) fix[n_fix++] = high[i];
  if (n_fix == 0) return FREQATTN_OK;
  HIP_TRY(c, hipMemcpyAsync(c->d_lists + c->off_fix, fix, (size_t)n_fix * sizeof(int32_t), hipMemcpyHostToDevice, st));
  const int32_t* list = c->d_lists + c->off_fix;
  HIP_TRY(c, forward_transform_mfma(*c, q, c->specQ, st, list, n_fix, full, -1, -1));
  HIP_TRY(c, forward_transform_mfma(*c, k, c->specK, st, list, n_fix, full, -1, -1));
  bool v_too = false;
  for (int i = 0; i < n_fix; ++i) {
    v_too = v_too || !c->v_full[(size_t)fix[i]];
    c->v_full[(size_t)fix[i]] = 1;
  }
  if (v_too) HIP_TRY(c, forward_transform_mfma(*c, v, c->specV, st, list, n_fix, full, -1, -1));
  return FREQATTN_OK;
}

// Sections 3.3-3.6 on the band-major buffers: compression, band operators, expansion, summaries, exchange.  `v_in` is
// the untransformed V (for the high-band summaries of slices whose V~ stops at the low+mid box), or NULL when V~ exists
// on the whole grid for every slice.
static freqattn_status bands_core(freqattn_ctx* c, float scale, const void* v_in, hipStream_t st, StageTimer& tm,
                                   bool passed_bands_done = false) {
  const bool mf = c->path == FREQATTN_PATH_MFMA;
  const int is_half = mf ? 1 : 0;
  const int32_t* L = c->d_lists;
  // section 3.3: compression of the low band
  if (c->n_list[LOW] > 0) {
    const int32_t* lst = L + c->off_list[LOW];
    HIP_TRY(c, launch_pool_low(c->specQ, c->lowQ, lst, c->n_list[LOW], c->N, c->d, c->band_n[LOW], c->nbar, c->cfg.low_compress, is_half, st));
    HIP_TRY(c, launch_pool_low(c->specK, c->lowK, lst, c->n_list[LOW], c->N, c->d, c->band_n[LOW], c->nbar, c->cfg.low_compress, is_half, st));
    HIP_TRY(c, launch_pool_low(c->specV, c->lowV, lst, c->n_list[LOW], c->N, c->d, c->band_n[LOW], c->nbar, c->cfg.low_compress, is_half, st));
  }
  tm.done("low_compress");

  // section 3.6, first half: summary tokens.  Band l of a slice is summarised only if another band of the slice is active
  // (the exchange of that band is the only reader).  For slices that do not run the high band (their V~ may stop at the
  // low+mid box) the high band's summaries are summed from V instead of pooled - by the allocation alone, also where V~
  // happens to exist on the whole grid: the result must not depend on a prediction.
  // which = 0: every band; 1: only bands the slice passes through (pooled from V~: can run before the band operators);
  // 2: only bands the slice runs (pooled from the band outputs).
  AttnParams ap;
  fill_attn_params(*c, ap, scale);
  auto summaries = [&](int which) -> freqattn_status {
    uint64_t skip[NBMAX][4] = {{0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}, {0, 0, 0, 0}}, sel[4] = {0, 0, 0, 0};
    const int all_bands = (1 << c->nb) - 1;
    int nsel = 0, npool = 0;
    if (c->slices <= 256) {
      for (int s = 0; s < c->slices; ++s) {
        const int mask = c->h_alloc[(size_t)(s % c->shape.heads)];
        for (int l = 0; l < c->nb; ++l) {
          const bool active = (mask >> l) & 1;
          bool skp = (mask & ~(1 << l) & all_bands) == 0 || (which == 1 && active) || (which == 2 && !active);
          if (passed_bands_done && !active) skp = true;   // (projected forward: those tokens are in their slots already, and V~ does not exist there)
          if (l == 2 && mf && c->v_box_ok && v_in && !(mask & 4)) {
            skp = true;
            if (mask != 0 && which != 2) { sel[s >> 6] |= 1ull << (s & 63); ++nsel; }
          }
          if (skp) skip[l][s >> 6] |= 1ull << (s & 63);
          else ++npool;
        }
      }
    } else {
      npool = 1;
    }
    if (npool > 0)
      HIP_TRY(c, launch_summaries(c->Y, c->specV, c->Cbuf, L + c->off_masks, c->slices, c->N, c->d, c->nb, c->band_off, c->band_n, c->m_eff, ap.m2, is_half, &skip[0][0], c->d_pool_part, st));
    if (nsel > 0) {
      int nsplit = std::max(1, c->vsum_nsplit / nsel);   // nsel * nsplit <= 2 CUs' worth + nsel, what the scratch holds
      nsplit = (int)std::max<int64_t>(1, std::min<int64_t>(nsplit, c->N / 64 / 8));   // at least eight tiles per range
      HIP_TRY(c, launch_vsum(v_in, c->d_wsum, c->d_vsum_part, c->Cbuf, sel, nsel, c->N, c->d, nsplit, c->band_n[HIGH], c->m_eff, ap.m2, st));
    }
    return FREQATTN_OK;
  };
  // Slices that run a single band carry its exchange inside the band items (see build_lists): the summary tokens of
  // the bands they pass through are needed before the launch.
  const bool split_summaries = mf && c->exchange_fusion && c->cfg.n_summary > 0 && c->slices <= 256;
  if (split_summaries) {
    freqattn_status fs = summaries(1);
    if (fs != FREQATTN_OK) return fs;
    tm.done("summaries");
  }

  // section 3.4: the three band operators
  if (mf) {
    if (c->launch_mode == FREQATTN_LAUNCH_FUSED) {
      HIP_TRY(c, launch_mfma_attn(ap, (const AttnItem*)(L + c->off_items), c->n_items_branch, c->attn_rows, c->num_cu, st));
      tm.done("band_attention_fused");
    } else {
      static const char* nm[3] = {"low_attention", "mid_attention", "high_attention"};
      for (int kd = 0; kd < 3; ++kd) {
        HIP_TRY(c, launch_mfma_attn(ap, (const AttnItem*)(L + c->off_items_kind[kd]), c->n_items_kind[kd], c->attn_rows, c->num_cu, st));
        tm.done(nm[kd]);
      }
    }
  } else {
    const int64_t Nd = c->N * c->d;
    GenericAttnArgs g{};
    g.d = c->d; g.scale = scale;
    if (c->n_list[LOW] > 0) {
      g.Q = (const float*)c->lowQ; g.K = (const float*)c->lowK; g.V = (const float*)c->lowV; g.O = (float*)c->lowY;
      g.slice_list = L + c->off_list[LOW]; g.n_slices = c->n_list[LOW];
      g.slice_stride = g.kv_slice_stride = c->nbar * c->d; g.nq = g.nk = (int)c->nbar; g.mode = 0;
      HIP_TRY(c, launch_generic_attn(g, st));
    }
    tm.done("low_attention");
    if (c->n_list[MID] > 0) {
      const int64_t o = c->band_off[MID] * c->d;
      g.Q = (const float*)c->specQ + o; g.K = (const float*)c->specK + o; g.V = (const float*)c->specV + o;
      g.O = (float*)c->Y + o; g.slice_list = L + c->off_list[MID]; g.n_slices = c->n_list[MID];
      g.slice_stride = g.kv_slice_stride = Nd; g.nq = g.nk = (int)c->band_n[MID]; g.mode = 1;
      g.row_ptr = c->d_row_ptr; g.col_idx = c->d_col_idx; g.block = c->cfg.mid_block;
      HIP_TRY(c, launch_generic_attn(g, st));
    }
    if (c->nb > 3 && c->n_list[MID2] > 0) {   // the second mid band: the same operator on its own rows and block list
      const int64_t o = c->band_off[MID2] * c->d;
      g.Q = (const float*)c->specQ + o; g.K = (const float*)c->specK + o; g.V = (const float*)c->specV + o;
      g.O = (float*)c->Y + o; g.slice_list = L + c->off_list[MID2]; g.n_slices = c->n_list[MID2];
      g.slice_stride = g.kv_slice_stride = Nd; g.nq = g.nk = (int)c->band_n[MID2]; g.mode = 1;
      g.row_ptr = c->d_row_ptr2; g.col_idx = c->d_col_idx2; g.block = c->cfg.mid_block;
      HIP_TRY(c, launch_generic_attn(g, st));
    }
    tm.done("mid_attention");
    if (c->n_list[HIGH] > 0) {
      const int64_t o = c->band_off[HIGH] * c->d;
      g.Q = (const float*)c->specQ + o; g.K = (const float*)c->specK + o; g.V = (const float*)c->specV + o;
      g.O = (float*)c->Y + o; g.slice_list = L + c->off_list[HIGH]; g.n_slices = c->n_list[HIGH];
      g.slice_stride = g.kv_slice_stride = Nd; g.nq = g.nk = (int)c->band_n[HIGH]; g.mode = 2;
      g.window = c->cfg.high_window;
      HIP_TRY(c, launch_generic_attn(g, st));
    }
    tm.done("high_attention");
  }
  if (c->n_list[LOW] > 0)
    HIP_TRY(c, launch_expand_low(c->lowY, c->Y, L + c->off_list[LOW], c->n_list[LOW], c->N, c->d, c->band_n[LOW], c->nbar, c->cfg.low_compress, is_half, st));
  tm.done("low_expand");

  // section 3.6: remaining summary tokens (of the bands a slice runs, from the band outputs), then the exchange of
  // the slices that run more than one band
  if (c->cfg.n_summary > 0) {
    freqattn_status fs = summaries(split_summaries ? 2 : 0);
    if (fs != FREQATTN_OK) return fs;
    tm.done(split_summaries ? "summaries_active" : "summaries");
    if (mf) {
      HIP_TRY(c, launch_mfma_attn(ap, (const AttnItem*)(L + c->off_items_xchg), c->n_items_xchg, c->attn_rows, c->num_cu, st));
    } else {
      for (int l = 0; l < c->nb; ++l) {
        if (c->n_list[l] == 0 || c->n_c[l] == 0) continue;
        GenericAttnArgs g{};
        g.d = c->d; g.scale = scale; g.mode = 0; g.residual = 1;
        g.Q = (const float*)c->Y + c->band_off[l] * c->d; g.O = (float*)c->Y + c->band_off[l] * c->d;
        g.K = g.V = (const float*)c->Cbuf + (int64_t)l * ap.m2 * c->d;
        g.slice_list = L + c->off_list[l]; g.n_slices = c->n_list[l];
        g.slice_stride = c->N * c->d; g.kv_slice_stride = (int64_t)c->nb * ap.m2 * c->d;
        g.nq = (int)c->band_n[l]; g.nk = c->n_c[l];
        HIP_TRY(c, launch_generic_attn(g, st));
      }
    }
    tm.done("exchange");
  }
  return FREQATTN_OK;
}

static freqattn_status bands_phase(freqattn_ctx* c, float scale, const void* v_in, void* out, hipStream_t st,
                                   StageTimer& tm) {
  freqattn_status fs = bands_core(c, scale, v_in, st, tm);
  if (fs != FREQATTN_OK) return fs;
  // section 3.7: scatter + inverse transform
  HIP_TRY(c, inverse_transform(*c, out, v_in, st));
  tm.done("inverse_transform");
  return FREQATTN_OK;
}

static freqattn_status check_forward_args(freqattn_ctx* c, const void* q, const void* k, const void* v,
                                          const freqattn_band_cfg* band_cfg, const void* out, const char* who) {
  if (!q || !k || !v || !band_cfg || !out) return fail(c, FREQATTN_EINVAL, std::string(who) + ": NULL argument");
  if (c->path == FREQATTN_PATH_TABLES_ONLY) return fail(c, FREQATTN_EUNSUPPORTED, std::string(who) + ": tables-only context");
  if (!same_cfg(*band_cfg, c->cfg))
    return fail(c, FREQATTN_EINVAL, std::string(who) + ": band_cfg differs from the one given to freqattn_create");
  if (out == q || out == k || out == v) return fail(c, FREQATTN_EINVAL, std::string(who) + ": out aliases an input");
  return FREQATTN_OK;
}

static freqattn_status forward_impl(freqattn_ctx* c, const void* q, const void* k, const void* v,
                                    const freqattn_band_cfg* band_cfg, const int32_t* head_alloc, void* out,
                                    hipStream_t st, const char* who) {
  if (!head_alloc) return fail(c, FREQATTN_EINVAL, std::string(who) + ": NULL argument");
  freqattn_status fs = check_forward_args(c, q, k, v, band_cfg, out, who);
  if (fs != FREQATTN_OK) return fs;
  for (int h = 0; h < c->shape.heads; ++h)
    if (head_alloc[h] < 0 || head_alloc[h] >= (1 << c->nb))
      return fail(c, FREQATTN_EINVAL, std::string(who) + (c->nb > 3 ? ": head_alloc entry outside 0..15" : ": head_alloc entry outside 0..7"));
  const float scale = band_cfg->softmax_scale > 0.f ? band_cfg->softmax_scale : 1.0f / std::sqrt((float)c->d);
  fs = ensure_lists(c, head_alloc, st);
  if (fs != FREQATTN_OK) return fs;
  StageTimer tm(*c, st);
  fs = transforms_phase(c, q, k, v, st, false);
  if (fs != FREQATTN_OK) return fs;
  tm.done("forward_transform");
  return bands_phase(c, scale, v, out, st, tm);
}

extern "C" freqattn_status freqattn_forward(freqattn_ctx* c, const void* q, const void* k, const void* v,
                                            const freqattn_band_cfg* band_cfg, const int32_t* head_alloc, void* out,
                                            void* stream) {
  if (!c) return FREQATTN_EINVAL;
  return guarded(c, "freqattn_forward", [&]() -> freqattn_status {
    return forward_impl(c, q, k, v, band_cfg, head_alloc, out, (hipStream_t)stream, "freqattn_forward");
  });
}

// ------------------------------------------------------------------------------------------------ static scratch
// freqattn_forward_static: the same forward with every device buffer - tables, spectral scratch, work lists - inside
// one file-scope device array instead of memory from hipMalloc.  Each device has its own copy of the array at its own
// address; the address is looked up once per device.  A shadow context per device holds the carving of the array for
// the context it last served.
#define FREQATTN_STATIC_BYTES ((size_t)128 << 20)
static __device__ __align__(256) unsigned char scratch[FREQATTN_STATIC_BYTES];

namespace {
struct StaticSlot {
  char* ptr = nullptr;              // device address of this device's copy of `scratch`
  freqattn_ctx* shadow = nullptr;   // context whose device pointers point into it
  uint64_t owner_uid = 0;           // uid of the caller's context the shadow was built for
};
constexpr int kMaxDevices = 64;
StaticSlot g_static[kMaxDevices];
}  // namespace

extern "C" freqattn_status freqattn_forward_static(freqattn_ctx* c, const void* q, const void* k, const void* v,
                                                   const freqattn_band_cfg* band_cfg, const int32_t* head_alloc,
                                                   void* out, void* stream) {
  if (!c) return FREQATTN_EINVAL;
  return guarded(c, "freqattn_forward_static", [&]() -> freqattn_status {
    hipStream_t st = (hipStream_t)stream;
    if (!q || !k || !v || !band_cfg || !head_alloc || !out)
      return fail(c, FREQATTN_EINVAL, "freqattn_forward_static: NULL argument");
    if (!same_cfg(*band_cfg, c->cfg))
      return fail(c, FREQATTN_EINVAL, "freqattn_forward_static: band_cfg differs from the one given to freqattn_create");
    int dev = 0;
    HIP_TRY(c, hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_forward_static: device index too large");
    StaticSlot& slot = g_static[dev];
    if (!slot.ptr) {
      void* p = nullptr;
      HIP_TRY(c, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
      if (!p) return fail(c, FREQATTN_EHIP, "freqattn_forward_static: the scratch array has no address on this device");
      slot.ptr = (char*)p;
    }
    if (!slot.shadow || slot.owner_uid != c->uid) {
      // Another context (or none) owns the carving: wait for whatever still uses the array on this stream, then lay
      // the new context out in it.  Steady-state calls for one context skip all of this.
      HIP_TRY(c, hipStreamSynchronize(st));
      if (slot.shadow) { free_all(slot.shadow); delete slot.shadow; slot.shadow = nullptr; slot.owner_uid = 0; }
      freqattn_ctx* sh = nullptr;
      const int32_t path = c->path == FREQATTN_PATH_TABLES_ONLY ? (int32_t)FREQATTN_PATH_AUTO : c->path;
      freqattn_status fs = host_setup(&c->shape, &c->cfg, path, &sh);
      if (fs != FREQATTN_OK) return fail(c, fs, std::string("freqattn_forward_static: ") + g_create_error);
      sh->arena_base = slot.ptr; sh->arena_cap = FREQATTN_STATIC_BYTES; sh->arena_need = 0;
      const hipError_t e = device_setup(sh, st);
      if (e != hipSuccess) {
        const size_t need = sh->arena_need;
        free_all(sh);
        delete sh;
        (void)hipGetLastError();
        if (e == hipErrorOutOfMemory)
          return fail(c, FREQATTN_ENOMEM, "freqattn_forward_static: this shape needs at least " + std::to_string(need) +
                                          " bytes of scratch, the static array holds " + std::to_string(FREQATTN_STATIC_BYTES));
        return fail(c, FREQATTN_EHIP, std::string("freqattn_forward_static: ") + hipGetErrorString(e));
      }
      slot.shadow = sh;
      slot.owner_uid = c->uid;
    }
    const freqattn_status fs = forward_impl(slot.shadow, q, k, v, band_cfg, head_alloc, out, st, "freqattn_forward_static");
    if (fs != FREQATTN_OK) c->err = slot.shadow->err;
    return fs;
  });
}


// ------------------------------------------------------------------------------------------------ projected forward
// Sections 3.1 and 3.7 folded around the path: Q = X W_Q, K = X W_K, V = X W_V, output = concat(heads) W_O.  The
// transform acts on the token axes, the projections on channels, so F(X W) = F(X) W: X is transformed once (instead of
// Q, K and V), the projections run on band-major spectral rows - Q~ and K~ only on the rows of the bands a head runs -
// and W_O is applied to the band outputs before one inverse transform of model width.
static freqattn_status ensure_projection_buffers(freqattn_ctx* c, int d_model, hipStream_t st) {
  if (c->proj_d_model == d_model) return FREQATTN_OK;
  HIP_TRY(c, hipStreamSynchronize(st));
  auto F = [&](auto*& p) { if (p) { (void)hipFree((void*)p); p = nullptr; } };
  F(c->projX); F(c->projZ); F(c->projWq); F(c->projWk); F(c->projWv); F(c->projWo); F(c->proj_ones);
  F(c->projWvN); F(c->projM); F(c->projPool); F(c->projCtmp);
  F(c->d_gemm_prob); F(c->d_gemm_seg);
  if (c->h_gemm_prob) { (void)hipHostFree(c->h_gemm_prob); c->h_gemm_prob = nullptr; }
  if (c->h_gemm_seg) { (void)hipHostFree(c->h_gemm_seg); c->h_gemm_seg = nullptr; }
  c->proj_d_model = 0;
  c->gemm_tables_valid = false;
  const int B = c->shape.batch, heads = c->shape.heads, hd = heads * c->d;
  const size_t wide = (size_t)B * (size_t)c->N * (size_t)d_model * sizeof(half_t);
  hipError_t e = hipSuccess;
  auto A = [&](hipError_t r) { if (e == hipSuccess) e = r; };
  A(dev_alloc_bytes(*c, &c->projX, wide));
  A(dev_alloc_bytes(*c, &c->projZ, wide));
  A(dev_alloc(*c, &c->projWq, (size_t)hd * d_model));
  A(dev_alloc(*c, &c->projWk, (size_t)hd * d_model));
  A(dev_alloc(*c, &c->projWv, (size_t)hd * d_model));
  A(dev_alloc(*c, &c->projWo, (size_t)hd * d_model));
  A(dev_alloc(*c, &c->proj_ones, (size_t)B));
  const size_t mrows = (size_t)std::max(c->cfg.n_summary, 1);
  A(dev_alloc(*c, &c->projWvN, (size_t)hd * d_model));
  A(dev_alloc(*c, &c->projM, (size_t)c->nb * d_model * d_model));
  A(dev_alloc(*c, &c->projPool, (size_t)B * c->nb * mrows * d_model));
  A(dev_alloc(*c, &c->projCtmp, (size_t)c->slices * c->nb * mrows * c->d));
  // problems: Q~, K~, V~ per slice; output projection per (batch entry, band); pass-through weights per band; pooled rows
  // per slice.  Segments: one per projection; heads + 1 per output projection; heads per pass-through weight.
  c->gemm_cap_prob = 3 * B * heads + c->nb * B + c->nb + B * heads;
  c->gemm_cap_seg = 3 * B * heads + c->nb * B * (heads + 1) + c->nb * heads + B * heads;
  A(dev_alloc(*c, &c->d_gemm_prob, (size_t)c->gemm_cap_prob));
  A(dev_alloc(*c, &c->d_gemm_seg, (size_t)c->gemm_cap_seg));
  if (e == hipSuccess) e = hipHostMalloc((void**)&c->h_gemm_prob, (size_t)c->gemm_cap_prob * sizeof(GemmProblem), hipHostMallocDefault);
  if (e == hipSuccess) e = hipHostMalloc((void**)&c->h_gemm_seg, (size_t)c->gemm_cap_seg * sizeof(GemmSeg), hipHostMallocDefault);
  if (e == hipSuccess) {
    std::vector<int32_t> ones((size_t)B, (1 << NBMAX) - 1);
    e = hipMemcpy(c->proj_ones, ones.data(), (size_t)B * sizeof(int32_t), hipMemcpyHostToDevice);
  }
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(c, e == hipErrorOutOfMemory ? FREQATTN_ENOMEM : FREQATTN_EHIP,
                std::string("freqattn_forward_projected: ") + hipGetErrorString(e));
  }
  c->proj_d_model = d_model;
  return FREQATTN_OK;
}

// Problem tables of the product launches for the current allocation.  A launch takes problems with the same rows of
// A.  Stage 0: [Q~, K~ (and, with `fold`, V~) of all heads with the same hull of active bands, per batch entry]
// [without `fold`: V~ of all heads on every row, per batch entry].  Stage 1: output projection per (batch, band), K
// running over the heads.  Without `fold` a head contributes the band output where it runs the band and V~ where it
// passes through.  With `fold` only the heads that run the band contribute their output; the passing heads' share
// X~ W_V,h W_O,h is one more segment, X~ times the band's pass-through weight (stage 2: the sum over the passing heads
// of W_V,h W_O,h, transposed, one product per band), so their V~ is never formed on that band; their summary tokens
// there (section 3.6) are the pooled rows of X~ times W_V,h (stage 3, per batch entry).
static int build_gemm_tables(Ctx& c, bool fold) {
  const int B = c.shape.batch, heads = c.shape.heads, d = c.d, dm = c.proj_d_model, hd = heads * d;
  half_t* X = (half_t*)c.projX;
  int np = 0, ns = 0;
  c.gemm_groups.clear();
  auto hull = [&](int h, int64_t& r0, int64_t& r1) -> bool {
    const int mask = c.h_alloc[(size_t)h];
    int lo = -1, hi = -1;
    for (int l = 0; l < c.nb; ++l)   // (bands lie in the order of their indices: the hull is one run of rows)
      if (((mask >> l) & 1) && c.band_n[l] > 0) { if (lo < 0) lo = l; hi = l; }
    if (lo < 0) return false;
    r0 = c.band_off[lo]; r1 = c.band_off[hi] + c.band_n[hi];
    return true;
  };
  for (int b = 0; b < B; ++b) {
    std::vector<char> done((size_t)heads, 0);
    for (int h0 = 0; h0 < heads; ++h0) {
      int64_t r0, r1;
      if (done[(size_t)h0] || !hull(h0, r0, r1)) continue;
      const int first = np;
      for (int h = h0; h < heads; ++h) {
        int64_t q0, q1;
        if (done[(size_t)h] || !hull(h, q0, q1) || q0 != r0 || q1 != r1) continue;
        done[(size_t)h] = 1;
        const int64_t slice = (int64_t)b * heads + h;
        for (int which = 0; which < (fold ? 3 : 2); ++which) {
          const half_t* Wt = (which == 0 ? c.projWq : which == 1 ? c.projWk : c.projWv) + (size_t)h * d * dm;
          half_t* spec = (half_t*)(which == 0 ? c.specQ : which == 1 ? c.specK : c.specV) + (slice * c.N + r0) * d;
          c.h_gemm_seg[ns] = GemmSeg{X + ((int64_t)b * c.N + r0) * dm, Wt, dm, dm, dm, 0};
          c.h_gemm_prob[np++] = GemmProblem{spec, d, (int)(r1 - r0), d, ns++, 1, 0};
        }
      }
      c.gemm_groups.push_back({first, np - first, (int)(r1 - r0), d, 0});
    }
    if (!fold) {
      const int first = np;
      for (int h = 0; h < heads; ++h) {
        const int64_t slice = (int64_t)b * heads + h;
        c.h_gemm_seg[ns] = GemmSeg{X + (int64_t)b * c.N * dm, c.projWv + (size_t)h * d * dm, dm, dm, dm, 0};
        c.h_gemm_prob[np++] = GemmProblem{(half_t*)c.specV + slice * c.N * d, d, (int)c.N, d, ns++, 1, 0};
      }
      c.gemm_groups.push_back({first, heads, (int)c.N, d, 0});
    }
  }
  bool passing[NBMAX] = {false, false, false, false};
  if (fold)
    for (int l = 0; l < c.nb; ++l) {
      if (c.band_n[l] <= 0) continue;
      const int seg0 = ns;
      for (int h = 0; h < heads; ++h)
        if (!((c.h_alloc[(size_t)h] >> l) & 1))   // (W_V,h W_O,h)^T[i][j] = sum_c W_O^T[i][h d + c] W_V[j][h d + c]
          c.h_gemm_seg[ns++] = GemmSeg{c.projWo + (size_t)h * d, c.projWvN + (size_t)h * d, hd, hd, d, 0};
      if (ns == seg0) continue;
      passing[l] = true;
      c.h_gemm_prob[np] = GemmProblem{c.projM + (size_t)l * dm * dm, dm, dm, dm, seg0, ns - seg0, 0};
      c.gemm_groups.push_back({np, 1, dm, dm, 2});
      ++np;
    }
  if (fold && c.cfg.n_summary > 0) {
    const int mrows = c.cfg.n_summary;
    for (int b = 0; b < B; ++b) {
      const int first = np;
      for (int h = 0; h < heads; ++h) {
        const int64_t slice = (int64_t)b * heads + h;
        c.h_gemm_seg[ns] = GemmSeg{c.projPool + (size_t)b * c.nb * mrows * dm, c.projWv + (size_t)h * d * dm, dm, dm, dm, 0};
        c.h_gemm_prob[np++] = GemmProblem{c.projCtmp + (size_t)slice * c.nb * mrows * d, d, c.nb * mrows, d, ns++, 1, 0};
      }
      c.gemm_groups.push_back({first, heads, c.nb * mrows, d, 3});
    }
  }
  for (int b = 0; b < B; ++b)
    for (int l = 0; l < c.nb; ++l) {
      if (c.band_n[l] <= 0) continue;
      const int seg0 = ns;
      for (int h = 0; h < heads; ++h) {
        const int64_t slice = (int64_t)b * heads + h;
        const bool active = (c.h_alloc[(size_t)h] >> l) & 1;
        if (fold && !active) continue;
        const half_t* src = (const half_t*)(active ? c.Y : c.specV) + (slice * c.N + c.band_off[l]) * d;
        c.h_gemm_seg[ns++] = GemmSeg{src, c.projWo + (size_t)h * d, d, hd, d, 0};
      }
      if (fold && passing[l])
        c.h_gemm_seg[ns++] = GemmSeg{X + ((int64_t)b * c.N + c.band_off[l]) * dm, c.projM + (size_t)l * dm * dm, dm, dm, dm, 0};
      c.h_gemm_prob[np] = GemmProblem{(half_t*)c.projZ + ((int64_t)b * c.N + c.band_off[l]) * dm, dm, (int)c.band_n[l], dm, seg0, ns - seg0, 0};
      c.gemm_groups.push_back({np, 1, (int)c.band_n[l], dm, 1});
      ++np;
    }
  return np;
}

extern "C" freqattn_status freqattn_forward_projected(freqattn_ctx* c, const void* x, int32_t d_model, const void* wq,
                                                      const void* wk, const void* wv, const void* wo,
                                                      const freqattn_band_cfg* band_cfg, const int32_t* head_alloc,
                                                      void* out, void* stream) {
  if (!c) return FREQATTN_EINVAL;
  return guarded(c, "freqattn_forward_projected", [&]() -> freqattn_status {
    if (!x || !wq || !wk || !wv || !wo || !band_cfg || !head_alloc || !out)
      return fail(c, FREQATTN_EINVAL, "freqattn_forward_projected: NULL argument");
    if (c->path != FREQATTN_PATH_MFMA)
      return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_forward_projected: needs a context on the matrix-core path");
    if (!same_cfg(*band_cfg, c->cfg))
      return fail(c, FREQATTN_EINVAL, "freqattn_forward_projected: band_cfg differs from the one given to freqattn_create");
    if (out == x) return fail(c, FREQATTN_EINVAL, "freqattn_forward_projected: out aliases x");
    const int heads = c->shape.heads, B = c->shape.batch;
    if (d_model < 64 || d_model % 64 != 0 || (int64_t)d_model > (int64_t)heads * c->d)
      return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_forward_projected: d_model must be a multiple of 64 and at most "
                                            "heads * head_dim (the transform passes share the context's scratch)");
    for (int h = 0; h < heads; ++h)
      if (head_alloc[h] < 0 || head_alloc[h] >= (1 << c->nb))
        return fail(c, FREQATTN_EINVAL, c->nb > 3 ? "freqattn_forward_projected: head_alloc entry outside 0..15" : "freqattn_forward_projected: head_alloc entry outside 0..7");
    hipStream_t st = (hipStream_t)stream;
    const float scale = band_cfg->softmax_scale > 0.f ? band_cfg->softmax_scale : 1.0f / std::sqrt((float)c->d);
    freqattn_status fs = ensure_lists(c, head_alloc, st);
    if (fs != FREQATTN_OK) return fs;
    fs = ensure_projection_buffers(c, d_model, st);
    if (fs != FREQATTN_OK) return fs;
    // Pass-through folding (see build_gemm_tables): on by default wherever the summaries' per-slice bookkeeping reaches
    // (256 slices); FREQATTN_PROJ_FOLD=0, read at every call, keeps V~ on every row instead.
    const char* fold_env = getenv("FREQATTN_PROJ_FOLD");
    const bool fold = c->slices <= 256 && !(fold_env && atoi(fold_env) == 0);
    if (fold != c->proj_fold) {
      if (c->gemm_tables_valid) HIP_TRY(c, hipStreamSynchronize(st));   // the tables of the other mode may still be read
      c->proj_fold = fold;
      c->gemm_tables_valid = false;
    }
    if (!c->gemm_tables_valid) {
      // (ensure_lists or ensure_projection_buffers waited for the stream when they invalidated the tables)
      const int np = build_gemm_tables(*c, fold);
      int ns = 0;
      for (int i = 0; i < np; ++i) ns = std::max(ns, c->h_gemm_prob[i].seg0 + c->h_gemm_prob[i].nseg);
      if (np > 0) HIP_TRY(c, hipMemcpyAsync(c->d_gemm_prob, c->h_gemm_prob, (size_t)np * sizeof(GemmProblem), hipMemcpyHostToDevice, st));
      if (ns > 0) HIP_TRY(c, hipMemcpyAsync(c->d_gemm_seg, c->h_gemm_seg, (size_t)ns * sizeof(GemmSeg), hipMemcpyHostToDevice, st));
      c->gemm_tables_valid = true;
    }
    StageTimer tm(*c, st);
    const int hd = heads * c->d;
    HIP_TRY(c, launch_transpose_bf16_to_f16(wq, c->projWq, d_model, hd, st));
    HIP_TRY(c, launch_transpose_bf16_to_f16(wk, c->projWk, d_model, hd, st));
    HIP_TRY(c, launch_transpose_bf16_to_f16(wv, c->projWv, d_model, hd, st));
    HIP_TRY(c, launch_transpose_bf16_to_f16(wo, c->projWo, hd, d_model, st));
    auto products = [&](int stage) -> freqattn_status {
      for (const Ctx::GemmGroup& gg : c->gemm_groups)
        if (gg.stage == stage) HIP_TRY(c, launch_gemm_nt(c->d_gemm_prob + gg.first, c->d_gemm_seg, gg.per, gg.m, gg.n, st));
      return FREQATTN_OK;
    };
    if (fold) {
      HIP_TRY(c, launch_convert_16(wv, c->projWvN, (int64_t)d_model * hd, 0, st));
      fs = products(2);   // pass-through weights per band
      if (fs != FREQATTN_OK) return fs;
    }
    tm.done("weights");
    const int full[3] = {c->shape.T, c->shape.H, c->shape.W};
    HIP_TRY(c, forward_transform_mfma(*c, x, c->projX, st, nullptr, B, full, -1, -1, d_model));
    tm.done("x_transform");
    fs = products(0);
    if (fs != FREQATTN_OK) return fs;
    tm.done("qkv_projection");
    if (fold && c->cfg.n_summary > 0) {
      // summary tokens of the bands a head passes through: chunk means of X~, times every head's W_V, into the slots
      const int mrows = c->cfg.n_summary;
      HIP_TRY(c, launch_pool_wide(c->projX, c->projPool, B, c->N, d_model, c->nb, c->band_off, c->band_n, c->m_eff, mrows, st));
      fs = products(3);
      if (fs != FREQATTN_OK) return fs;
      HIP_TRY(c, launch_place_summaries(c->projCtmp, c->Cbuf, c->d_lists + c->off_masks, c->slices, c->d, c->nb, c->m_eff, mrows,
                                        (c->nb - 1) * std::max(c->cfg.n_summary, 1), st));
      tm.done("summaries_passed_bands");
    }
    c->v_full.assign((size_t)c->slices, 1);
    fs = bands_core(c, scale, nullptr, st, tm, fold);
    if (fs != FREQATTN_OK) return fs;
    fs = products(1);
    if (fs != FREQATTN_OK) return fs;
    tm.done("o_projection");
    HIP_TRY(c, inverse_transform_mfma(*c, out, nullptr, st, nullptr, B, full, false, c->projZ, d_model, c->proj_ones));
    tm.done("inverse_transform");
    return FREQATTN_OK;
  });
}

static freqattn_status router_from_spectral(freqattn_ctx* c, float t, int32_t hidden, const float* w1, const float* b1,
                                            const float* w2, const float* b2, int32_t* head_alloc, float pi[3],
                                            float* stats_out, hipStream_t st, bool* high_unreliable = nullptr);

extern "C" freqattn_status freqattn_forward_routed(freqattn_ctx* c, const void* q, const void* k, const void* v,
                                                   const freqattn_band_cfg* band_cfg, float t, int32_t hidden,
                                                   const float* w1, const float* b1, const float* w2, const float* b2,
                                                   void* out, int32_t* head_alloc_out, float pi_out[3], void* stream) {
  return guarded(c, "freqattn_forward_routed", [&]() -> freqattn_status {
  if (!c) return FREQATTN_EINVAL;
  if (!w1 || !b1 || !w2 || !b2 || !head_alloc_out || !pi_out || hidden < 1)
    return fail(c, FREQATTN_EINVAL, "freqattn_forward_routed: NULL argument or hidden < 1");
  freqattn_status fs = check_forward_args(c, q, k, v, band_cfg, out, "freqattn_forward_routed");
  if (fs != FREQATTN_OK) return fs;
  if (c->d % 64 != 0) return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_forward_routed: head_dim must be a multiple of 64");
  if (c->nb != 3) return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_forward_routed: the router scores three bands (section 3.5); a four-band context takes its allocation from the caller");
  hipStream_t st = (hipStream_t)stream;
  const float scale = band_cfg->softmax_scale > 0.f ? band_cfg->softmax_scale : 1.0f / std::sqrt((float)c->d);
  StageTimer tm(*c, st);
  fs = transforms_phase(c, q, k, v, st, true, c->predict_alloc != 0);
  if (fs != FREQATTN_OK) return fs;
  tm.done("forward_transform");
  bool redo = false;
  fs = router_from_spectral(c, t, hidden, w1, b1, w2, b2, head_alloc_out, pi_out, nullptr, st, &redo);
  if (fs != FREQATTN_OK) return fs;
  if (redo) {
    // the high band holds too little energy for the difference form: whole-grid transforms with direct statistics
    fs = transforms_phase(c, q, k, v, st, true, false, true);
    if (fs != FREQATTN_OK) return fs;
    fs = router_from_spectral(c, t, hidden, w1, b1, w2, b2, head_alloc_out, pi_out, nullptr, st);
    if (fs != FREQATTN_OK) return fs;
  }
  fs = ensure_lists(c, head_alloc_out, st);
  if (fs != FREQATTN_OK) return fs;
  tm.done("router");
  fs = complete_qk_for_high(c, q, k, v, st);
  if (fs != FREQATTN_OK) return fs;
  tm.done("forward_transform_high_qk");
  return bands_phase(c, scale, v, out, st, tm);
  });
}


extern "C" freqattn_status freqattn_dense_forward(freqattn_ctx* c, const void* q, const void* k, const void* v, void* out,
                                                  void* stream) {
  return guarded(c, "freqattn_dense_forward", [&]() -> freqattn_status {
  if (!c) return FREQATTN_EINVAL;
  if (!q || !k || !v || !out) return fail(c, FREQATTN_EINVAL, "freqattn_dense_forward: NULL argument");
  if (c->path != FREQATTN_PATH_MFMA) return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_dense_forward: MFMA path only");
  hipStream_t st = (hipStream_t)stream;
  if (!c->alloc_valid) {   // the dense item list is uploaded with the first allocation's lists
    std::vector<int32_t> zero((size_t)c->shape.heads, 0);
    freqattn_status fs = ensure_lists(c, zero.data(), st);
    if (fs != FREQATTN_OK) return fs;
  }
  AttnParams ap;
  const float scale = c->cfg.softmax_scale > 0.f ? c->cfg.softmax_scale : 1.0f / std::sqrt((float)c->d);
  fill_attn_params(*c, ap, scale);
  StageTimer tm(*c, st);
  // The attention kernel reads fp16 tensors (tiles copied straight into LDS): the bf16 inputs are converted into the
  // context's spectral scratch first, and the fp16 result back into the caller's bf16 tensor - two element-wise
  // passes beside an N^2 kernel.
  const int64_t n_el = (int64_t)c->slices * c->N * c->d;   // a multiple of 64 on this path
  HIP_TRY(c, launch_convert_16(q, c->specQ, n_el, 0, st));
  HIP_TRY(c, launch_convert_16(k, c->specK, n_el, 0, st));
  HIP_TRY(c, launch_convert_16(v, c->specV, n_el, 0, st));
  ap.denseQ = c->specQ; ap.denseK = c->specK; ap.denseV = c->specV; ap.denseO = c->Y;
  HIP_TRY(c, launch_mfma_attn(ap, (const AttnItem*)(c->d_lists + c->off_items_dense), c->n_items_dense, c->attn_rows, c->num_cu, st));
  HIP_TRY(c, launch_convert_16(c->Y, out, n_el, 1, st));
  tm.done("dense_attention");
  return FREQATTN_OK;
  });
}

extern "C" freqattn_status freqattn_read_spectral(freqattn_ctx* c, int32_t which, int32_t slice, int32_t band,
                                                  float* host_out, void* stream) {
  return guarded(c, "freqattn_read_spectral", [&]() -> freqattn_status {
  if (!c || !host_out || which < 0 || which > 3 || slice < 0 || slice >= c->slices || band < 0 || band >= c->nb)
    return FREQATTN_EINVAL;
  if (c->path == FREQATTN_PATH_TABLES_ONLY) return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_read_spectral: tables-only context");
  HIP_TRY(c, hipStreamSynchronize((hipStream_t)stream));
  const void* src = which == 0 ? c->specQ : which == 1 ? c->specK : which == 2 ? c->specV : c->Y;
  if (band == 2 && (which == 2 || (which == 3 && c->alloc_valid && !((c->h_alloc[slice % c->shape.heads] >> band) & 1))) &&
      (size_t)slice < c->v_full.size() && !c->v_full[(size_t)slice])
    return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_read_spectral: V~ of this slice was only computed on the low+mid box");
  if (which == 3) {
    if (!c->alloc_valid) return fail(c, FREQATTN_EINVAL, "freqattn_read_spectral: no forward has run");
    if (!((c->h_alloc[slice % c->shape.heads] >> band) & 1)) src = c->specV;
  }
  const size_t cnt = (size_t)c->band_n[band] * c->d;
  const size_t off = ((size_t)slice * c->N + c->band_off[band]) * c->d;
  if (cnt == 0) return FREQATTN_OK;
  if (c->path == FREQATTN_PATH_MFMA) {
    std::vector<half_t> tmp(cnt);
    HIP_TRY(c, hipMemcpy(tmp.data(), (const half_t*)src + off, cnt * sizeof(half_t), hipMemcpyDeviceToHost));
    for (size_t i = 0; i < cnt; ++i) host_out[i] = (float)tmp[i];
  } else {
    HIP_TRY(c, hipMemcpy(host_out, (const float*)src + off, cnt * sizeof(float), hipMemcpyDeviceToHost));
  }
  return FREQATTN_OK;
  });
}

// ------------------------------------------------------------------------------------------------ router
static freqattn_status router_from_spectral(freqattn_ctx* c, float t, int32_t hidden, const float* w1, const float* b1,
                                            const float* w2, const float* b2, int32_t* head_alloc, float pi[3],
                                            float* stats_out, hipStream_t st, bool* high_unreliable) {
  const int d = c->d, DR = 64, DT = 64;
  HIP_TRY(c, hipMemcpyAsync(c->h_stats, c->d_stats, 3 * d * sizeof(float), hipMemcpyDeviceToHost, st));
  HIP_TRY(c, hipMemcpyAsync(c->h_stats + 3 * d, c->d_range_flag, sizeof(int32_t), hipMemcpyDeviceToHost, st));
  HIP_TRY(c, hipStreamSynchronize(st));
  if (c->h_stats[3 * d] != 0.f) {   // (any set bit pattern of the flag reads as a non-zero float)
    (void)launch_fill_zero((float*)c->d_range_flag, 1, st);
    return fail(c, FREQATTN_ERANGE, "spectral coefficients leave the fp16 range of the matrix-core path: the inputs must "
                                    "satisfy sqrt(N) * max|x| < 65504 (or use the fp32 path)");
  }
  for (int i = 0; i < 3 * d; ++i)
    if (!std::isfinite(c->h_stats[i]))
      return fail(c, FREQATTN_ERANGE, "router statistics are not finite: the inputs leave the fp16 range of the spectral "
                                      "buffers (sqrt(N) * max|x| must stay below 65504) or are not finite themselves");
  if (high_unreliable) {
    // High-band energy taken as total minus low minus mid (section 5: the transform is orthonormal) inherits the
    // rounding of the fp16 transform, about 1e-4 of the total; below 1 % of a channel's total it is not trusted.
    *high_unreliable = false;
    if (c->path == FREQATTN_PATH_MFMA && c->qk_on_mid_box)
      for (int ch = 0; ch < d; ++ch) {
        const double tot = (double)c->h_stats[ch] + c->h_stats[d + ch] + c->h_stats[2 * d + ch];
        if ((double)c->h_stats[2 * d + ch] < 0.01 * tot) *high_unreliable = true;
      }
  }
  // g: log(eps + mean energy) per band and channel group, centred (section 3.5 "pooled statistics")
  double x[3 * 64 + 64];
  const int per = d / DR;
  double mean_log = 0.0;
  for (int l = 0; l < 3; ++l)
    for (int r = 0; r < DR; ++r) {
      double sum = 0.0;
      for (int u = 0; u < per; ++u) sum += (double)c->h_stats[l * d + r * per + u];
      const double cnt = 3.0 * c->slices * (double)std::max<int64_t>(c->band_n[l], 1);
      const double e = sum / cnt / per;
      x[l * DR + r] = std::log(1e-6 + e);
      mean_log += x[l * DR + r];
    }
  mean_log /= 3.0 * DR;
  for (int i = 0; i < 3 * DR; ++i) x[i] -= mean_log;
  if (stats_out)
    for (int i = 0; i < 3 * DR; ++i) stats_out[i] = (float)x[i];
  // e(t): sin then cos of 1000 t 10000^(-2i/64)
  for (int i = 0; i < DT / 2; ++i) {
    const double ang = 1000.0 * (double)t * std::pow(10000.0, -2.0 * i / DT);
    x[3 * DR + i] = std::sin(ang);
    x[3 * DR + DT / 2 + i] = std::cos(ang);
  }
  const int DIN = 3 * DR + DT;
  std::vector<double> hdn(hidden);
  for (int j = 0; j < hidden; ++j) {
    double s = b1[j];
    for (int i = 0; i < DIN; ++i) s += x[i] * (double)w1[(size_t)i * hidden + j];
    hdn[j] = s > 0 ? s : 0;
  }
  double z[3];
  const double prior[3] = {1.0, 0.0, -1.0};
  for (int o = 0; o < 3; ++o) {
    double s = b2[o];
    for (int j = 0; j < hidden; ++j) s += hdn[j] * (double)w2[(size_t)j * 3 + o];
    z[o] = s + 1.5 * (2.0 * (double)t - 1.0) * prior[o];
  }
  const double zm = std::max(z[0], std::max(z[1], z[2]));
  double p[3], ps = 0;
  for (int o = 0; o < 3; ++o) { p[o] = std::exp(z[o] - zm); ps += p[o]; }
  for (int o = 0; o < 3; ++o) { p[o] /= ps; pi[o] = (float)p[o]; }
  if (!(std::isfinite(p[0]) && std::isfinite(p[1]) && std::isfinite(p[2])))
    return fail(c, FREQATTN_ERANGE, "router: allocation probabilities are not finite (non-finite router weights?)");
  // apportionment: one head per band when heads >= 3, the rest by largest remainder, ties to the lower band
  const int heads = c->shape.heads;
  const int base = heads >= 3 ? 1 : 0;
  const int rest = heads - 3 * base;
  int cnt[3]; double rem[3]; int given = 0;
  for (int o = 0; o < 3; ++o) {
    const double quota = p[o] * rest;
    cnt[o] = (int)std::floor(quota);
    rem[o] = quota - cnt[o];
    given += cnt[o];
  }
  for (int r = given; r < rest; ++r) {
    int best = 0;
    for (int o = 1; o < 3; ++o)
      if (rem[o] > rem[best]) best = o;
    cnt[best] += 1;
    rem[best] = -1.0;
  }
  return freqattn_route_fixed(heads, cnt[0] + base, cnt[1] + base, cnt[2] + base, head_alloc);
}


extern "C" freqattn_status freqattn_route_mlp(freqattn_ctx* c, const void* q, const void* k, const void* v, float t,
                                              int32_t hidden, const float* w1, const float* b1, const float* w2,
                                              const float* b2, int32_t* head_alloc, float pi[3], float* stats_out,
                                              void* stream) {
  return guarded(c, "freqattn_route_mlp", [&]() -> freqattn_status {
  if (!c) return FREQATTN_EINVAL;
  if (!q || !k || !v || !w1 || !b1 || !w2 || !b2 || !head_alloc || !pi || hidden < 1)
    return fail(c, FREQATTN_EINVAL, "freqattn_route_mlp: NULL argument or hidden < 1");
  if (c->path == FREQATTN_PATH_TABLES_ONLY) return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_route_mlp: tables-only context");
  if (c->d % 64 != 0) return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_route_mlp: head_dim must be a multiple of 64");
  if (c->nb != 3) return fail(c, FREQATTN_EUNSUPPORTED, "freqattn_route_mlp: the router scores three bands (section 3.5); a four-band context takes its allocation from the caller");
  hipStream_t st = (hipStream_t)stream;
  freqattn_status fs = transforms_phase(c, q, k, v, st, true);
  if (fs != FREQATTN_OK) return fs;
  bool redo = false;
  fs = router_from_spectral(c, t, hidden, w1, b1, w2, b2, head_alloc, pi, stats_out, st, &redo);
  if (fs != FREQATTN_OK || !redo) return fs;
  fs = transforms_phase(c, q, k, v, st, true, false, true);
  if (fs != FREQATTN_OK) return fs;
  return router_from_spectral(c, t, hidden, w1, b1, w2, b2, head_alloc, pi, stats_out, st);
  });
}

// ------------------------------------------------------------------------------------------------ stage timing
extern "C" freqattn_status freqattn_set_stage_timing(freqattn_ctx* c, int32_t enabled) {
  if (!c) return FREQATTN_EINVAL;
  c->timing = enabled != 0;
  c->n_stages = 0;
  c->timed_steps = 0;
  return FREQATTN_OK;
}

extern "C" freqattn_status freqattn_stage_times(freqattn_ctx* c, int32_t max_stages, const char** names_out, float* ms_out,
                                                int32_t* n_stages) {
  if (!c || !names_out || !ms_out || !n_stages) return FREQATTN_EINVAL;
  *n_stages = 0;
  if (!c->timing || c->n_stages == 0 || c->timed_steps == 0) return FREQATTN_OK;
  const int last = (int)((c->timed_steps - 1) % Ctx::MAX_TIMED);
  HIP_TRY(c, hipEventSynchronize(c->ev[last][c->n_stages]));
  const int n = std::min<int>(c->n_stages, max_stages);
  const int kept = (int)std::min<int64_t>(c->timed_steps, Ctx::MAX_TIMED);
  for (int i = 0; i < n; ++i) {
    names_out[i] = c->stage_name[i];
    double sum = 0.0;
    for (int t = 0; t < kept; ++t) {
      float ms = 0.f;
      HIP_TRY(c, hipEventElapsedTime(&ms, c->ev[t][i], c->ev[t][i + 1]));
      sum += ms;
    }
    ms_out[i] = (float)(sum / kept);
  }
  *n_stages = n;
  return FREQATTN_OK;
}
