// Host-side integer tables and transform matrices of libfreqattn.
#include <cstring>
#include <cmath>

#include "ctx.h"

namespace fa {

// Orthonormal DCT-II matrix of paper section 3.2: F[k][j] = s_k sqrt(2/n) cos(pi (2j+1) k / (2n)), s_0 = 1/sqrt 2.
// The angle is reduced in integers first ((2j+1)k mod 4n) so that cos sees an argument in [0, 2 pi).
void build_dct_matrix(int n, std::vector<double>& F) {
  F.assign((size_t)n * n, 0.0);
  const double pi = 3.14159265358979323846264338327950288;
  const double amp = std::sqrt(2.0 / n);
  for (int k = 0; k < n; ++k) {
    const double sk = (k == 0) ? std::sqrt(0.5) : 1.0;
    for (int j = 0; j < n; ++j) {
      const long m = ((long)(2 * j + 1) * k) % (4L * n);
      F[(size_t)k * n + j] = sk * amp * std::cos(pi * (double)m / (2.0 * n));
    }
  }
}

// Orthonormal Haar wavelet matrix of order n = 2^p (section 3.2 names wavelets as the alternative): row 0 is
// 1/sqrt(n); row 2^j + i is +-sqrt(2^j / n) on the two halves of [i n/2^j, (i+1) n/2^j) and zero elsewhere.
void build_haar_matrix(int n, std::vector<double>& F) {
  F.assign((size_t)n * n, 0.0);
  for (int j = 0; j < n; ++j) F[j] = 1.0 / std::sqrt((double)n);
  for (int lev = 0; (1 << lev) < n; ++lev) {
    const int s = n >> lev;
    const double a = std::sqrt((double)(1 << lev) / n);
    for (int i = 0; i < (1 << lev); ++i)
      for (int j = 0; j < s; ++j) F[(size_t)((1 << lev) + i) * n + i * s + j] = (j < s / 2) ? a : -a;
  }
}

// Band membership of section 3.3 with rational edges, decided in 64-bit integers; band-major order is the order of
// the ascending flat index (kt*H + kh)*W + kw inside each band.  perm maps a flat index to its band-major row, where
// the low band occupies rows [0, n_low), the mid band the next n_mid rows, the high band the rows after that and - in a
// four-band layout (cfg.mid2_num > 0: coefficients inside the third edge but outside the mid edge) - the second mid
// band the rest: the bands lie in the order of their indices, and a three-band layout is a four-band one without its
// last band.
void build_bands(Ctx& c) {
  const int T = c.shape.T, H = c.shape.H, W = c.shape.W;
  const freqattn_band_cfg& g = c.cfg;
  c.nb = g.mid2_num > 0 ? 4 : 3;
  for (int l = 0; l < NBMAX; ++l) c.h_band_index[l].clear();
  for (int kt = 0; kt < T; ++kt)
    for (int kh = 0; kh < H; ++kh)
      for (int kw = 0; kw < W; ++kw) {
        const int64_t flat = ((int64_t)kt * H + kh) * W + kw;
        auto inside = [&](int64_t num, int64_t den) {
          return kt * den < num * T && kh * den < num * H && kw * den < num * W;
        };
        int l = inside(g.low_num, g.low_den) ? LOW : inside(g.mid_num, g.mid_den) ? MID : HIGH;
        if (l == HIGH && c.nb == 4 && inside(g.mid2_num, g.mid2_den)) l = MID2;
        c.h_band_index[l].push_back((int32_t)flat);
      }
  int64_t off = 0;
  for (int l = 0; l < NBMAX; ++l) {
    c.band_n[l] = (int64_t)c.h_band_index[l].size();
    c.band_off[l] = off;
    off += c.band_n[l];
  }
  c.h_perm.assign((size_t)c.N, 0);
  for (int l = 0; l < NBMAX; ++l)
    for (size_t r = 0; r < c.h_band_index[l].size(); ++r)
      c.h_perm[c.h_band_index[l][r]] = (int32_t)(c.band_off[l] + (int64_t)r);
}

// Block list of the mid-band pattern (section 3.4.2): query block I sees key block J iff |I-J| <= diag, or
// (I-J) mod stride == 0, or J == 0 when block0 is on.  Columns ascend within a row.  One list per block-sparse band.
static int64_t block_list(const freqattn_band_cfg& g, int64_t n_rows, std::vector<int32_t>& row_ptr, std::vector<int32_t>& col_idx) {
  const int64_t nb = (n_rows + g.mid_block - 1) / g.mid_block;
  row_ptr.assign((size_t)nb + 1, 0);
  col_idx.clear();
  for (int64_t I = 0; I < nb; ++I) {
    for (int64_t J = 0; J < nb; ++J) {
      const int64_t diff = I - J;
      const int64_t ad = diff < 0 ? -diff : diff;
      int64_t mod = diff % g.mid_stride;
      if (mod < 0) mod += g.mid_stride;
      if (ad <= g.mid_diag || mod == 0 || (g.mid_block0 && J == 0)) col_idx.push_back((int32_t)J);
    }
    row_ptr[(size_t)I + 1] = (int32_t)col_idx.size();
  }
  return nb;
}
void build_mid_blocks(Ctx& c) {
  c.nb_mid = block_list(c.cfg, c.band_n[MID], c.h_row_ptr, c.h_col_idx);
  c.nb_mid2 = block_list(c.cfg, c.band_n[MID2], c.h_row_ptr2, c.h_col_idx2);
}

// Weights of a band's summary tokens as functionals of the untransformed input (section 3.6, U = I):
//   w[u][(t,h,w)] = sum over the rows (kt,kh,kw) of chunk u of F_T[kt][t] F_H[kh][h] F_W[kw][w],
// chunk u = band rows [floor(u n / m), floor((u+1) n / m)), rows in ascending flat order.  Separable per row, so a
// chunk is summed kw-run by kw-run into a per-kt plane G[h][w], and each plane goes into the volume with F_T's row.
// Output: [m][N] in token order.
void build_summary_weights(const Ctx& c, int band, std::vector<float>& out) {
  const int T = c.shape.T, H = c.shape.H, W = c.shape.W;
  const int64_t N = c.N, HW = (int64_t)H * W;
  const std::vector<int32_t>& idx = c.h_band_index[band];
  const int64_t nb = (int64_t)idx.size();
  const int m = c.m_eff[band];
  const double* Ft = c.h_F[0].data();
  const double* Fh = c.h_F[1].data();
  const double* Fw = c.h_F[2].data();
  out.assign((size_t)m * N, 0.f);
  std::vector<double> acc((size_t)N), G((size_t)HW), srow((size_t)W);
  for (int u = 0; u < m; ++u) {
    const int64_t r0 = ((int64_t)u * nb) / m, r1 = ((int64_t)(u + 1) * nb) / m;
    std::fill(acc.begin(), acc.end(), 0.0);
    int64_t r = r0;
    while (r < r1) {
      const int kt = (int)(idx[(size_t)r] / HW);
      std::fill(G.begin(), G.end(), 0.0);
      while (r < r1 && idx[(size_t)r] / HW == kt) {
        const int64_t rowid = idx[(size_t)r] / W;   // kt*H + kh
        const int kh = (int)(rowid % H);
        std::fill(srow.begin(), srow.end(), 0.0);
        while (r < r1 && idx[(size_t)r] / W == rowid) {
          const double* fw = Fw + (size_t)(idx[(size_t)r] % W) * W;
          for (int w = 0; w < W; ++w) srow[(size_t)w] += fw[w];
          ++r;
        }
        const double* fh = Fh + (size_t)kh * H;
        for (int h = 0; h < H; ++h) {
          const double a = fh[h];
          double* g = G.data() + (size_t)h * W;
          for (int w = 0; w < W; ++w) g[w] += a * srow[(size_t)w];
        }
      }
      const double* ft = Ft + (size_t)kt * T;
      for (int t = 0; t < T; ++t) {
        const double a = ft[t];
        double* dst = acc.data() + (size_t)t * HW;
        for (int64_t i = 0; i < HW; ++i) dst[i] += a * G[(size_t)i];
      }
    }
    float* row = out.data() + (size_t)u * N;
    for (int64_t n = 0; n < N; ++n) row[n] = (float)acc[(size_t)n];
  }
}

// The layout the summing kernel reads: bf16, [N/64][64][64] (tile of 64 tokens, chunk, token; chunks >= m are zero);
// inside every group of 16 tokens the order is the one in which the kernel's transposing LDS reads deliver them
// (stored position 8 g + 4 h + e holds token 8 h + 4 g + e).
void pack_vsum_weights(const std::vector<float>& w, int m, int64_t N, std::vector<uint16_t>& out) {
  out.assign((size_t)64 * N, 0);
  for (int u = 0; u < m; ++u)
    for (int64_t n = 0; n < N; ++n) {
      const float f = w[(size_t)u * N + n];
      uint32_t b;
      std::memcpy(&b, &f, 4);
      b += 0x7fffu + ((b >> 16) & 1u);   // round to nearest even (the weights are finite)
      const int o = (int)(n & 15), hh = (o >> 3) & 1, gg = (o >> 2) & 1, e = o & 3;
      out[(size_t)((n >> 6) * 4096 + (int64_t)u * 64 + ((n & 48) + 8 * gg + 4 * hh + e))] = (uint16_t)(b >> 16);
    }
}

}  // namespace fa
