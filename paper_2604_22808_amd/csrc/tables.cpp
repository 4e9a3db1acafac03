// Host-side integer tables and transform matrices of libfreqattn.
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
// the low band occupies rows [0, n_low), the mid band the next n_mid rows and the high band the rest.
void build_bands(Ctx& c) {
  const int T = c.shape.T, H = c.shape.H, W = c.shape.W;
  const freqattn_band_cfg& g = c.cfg;
  for (int l = 0; l < 3; ++l) c.h_band_index[l].clear();
  std::vector<int8_t> band((size_t)c.N);
  for (int kt = 0; kt < T; ++kt)
    for (int kh = 0; kh < H; ++kh)
      for (int kw = 0; kw < W; ++kw) {
        const int64_t flat = ((int64_t)kt * H + kh) * W + kw;
        auto inside = [&](int64_t num, int64_t den) {
          return kt * den < num * T && kh * den < num * H && kw * den < num * W;
        };
        const int l = inside(g.low_num, g.low_den) ? LOW : inside(g.mid_num, g.mid_den) ? MID : HIGH;
        band[flat] = (int8_t)l;
        c.h_band_index[l].push_back((int32_t)flat);
      }
  int64_t off = 0;
  for (int l = 0; l < 3; ++l) {
    c.band_n[l] = (int64_t)c.h_band_index[l].size();
    c.band_off[l] = off;
    off += c.band_n[l];
  }
  c.h_perm.assign((size_t)c.N, 0);
  for (int l = 0; l < 3; ++l)
    for (size_t r = 0; r < c.h_band_index[l].size(); ++r)
      c.h_perm[c.h_band_index[l][r]] = (int32_t)(c.band_off[l] + (int64_t)r);
}

// Block list of the mid-band pattern (section 3.4.2): query block I sees key block J iff |I-J| <= diag, or
// (I-J) mod stride == 0, or J == 0 when block0 is on.  Columns ascend within a row.
void build_mid_blocks(Ctx& c) {
  const freqattn_band_cfg& g = c.cfg;
  const int64_t nb = (c.band_n[MID] + g.mid_block - 1) / g.mid_block;
  c.nb_mid = nb;
  c.h_row_ptr.assign((size_t)nb + 1, 0);
  c.h_col_idx.clear();
  for (int64_t I = 0; I < nb; ++I) {
    for (int64_t J = 0; J < nb; ++J) {
      const int64_t diff = I - J;
      const int64_t ad = diff < 0 ? -diff : diff;
      int64_t mod = diff % g.mid_stride;
      if (mod < 0) mod += g.mid_stride;
      if (ad <= g.mid_diag || mod == 0 || (g.mid_block0 && J == 0)) c.h_col_idx.push_back((int32_t)J);
    }
    c.h_row_ptr[(size_t)I + 1] = (int32_t)c.h_col_idx.size();
  }
}

}  // namespace fa
