// CPU ORACLE — TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, fp64 implementation of what the per-chunk attention step computes:
// per-axis rotary tables, global position decode, qk-RMSNorm, 3D rotation with a global
// latent-frame time index, and softmax attention of the chunk's queries over all visible
// keys.  It shares no code with the HIP path and is never used by it; only tests, the
// smoke check and the bench's cpu_baseline leg may call it.
//
// Every function is the definition written out: no tiling, no online softmax, no fusion.
// OpenMP only spreads independent (row, head) pairs over host cores.
//
// Pins (tests marked "not gpu"): closed forms for the tables, exhaustive decode against
// numpy.unravel_index, norm preservation, identity at the origin, the relative-position
// identity, a complex-number re-derivation of the rotation that follows Algorithm 2,
// library softmax-attention in fp64, row sums, permutation invariance, and streaming ==
// one-shot block-causal attention; for the projection: a library matmul, an identity
// weight (projection == its input), a zero input (projection == bias) and linearity.  End-to-end numeric values are not printed anywhere in
// the paper, so there is no printed-value pin ("parity unpinned by printed values").
#include <cmath>
#include <cstdint>
#include <cstddef>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

extern "C" {

int oracle_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

// Frequency of pair j on an axis that owns dim_a channels: theta^(-2j/dim_a).
// (The paper gives three per-axis frequency tables, Algorithm 2; the law itself is the
// standard rotary one, applied per axis with that axis's own width.)
static inline double axis_omega(int j, int dim_a, double theta) {
  return std::pow(theta, -2.0 * (double)j / (double)dim_a);
}

// out[p][j][0] = cos(p * omega_j), out[p][j][1] = sin(p * omega_j), p < n_pos, j < dim_a/2.
// Algorithm 2's freqs[axis]; Section 3.4.1 item 2 (precomputed, contiguous).
void oracle_axis_table(int dim_a, double theta, int n_pos, double* out) {
  const int np2 = dim_a / 2;
  for (int p = 0; p < n_pos; ++p)
    for (int j = 0; j < np2; ++j) {
      const double phi = (double)p * axis_omega(j, dim_a, theta);
      out[((size_t)p * np2 + j) * 2 + 0] = std::cos(phi);
      out[((size_t)p * np2 + j) * 2 + 1] = std::sin(phi);
    }
}

// Section 3.3.3: i_global = Delta + i_local; t_global = s + floor(i_global / (Hg*Wg));
// (h, w) from the row-major (F, Hg, Wg) flattening used by Algorithm 2's expand().
void oracle_decode(int64_t i_local, int64_t delta, int s, int grid_h, int grid_w,
                   int* t_global, int* h, int* w) {
  const int64_t hw = (int64_t)grid_h * grid_w;
  const int64_t ig = delta + i_local;
  const int64_t f = ig / hw;
  const int64_t r = ig % hw;
  *t_global = (int)(s + f);
  *h = (int)(r / grid_w);
  *w = (int)(r % grid_w);
}

// RMSNorm per token over a group of `group` consecutive channels (group = H*D: the whole
// projection vector; group = D: per head).  y_c = x_c * g_c / sqrt(mean_G(x^2) + eps).
// x, y: [n][H*D]; gain: [H*D].
void oracle_rmsnorm(const double* x, const double* gain, double eps, int64_t n, int hd,
                    int group, double* y) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    const double* xi = x + (size_t)i * hd;
    double* yi = y + (size_t)i * hd;
    for (int g0 = 0; g0 < hd; g0 += group) {
      double ss = 0.0;
      for (int c = 0; c < group; ++c) ss += xi[g0 + c] * xi[g0 + c];
      const double r = 1.0 / std::sqrt(ss / (double)group + eps);
      for (int c = 0; c < group; ++c) yi[g0 + c] = xi[g0 + c] * gain[g0 + c] * r;
    }
  }
}

// 3D rotation (Section 3.3.2 item 2, Algorithm 2): within each head, channels (2j, 2j+1)
// form one complex number that is multiplied by exp(i*phi_j).  Pairs 0..dt/2-1 take the
// time angle t_global*omega_T, the next dh/2 pairs the height angle, the last dw/2 the
// width angle (concatenation order T, H, W).  x, out: [n][H][D], D = dt+dh+dw.
void oracle_rotate(const double* x, int64_t n, int n_heads, int dt, int dh, int dw,
                   double theta, int grid_h, int grid_w, int s, int64_t delta, double* out) {
  const int D = dt + dh + dw;
  const int pt = dt / 2, ph = dh / 2;
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i) {
    int tg, h, w;
    oracle_decode(i, delta, s, grid_h, grid_w, &tg, &h, &w);
    for (int head = 0; head < n_heads; ++head) {
      const double* xi = x + ((size_t)i * n_heads + head) * D;
      double* oi = out + ((size_t)i * n_heads + head) * D;
      for (int j = 0; j < D / 2; ++j) {
        double phi;
        if (j < pt) phi = (double)tg * axis_omega(j, dt, theta);
        else if (j < pt + ph) phi = (double)h * axis_omega(j - pt, dh, theta);
        else phi = (double)w * axis_omega(j - pt - ph, dw, theta);
        const double c = std::cos(phi), sn = std::sin(phi);
        const double a = xi[2 * j], b = xi[2 * j + 1];
        oi[2 * j] = a * c - b * sn;      // Re[(a+ib)(c+i sn)]
        oi[2 * j + 1] = a * sn + b * c;  // Im
      }
    }
  }
}

// Softmax attention, per head and query row, two passes (Algorithm 3 step 6):
//   s_m = scale*<q, k_m>, M = max s_m, p_m = exp(s_m-M)/sum, o = sum p_m v_m,
//   lse = M + log(sum exp(s_m-M)).
// q, o: [Lq][H][D]; k, v: [Lk][H][D]; lse: [H][Lq]; P (optional): [H][Lq][Lk].
// Optional block mask: key m visible to query i iff k_block[m] <= q_block[i].
void oracle_attention(const double* q, const double* k, const double* v, int64_t Lq,
                      int64_t Lk, int n_heads, int D, double scale, const int32_t* q_block,
                      const int32_t* k_block, double* o, double* lse, double* P) {
  const int64_t jobs = Lq * n_heads;
#pragma omp parallel
  {
    std::vector<double> sc((size_t)Lk);
#pragma omp for schedule(dynamic, 4)
    for (int64_t job = 0; job < jobs; ++job) {
      const int64_t i = job / n_heads;
      const int head = (int)(job % n_heads);
      const double* qi = q + ((size_t)i * n_heads + head) * D;
      double M = -INFINITY;
      for (int64_t m = 0; m < Lk; ++m) {
        const bool vis = !(q_block && k_block) || k_block[m] <= q_block[i];
        if (!vis) { sc[m] = -INFINITY; continue; }
        const double* km = k + ((size_t)m * n_heads + head) * D;
        double dot = 0.0;
        for (int c = 0; c < D; ++c) dot += qi[c] * km[c];
        sc[m] = scale * dot;
        if (sc[m] > M) M = sc[m];
      }
      double Z = 0.0;
      for (int64_t m = 0; m < Lk; ++m) {
        sc[m] = (sc[m] == -INFINITY) ? 0.0 : std::exp(sc[m] - M);
        Z += sc[m];
      }
      double* oi = o + ((size_t)i * n_heads + head) * D;
      for (int c = 0; c < D; ++c) oi[c] = 0.0;
      for (int64_t m = 0; m < Lk; ++m) {
        const double p = sc[m] / Z;
        if (P) P[((size_t)head * Lq + i) * Lk + m] = p;
        const double* vm = v + ((size_t)m * n_heads + head) * D;
        for (int c = 0; c < D; ++c) oi[c] += p * vm[c];
      }
      if (lse) lse[(size_t)head * Lq + i] = M + std::log(Z);
    }
  }
}

// Algorithm 3 step 1, the local QKV projection: y[i][o] = sum_c x[i][c] * w[o][c] + bias[o]
// (weights stored [out][in] like a linear layer; bias may be null).  Columns 0..HD-1 of y
// are q, the next HD are k, the last HD are v.
void oracle_project(const double* x, const double* w, const double* bias, int64_t n, int64_t c_in,
                    int64_t n_out, double* y) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < n; ++i)
    for (int64_t o = 0; o < n_out; ++o) {
      double acc = 0.0;
      for (int64_t c = 0; c < c_in; ++c) acc += x[i * c_in + c] * w[o * c_in + c];
      y[i * n_out + o] = acc + (bias ? bias[o] : 0.0);
    }
}

}  // extern "C"
