// Radial / spherical basis functions (named in paper Sec. 3.3; standard definitions).
// Per-edge quantities are evaluated in fp64 and rounded once to fp32 (E values only, the cost is
// negligible); per-triplet quantities (cosines, Legendre factors) are fp32.
#include <math.h>
#include <stdarg.h>

#include "common.h"

namespace {

constexpr int MAX_S = 8;
constexpr int MAX_R_BESSEL = 16;

struct bessel_table {
  double z[MAX_S * MAX_R_BESSEL];     // z[l*R + n]  zeros of j_l
  double norm[MAX_S * MAX_R_BESSEL];  // sqrt(2 / (c^3 j_{l+1}(z)^2))
};

// j_l(x), x > 0: ascending series below the turning point, upward recurrence above it.
__host__ __device__ inline double sph_bessel(int l, double x) {
  if (x < (double)l + 1.0 && l >= 2) {
    double q = -0.5 * x * x, term = 1.0, sum = 1.0;
    for (int k = 1; k <= 40; ++k) {
      term *= q / ((double)k * (double)(2 * l + 2 * k + 1));
      sum += term;
    }
    double pref = 1.0;
    for (int k = 1; k <= l; ++k) pref *= x / (double)(2 * k + 1);
    return pref * sum;
  }
  double s = sin(x), c = cos(x);
  double j0 = s / x;
  if (l == 0) return j0;
  double j1 = s / (x * x) - c / x;
  for (int k = 1; k < l; ++k) {
    double j2 = (double)(2 * k + 1) / x * j1 - j0;
    j0 = j1;
    j1 = j2;
  }
  return j1;
}

__host__ __device__ inline double envelope_d(double x, int p) {
  double xp = 1.0;
  for (int k = 0; k < p; ++k) xp *= x;
  double a = -0.5 * (p + 1) * (p + 2), b = (double)p * (p + 2), c = -0.5 * p * (p + 1);
  return 1.0 + xp * (a + x * (b + x * c));
}

// zeros of j_l by bisection between consecutive zeros of j_{l-1}
void make_bessel_table(int S, int R, double cutoff, bessel_table* t) {
  const int n0 = R + S;
  double prev[MAX_S + MAX_R_BESSEL], cur[MAX_S + MAX_R_BESSEL];
  for (int n = 0; n < n0; ++n) prev[n] = M_PI * (n + 1);
  for (int n = 0; n < R; ++n) t->z[n] = prev[n];
  for (int l = 1; l < S; ++l) {
    for (int n = 0; n < n0 - l; ++n) {
      double a = prev[n], b = prev[n + 1], fa = sph_bessel(l, a);
      for (int it = 0; it < 200 && (b - a) > 1e-15 * b; ++it) {
        double mid = 0.5 * (a + b), fm = sph_bessel(l, mid);
        if ((fm > 0) == (fa > 0)) { a = mid; fa = fm; } else { b = mid; }
      }
      cur[n] = 0.5 * (a + b);
    }
    for (int n = 0; n < n0 - l; ++n) prev[n] = cur[n];
    for (int n = 0; n < R; ++n) t->z[l * R + n] = prev[n];
  }
  for (int l = 0; l < S; ++l)
    for (int n = 0; n < R; ++n) {
      double j = sph_bessel(l + 1, t->z[l * R + n]);
      t->norm[l * R + n] = sqrt(2.0 / (cutoff * cutoff * cutoff * j * j));
    }
}

// variant D: rbf[E,R] and rad[E,S*R]; one thread per (edge, row) with row 0 = rbf, row 1+l = rad l
__global__ void basis_edge_D_kernel(const float* __restrict__ dist, int64_t n_edges, int S, int R, int p,
                                    double cutoff, bessel_table tab, float* __restrict__ rbf,
                                    float* __restrict__ rad) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int rows = S + 1;
  if (idx >= n_edges * rows) return;
  int64_t e = idx / rows;
  int row = (int)(idx % rows);
  double d = (double)dist[e];
  double x = d / cutoff;
  double u = envelope_d(x, p);
  if (row == 0) {
    if (!rbf) return;
    double pre = u * sqrt(2.0 / cutoff) / d;
    for (int n = 0; n < R; ++n) rbf[e * R + n] = (float)(pre * sin((double)(n + 1) * M_PI * x));
  } else {
    if (!rad) return;
    int l = row - 1;
    for (int n = 0; n < R; ++n)
      rad[e * S * R + l * R + n] = (float)(u * tab.norm[l * R + n] * sph_bessel(l, tab.z[l * R + n] * x));
  }
}

// variant D, for forces: gd[e] = sum_n grad_rbf[e,n] d rbf_n / dd + sum_{l,n} grad_rad[e,l,n] d rad_ln / dd with
//   rbf_n(d) = u(x) sqrt(2/c) sin(k x) / d,  k = (n+1) pi,  x = d / c
//   rad_ln(d) = u(x) N_ln j_l(z_ln x),  j_l'(y) = j_{l-1}(y) - (l+1)/y j_l(y)  (j_0' = -j_1)
// one thread per edge (a few dozen terms in fp64; not a hot kernel)
__global__ void grad_dist_bessel_kernel(const float* __restrict__ dist, const float* __restrict__ grad_rbf,
                                        const float* __restrict__ grad_rad, int64_t n_edges, int S, int R, int p, double cutoff,
                                        bessel_table tab, float* __restrict__ gd) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= n_edges) return;
  const double d = (double)dist[e], x = d / cutoff;
  double xp1 = 1.0;                       // x^(p-1)
  for (int k = 0; k < p - 1; ++k) xp1 *= x;
  const double a = -0.5 * (p + 1) * (p + 2), b = (double)p * (p + 2), c = -0.5 * p * (p + 1);
  const double u = 1.0 + xp1 * x * (a + x * (b + x * c));
  const double du = xp1 * (p * a + x * ((p + 1) * b + x * (p + 2) * c)) / cutoff;   // du/dd
  double s = 0.0;
  if (grad_rbf) {
    const double pre = sqrt(2.0 / cutoff);
    for (int n = 0; n < R; ++n) {
      const double k = (double)(n + 1) * M_PI, sn = sin(k * x), cs = cos(k * x);
      s += (double)grad_rbf[e * R + n] * pre * (du * sn / d + u * (k / cutoff * cs / d - sn / (d * d)));
    }
  }
  if (grad_rad) {
    for (int l = 0; l < S; ++l)
      for (int n = 0; n < R; ++n) {
        const double z = tab.z[l * R + n], y = z * x;
        const double jl = sph_bessel(l, y);
        const double djl = l == 0 ? -sph_bessel(1, y) : sph_bessel(l - 1, y) - (double)(l + 1) / y * jl;
        s += (double)grad_rad[e * S * R + l * R + n] * tab.norm[l * R + n] * (du * jl + u * z / cutoff * djl);
      }
  }
  gd[e] = (float)s;
}

// variant G: g[E,R] Gaussian radial basis
__global__ void basis_edge_G_kernel(const float* __restrict__ dist, int64_t n_edges, int R, int p,
                                    double cutoff, float* __restrict__ g) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_edges * R) return;
  int64_t e = idx / R;
  int n = (int)(idx % R);
  double x = (double)dist[e] / cutoff;
  double a = (x - (double)n / (double)(R - 1)) * (double)(R - 1);
  g[idx] = (float)(envelope_d(x, p) * exp(-0.5 * a * a));
}

__global__ void cos_alpha_kernel(const float* __restrict__ unit, const int32_t* __restrict__ idx_kj,
                                 const int32_t* __restrict__ idx_ji, int64_t n_triplets,
                                 float* __restrict__ cos_alpha) {
  int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= n_triplets) return;
  const float* a = unit + 3 * (int64_t)idx_ji[t];
  const float* b = unit + 3 * (int64_t)idx_kj[t];
  float c = -(a[0] * b[0] + a[1] * b[1] + a[2] * b[2]);
  cos_alpha[t] = fminf(1.0f, fmaxf(-1.0f, c));
}

// out[q] = in[perm[q]].  For the kj-major copy of cos alpha the gathered values of neighbouring q lie a whole in-degree apart
// (each its own 64-byte sector), but all rows of a centre atom gather from the same d_in x d_out block; workgroup ids are
// dealt round-robin to the 8 XCDs, so they are renumbered to give each XCD a contiguous range of q: the block of an atom
// is then fetched into one L2 and hit there by the atom's other rows (3.5 GB fetched for 0.4 GB used otherwise).
__global__ void permute_kernel(const float* __restrict__ in, const int32_t* __restrict__ perm, int64_t n,
                               float* __restrict__ out) {
  const int64_t nb = gridDim.x, per = nb >> 3, rem = nb & 7;
  const int64_t x = blockIdx.x & 7, i = blockIdx.x >> 3;
  const int64_t blk = x * per + (x < rem ? x : rem) + i;
  const int64_t q = blk * blockDim.x + threadIdx.x;
  if (q < n) out[q] = in[perm[q]];
}

// materialised spherical basis, one thread per (triplet, l)
__global__ void sbf_kernel(const float* __restrict__ rad, const float* __restrict__ cos_alpha,
                           const int32_t* __restrict__ idx_kj, int64_t n_triplets, int S, int R,
                           float* __restrict__ sbf) {
  int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= n_triplets * S) return;
  int64_t t = idx / S;
  int l = (int)(idx % S);
  float c = cos_alpha[t];
  float p0 = 1.0f, p1 = c;
  for (int k = 1; k < l; ++k) {
    float p2 = ((2 * k + 1) * c * p1 - k * p0) / (float)(k + 1);
    p0 = p1;
    p1 = p2;
  }
  float P = (l == 0) ? 1.0f : p1;
  float Y = sqrtf((float)(2 * l + 1) / (4.0f * (float)M_PI)) * P;
  const float* r = rad + ((int64_t)idx_kj[t] * S + l) * R;
  float* o = sbf + (t * S + l) * R;
  for (int n = 0; n < R; ++n) o[n] = r[n] * Y;
}

inline int nblk(int64_t n) { return (int)((n + 255) / 256); }

}  // namespace

extern "C" int gp_basis_forward(gp_ctx* ctx, const gp_dims* dims, const float* dist, const float* unit,
                                const int32_t* idx_kj, const int32_t* idx_ji, const int32_t* perm_kj,
                                int64_t n_edges, int64_t n_triplets, float* rbf, float* rad,
                                float* cos_alpha, float* cos_alpha_kj, float* sbf) {
  if (!ctx) return GP_BAD_ARG;
  GP_REQUIRE(ctx, dims, "gp_basis_forward: dims is NULL");
  GP_REQUIRE(ctx, n_edges >= 0 && n_triplets >= 0, "gp_basis_forward: negative size");
  GP_REQUIRE(ctx, dims->cutoff > 0.f, "gp_basis_forward: cutoff must be positive");
  const int S = dims->num_spherical, R = dims->num_radial, p = dims->envelope_p;
  if (S < 1 || S > MAX_S || R < 1 || p < 1 || p > 16)
    return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_basis_forward: num_spherical=%d num_radial=%d p=%d unsupported", S, R, p);
  GP_HIP(ctx, hipSetDevice(ctx->device));
  hipStream_t st = ctx->stream;
  if (n_edges > 0 && (rbf || rad)) {
    GP_REQUIRE(ctx, dist, "gp_basis_forward: dist is NULL");
    if (dims->variant == GP_VARIANT_D) {
      if (R > MAX_R_BESSEL) return gp_fail(ctx, GP_UNSUPPORTED_DIMS, "gp_basis_forward: num_radial=%d > %d", R, MAX_R_BESSEL);
      bessel_table tab;
      make_bessel_table(S, R, (double)dims->cutoff, &tab);
      basis_edge_D_kernel<<<nblk(n_edges * (S + 1)), 256, 0, st>>>(dist, n_edges, S, R, p, (double)dims->cutoff, tab, rbf, rad);
      GP_LAUNCH_CHECK(ctx, "basis_edge_D_kernel");
    } else if (dims->variant == GP_VARIANT_G) {
      GP_REQUIRE(ctx, R >= 2, "gp_basis_forward: Gaussian basis needs num_radial >= 2");
      if (rbf) {
        basis_edge_G_kernel<<<nblk(n_edges * R), 256, 0, st>>>(dist, n_edges, R, p, (double)dims->cutoff, rbf);
        GP_LAUNCH_CHECK(ctx, "basis_edge_G_kernel");
      }
    } else {
      return gp_fail(ctx, GP_BAD_ARG, "gp_basis_forward: unknown variant %d", dims->variant);
    }
  }
  if (n_triplets > 0 && cos_alpha) {
    GP_REQUIRE(ctx, unit && idx_kj && idx_ji, "gp_basis_forward: unit/idx_kj/idx_ji is NULL");
    cos_alpha_kernel<<<nblk(n_triplets), 256, 0, st>>>(unit, idx_kj, idx_ji, n_triplets, cos_alpha);
    GP_LAUNCH_CHECK(ctx, "cos_alpha_kernel");
    if (cos_alpha_kj) {
      GP_REQUIRE(ctx, perm_kj, "gp_basis_forward: cos_alpha_kj needs perm_kj");
      permute_kernel<<<nblk(n_triplets), 256, 0, st>>>(cos_alpha, perm_kj, n_triplets, cos_alpha_kj);
      GP_LAUNCH_CHECK(ctx, "permute_kernel");
    }
    if (sbf) {
      GP_REQUIRE(ctx, rad && dims->variant == GP_VARIANT_D, "gp_basis_forward: sbf needs rad (variant D)");
      sbf_kernel<<<nblk(n_triplets * S), 256, 0, st>>>(rad, cos_alpha, idx_kj, n_triplets, S, R, sbf);
      GP_LAUNCH_CHECK(ctx, "sbf_kernel");
    }
  } else if (n_triplets > 0) {
    GP_REQUIRE(ctx, !cos_alpha_kj && !sbf, "gp_basis_forward: cos_alpha_kj/sbf need cos_alpha");
  }
  return GP_OK;
}

// dL/dd per edge from the gradients with respect to the Bessel radial basis and the radial part of the spherical
// basis (either may be NULL)
int gp_grad_dist_bessel(gp_ctx* ctx, const gp_dims* dims, const float* dist, const float* grad_rbf, const float* grad_rad,
                        int64_t n_edges, float* gd) {
  if (n_edges == 0) return GP_OK;
  const int S = dims->num_spherical, R = dims->num_radial;
  GP_REQUIRE(ctx, S >= 1 && S <= MAX_S && R >= 1 && R <= MAX_R_BESSEL, "grad_dist_bessel: basis sizes out of range");
  bessel_table tab;
  make_bessel_table(S, R, (double)dims->cutoff, &tab);
  grad_dist_bessel_kernel<<<(unsigned)((n_edges + 255) / 256), 256, 0, ctx->stream>>>(dist, grad_rbf, grad_rad, n_edges, S, R,
                                                                                      dims->envelope_p, (double)dims->cutoff, tab, gd);
  GP_LAUNCH_CHECK(ctx, "grad_dist_bessel_kernel");
  return GP_OK;
}
