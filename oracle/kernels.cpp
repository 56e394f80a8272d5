// CPU checker for the task kernels -- TEST INFRASTRUCTURE ONLY.
//
// Plain, serial, obviously-correct definitions of what each GPU task computes.
// Nothing in the product path may call into this file; it shares no code with
// the HIP library.  Floating-point results are accumulated in double unless a
// function says otherwise.  Every function is the textbook definition of its
// result written out as loops; there is no blocking, fusion or reordering.
//
// The paper (Sec. V-A "Workloads") runs third-party stencil, dense-algebra,
// neural-network and graph jobs; the kernels below are the synthetic stand-ins
// for those job classes, so each definition here is the mathematical one, not
// a passage of the paper.
#include <cstdint>
#include <cstring>
#include <cmath>
#include <vector>

extern "C" {

// ---- 5-point Jacobi sweep, zero Dirichlet ring ---------------------------
// v[i][j] = ((u[i-1][j] + u[i+1][j]) + (u[i][j-1] + u[i][j+1])) / 4 on the
// interior 1..n-2, ring cells keep their value.  `u` is n*n row-major and is
// overwritten with the state after `iters` sweeps.  Double precision.
void orc_jacobi_f64(double* u, uint32_t n, uint32_t iters) {
  if (n < 3) return;
  std::vector<double> tmp(u, u + (size_t)n * n);
  double* a = u;
  double* b = tmp.data();
  for (uint32_t t = 0; t < iters; ++t) {
    for (uint32_t i = 1; i + 1 < n; ++i)
      for (uint32_t j = 1; j + 1 < n; ++j)
        b[(size_t)i * n + j] = 0.25 * ((a[(size_t)(i - 1) * n + j] + a[(size_t)(i + 1) * n + j]) +
                                       (a[(size_t)i * n + j - 1] + a[(size_t)i * n + j + 1]));
    double* s = a; a = b; b = s;
  }
  if (a != u) std::memcpy(u, a, sizeof(double) * (size_t)n * n);
}

// Same sweep evaluated in single precision with the association fixed as
// (north + south) + (west + east), then * 0.25f.  Used for the bit-exact
// comparison: every operation is a correctly rounded IEEE fp32 add or an
// exact scaling, so any conforming evaluation gives the same bits.
void orc_jacobi_f32(float* u, uint32_t n, uint32_t iters) {
  if (n < 3) return;
  std::vector<float> tmp(u, u + (size_t)n * n);
  float* a = u;
  float* b = tmp.data();
  for (uint32_t t = 0; t < iters; ++t) {
    for (uint32_t i = 1; i + 1 < n; ++i)
      for (uint32_t j = 1; j + 1 < n; ++j) {
        volatile float ns = a[(size_t)(i - 1) * n + j] + a[(size_t)(i + 1) * n + j];
        volatile float we = a[(size_t)i * n + j - 1] + a[(size_t)i * n + j + 1];
        volatile float s = ns + we;
        b[(size_t)i * n + j] = 0.25f * s;
      }
    float* s = a; a = b; b = s;
  }
  if (a != u) std::memcpy(u, a, sizeof(float) * (size_t)n * n);
}

// ---- GEMM: C[i][j] = sum_k A[i][k] * B[k][j], row-major ------------------
// fp32 operands, exact products and sums carried in double, result in double.
void orc_gemm_f32(const float* A, const float* B, double* C, uint32_t m, uint32_t n, uint32_t k) {
  for (uint32_t i = 0; i < m; ++i)
    for (uint32_t j = 0; j < n; ++j) {
      double acc = 0.0;
      for (uint32_t p = 0; p < k; ++p)
        acc += (double)A[(size_t)i * k + p] * (double)B[(size_t)p * n + j];
      C[(size_t)i * n + j] = acc;
    }
}

// sum_k |A[i][k]| * |B[k][j]| -- the denominator of the componentwise error bound.
void orc_gemm_abs_f32(const float* A, const float* B, double* C, uint32_t m, uint32_t n, uint32_t k) {
  for (uint32_t i = 0; i < m; ++i)
    for (uint32_t j = 0; j < n; ++j) {
      double acc = 0.0;
      for (uint32_t p = 0; p < k; ++p)
        acc += std::fabs((double)A[(size_t)i * k + p]) * std::fabs((double)B[(size_t)p * n + j]);
      C[(size_t)i * n + j] = acc;
    }
}

// Selected entries only: out[s] = sum_k A[rows[s]][k]*B[k][cols[s]] and the
// matching |A||B| entry.  Lets full-size products be checked entry by entry.
void orc_gemm_f32_entries(const float* A, const float* B, uint32_t n, uint32_t k,
                          const uint32_t* rows, const uint32_t* cols, uint32_t count,
                          double* out, double* out_abs) {
  for (uint32_t s = 0; s < count; ++s) {
    double acc = 0.0, acca = 0.0;
    const float* a = A + (size_t)rows[s] * k;
    for (uint32_t p = 0; p < k; ++p) {
      double t = (double)a[p] * (double)B[(size_t)p * n + cols[s]];
      acc += t;
      acca += std::fabs(t);
    }
    out[s] = acc;
    if (out_abs) out_abs[s] = acca;
  }
}

static inline double bf16_to_double(uint16_t h) {
  uint32_t w = (uint32_t)h << 16;
  float f;
  std::memcpy(&f, &w, 4);
  return (double)f;
}

// round a double to the nearest bfloat16 (ties to even) via fp32: the value is
// first rounded to fp32 (as a device storing an fp32 accumulator would hold
// it) and then to bf16.
static inline uint16_t f32_to_bf16(float f) {
  uint32_t w;
  std::memcpy(&w, &f, 4);
  if ((w & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((w >> 16) | 0x40);  // NaN
  uint32_t r = ((w >> 16) & 1u) + 0x7fffu;
  return (uint16_t)((w + r) >> 16);
}

// bf16 operands (bit patterns), products/sums in double, result in double.
void orc_gemm_bf16(const uint16_t* A, const uint16_t* B, double* C, uint32_t m, uint32_t n, uint32_t k) {
  for (uint32_t i = 0; i < m; ++i)
    for (uint32_t j = 0; j < n; ++j) {
      double acc = 0.0;
      for (uint32_t p = 0; p < k; ++p)
        acc += bf16_to_double(A[(size_t)i * k + p]) * bf16_to_double(B[(size_t)p * n + j]);
      C[(size_t)i * n + j] = acc;
    }
}

void orc_gemm_bf16_entries(const uint16_t* A, const uint16_t* B, uint32_t n, uint32_t k,
                           const uint32_t* rows, const uint32_t* cols, uint32_t count, double* out) {
  for (uint32_t s = 0; s < count; ++s) {
    double acc = 0.0;
    for (uint32_t p = 0; p < k; ++p)
      acc += bf16_to_double(A[(size_t)rows[s] * k + p]) * bf16_to_double(B[(size_t)p * n + cols[s]]);
    out[s] = acc;
  }
}

// ---- 3x3 convolution + ReLU, pad 1, stride s ------------------------------
// x: N,H,W,C (bf16 bits); w: K,3,3,C (bf16 bits); y: N,Ho,Wo,K in double with
// Ho = (H + 2 - 3)/s + 1.  y = max(0, sum_{r,t,c} x[n][oh*s-1+r][ow*s-1+t][c] * w[k][r][t][c]);
// taps that fall outside the image contribute zero.
void orc_conv3x3_relu(const uint16_t* x, const uint16_t* w, double* y, uint32_t N, uint32_t H,
                      uint32_t W, uint32_t C, uint32_t K, uint32_t stride) {
  uint32_t Ho = (H + 2 - 3) / stride + 1, Wo = (W + 2 - 3) / stride + 1;
  for (uint32_t nb = 0; nb < N; ++nb)
    for (uint32_t oh = 0; oh < Ho; ++oh)
      for (uint32_t ow = 0; ow < Wo; ++ow)
        for (uint32_t kk = 0; kk < K; ++kk) {
          double acc = 0.0;
          for (uint32_t r = 0; r < 3; ++r)
            for (uint32_t t = 0; t < 3; ++t) {
              int64_t ih = (int64_t)oh * stride - 1 + r, iw = (int64_t)ow * stride - 1 + t;
              if (ih < 0 || iw < 0 || ih >= (int64_t)H || iw >= (int64_t)W) continue;
              const uint16_t* xp = x + (((size_t)nb * H + ih) * W + iw) * C;
              const uint16_t* wp = w + (((size_t)kk * 3 + r) * 3 + t) * C;
              for (uint32_t c = 0; c < C; ++c) acc += bf16_to_double(xp[c]) * bf16_to_double(wp[c]);
            }
          y[(((size_t)nb * Ho + oh) * Wo + ow) * K + kk] = acc > 0.0 ? acc : 0.0;
        }
}

// double activations -> bf16 bit patterns (via fp32, nearest even): the
// rounding applied between the layers of the network.
void orc_round_bf16(const double* x, uint16_t* out, uint64_t count) {
  for (uint64_t i = 0; i < count; ++i) out[i] = f32_to_bf16((float)x[i]);
}

// ---- BFS levels on a CSR graph -------------------------------------------
// level[v] = number of edges on a shortest path source -> v, -1 if unreachable.
void orc_bfs(const int32_t* row_ptr, const int32_t* col_idx, uint32_t n, uint32_t source,
             int32_t* level) {
  for (uint32_t v = 0; v < n; ++v) level[v] = -1;
  if (source >= n) return;
  std::vector<uint32_t> queue;
  queue.reserve(n);
  queue.push_back(source);
  level[source] = 0;
  for (size_t head = 0; head < queue.size(); ++head) {
    uint32_t u = queue[head];
    for (int32_t e = row_ptr[u]; e < row_ptr[u + 1]; ++e) {
      int32_t v = col_idx[e];
      if (level[v] < 0) {
        level[v] = level[u] + 1;
        queue.push_back((uint32_t)v);
      }
    }
  }
}

}  // extern "C"
