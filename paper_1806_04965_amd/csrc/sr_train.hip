// Kernels of one training window (Sec. 3: rollout window of size W; App. A2: loss): the reverse sweep
// over the window for fp32 graphs.  Every kernel is a plain gather: one thread owns one output element
// and adds its terms in a fixed order, so gradients are reproducible from run to run; sums that are cut
// across workgroups go through partial results that a second kernel adds in index order.
// States and gradients are dense NHWC floats.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sr_internal.h"

namespace {

inline int grid_for(long long n, int per_block) {
  long long b = (n + per_block - 1) / per_block;
  return (int)(b < 1 ? 1 : b);
}

// softmax cross-entropy of one frame (App. A2): terms[b] = -log softmax(z_b)[label_b];
// dz[b][c] += (softmax(z_b)[c] - [c == label_b]) * scale.  One thread per sample.
__global__ void sr_ce_kernel(const float* __restrict__ z, const int32_t* __restrict__ labels, int B, int C, float scale,
                             float* __restrict__ terms, float* __restrict__ dz) {
  const int b = blockIdx.x * blockDim.x + threadIdx.x;
  if (b >= B) return;
  const float* zb = z + (size_t)b * C;
  float zmax = zb[0];
  for (int c = 1; c < C; ++c) zmax = fmaxf(zmax, zb[c]);
  float sum = 0.f;
  for (int c = 0; c < C; ++c) sum += expf(zb[c] - zmax);
  const float lse = zmax + logf(sum);
  int lab = labels[b];
  lab = lab < 0 ? 0 : (lab >= C ? C - 1 : lab);   // the host checks nothing on the device: stay in bounds
  terms[b] = lse - zb[lab];
  float* d = dz + (size_t)b * C;
  for (int c = 0; c < C; ++c) d[c] += (expf(zb[c] - lse) - (c == lab ? 1.f : 0.f)) * scale;
}

// loss = scale * sum of the n terms, added in index order by one thread per 1/256 of them, then a tree
__global__ void sr_sum_terms_kernel(const float* __restrict__ terms, int n, float scale, float* __restrict__ out) {
  __shared__ float part[256];
  float acc = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) acc += terms[i];
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[0] = part[0] * scale;
}

// rectifier: the gradient passes where the state is positive (x = max(a, 0): a > 0 exactly there)
__global__ void sr_relu_mask_kernel(float* __restrict__ d, const float* __restrict__ x, size_t n) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n && !(x[i] > 0.f)) d[i] = 0.f;
}

// db[c] += sum over the M pixels of d[m][c]; one workgroup per channel
__global__ void sr_bias_grad_kernel(const float* __restrict__ d, int M, int C, float* __restrict__ db) {
  __shared__ float part[256];
  const int c = blockIdx.x;
  float acc = 0.f;
  for (int m = threadIdx.x; m < M; m += 256) acc += d[(size_t)m * C + c];
  part[threadIdx.x] = acc;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) {
    if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
    __syncthreads();
  }
  if (threadIdx.x == 0) db[c] += part[0];
}

// adjoint of nearest up-sampling: out[b][h][w][c] = sum of the up x up block of d
__global__ void sr_pool_sum_kernel(const float* __restrict__ d, int B, int Hs, int Ws, int C, int up,
                                   float* __restrict__ out) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n = (size_t)B * Hs * Ws * C;
  if (i >= n) return;
  const int c = (int)(i % C);
  size_t r = i / C;
  const int w = (int)(r % Ws); r /= Ws;
  const int h = (int)(r % Hs);
  const int b = (int)(r / Hs);
  float acc = 0.f;
  for (int a = 0; a < up; ++a)
    for (int e = 0; e < up; ++e)
      acc += d[(((size_t)b * Hs * up + (size_t)h * up + a) * Ws * up + (size_t)w * up + e) * C + c];
  out[i] = acc;
}

// dx[b][h][w][ci] (+)= sum over taps (i, j) with h = ho*s + i - p, w = wo*s + j - p and over co of
// theta[i][j][ci][co] * dy[b][ho][wo][co]
__global__ void sr_dgrad_kernel(SrConvGeom q, const float* __restrict__ theta, const float* __restrict__ dy,
                                float* __restrict__ dx, int accumulate) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n = (size_t)q.B * q.H * q.W * q.Cin;
  if (idx >= n) return;
  const int ci = (int)(idx % q.Cin);
  size_t r = idx / q.Cin;
  const int w = (int)(r % q.W); r /= q.W;
  const int h = (int)(r % q.H);
  const int b = (int)(r / q.H);
  float acc = 0.f;
  for (int i = 0; i < q.kh; ++i) {
    const int th = h + q.pad - i;
    if (th < 0 || th % q.stride) continue;
    const int ho = th / q.stride;
    if (ho >= q.Ho) continue;
    for (int j = 0; j < q.kw; ++j) {
      const int tw = w + q.pad - j;
      if (tw < 0 || tw % q.stride) continue;
      const int wo = tw / q.stride;
      if (wo >= q.Wo) continue;
      const float* d = dy + (((size_t)b * q.Ho + ho) * q.Wo + wo) * q.Cout;
      const float* t = theta + ((size_t)(i * q.kw + j) * q.Cin + ci) * q.Cout;
      for (int co = 0; co < q.Cout; ++co) acc += t[co] * d[co];
    }
  }
  dx[idx] = accumulate ? dx[idx] + acc : acc;
}

// part[s][i][j][ci][co] = sum over the pixels m = (b, ho, wo) of slice s of
// x[b][ho*s + i - p][wo*s + j - p][ci] * dy[m][co]     (grid: weight elements x slices)
__global__ void sr_wgrad_kernel(SrConvGeom q, const float* __restrict__ x, const float* __restrict__ dy,
                                int m_per_slice, float* __restrict__ part) {
  const size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t nw = (size_t)q.kh * q.kw * q.Cin * q.Cout;
  if (k >= nw) return;
  const int co = (int)(k % q.Cout);
  size_t r = k / q.Cout;
  const int ci = (int)(r % q.Cin); r /= q.Cin;
  const int j = (int)(r % q.kw);
  const int i = (int)(r / q.kw);
  const int M = q.B * q.Ho * q.Wo;
  const int m0 = blockIdx.y * m_per_slice;
  const int m1 = m0 + m_per_slice < M ? m0 + m_per_slice : M;
  float acc = 0.f;
  for (int m = m0; m < m1; ++m) {
    const int wo = m % q.Wo;
    const int ho = (m / q.Wo) % q.Ho;
    const int b = m / (q.Wo * q.Ho);
    const int hi = ho * q.stride + i - q.pad, wi = wo * q.stride + j - q.pad;
    if (hi < 0 || hi >= q.H || wi < 0 || wi >= q.W) continue;
    acc += x[(((size_t)b * q.H + hi) * q.W + wi) * q.Cin + ci] * dy[(size_t)m * q.Cout + co];
  }
  part[(size_t)blockIdx.y * nw + k] = acc;
}

// dst[k] += part[0][k] + part[1][k] + ... in slice order
__global__ void sr_add_slices_kernel(const float* __restrict__ part, size_t n, int slices, float* __restrict__ dst) {
  const size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (k >= n) return;
  float acc = 0.f;
  for (int s = 0; s < slices; ++s) acc += part[(size_t)s * n + k];
  dst[k] += acc;
}

// mean over the pixels of one image: out[b][c]
__global__ void sr_gap_mean_kernel(const float* __restrict__ x, int B, int HW, int C, float* __restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= B * C) return;
  const int c = i % C, b = i / C;
  float acc = 0.f;
  for (int p = 0; p < HW; ++p) acc += x[((size_t)b * HW + p) * C + c];
  out[i] = acc / (float)HW;
}

// adjoint of the mean: dx[b][p][c] += dmean[b][c] / HW
__global__ void sr_gap_spread_kernel(const float* __restrict__ dmean, int B, int HW, int C, float* __restrict__ dx) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n = (size_t)B * HW * C;
  if (i >= n) return;
  const int c = (int)(i % C);
  const int b = (int)(i / ((size_t)HW * C));
  dx[i] += dmean[(size_t)b * C + c] / (float)HW;
}

// RMSprop: a <- rho a + (1 - rho) g^2;  theta <- theta - lr g / (sqrt(a) + eps)
__global__ void sr_rmsprop_kernel(float* __restrict__ theta, float* __restrict__ a, const float* __restrict__ g,
                                  size_t n, float lr, float rho, float eps) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const float gi = g[i];
  const float ai = rho * a[i] + (1.f - rho) * gi * gi;
  a[i] = ai;
  theta[i] -= lr * gi / (sqrtf(ai) + eps);
}

}  // namespace

hipError_t sr_train_rmsprop(hipStream_t s, float* theta, float* a, const float* g, size_t n, float lr, float rho,
                            float eps) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(sr_rmsprop_kernel, dim3(grid_for((long long)n, 256)), dim3(256), 0, s, theta, a, g, n, lr, rho, eps);
  return hipGetLastError();
}

hipError_t sr_train_ce(hipStream_t s, const float* z, const int32_t* labels, int B, int C, float scale, float* terms,
                       float* dz) {
  hipLaunchKernelGGL(sr_ce_kernel, dim3(grid_for(B, 64)), dim3(64), 0, s, z, labels, B, C, scale, terms, dz);
  return hipGetLastError();
}

hipError_t sr_train_sum_terms(hipStream_t s, const float* terms, int n, float scale, float* out) {
  hipLaunchKernelGGL(sr_sum_terms_kernel, dim3(1), dim3(256), 0, s, terms, n, scale, out);
  return hipGetLastError();
}

hipError_t sr_train_relu_mask(hipStream_t s, float* d, const float* x, size_t n) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(sr_relu_mask_kernel, dim3(grid_for((long long)n, 256)), dim3(256), 0, s, d, x, n);
  return hipGetLastError();
}

hipError_t sr_train_bias_grad(hipStream_t s, const float* d, int M, int C, float* db) {
  hipLaunchKernelGGL(sr_bias_grad_kernel, dim3(C), dim3(256), 0, s, d, M, C, db);
  return hipGetLastError();
}

hipError_t sr_train_pool_sum(hipStream_t s, const float* d, int B, int Hs, int Ws, int C, int up, float* out) {
  const long long n = (long long)B * Hs * Ws * C;
  hipLaunchKernelGGL(sr_pool_sum_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, d, B, Hs, Ws, C, up, out);
  return hipGetLastError();
}

hipError_t sr_train_dgrad(hipStream_t s, const SrConvGeom& q, const float* theta, const float* dy, float* dx,
                          int accumulate) {
  const long long n = (long long)q.B * q.H * q.W * q.Cin;
  hipLaunchKernelGGL(sr_dgrad_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, q, theta, dy, dx, accumulate);
  return hipGetLastError();
}

int sr_train_wgrad_slices(const SrConvGeom& q) {
  const long long nw = (long long)q.kh * q.kw * q.Cin * q.Cout;
  const long long M = (long long)q.B * q.Ho * q.Wo;
  long long want = (2048LL * 256 + nw - 1) / nw;   // about 2048 workgroups in all
  if (want > SR_TRAIN_MAX_SLICES) want = SR_TRAIN_MAX_SLICES;
  if (want > M) want = M;
  return (int)(want < 1 ? 1 : want);
}

hipError_t sr_train_wgrad(hipStream_t s, const SrConvGeom& q, const float* x, const float* dy, float* part,
                          float* dtheta) {
  const long long nw = (long long)q.kh * q.kw * q.Cin * q.Cout;
  const int M = q.B * q.Ho * q.Wo;
  const int slices = sr_train_wgrad_slices(q);
  const int per = (M + slices - 1) / slices;
  const int used = (M + per - 1) / per;
  hipLaunchKernelGGL(sr_wgrad_kernel, dim3(grid_for(nw, 256), used), dim3(256), 0, s, q, x, dy, per, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(sr_add_slices_kernel, dim3(grid_for(nw, 256)), dim3(256), 0, s, part, (size_t)nw, used, dtheta);
  return hipGetLastError();
}

hipError_t sr_train_gap_mean(hipStream_t s, const float* x, int B, int HW, int C, float* out) {
  hipLaunchKernelGGL(sr_gap_mean_kernel, dim3(grid_for((long long)B * C, 256)), dim3(256), 0, s, x, B, HW, C, out);
  return hipGetLastError();
}

hipError_t sr_train_gap_spread(hipStream_t s, const float* dmean, int B, int HW, int C, float* dx) {
  const long long n = (long long)B * HW * C;
  hipLaunchKernelGGL(sr_gap_spread_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, dmean, B, HW, C, dx);
  return hipGetLastError();
}
