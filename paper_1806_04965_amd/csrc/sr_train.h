// Launchers of the training-window kernels (sr_train.hip), used by sr_train_host.cpp.
#ifndef SR_TRAIN_H_
#define SR_TRAIN_H_

#include <hip/hip_runtime_api.h>
#include <stddef.h>
#include <stdint.h>

// ---------------------------------------------------------------------------
// training window (fp32 graphs): reverse sweep over the rollout window (Sec. 3; loss of App. A2)
// ---------------------------------------------------------------------------
struct SrConvGeom {   // y[b][ho][wo][co] = sum x[b][ho*stride + i - pad][wo*stride + j - pad][ci] * theta[i][j][ci][co]
  int B, H, W, Cin, Ho, Wo, Cout, kh, kw, stride, pad;
  // state gradient of a strided edge, one launch per phase (ph, pw) of the source pixels: rows are the pixels
  // h = hh*stride + ph, w = ww*stride + pw of a Hp x Wp grid, which pair only with the taps i = ti0 + a*stride,
  // j = tj0 + c*stride (a < nti, c < ntj).  Stride 1: one phase, the whole image, all taps.
  int ph, pw, Hp, Wp, ti0, tj0, nti, ntj;
  // divisions by Wo, Ho*Wo, Cout, Cin and kw as multiply-high, add, shift (exact for dividends below 2^31);
  // filled by the launchers of the tiled kernels
  uint32_t mul_wo, sh_wo, mul_howo, sh_howo, mul_cout, sh_cout, mul_cin, sh_cin, mul_kw, sh_kw;
  int tall_from;   // host side only: workgroups from which a launch takes the taller tile shape
};
#define SR_TRAIN_TILED_MIN_MACS 1.0e6   // smaller contractions stay on the one-thread-per-output kernels
#define SR_TRAIN_MAX_SLICES 256  // a weight gradient's pixel sum is cut into at most this many partial sums
hipError_t sr_train_ce(hipStream_t s, const float* z, const int32_t* labels, int B, int C, float scale, float* terms,
                       float* dz);
hipError_t sr_train_sum_terms(hipStream_t s, const float* terms, int n, float scale, float* out);
// d <- d * m * sigma'(a) for x = m * sigma(a) (m may be null)
hipError_t sr_train_act_grad(hipStream_t s, float* d, const float* x, const float* m, size_t n, int act);
int sr_train_bias_slices(int M);
// part: sr_train_bias_slices(M) * C floats of scratch; db += the gradient
hipError_t sr_train_bias_grad(hipStream_t s, const float* d, int M, int C, float* part, float* db);
hipError_t sr_train_pool_sum(hipStream_t s, const float* d, int B, int Hs, int Ws, int C, int up, float* out);
hipError_t sr_train_dgrad(hipStream_t s, const SrConvGeom& q, const float* theta, const float* dy, float* dx,
                          int accumulate);
// forward of one edge into y (dense [B][Ho][Wo][Cout]); accumulate: y += the edge's result
hipError_t sr_train_fwd(hipStream_t s, const SrConvGeom& q, const float* x, const float* theta, float* y,
                        int accumulate);
int sr_train_fwd_is_tiled(const SrConvGeom& q);   // would sr_train_fwd take this edge to the tiled kernel?
hipError_t sr_train_upsample_add(hipStream_t s, const float* y, int B, int H, int W, int C, int up, float* dst,
                                 int accumulate);
hipError_t sr_train_bias_act(hipStream_t s, float* a, const float* bias, const float* m, int C, size_t n, int act);
int sr_train_wgrad_slices(const SrConvGeom& q);
// part: sr_train_wgrad_slices(q) * (number of weights) floats of scratch; dtheta += the gradient
hipError_t sr_train_wgrad(hipStream_t s, const SrConvGeom& q, const float* x, const float* dy, float* part,
                          float* dtheta);
hipError_t sr_train_gap_mean(hipStream_t s, const float* x, int B, int HW, int C, float* out);
hipError_t sr_train_rmsprop(hipStream_t s, float* theta, float* a, const float* g, size_t n, float lr, float rho,
                            float eps);
hipError_t sr_train_gap_spread(hipStream_t s, const float* dmean, int B, int HW, int C, float* dx);

#endif  // SR_TRAIN_H_
