// Kernels of one training window (Sec. 3: rollout window of size W; App. A2: loss) for fp32 graphs: forward
// pass and reverse sweep.  Contractions with enough work run as tiles on the fp32 matrix cores, the rest as
// plain gathers (one thread owns one output element).  Every sum is taken in a fixed order, so gradients are
// reproducible from run to run; sums that are cut across workgroups go through partial results that a second
// kernel adds in a fixed order.  States and gradients are dense NHWC floats.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <algorithm>

#include "sr_internal.h"
#include "sr_train.h"

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

// gradient through the node map x = m * sigma(a): for the rectifier the gradient passes where the state is positive
// (x = m * max(a, 0) > 0 exactly where a > 0 and m > 0); m: dropout multipliers or null
__global__ void sr_act_grad_kernel(float* __restrict__ d, const float* __restrict__ x, const float* __restrict__ m,
                                   size_t n, int act) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = d[i];
  if (act == 1 && !(x[i] > 0.f)) v = 0.f;
  if (m) v *= m[i];
  d[i] = v;
}

// db[c] += sum over the M pixels of d[m][c]; one workgroup per channel (few pixels: one launch, no scratch)
__global__ void sr_bias_grad_small_kernel(const float* __restrict__ d, int M, int C, float* __restrict__ db) {
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

// part[s][c] = sum over the pixels m of slice s of d[m][c]: a workgroup takes 64 channels x one slice of pixels,
// four pixel lanes per channel (each adds every fourth pixel of the slice in order, then the four in order)
__global__ void sr_bias_grad_kernel(const float* __restrict__ d, int M, int C, int m_per_slice, float* __restrict__ part) {
  __shared__ float lanes[4][64];
  const int c = blockIdx.x * 64 + (threadIdx.x & 63), pl = threadIdx.x >> 6;
  const int m0 = blockIdx.y * m_per_slice;
  const int m1 = min(M, m0 + m_per_slice);
  float acc = 0.f;
  if (c < C)
    for (int m = m0 + pl; m < m1; m += 32) {   // eight loads in flight at a time, added in order
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = (m + 4 * u < m1) ? d[(size_t)(m + 4 * u) * C + c] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) acc += v[u];
    }
  lanes[pl][threadIdx.x & 63] = acc;
  __syncthreads();
  if (pl == 0 && c < C)
    part[(size_t)blockIdx.y * C + c] = ((lanes[0][threadIdx.x] + lanes[1][threadIdx.x]) + lanes[2][threadIdx.x]) + lanes[3][threadIdx.x];
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

// dst[k] += the sum over the slices of part[s][k], in a fixed order: a workgroup takes 64 elements, four slice
// lanes per element (each adds every fourth slice in order, eight loads in flight at a time; then the four in order)
__global__ void sr_add_slices_kernel(const float* __restrict__ part, size_t n, int slices, float* __restrict__ dst) {
  __shared__ float lanes[4][64];
  const size_t k = (size_t)blockIdx.x * 64 + (threadIdx.x & 63);
  const int pl = threadIdx.x >> 6;
  float acc = 0.f;
  if (k < n)
    for (int s0 = pl; s0 < slices; s0 += 32) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = (s0 + 4 * u < slices) ? part[(size_t)(s0 + 4 * u) * n + k] : 0.f;
#pragma unroll
      for (int u = 0; u < 8; ++u) acc += v[u];
    }
  lanes[pl][threadIdx.x & 63] = acc;
  __syncthreads();
  if (pl == 0 && k < n)
    dst[k] += ((lanes[0][threadIdx.x] + lanes[1][threadIdx.x]) + lanes[2][threadIdx.x]) + lanes[3][threadIdx.x];
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

// ---------------------------------------------------------------------------
// The two gradient contractions of a convolution as tiled matrix products on the fp32 matrix cores
// (v_mfma_f32_32x32x2_f32): C[i][j] (+)= sum_r A[i][r] * B[r][j], operands gathered on the fly.
//   state gradient  (MODE 0): i = source pixel (b, h, w), j = ci, r = (tap, co);
//                             A = dy at the output pixel that tap pairs with (h, w), B = theta[tap][j][co]
//   forward         (MODE 2): i = output pixel m = (b, ho, wo), j = co, r = (tap, ci);
//                             A = x at the source pixel that tap pairs with m, B = theta[tap][ci][j]
//   weight gradient (MODE 1): i = (tap, ci), j = co, r = output pixel m = (b, ho, wo);
//                             A = x at the source pixel that tap pairs with m, B = dy[m][j]
// One workgroup (4 waves) owns a TI x TJ tile of C; the waves lie WJN along j and 4 / WJN along i, each
// with MI x MJ MFMA tiles of 32 x 32.  The reduction runs in steps of 16 through LDS (A and B tiles stored
// r-major, so a wave's operand read is 32 consecutive floats); blockIdx.z cuts the reduction into slices
// (weight gradient: partial sums that a second kernel adds in slice order).  Every sum has a fixed order
// whatever the tile shape: same call, same bits.
typedef float sr_f32x16 __attribute__((ext_vector_type(16)));
__device__ const float sr_zero_word = 0.f;   // what an operand element outside its tensor reads

// n / d for n < 2^31 with the pair the host made for d (Granlund & Montgomery: l = ceil(log2 d),
// m = floor(2^32 (2^l - d) / d) + 1, q = (mulhi(m, n) + n) >> l; no overflow while n < 2^31)
__device__ __forceinline__ int sr_fdiv(int n, uint32_t mul, uint32_t sh) {
  return (int)((__umulhi((uint32_t)n, mul) + (uint32_t)n) >> sh);
}
// the pair for d >= 1, made on the device (a phase's own divisors)
__device__ __forceinline__ void sr_fdiv_make(uint32_t d, uint32_t* mul, uint32_t* sh) {
  const uint32_t l = (d <= 1) ? 0u : 32u - (uint32_t)__clz((int)(d - 1));
  *mul = (uint32_t)((((1ull << l) - d) << 32) / d + 1);
  *sh = l;
}
#define SR_GT 128   // edge of the largest tile
#define SR_GR 16    // reduction step

// State gradient of a stride-s edge: grid plane z is the phase (ph, pw) of the source pixels.  A stride-s edge
// pairs a pixel only with the taps of its own residues, so each phase is a contraction of its own (without the
// split all but 1/s^2 of the products would be zeros).  Fills the phase's fields of q and returns its row count
// I and reduction length R (the launch is sized for phase (0, 0), the largest).
__device__ __forceinline__ void sr_phase_of_plane(SrConvGeom& q, int z, int* I, int* R) {
  q.ph = z / q.stride;
  q.pw = z % q.stride;
  q.Hp = (q.H - q.ph + q.stride - 1) / q.stride;
  q.Wp = (q.W - q.pw + q.stride - 1) / q.stride;
  q.ti0 = (q.ph + q.pad) % q.stride;
  q.tj0 = (q.pw + q.pad) % q.stride;
  q.nti = q.ti0 < q.kh ? (q.kh - q.ti0 + q.stride - 1) / q.stride : 0;
  q.ntj = q.tj0 < q.kw ? (q.kw - q.tj0 + q.stride - 1) / q.stride : 0;
  *I = q.B * max(q.Hp, 0) * max(q.Wp, 0);
  *R = q.nti * q.ntj * q.Cout;
}

// A wave's accumulators into C (row-major, J columns; MODE 0: a row of the phase grid goes to its source pixel).
// Register v of lane l holds row 8 * (v / 4) + 4 * (l / 32) + v % 4 of an MFMA tile's 32, column l % 32.
template <int MODE, int MI, int MJ>
__device__ __forceinline__ void sr_store_tile(const sr_f32x16 (&acc)[MI][MJ], const SrConvGeom& q, float* out, int i_wave,
                                              int j_wave, int lane, int I, int J, uint32_t mul_wp, uint32_t sh_wp,
                                              uint32_t mul_hpwp, uint32_t sh_hpwp, int accumulate) {
#pragma unroll
  for (int x = 0; x < MI; ++x)
#pragma unroll
    for (int y = 0; y < MJ; ++y)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int i = i_wave + x * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int j = j_wave + y * 32 + (lane & 31);
        if (i < I && j < J) {
          size_t row = (size_t)i;
          if (MODE == 0) {
            const int b = sr_fdiv(i, mul_hpwp, sh_hpwp), rem = i - b * (q.Wp * q.Hp);
            const int hh = sr_fdiv(rem, mul_wp, sh_wp), ww = rem - hh * q.Wp;
            row = ((size_t)b * q.H + hh * q.stride + q.ph) * q.W + ww * q.stride + q.pw;
          }
          float* dst = out + row * J + j;
          *dst = accumulate ? *dst + acc[x][y][v] : acc[x][y][v];
        }
      }
}

template <int MODE, int TI, int TJ, int WJN>
__global__ __launch_bounds__(256, 2) void sr_conv_gemm_kernel(SrConvGeom q, const float* __restrict__ pa,
                                                              const float* __restrict__ pb, float* __restrict__ pc,
                                                              int I, int J, int R, int r_per_slice, int accumulate) {
  constexpr int WIN = 4 / WJN;                                // waves along i
  constexpr int MI = TI / (32 * WIN), MJ = TJ / (32 * WJN);   // MFMA tiles of a wave
  constexpr int NA = TI / 16, NB = TJ / 16;                   // operand elements a thread gathers per step
  static_assert(MI >= 1 && MJ >= 1 && MI * 32 * WIN == TI && MJ * 32 * WJN == TJ, "tile shape");
  __shared__ float As[SR_GR][TI + 4];
  __shared__ float Bs[SR_GR][TJ + 4];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int i0 = blockIdx.x * TI, j0 = blockIdx.y * TJ;
  if (MODE == 0) {
    sr_phase_of_plane(q, blockIdx.z, &I, &R);
    r_per_slice = R;
    if (i0 >= I || (R == 0 && accumulate)) return;   // the whole workgroup: this phase has fewer pixels, or no tap reaches it
  }
  const int r_begin = (MODE == 1) ? blockIdx.z * r_per_slice : 0;
  const int r_end = min(R, r_begin + r_per_slice);
  const int wi = wave / WJN, wj = wave % WJN;

  // Operand addresses are byte offsets in 32 bits (the launchers send only tensors below 2^30 bytes here), split
  // into a part fixed per thread and row, made once, and a part per reduction step, made once per thread and
  // step; an element costs one add for its address and two compares for its bounds.  Every load is unconditional:
  // no branch per element.
  constexpr int FAR = 1 << 20;      // added to a coordinate, puts it out of every range
  // MODE 0, 2: A is gathered r-fastest (r = t % 16, rows t / 16 + 16 n)
  // MODE 1:    A and B are gathered i- / j-fastest (i = t % TI, r = t / TI + (256 / TI) n; B alike with TJ)
  int ah[NA], aw[NA], aoff[NA];     // MODE 0, 2: per row, the coordinates the taps move and the byte offset at tap 0
  int ati = 0, atj = 0, a1off = 0;  // MODE 1: tap and byte offset of the thread's A row
  uint32_t mul_wp = 0, sh_wp = 0, mul_hpwp = 0, sh_hpwp = 0, mul_ntj = 0, sh_ntj = 0;   // MODE 0: the phase's divisors
  if (MODE == 2) {
#pragma unroll
    for (int n = 0; n < NA; ++n) {
      const int i = i0 + (t >> 4) + 16 * n;
      const int b = sr_fdiv(i, q.mul_howo, q.sh_howo), rem = i - b * (q.Ho * q.Wo);
      const int ho = sr_fdiv(rem, q.mul_wo, q.sh_wo), wo = rem - ho * q.Wo;
      // top-left corner of the output pixel's window in the source
      ah[n] = (i < I) ? ho * q.stride - q.pad : FAR;
      aw[n] = wo * q.stride - q.pad;
      aoff[n] = (((b * q.H + ho * q.stride - q.pad) * q.W + aw[n]) * q.Cin) * 4;
    }
  } else if (MODE == 0) {
    const int lgs = (q.stride == 1) ? 0 : (q.stride == 2 ? 1 : (q.stride == 4 ? 2 : -1));   // strides 1, 2, 4 by shifts
    sr_fdiv_make((uint32_t)max(q.Wp, 1), &mul_wp, &sh_wp);
    sr_fdiv_make((uint32_t)max(q.Wp * q.Hp, 1), &mul_hpwp, &sh_hpwp);
    sr_fdiv_make((uint32_t)max(q.ntj, 1), &mul_ntj, &sh_ntj);
#pragma unroll
    for (int n = 0; n < NA; ++n) {
      const int i = i0 + (t >> 4) + 16 * n;
      const int b = sr_fdiv(i, mul_hpwp, sh_hpwp), rem = i - b * (q.Wp * q.Hp);
      const int hh = sr_fdiv(rem, mul_wp, sh_wp), ww = rem - hh * q.Wp;
      // source pixel (hh*s + ph, ww*s + pw) pairs through the phase's tap (a, c) with output pixel (hq - a, wq - c):
      // (h + pad - ti0) is a multiple of the stride and not negative
      const int hn = hh * q.stride + q.ph + q.pad - q.ti0, wn = ww * q.stride + q.pw + q.pad - q.tj0;
      const int hq = lgs >= 0 ? hn >> lgs : hn / q.stride, wq = lgs >= 0 ? wn >> lgs : wn / q.stride;
      ah[n] = (i < I) ? hq : -FAR;
      aw[n] = wq;
      aoff[n] = (((b * q.Ho + hq) * q.Wo + wq) * q.Cout) * 4;
    }
  } else {
    const int i = i0 + (t % TI);
    const int tap = sr_fdiv(i, q.mul_cin, q.sh_cin), ci = i - tap * q.Cin;
    ati = sr_fdiv(tap, q.mul_kw, q.sh_kw);
    atj = tap - ati * q.kw;
    a1off = (((ati * q.W + atj) * q.Cin) + ci) * 4;
    if (i >= I) ati = FAR;
  }
  // B: byte offset of the thread's first element at reduction index 0, and whether its column exists
  int boff = 0;
  bool b_col_ok = false;
  if (MODE == 0) {
    const int j = j0 + (t >> 4);
    boff = j * q.Cout * 4;                      // theta[tap][j][co]: + 16 n Cout per element, + (tap Cin Cout + co) per step
  } else {
    const int j = j0 + (t % TJ);
    b_col_ok = j < J;
    boff = ((t / TJ) * q.Cout + j) * 4;         // [r][j] with Cout columns: + (256 / TJ) n Cout per element, + rs Cout per step
  }

  sr_f32x16 acc[MI][MJ];
#pragma unroll
  for (int x = 0; x < MI; ++x)
#pragma unroll
    for (int y = 0; y < MJ; ++y)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;

  // an element out of range is read from a word that holds zero: no use of a loaded value before the step that
  // stores it (a select after the load would wait for the load right where it was issued)
  auto at = [](const float* base, bool ok, int byte_off) {
    typedef const __attribute__((address_space(1))) float* global_ptr;   // both are global memory: say so
    const global_ptr p = ok ? (global_ptr)((const char*)base + (uint32_t)byte_off) : (global_ptr)&sr_zero_word;
    return *p;
  };
  // the operands of one reduction step, from global memory into registers
  auto gather = [&](int rs, float (&va)[NA], float (&vb)[NB]) {
    if (MODE == 2) {
      const int r = rs + (t & 15);
      const int tap = sr_fdiv(r, q.mul_cin, q.sh_cin), ci = r - tap * q.Cin;
      int ti = sr_fdiv(tap, q.mul_kw, q.sh_kw);
      const int tj = tap - ti * q.kw;
      const int toff = ((ti * q.W + tj) * q.Cin + ci) * 4;
      if (r >= r_end) ti = FAR;
#pragma unroll
      for (int n = 0; n < NA; ++n) {
        const bool ok = (unsigned)(ah[n] + ti) < (unsigned)q.H && (unsigned)(aw[n] + tj) < (unsigned)q.W;
        va[n] = at(pa, ok, aoff[n] + toff);
      }
      const int sb = boff + rs * q.Cout * 4;
#pragma unroll
      for (int n = 0; n < NB; ++n) {
        const bool okb = b_col_ok && rs + t / TJ + (256 / TJ) * n < r_end;
        vb[n] = at(pb, okb, sb + n * (256 / TJ) * q.Cout * 4);
      }
    } else if (MODE == 0) {
      const int r = rs + (t & 15);
      const bool r_ok = r < r_end;
      const int vt = sr_fdiv(r, q.mul_cout, q.sh_cout), co = r - vt * q.Cout;   // vt: index among the phase's taps
      int vi = sr_fdiv(vt, mul_ntj, sh_ntj);
      const int vj = vt - vi * q.ntj;
      const int tap = (q.ti0 + vi * q.stride) * q.kw + q.tj0 + vj * q.stride;
      const int toff = (co - (vi * q.Wo + vj) * q.Cout) * 4;
      if (!r_ok) vi = 2 * FAR;
#pragma unroll
      for (int n = 0; n < NA; ++n) {
        const bool ok = (unsigned)(ah[n] - vi) < (unsigned)q.Ho && (unsigned)(aw[n] - vj) < (unsigned)q.Wo;
        va[n] = at(pa, ok, aoff[n] + toff);
      }
      const int sb = boff + (tap * q.Cin * q.Cout + co) * 4;
#pragma unroll
      for (int n = 0; n < NB; ++n) {
        const bool okb = r_ok && j0 + (t >> 4) + 16 * n < J;
        vb[n] = at(pb, okb, sb + n * 16 * q.Cout * 4);
      }
    } else {
      // a wave's threads share their reduction indices: the pixel's decoding runs on the scalar unit
      const int rl = __builtin_amdgcn_readfirstlane(rs + t / TI);
#pragma unroll
      for (int n = 0; n < NA; ++n) {
        const int r = rl + (256 / TI) * n;
        const int b = sr_fdiv(r, q.mul_howo, q.sh_howo), rem = r - b * (q.Ho * q.Wo);
        const int ho = sr_fdiv(rem, q.mul_wo, q.sh_wo), wo = rem - ho * q.Wo;
        const int h0 = (r < r_end) ? ho * q.stride - q.pad : FAR, w0 = wo * q.stride - q.pad;
        const int sbase = (((b * q.H + ho * q.stride - q.pad) * q.W + w0) * q.Cin) * 4;
        const bool ok = (unsigned)(h0 + ati) < (unsigned)q.H && (unsigned)(w0 + atj) < (unsigned)q.W;
        va[n] = at(pa, ok, sbase + a1off);
      }
      const int sb = boff + rs * q.Cout * 4;
#pragma unroll
      for (int n = 0; n < NB; ++n) {
        const bool okb = b_col_ok && rs + t / TJ + (256 / TJ) * n < r_end;
        vb[n] = at(pb, okb, sb + n * (256 / TJ) * q.Cout * 4);
      }
    }
  };

  // one reduction step from the register set that holds its operands; the set is then refilled with the operands
  // of the step after the next, so that two steps' loads are in flight while a step's products run
  auto step = [&](int rs, float (&va)[NA], float (&vb)[NB]) {
    __syncthreads();   // the previous step's operand reads are done
    if (MODE == 1) {
#pragma unroll
      for (int n = 0; n < NA; ++n) As[t / TI + (256 / TI) * n][t % TI] = va[n];
    } else {
#pragma unroll
      for (int n = 0; n < NA; ++n) As[t & 15][(t >> 4) + 16 * n] = va[n];
    }
    if (MODE == 0) {
#pragma unroll
      for (int n = 0; n < NB; ++n) Bs[t & 15][(t >> 4) + 16 * n] = vb[n];
    } else {
#pragma unroll
      for (int n = 0; n < NB; ++n) Bs[t / TJ + (256 / TJ) * n][t % TJ] = vb[n];
    }
    __syncthreads();
    // unconditional (past the end every element reads the zero word): the count of loads in flight is then the
    // same at every step, and a step waits only for its own set
    gather(rs + 2 * SR_GR, va, vb);
#pragma unroll
    for (int kk = 0; kk < SR_GR / 2; ++kk) {
      const int rr = 2 * kk + (lane >> 5);
      float a[MI], b[MJ];
#pragma unroll
      for (int x = 0; x < MI; ++x) a[x] = As[rr][wi * 32 * MI + 32 * x + (lane & 31)];
#pragma unroll
      for (int y = 0; y < MJ; ++y) b[y] = Bs[rr][wj * 32 * MJ + 32 * y + (lane & 31)];
#pragma unroll
      for (int x = 0; x < MI; ++x)
#pragma unroll
        for (int y = 0; y < MJ; ++y) acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[x], b[y], acc[x][y], 0, 0, 0);
    }
  };
  float va0[NA], vb0[NB], va1[NA], vb1[NB];
  gather(r_begin, va0, vb0);
  // keep the two sets' loads apart in issue order, as they are inside the loop: a step's wait for its own set is
  // counted from the order of issue
  __builtin_amdgcn_sched_barrier(0);
  gather(r_begin + SR_GR, va1, vb1);
  // pairs of steps, then the odd one: a loop with one way round, so that the order in which the two sets' loads
  // were issued is the same whenever a step is reached (every condition here is the same for the whole workgroup)
  int rs = r_begin;
  for (; rs + SR_GR < r_end; rs += 2 * SR_GR) {
    step(rs, va0, vb0);
    step(rs + SR_GR, va1, vb1);
  }
  if (rs < r_end) step(rs, va0, vb0);
  float* out = pc + ((MODE == 1) ? (size_t)blockIdx.z * I * J : (size_t)0);
  sr_store_tile<MODE, MI, MJ>(acc, q, out, i0 + wi * 32 * MI, j0 + wj * 32 * MJ, lane, I, J, mul_wp, sh_wp, mul_hpwp,
                              sh_hpwp, accumulate);
}

// The same contraction for channel counts that are multiples of four: every operand is gathered 16 bytes at a
// time along its channel axis (a quarter of the loads and of the address arithmetic).  Operands whose channel
// axis is the reduction index (A of the forward and of the state gradient, B of the state gradient) lie in LDS row
// by row, a row's 16 reduction indices side by side, so a gather is one 16-byte LDS write and a wave reads its
// operand for a whole step with two 16-byte reads; the others (channel axis = tile row or column) lie reduction
// index by reduction index as above.  Reduction index of MFMA kk in lane half h: 8 h + kk.
typedef float sr_f32x4 __attribute__((ext_vector_type(4)));
__device__ __align__(16) const float sr_zero_quad[4] = {0.f, 0.f, 0.f, 0.f};

template <int MODE, int TI, int TJ, int WJN>
__global__ __launch_bounds__(256, 2) void sr_conv_gemm4_kernel(SrConvGeom q, const float* __restrict__ pa,
                                                               const float* __restrict__ pb, float* __restrict__ pc,
                                                               int I, int J, int R, int r_per_slice, int accumulate) {
  constexpr int WIN = 4 / WJN;
  constexpr int MI = TI / (32 * WIN), MJ = TJ / (32 * WJN);
  constexpr int NAV = TI / 64;                    // 16-byte pieces of A a thread gathers per step
  constexpr int NBV = TJ >= 64 ? TJ / 64 : 1;     // ... of B (a 32-wide tile: half the threads, one piece each)
  constexpr bool A_ROWS = MODE != 1, B_ROWS = MODE == 0;
  constexpr int RP = SR_GR + 4;                   // pitch of a row-by-row operand: eight lanes' 16-byte reads hit eight columns
  static_assert(MI >= 1 && MJ >= 1 && MI * 32 * WIN == TI && MJ * 32 * WJN == TJ && NAV >= 1, "tile shape");
  __shared__ __align__(16) float As[A_ROWS ? TI * RP : SR_GR * (TI + 4)];
  __shared__ __align__(16) float Bs[B_ROWS ? TJ * RP : SR_GR * (TJ + 4)];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int i0 = blockIdx.x * TI, j0 = blockIdx.y * TJ;
  if (MODE == 0) {
    sr_phase_of_plane(q, blockIdx.z, &I, &R);
    r_per_slice = R;
    if (i0 >= I || (R == 0 && accumulate)) return;   // the whole workgroup: this phase has fewer pixels, or no tap reaches it
  }
  const int r_begin = (MODE == 1) ? blockIdx.z * r_per_slice : 0;
  const int r_end = min(R, r_begin + r_per_slice);
  const int wi = wave / WJN, wj = wave % WJN;

  constexpr int FAR = 1 << 20;
  // MODE 0, 2: a thread's A pieces are reduction indices 4 (t % 4) .. + 3 of the rows t / 4 + 64 n
  // MODE 1:    rows 4 (t % (TI / 4)) .. + 3 at the reduction indices t / (TI / 4) + (1024 / TI) n
  int ah[NAV], aw[NAV], aoff[NAV];
  int ati = 0, atj = 0, a1off = 0;
  uint32_t mul_wp = 0, sh_wp = 0, mul_hpwp = 0, sh_hpwp = 0, mul_ntj = 0, sh_ntj = 0;
  if (MODE == 2) {
#pragma unroll
    for (int n = 0; n < NAV; ++n) {
      const int i = i0 + (t >> 2) + 64 * n;
      const int b = sr_fdiv(i, q.mul_howo, q.sh_howo), rem = i - b * (q.Ho * q.Wo);
      const int ho = sr_fdiv(rem, q.mul_wo, q.sh_wo), wo = rem - ho * q.Wo;
      ah[n] = (i < I) ? ho * q.stride - q.pad : FAR;
      aw[n] = wo * q.stride - q.pad;
      aoff[n] = (((b * q.H + ho * q.stride - q.pad) * q.W + aw[n]) * q.Cin) * 4;
    }
  } else if (MODE == 0) {
    const int lgs = (q.stride == 1) ? 0 : (q.stride == 2 ? 1 : (q.stride == 4 ? 2 : -1));
    sr_fdiv_make((uint32_t)max(q.Wp, 1), &mul_wp, &sh_wp);
    sr_fdiv_make((uint32_t)max(q.Wp * q.Hp, 1), &mul_hpwp, &sh_hpwp);
    sr_fdiv_make((uint32_t)max(q.ntj, 1), &mul_ntj, &sh_ntj);
#pragma unroll
    for (int n = 0; n < NAV; ++n) {
      const int i = i0 + (t >> 2) + 64 * n;
      const int b = sr_fdiv(i, mul_hpwp, sh_hpwp), rem = i - b * (q.Wp * q.Hp);
      const int hh = sr_fdiv(rem, mul_wp, sh_wp), ww = rem - hh * q.Wp;
      const int hn = hh * q.stride + q.ph + q.pad - q.ti0, wn = ww * q.stride + q.pw + q.pad - q.tj0;
      const int hq = lgs >= 0 ? hn >> lgs : hn / q.stride, wq = lgs >= 0 ? wn >> lgs : wn / q.stride;
      ah[n] = (i < I) ? hq : -FAR;
      aw[n] = wq;
      aoff[n] = (((b * q.Ho + hq) * q.Wo + wq) * q.Cout) * 4;
    }
  } else {
    const int i = i0 + 4 * (t % (TI / 4));
    const int tap = sr_fdiv(i, q.mul_cin, q.sh_cin), ci = i - tap * q.Cin;
    ati = sr_fdiv(tap, q.mul_kw, q.sh_kw);
    atj = tap - ati * q.kw;
    a1off = (((ati * q.W + atj) * q.Cin) + ci) * 4;
    if (i >= I) ati = FAR;
  }
  // B: byte offset of the thread's first piece at reduction index 0, and whether the thread has a piece at all
  int boff = 0;
  bool b_ok = false;
  if (MODE == 0) {
    const int j = j0 + (t >> 2);                 // theta[tap][j][co .. co + 3]: + 64 n Cout per piece, + (tap Cin Cout + co) per step
    boff = j * q.Cout * 4;
    b_ok = (t >> 2) < TJ;
  } else {
    const int j = j0 + 4 * (t % (TJ / 4));       // [r][j .. j + 3] with Cout columns
    b_ok = j < J && t / (TJ / 4) < SR_GR;
    boff = ((t / (TJ / 4)) * q.Cout + j) * 4;
  }

  sr_f32x16 acc[MI][MJ];
#pragma unroll
  for (int x = 0; x < MI; ++x)
#pragma unroll
    for (int y = 0; y < MJ; ++y)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[x][y][v] = 0.f;

  auto at4 = [](const float* base, bool ok, int byte_off) {
    typedef const __attribute__((address_space(1))) sr_f32x4* global_ptr;
    const global_ptr p = ok ? (global_ptr)((const char*)base + (uint32_t)byte_off) : (global_ptr)sr_zero_quad;
    return *p;
  };
  auto gather = [&](int rs, sr_f32x4 (&va)[NAV], sr_f32x4 (&vb)[NBV]) {
    if (MODE == 2) {
      const int r = rs + 4 * (t & 3);
      const int tap = sr_fdiv(r, q.mul_cin, q.sh_cin), ci = r - tap * q.Cin;
      int ti = sr_fdiv(tap, q.mul_kw, q.sh_kw);
      const int tj = tap - ti * q.kw;
      const int toff = ((ti * q.W + tj) * q.Cin + ci) * 4;
      if (r >= r_end) ti = FAR;
#pragma unroll
      for (int n = 0; n < NAV; ++n) {
        const bool ok = (unsigned)(ah[n] + ti) < (unsigned)q.H && (unsigned)(aw[n] + tj) < (unsigned)q.W;
        va[n] = at4(pa, ok, aoff[n] + toff);
      }
      const int sb = boff + rs * q.Cout * 4;
#pragma unroll
      for (int n = 0; n < NBV; ++n) {
        const bool okb = b_ok && rs + t / (TJ / 4) + (1024 / TJ) * n < r_end;
        vb[n] = at4(pb, okb, sb + n * (1024 / TJ) * q.Cout * 4);
      }
    } else if (MODE == 0) {
      const int r = rs + 4 * (t & 3);
      const bool r_ok = r < r_end;
      const int vt = sr_fdiv(r, q.mul_cout, q.sh_cout), co = r - vt * q.Cout;
      int vi = sr_fdiv(vt, mul_ntj, sh_ntj);
      const int vj = vt - vi * q.ntj;
      const int tap = (q.ti0 + vi * q.stride) * q.kw + q.tj0 + vj * q.stride;
      const int toff = (co - (vi * q.Wo + vj) * q.Cout) * 4;
      if (!r_ok) vi = 2 * FAR;
#pragma unroll
      for (int n = 0; n < NAV; ++n) {
        const bool ok = (unsigned)(ah[n] - vi) < (unsigned)q.Ho && (unsigned)(aw[n] - vj) < (unsigned)q.Wo;
        va[n] = at4(pa, ok, aoff[n] + toff);
      }
      const int sb = boff + (tap * q.Cin * q.Cout + co) * 4;
#pragma unroll
      for (int n = 0; n < NBV; ++n) {
        const bool okb = b_ok && r_ok && j0 + (t >> 2) + 64 * n < J;
        vb[n] = at4(pb, okb, sb + n * 64 * q.Cout * 4);
      }
    } else {
#pragma unroll
      for (int n = 0; n < NAV; ++n) {
        const int r = rs + t / (TI / 4) + (1024 / TI) * n;
        const int b = sr_fdiv(r, q.mul_howo, q.sh_howo), rem = r - b * (q.Ho * q.Wo);
        const int ho = sr_fdiv(rem, q.mul_wo, q.sh_wo), wo = rem - ho * q.Wo;
        const int h0 = (r < r_end) ? ho * q.stride - q.pad : FAR, w0 = wo * q.stride - q.pad;
        const int sbase = (((b * q.H + ho * q.stride - q.pad) * q.W + w0) * q.Cin) * 4;
        const bool ok = (unsigned)(h0 + ati) < (unsigned)q.H && (unsigned)(w0 + atj) < (unsigned)q.W;
        va[n] = at4(pa, ok, sbase + a1off);
      }
      const int sb = boff + rs * q.Cout * 4;
#pragma unroll
      for (int n = 0; n < NBV; ++n) {
        const bool okb = b_ok && rs + t / (TJ / 4) + (1024 / TJ) * n < r_end;
        vb[n] = at4(pb, okb, sb + n * (1024 / TJ) * q.Cout * 4);
      }
    }
  };
  auto step = [&](int rs, sr_f32x4 (&va)[NAV], sr_f32x4 (&vb)[NBV]) {
    __syncthreads();
    if (A_ROWS) {
#pragma unroll
      for (int n = 0; n < NAV; ++n) *(sr_f32x4*)&As[((t >> 2) + 64 * n) * RP + 4 * (t & 3)] = va[n];
    } else {
#pragma unroll
      for (int n = 0; n < NAV; ++n) *(sr_f32x4*)&As[(t / (TI / 4) + (1024 / TI) * n) * (TI + 4) + 4 * (t % (TI / 4))] = va[n];
    }
    if (B_ROWS) {
#pragma unroll
      for (int n = 0; n < NBV; ++n)
        if ((t >> 2) + 64 * n < TJ) *(sr_f32x4*)&Bs[((t >> 2) + 64 * n) * RP + 4 * (t & 3)] = vb[n];
    } else {
#pragma unroll
      for (int n = 0; n < NBV; ++n)
        if (t / (TJ / 4) + (1024 / TJ) * n < SR_GR)
          *(sr_f32x4*)&Bs[(t / (TJ / 4) + (1024 / TJ) * n) * (TJ + 4) + 4 * (t % (TJ / 4))] = vb[n];
    }
    __syncthreads();
    gather(rs + 2 * SR_GR, va, vb);   // unconditional: see sr_conv_gemm_kernel
    const int h8 = (lane >> 5) * 8;
    float a[MI][8], b[MJ][8];
#pragma unroll
    for (int x = 0; x < MI; ++x) {
      const int row = wi * 32 * MI + 32 * x + (lane & 31);
      if (A_ROWS) {
        const sr_f32x4 lo = *(const sr_f32x4*)&As[row * RP + h8], hi = *(const sr_f32x4*)&As[row * RP + h8 + 4];
        a[x][0] = lo.x; a[x][1] = lo.y; a[x][2] = lo.z; a[x][3] = lo.w;
        a[x][4] = hi.x; a[x][5] = hi.y; a[x][6] = hi.z; a[x][7] = hi.w;
      } else {
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) a[x][kk] = As[(h8 + kk) * (TI + 4) + row];
      }
    }
#pragma unroll
    for (int y = 0; y < MJ; ++y) {
      const int col = wj * 32 * MJ + 32 * y + (lane & 31);
      if (B_ROWS) {
        const sr_f32x4 lo = *(const sr_f32x4*)&Bs[col * RP + h8], hi = *(const sr_f32x4*)&Bs[col * RP + h8 + 4];
        b[y][0] = lo.x; b[y][1] = lo.y; b[y][2] = lo.z; b[y][3] = lo.w;
        b[y][4] = hi.x; b[y][5] = hi.y; b[y][6] = hi.z; b[y][7] = hi.w;
      } else {
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) b[y][kk] = Bs[(h8 + kk) * (TJ + 4) + col];
      }
    }
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
#pragma unroll
      for (int x = 0; x < MI; ++x)
#pragma unroll
        for (int y = 0; y < MJ; ++y)
          acc[x][y] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[x][kk], b[y][kk], acc[x][y], 0, 0, 0);
  };
  sr_f32x4 va0[NAV], vb0[NBV], va1[NAV], vb1[NBV];
  gather(r_begin, va0, vb0);
  __builtin_amdgcn_sched_barrier(0);
  gather(r_begin + SR_GR, va1, vb1);
  int rs = r_begin;
  for (; rs + SR_GR < r_end; rs += 2 * SR_GR) {
    step(rs, va0, vb0);
    step(rs + SR_GR, va1, vb1);
  }
  if (rs < r_end) step(rs, va0, vb0);
  float* out = pc + ((MODE == 1) ? (size_t)blockIdx.z * I * J : (size_t)0);
  sr_store_tile<MODE, MI, MJ>(acc, q, out, i0 + wi * 32 * MI, j0 + wj * 32 * MJ, lane, I, J, mul_wp, sh_wp, mul_hpwp,
                              sh_hpwp, accumulate);
}

// forward of one edge, one thread per output element: y[b][ho][wo][co] (+)= sum x * theta
__global__ void sr_fwd_kernel(SrConvGeom q, const float* __restrict__ x, const float* __restrict__ theta,
                              float* __restrict__ y, int accumulate) {
  const size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n = (size_t)q.B * q.Ho * q.Wo * q.Cout;
  if (idx >= n) return;
  const int co = (int)(idx % q.Cout);
  size_t r = idx / q.Cout;
  const int wo = (int)(r % q.Wo); r /= q.Wo;
  const int ho = (int)(r % q.Ho);
  const int b = (int)(r / q.Ho);
  float acc = 0.f;
  for (int i = 0; i < q.kh; ++i) {
    const int hi = ho * q.stride + i - q.pad;
    if (hi < 0 || hi >= q.H) continue;
    for (int j = 0; j < q.kw; ++j) {
      const int wi = wo * q.stride + j - q.pad;
      if (wi < 0 || wi >= q.W) continue;
      const float* xs = x + (((size_t)b * q.H + hi) * q.W + wi) * q.Cin;
      const float* t = theta + (size_t)(i * q.kw + j) * q.Cin * q.Cout + co;
      for (int ci = 0; ci < q.Cin; ++ci) acc += xs[ci] * t[(size_t)ci * q.Cout];
    }
  }
  y[idx] = accumulate ? y[idx] + acc : acc;
}

// the same for few outputs with long sums (dense edges): one wave per output element, the lanes take every 64th
// term of the (tap, ci) sum in order, then a fixed tree over the lanes
__global__ void sr_fwd_wide_kernel(SrConvGeom q, const float* __restrict__ x, const float* __restrict__ theta,
                                   float* __restrict__ y, int accumulate) {
  const size_t idx = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const size_t n = (size_t)q.B * q.Ho * q.Wo * q.Cout;
  if (idx >= n) return;                       // a whole wave
  const int lane = threadIdx.x & 63;
  const int co = (int)(idx % q.Cout);
  size_t r = idx / q.Cout;
  const int wo = (int)(r % q.Wo); r /= q.Wo;
  const int ho = (int)(r % q.Ho);
  const int b = (int)(r / q.Ho);
  const int K = q.kh * q.kw * q.Cin;
  float acc = 0.f;
  for (int k = lane; k < K; k += 64) {
    const int ci = k % q.Cin, tap = k / q.Cin;
    const int hi = ho * q.stride + tap / q.kw - q.pad, wi = wo * q.stride + tap % q.kw - q.pad;
    if (hi >= 0 && hi < q.H && wi >= 0 && wi < q.W)
      acc += x[(((size_t)b * q.H + hi) * q.W + wi) * q.Cin + ci] * theta[(size_t)k * q.Cout + co];
  }
  for (int m = 32; m > 0; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if (lane == 0) y[idx] = accumulate ? y[idx] + acc : acc;
}

// the same for a narrow target (at most 32 channels, long sums: the edge into the logits): one workgroup per output
// pixel; a thread takes every 256th term of the (tap, ci) sum in order for up to 16 output channels at a time,
// reading its source element once for all of them; then a fixed tree over the lanes and the four waves in order
__global__ __launch_bounds__(256) void sr_fwd_pixel_kernel(SrConvGeom q, const float* __restrict__ x,
                                                            const float* __restrict__ theta, float* __restrict__ y,
                                                            int accumulate) {
  __shared__ float part[4][16];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int m = blockIdx.x;   // output pixel (b, ho, wo)
  const int b = sr_fdiv(m, q.mul_howo, q.sh_howo), rem = m - b * (q.Ho * q.Wo);
  const int ho = sr_fdiv(rem, q.mul_wo, q.sh_wo), wo = rem - ho * q.Wo;
  const int K = q.kh * q.kw * q.Cin;
  for (int c0 = 0; c0 < q.Cout; c0 += 16) {
    float acc[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) acc[c] = 0.f;
    const int nc = min(16, q.Cout - c0);
    // every load unconditional (a source element outside the image is read from a word that holds zero), so the
    // unrolled loop has four terms' loads in flight at a time
#pragma unroll 4
    for (int k = t; k < K; k += 256) {
      const int tap = sr_fdiv(k, q.mul_cin, q.sh_cin), ci = k - tap * q.Cin;
      const int ti = sr_fdiv(tap, q.mul_kw, q.sh_kw), tj = tap - ti * q.kw;
      const int hi = ho * q.stride + ti - q.pad, wi = wo * q.stride + tj - q.pad;
      const bool ok = (unsigned)hi < (unsigned)q.H && (unsigned)wi < (unsigned)q.W;
      const float* px = ok ? x + (((size_t)b * q.H + hi) * q.W + wi) * q.Cin + ci : &sr_zero_word;
      const float xv = *px;
      const float* row = theta + (size_t)k * q.Cout + c0;
#pragma unroll
      for (int c = 0; c < 16; ++c) acc[c] += xv * row[c < nc ? c : 0];   // channels past the last: not written out
    }
#pragma unroll
    for (int c = 0; c < 16; ++c) {
      float v = acc[c];
      for (int w = 32; w > 0; w >>= 1) v += __shfl_xor(v, w, 64);
      if (lane == 0) part[wave][c] = v;
    }
    __syncthreads();
    if (t < 16 && c0 + t < q.Cout) {
      const float v = ((part[0][t] + part[1][t]) + part[2][t]) + part[3][t];
      float* dst = y + (size_t)m * q.Cout + c0 + t;
      *dst = accumulate ? *dst + v : v;
    }
    __syncthreads();
  }
}

// nearest up-sampling of an edge's result into its target: dst[b][h][w][c] (+)= y[b][h / up][w / up][c]
__global__ void sr_upsample_add_kernel(const float* __restrict__ y, int B, int H, int W, int C, int up,
                                       float* __restrict__ dst, int accumulate) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t n = (size_t)B * H * W * C;
  if (i >= n) return;
  const int c = (int)(i % C);
  size_t r = i / C;
  const int w = (int)(r % W); r /= W;
  const int h = (int)(r % H);
  const int b = (int)(r / H);
  const float v = y[(((size_t)b * (H / up) + h / up) * (W / up) + w / up) * C + c];
  dst[i] = accumulate ? dst[i] + v : v;
}

// x = m * sigma(a + b_c) in place (App. A1.2 node map; m: dropout multipliers or null)
__global__ void sr_bias_act_kernel(float* __restrict__ a, const float* __restrict__ bias, const float* __restrict__ m,
                                   int C, size_t n, int act) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float v = a[i] + bias[i % C];
  if (act == 1) v = fmaxf(v, 0.f);
  a[i] = m ? v * m[i] : v;
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

hipError_t sr_train_act_grad(hipStream_t s, float* d, const float* x, const float* m, size_t n, int act) {
  if (n == 0 || (act != 1 && !m)) return hipSuccess;
  hipLaunchKernelGGL(sr_act_grad_kernel, dim3(grid_for((long long)n, 256)), dim3(256), 0, s, d, x, m, n, act);
  return hipGetLastError();
}

int sr_train_bias_slices(int M) {
  const int want = (M + 255) / 256;   // 256 pixels per slice or more
  return want < 1 ? 1 : (want > SR_TRAIN_MAX_SLICES ? SR_TRAIN_MAX_SLICES : want);
}

hipError_t sr_train_bias_grad(hipStream_t s, const float* d, int M, int C, float* part, float* db) {
  if (M <= 2048) {
    hipLaunchKernelGGL(sr_bias_grad_small_kernel, dim3(C), dim3(256), 0, s, d, M, C, db);
    return hipGetLastError();
  }
  const int slices = sr_train_bias_slices(M);
  const int per = (M + slices - 1) / slices;
  const int used = (M + per - 1) / per;
  hipLaunchKernelGGL(sr_bias_grad_kernel, dim3((C + 63) / 64, used), dim3(256), 0, s, d, M, C, per, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(sr_add_slices_kernel, dim3(grid_for(C, 64)), dim3(256), 0, s, part, (size_t)C, used, db);
  return hipGetLastError();
}

hipError_t sr_train_pool_sum(hipStream_t s, const float* d, int B, int Hs, int Ws, int C, int up, float* out) {
  const long long n = (long long)B * Hs * Ws * C;
  hipLaunchKernelGGL(sr_pool_sum_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, d, B, Hs, Ws, C, up, out);
  return hipGetLastError();
}

static void sr_fastdiv(uint32_t d, uint32_t* mul, uint32_t* sh) {
  uint32_t l = 0;
  while ((1ull << l) < d) ++l;
  *mul = (uint32_t)(((1ull << 32) * ((1ull << l) - d)) / d + 1);
  *sh = l;
}
static SrConvGeom sr_with_divisors(const SrConvGeom& q) {
  SrConvGeom p = q;
  sr_fastdiv((uint32_t)q.Wo, &p.mul_wo, &p.sh_wo);
  sr_fastdiv((uint32_t)(q.Ho * q.Wo), &p.mul_howo, &p.sh_howo);
  sr_fastdiv((uint32_t)q.Cout, &p.mul_cout, &p.sh_cout);
  sr_fastdiv((uint32_t)q.Cin, &p.mul_cin, &p.sh_cin);
  sr_fastdiv((uint32_t)q.kw, &p.mul_kw, &p.sh_kw);
  return p;
}

// Tile shape of a contraction with I rows and J columns in `planes` grid planes: the narrowest column tile that
// holds J, then the taller row tile only where the launch still has tall_from workgroups, some thousands by
// default (a launch of few tall tiles is a few long dependent chains on an otherwise idle chip; on the measured
// windows the smaller tile was the faster or equal one for every launch below that)
struct SrTileShape { int ti, tj, wjn; };
static SrTileShape sr_pick_tile(long long I, long long J, long long planes, int tall_from) {
  static const SrTileShape wide[] = {{128, 128, 2}, {64, 64, 2}}, mid[] = {{128, 64, 2}, {64, 64, 2}},
                           slim[] = {{256, 32, 1}, {128, 32, 1}};
  const SrTileShape* c = J <= 32 ? slim : (J <= 64 ? mid : wide);
  const long long first = (I + c[0].ti - 1) / c[0].ti * ((J + c[0].tj - 1) / c[0].tj) * planes;
  return first >= tall_from ? c[0] : c[1];
}
template <int MODE>
static hipError_t sr_launch_gemm(hipStream_t s, SrTileShape ts, int planes, const SrConvGeom& q, const float* pa,
                                 const float* pb, float* pc, int I, int J, int R, int per, int accumulate) {
  const dim3 grid((I + ts.ti - 1) / ts.ti, (J + ts.tj - 1) / ts.tj, planes);
  const bool quads = q.Cin % 4 == 0 && q.Cout % 4 == 0;   // every channel axis in 16-byte pieces
#define SR_GEMM_CASE(TI, TJ, WJN)                                                                                    \
  if (ts.ti == TI && ts.tj == TJ && ts.wjn == WJN) {                                                                 \
    if (quads)                                                                                                       \
      hipLaunchKernelGGL((sr_conv_gemm4_kernel<MODE, TI, TJ, WJN>), grid, dim3(256), 0, s, q, pa, pb, pc, I, J, R,   \
                         per, accumulate);                                                                           \
    else                                                                                                             \
      hipLaunchKernelGGL((sr_conv_gemm_kernel<MODE, TI, TJ, WJN>), grid, dim3(256), 0, s, q, pa, pb, pc, I, J, R,    \
                         per, accumulate);                                                                           \
    return hipGetLastError();                                                                                        \
  }
  SR_GEMM_CASE(128, 128, 2)
  SR_GEMM_CASE(128, 64, 2)
  SR_GEMM_CASE(64, 64, 2)
  SR_GEMM_CASE(256, 32, 1)
  SR_GEMM_CASE(128, 32, 1)
#undef SR_GEMM_CASE
  return hipErrorInvalidValue;
}

// Which contractions go to the tiled matrix-core kernel: those with enough multiply-adds whose 128 x 128 tiles are
// reasonably full and numerous (else the one-thread-per-output kernels, which spread over the chip whatever the shape)
static bool sr_train_big(const SrConvGeom& q) {
  // the tiled kernel addresses its operands by byte offsets in 32 bits, with room for a padding row either side
  const double lim = (double)(1u << 30);
  if (4.0 * q.B * q.H * q.W * q.Cin >= lim || 4.0 * q.B * q.Ho * q.Wo * q.Cout >= lim ||
      4.0 * q.kh * q.kw * q.Cin * q.Cout >= lim)
    return false;
  return (double)q.B * q.Ho * q.Wo * q.Cout * q.Cin * q.kh * q.kw >= SR_TRAIN_TILED_MIN_MACS;
}
static long long sr_wgrad_tiles(const SrConvGeom& q) {
  return ((long long)q.kh * q.kw * q.Cin + SR_GT - 1) / SR_GT * ((q.Cout + SR_GT - 1) / SR_GT);
}
static long long sr_wgrad_max_slices(const SrConvGeom& q) {   // slices of at least 128 pixels
  const long long M = (long long)q.B * q.Ho * q.Wo;
  return std::min<long long>(SR_TRAIN_MAX_SLICES, std::max<long long>(1, M / 128));
}
static bool sr_dgrad_tiled(const SrConvGeom& q) {
  return sr_train_big(q) && q.Cin >= 16 && ((long long)q.B * q.H * q.W + 63) / 64 >= 2;
}
static bool sr_wgrad_tiled(const SrConvGeom& q) {
  return sr_train_big(q) && q.Cout >= 16;
}

hipError_t sr_train_dgrad(hipStream_t s, const SrConvGeom& q, const float* theta, const float* dy, float* dx,
                          int accumulate) {
  const long long n = (long long)q.B * q.H * q.W * q.Cin;
  if (sr_dgrad_tiled(q)) {
    // grid z: the stride^2 phases of the source pixels; x is sized for phase (0, 0), which has the most pixels
    const int Hp = (q.H + q.stride - 1) / q.stride, Wp = (q.W + q.stride - 1) / q.stride;
    const int I = q.B * Hp * Wp, J = q.Cin;
    const int planes = q.stride * q.stride;
    return sr_launch_gemm<0>(s, sr_pick_tile(I, J, planes, q.tall_from), planes, sr_with_divisors(q), dy, theta, dx, I, J, 0, 0, accumulate);
  }
  hipLaunchKernelGGL(sr_dgrad_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, q, theta, dy, dx, accumulate);
  return hipGetLastError();
}

static bool sr_fwd_tiled(const SrConvGeom& q) {
  return sr_train_big(q) && q.Cout >= 16 && ((long long)q.B * q.Ho * q.Wo + 63) / 64 >= 2;
}
int sr_train_fwd_is_tiled(const SrConvGeom& q) { return sr_fwd_tiled(q) ? 1 : 0; }

hipError_t sr_train_fwd(hipStream_t s, const SrConvGeom& q, const float* x, const float* theta, float* y,
                        int accumulate) {
  if (sr_fwd_tiled(q)) {
    const SrConvGeom p = sr_with_divisors(q);
    const int I = q.B * q.Ho * q.Wo, J = q.Cout, R = q.kh * q.kw * q.Cin;
    return sr_launch_gemm<2>(s, sr_pick_tile(I, J, 1, q.tall_from), 1, p, x, theta, y, I, J, R, R, accumulate);
  }
  const long long n = (long long)q.B * q.Ho * q.Wo * q.Cout;
  if (q.Cout <= 32 && n / q.Cout <= 65536 && (long long)q.kh * q.kw * q.Cin >= 1024) {   // a workgroup per output pixel
    hipLaunchKernelGGL(sr_fwd_pixel_kernel, dim3((unsigned)(n / q.Cout)), dim3(256), 0, s, sr_with_divisors(q), x, theta, y,
                       accumulate);
    return hipGetLastError();
  }
  if (n <= 65536 && (long long)q.kh * q.kw * q.Cin >= 256) {   // few outputs, long sums: a wave per output
    hipLaunchKernelGGL(sr_fwd_wide_kernel, dim3(grid_for(n, 4)), dim3(256), 0, s, q, x, theta, y, accumulate);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(sr_fwd_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, q, x, theta, y, accumulate);
  return hipGetLastError();
}

hipError_t sr_train_upsample_add(hipStream_t s, const float* y, int B, int H, int W, int C, int up, float* dst,
                                 int accumulate) {
  const long long n = (long long)B * H * W * C;
  hipLaunchKernelGGL(sr_upsample_add_kernel, dim3(grid_for(n, 256)), dim3(256), 0, s, y, B, H, W, C, up, dst, accumulate);
  return hipGetLastError();
}

hipError_t sr_train_bias_act(hipStream_t s, float* a, const float* bias, const float* m, int C, size_t n, int act) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(sr_bias_act_kernel, dim3(grid_for((long long)n, 256)), dim3(256), 0, s, a, bias, m, C, n, act);
  return hipGetLastError();
}

int sr_train_wgrad_slices(const SrConvGeom& q) {
  const long long nw = (long long)q.kh * q.kw * q.Cin * q.Cout;
  const long long M = (long long)q.B * q.Ho * q.Wo;
  if (sr_wgrad_tiled(q)) {   // about 1024 workgroups
    const long long tiles = sr_wgrad_tiles(q);
    const long long want = std::min<long long>((1024 + tiles - 1) / tiles, sr_wgrad_max_slices(q));
    return (int)std::max<long long>(1, want);
  }
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
  if (sr_wgrad_tiled(q)) {
    const int I = q.kh * q.kw * q.Cin, J = q.Cout;
    const int per = ((M + slices - 1) / slices + SR_GR - 1) / SR_GR * SR_GR;
    const int used = (M + per - 1) / per;
    if (used == 1)   // one slice: straight onto the gradient
      return sr_launch_gemm<1>(s, sr_pick_tile(I, J, 1, q.tall_from), 1, sr_with_divisors(q), x, dy, dtheta, I, J, M, per, 1);
    hipError_t e = sr_launch_gemm<1>(s, sr_pick_tile(I, J, used, q.tall_from), used, sr_with_divisors(q), x, dy, part, I, J, M, per, 0);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(sr_add_slices_kernel, dim3(grid_for(nw, 64)), dim3(256), 0, s, part, (size_t)nw, used, dtheta);
    return hipGetLastError();
  }
  const int per = (M + slices - 1) / slices;
  const int used = (M + per - 1) / per;
  hipLaunchKernelGGL(sr_wgrad_kernel, dim3(grid_for(nw, 256), used), dim3(256), 0, s, q, x, dy, per, part);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(sr_add_slices_kernel, dim3(grid_for(nw, 64)), dim3(256), 0, s, part, (size_t)nw, used, dtheta);
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
