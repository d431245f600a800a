// HIP kernels of the streaming-rollout frame update for gfx950 (CDNA4).
//
//   x_v(t) = sigma_v( b_v + sum_{e=(u,v)} f_e(theta_e, x_u(t - R(e))) )      (App. A1.2, Eq. 2)
//
// sr_mfma_kernel   node-centric implicit-GEMM tiles on the bf16 matrix cores: one workgroup owns a
//                  tile (pixels x output channels) of one node and walks over all incoming edges,
//                  accumulating into the same float accumulators (the sum over edges is one
//                  convolution over the concatenated sources, App. A2); bias, activation, rounding
//                  and the NHWC store are fused behind the last edge.
// sr_direct_kernel one thread per output element, float accumulation; fp32 graphs, and nodes the
//                  tile kernel does not take.
// head kernels     global average pool + dense.
// plus input staging, state packing, output recording and the frame counter.
//
// Every kernel takes the frame counter from SrCtx: the copy written at frame t is t & 1.
#include <hip/hip_runtime.h>
#include <hip/hip_bf16.h>
#include "sr_internal.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

// ---------------------------------------------------------------------------
// bfloat16 <-> float (round to nearest even)
// ---------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_float(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

__device__ __forceinline__ uint16_t float_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

template <typename T> struct Store;
template <> struct Store<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Store<uint16_t> {
  static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_bits_to_float(*p); }
  static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = float_to_bf16_bits(v); }
};

// ---------------------------------------------------------------------------
// bookkeeping kernels
// ---------------------------------------------------------------------------
__global__ void sr_set_ctx_kernel(SrCtx* ctx, SrCtx v, int set_frame) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    int frame = ctx->frame;
    *ctx = v;
    if (!set_frame) ctx->frame = frame;
  }
}

__global__ void sr_tick_kernel(SrCtx* ctx) {
  if (threadIdx.x == 0 && blockIdx.x == 0) ctx->frame = ctx->frame + 1;
}

__global__ void sr_fill_zero_kernel(uint4* p, size_t n16, unsigned char* tail, size_t ntail) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
  if (blockIdx.x == 0 && threadIdx.x < ntail) tail[threadIdx.x] = 0;
}

// state[frame & 1] of every input node := this frame's input, channel pitch C -> Cp
template <typename T>
__global__ void sr_stage_inputs_kernel(const SrCtx* __restrict__ ctx, const SrStageNode* __restrict__ nodes) {
  const SrStageNode nd = nodes[blockIdx.y];
  const int frame = ctx->frame;
  const char* base = (const char*)ctx->in_ptr[nd.input_slot];
  if (base == nullptr) return;
  const T* in = (const T*)(base + (int64_t)(frame - ctx->in_base) * ctx->in_stride[nd.input_slot]);
  T* out = (T*)nd.state[frame & 1];
  const int total = nd.elems_px * nd.Cp;
  for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
    int p = idx / nd.Cp, c = idx - p * nd.Cp;
    out[idx] = (c < nd.C) ? in[(size_t)p * nd.C + c] : (T)0;
  }
}

// dense [px][C]  <->  pitched [px][Cp]
template <typename T>
__global__ void sr_pack_kernel(T* __restrict__ dst, const T* __restrict__ src, int px, int C, int Cp, int unpack) {
  const int total = unpack ? px * C : px * Cp;
  for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
    if (unpack) {
      int p = idx / C, c = idx - p * C;
      dst[idx] = src[(size_t)p * Cp + c];
    } else {
      int p = idx / Cp, c = idx - p * Cp;
      dst[idx] = (c < C) ? src[(size_t)p * C + c] : (T)0;
    }
  }
}

template <typename T>
__global__ void sr_record_output_kernel(const SrCtx* __restrict__ ctx, const T* s0, const T* s1, int px, int C, int Cp) {
  char* base = (char*)ctx->out_ptr;
  if (base == nullptr) return;
  const int frame = ctx->frame;
  T* dst = (T*)(base + (int64_t)(frame - ctx->out_base) * ctx->out_stride);
  const T* src = (frame & 1) ? s1 : s0;
  const int total = px * C;
  for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += gridDim.x * blockDim.x) {
    int p = idx / C, c = idx - p * C;
    dst[idx] = src[(size_t)p * Cp + c];
  }
}

// ---------------------------------------------------------------------------
// direct path
// ---------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void sr_direct_kernel(const SrCtx* __restrict__ ctx,
                                                        const SrDirectNode* __restrict__ nodes,
                                                        const SrDirectEdge* __restrict__ edges,
                                                        const SrDirectBlock* __restrict__ blocks, int batch) {
  const SrDirectBlock blk = blocks[blockIdx.x];
  const SrDirectNode nd = nodes[blk.node];
  const int cur = ctx->frame & 1;
  const int idx = blk.first + threadIdx.x;
  const int HW = nd.H * nd.W;
  if (idx >= batch * HW * nd.C) return;
  const int m = idx / nd.C, co = idx - m * nd.C;
  const int b = m / HW, r = m - b * HW;
  const int oy = r / nd.W, ox = r - oy * nd.W;
  float acc = nd.bias[co];
  for (int ei = 0; ei < nd.edge_count; ++ei) {
    const SrDirectEdge e = edges[nd.edge_begin + ei];
    const T* src = (const T*)e.src[e.bridge ? (cur ^ 1) : cur];
    if (e.kind == 0) {
      const int sy = (oy / e.up) * e.stride - e.pad;
      const int sx = (ox / e.up) * e.stride - e.pad;
      for (int i = 0; i < e.kh; ++i) {
        const int iy = sy + i;
        if (iy < 0 || iy >= e.Hs) continue;
        for (int j = 0; j < e.kw; ++j) {
          const int ix = sx + j;
          if (ix < 0 || ix >= e.Ws) continue;
          const T* px = src + ((size_t)(b * e.Hs + iy) * e.Ws + ix) * e.Csp;
          const float* w = e.w + (size_t)(i * e.kw + j) * e.Cin * nd.C + co;
          for (int ci = 0; ci < e.Cin; ++ci) acc += Store<T>::load(px + ci) * w[(size_t)ci * nd.C];
        }
      }
    } else {  // mean over (h,w), then dense
      const int n = e.Hs * e.Ws;
      const float inv = 1.0f / (float)n;
      const T* img = src + (size_t)b * n * e.Csp;
      for (int ci = 0; ci < e.Cin; ++ci) {
        float s = 0.f;
        for (int p = 0; p < n; ++p) s += Store<T>::load(img + (size_t)p * e.Csp + ci);
        acc += (s * inv) * e.w[(size_t)ci * nd.C + co];
      }
    }
  }
  if (nd.act == 1) acc = fmaxf(acc, 0.f);
  Store<T>::store((T*)nd.out[cur] + (size_t)m * nd.Cp + co, acc);
}

// ---------------------------------------------------------------------------
// GAP + dense head
// ---------------------------------------------------------------------------
// partial[b][s][c] = sum over the s-th slab of pixels of src[b][p][c]
template <typename T>
__global__ __launch_bounds__(256) void sr_gap_partial_kernel(const SrCtx* __restrict__ ctx,
                                                             const SrHead* __restrict__ heads) {
  const SrHead h = heads[blockIdx.z];
  const int b = blockIdx.y, s = blockIdx.x;
  if (b >= h.B || s >= h.splits) return;
  const int cur = ctx->frame & 1;
  const T* src = (const T*)h.src[h.bridge ? (cur ^ 1) : cur] + (size_t)b * h.HW * h.Csp;
  const int per = (h.HW + h.splits - 1) / h.splits;
  const int p0 = s * per, p1 = min(h.HW, p0 + per);
  for (int c = threadIdx.x; c < h.Cin; c += blockDim.x) {
    float sum = 0.f;
    for (int p = p0; p < p1; ++p) sum += Store<T>::load(src + (size_t)p * h.Csp + c);
    h.partial[((size_t)b * h.splits + s) * h.Cin + c] = sum;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void sr_head_dense_kernel(const SrCtx* __restrict__ ctx,
                                                            const SrHead* __restrict__ heads) {
  extern __shared__ float mean[];
  const SrHead h = heads[blockIdx.y];
  const int b = blockIdx.x;
  if (b >= h.B) return;
  const int cur = ctx->frame & 1;
  const float inv = 1.0f / (float)h.HW;
  for (int c = threadIdx.x; c < h.Cin; c += blockDim.x) {
    float sum = 0.f;
    for (int s = 0; s < h.splits; ++s) sum += h.partial[((size_t)b * h.splits + s) * h.Cin + c];
    mean[c] = sum * inv;
  }
  __syncthreads();
  for (int co = threadIdx.x; co < h.Cout; co += blockDim.x) {
    float acc = h.bias[co];
    for (int ci = 0; ci < h.Cin; ++ci) acc += mean[ci] * h.w[(size_t)ci * h.Cout + co];
    if (h.act == 1) acc = fmaxf(acc, 0.f);
    Store<T>::store((T*)h.out[cur] + (size_t)b * h.Cp + co, acc);
  }
}

// ---------------------------------------------------------------------------
// MFMA path
// ---------------------------------------------------------------------------
// Workgroup = 4 wave64 arranged waves_m x waves_n; each wave owns 128 pixels x (32*WN) channels:
// 4 x WN accumulator tiles of v_mfma_f32_32x32x16_bf16.  Operand layout of that instruction: lane l
// supplies row (A) / column (B) l % 32 and 8 consecutive k values selected by l / 32.
//
// A operand (pixels x channels of the source): the source patch that the tile's pixels touch is
// staged once per KC channels in LDS and re-read for every tap.  LDS slot (q, px): q = padded
// source row relative to the tile's first one, px = padded source column, stored column-phase
// major for strided edges so that consecutive output pixels read consecutive slots:
//     slot = q*RP + (px % stride)*PWs + px / stride,   SP = KC*2 + 16 bytes per slot
// (the 16 spare bytes rotate consecutive slots across the LDS banks).
//
// B operand (weights): pre-packed on the host in exactly the per-lane order of the instruction,
// [tap][k16 block][32-channel tile][lane][8], so a wave's fragment is one coalesced 1 KiB load
// straight into registers; it is prefetched one k-step ahead.
template <int WN>
__device__ __forceinline__ void sr_mfma_tile(const SrCtx* __restrict__ ctx, const SrMfmaNode& nd,
                                             const SrMfmaEdge* __restrict__ edges, const SrMfmaTile& t,
                                             unsigned char* lds) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm = wave / nd.waves_n;
  const int wn = wave - wm * nd.waves_n;
  const int cur = ctx->frame & 1;
  const int BM = 128 * nd.waves_m;
  const int HoWo = nd.Ho * nd.Wo;
  const int m_first = t.m0;
  const int m_last = min(t.m0 + BM, nd.M) - 1;
  const int wave_m0 = t.m0 + wm * 128;
  const int wave_n0 = t.n0 + wn * (32 * WN);
  const int ntile0 = wave_n0 >> 5;

  // pixel coordinates of this lane's 4 rows (clamped to the last valid pixel)
  int pb[4], py[4], pxo[4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    int m = min(wave_m0 + mi * 32 + (lane & 31), nd.M - 1);
    int b = m / HoWo;
    int r = m - b * HoWo;
    int oy = r / nd.Wo;
    pb[mi] = b; py[mi] = oy; pxo[mi] = r - oy * nd.Wo;
  }
  const int b_first = m_first / HoWo, oy_first = (m_first - b_first * HoWo) / nd.Wo;
  const int b_last = m_last / HoWo, oy_last = (m_last - b_last * HoWo) / nd.Wo;

  f32x16_t acc[4][WN];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int nj = 0; nj < WN; ++nj)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][nj][r] = 0.f;

  for (int ei = 0; ei < nd.edge_count; ++ei) {
    const SrMfmaEdge& e = edges[nd.edge_begin + ei];
    const unsigned char* src = (const unsigned char*)e.src[e.bridge ? (cur ^ 1) : cur];
    const int s = e.stride, lg = (s == 1) ? 0 : (s == 2 ? 1 : 2);
    const int Q0 = b_first * e.PH + (oy_first / e.up) * s;
    const int Q1 = b_last * e.PH + (oy_last / e.up) * s + e.kh - 1;
    const int n_items_row = e.PW;
    const int CH = e.KC >> 3;                 // 16-byte pieces per slot
    const int lgCH = (CH == 2) ? 1 : (CH == 4 ? 2 : 3);
    const int n_items = (Q1 - Q0 + 1) * n_items_row * CH;
    int abase[4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
      int q = pb[mi] * e.PH + (py[mi] / e.up) * s - Q0;
      abase[mi] = (q * e.RP + (pxo[mi] / e.up)) * e.SP + (lane >> 5) * 16;
    }
    const int ntaps = e.kh * e.kw;
    const int k16_per_chunk = e.KC >> 4;
    const int k16_total = e.Csp >> 4;
    const bf16x8_t* wlane = (const bf16x8_t*)e.wpk + (size_t)ntile0 * 64 + lane;

    for (int chunk = 0; chunk < e.nchunk; ++chunk) {
      __syncthreads();   // everyone has finished reading the previous patch
      // ---- stage the patch: KC channels of every padded source pixel the tile touches
      for (int item0 = tid; item0 < n_items; item0 += 256 * 4) {
        uint4 v[4];
        int dst[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int item = item0 + u * 256;
          v[u] = make_uint4(0, 0, 0, 0);
          dst[u] = -1;
          if (item < n_items) {
            const int ch = item & (CH - 1);
            const int sl = item >> lgCH;
            const int q = __umulhi((unsigned)sl, e.magicPW);
            const int px = sl - q * e.PW;
            const int Qg = Q0 + q;
            const int b = __umulhi((unsigned)Qg, e.magicPH);
            const int iy = Qg - b * e.PH - e.pad;
            const int ix = px - e.pad;
            if (iy >= 0 && iy < e.Hs && ix >= 0 && ix < e.Ws) {
              const size_t off = (((size_t)(b * e.Hs + iy) * e.Ws + ix) * e.Csp + chunk * e.KC + ch * 8) * 2;
              v[u] = *(const uint4*)(src + off);
            }
            dst[u] = (q * e.RP + (px & (s - 1)) * e.PWs + (px >> lg)) * e.SP + ch * 16;
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u)
          if (dst[u] >= 0) *(uint4*)(lds + dst[u]) = v[u];
      }
      __syncthreads();
      // ---- contract: taps x k16 steps of this chunk
      const bf16x8_t* wchunk = wlane + (size_t)(chunk * k16_per_chunk) * e.wstride8;
      bf16x8_t bcur[WN], bnxt[WN];
#pragma unroll
      for (int nj = 0; nj < WN; ++nj) bnxt[nj] = bcur[nj] = wchunk[nj * 64];
      for (int tap = 0; tap < ntaps; ++tap) {
        const int ti = tap / e.kw, tj = tap - ti * e.kw;
        const int toff = (ti * e.RP + (tj & (s - 1)) * e.PWs + (tj >> lg)) * e.SP;
        for (int k = 0; k < k16_per_chunk; ++k) {
          // prefetch the next step's weights (next k16 of this tap, else first k16 of the next tap)
          int ntap = tap, nk = k + 1;
          if (nk == k16_per_chunk) { nk = 0; ntap = tap + 1; }
          if (ntap < ntaps) {
            const bf16x8_t* wp = wchunk + ((size_t)ntap * k16_total + nk) * e.wstride8;
#pragma unroll
            for (int nj = 0; nj < WN; ++nj) bnxt[nj] = wp[nj * 64];
          }
          bf16x8_t a[4];
#pragma unroll
          for (int mi = 0; mi < 4; ++mi) a[mi] = *(const bf16x8_t*)(lds + abase[mi] + toff + k * 32);
#pragma unroll
          for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int nj = 0; nj < WN; ++nj)
              acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[mi], bcur[nj], acc[mi][nj], 0, 0, 0);
#pragma unroll
          for (int nj = 0; nj < WN; ++nj) bcur[nj] = bnxt[nj];
        }
      }
    }
  }

  // ---- epilogue: bias, activation, round to bf16, NHWC store.
  // Accumulator layout: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
  uint16_t* out = (uint16_t*)nd.out[cur];
#pragma unroll
  for (int nj = 0; nj < WN; ++nj) {
    const int col = wave_n0 + nj * 32 + (lane & 31);
    const float bias = nd.bias[col];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = wave_m0 + mi * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < nd.M) {
          float v = acc[mi][nj][r] + bias;
          if (nd.act == 1) v = fmaxf(v, 0.f);
          out[(size_t)row * nd.Cp + col] = float_to_bf16_bits(v);
        }
      }
    }
  }
}

__global__ __launch_bounds__(256, 2) void sr_mfma_kernel(const SrCtx* __restrict__ ctx,
                                                         const SrMfmaNode* __restrict__ nodes,
                                                         const SrMfmaEdge* __restrict__ edges,
                                                         const SrMfmaTile* __restrict__ tiles) {
  extern __shared__ __align__(16) unsigned char sr_lds[];
  const SrMfmaTile t = tiles[blockIdx.x];
  const SrMfmaNode nd = nodes[t.node];
  if (nd.wn_tiles == 2) sr_mfma_tile<2>(ctx, nd, edges, t, sr_lds);
  else sr_mfma_tile<1>(ctx, nd, edges, t, sr_lds);
}

// ---------------------------------------------------------------------------
// launch wrappers
// ---------------------------------------------------------------------------
static inline int blocks_for(long long n, int per) {
  long long b = (n + per - 1) / per;
  if (b < 1) b = 1;
  if (b > 65535LL * 16) b = 65535LL * 16;
  return (int)b;
}

hipError_t sr_launch_set_ctx(hipStream_t s, SrCtx* ctx, const SrCtx& values, int set_frame) {
  hipLaunchKernelGGL(sr_set_ctx_kernel, dim3(1), dim3(64), 0, s, ctx, values, set_frame);
  return hipGetLastError();
}

hipError_t sr_launch_tick(hipStream_t s, SrCtx* ctx) {
  hipLaunchKernelGGL(sr_tick_kernel, dim3(1), dim3(64), 0, s, ctx);
  return hipGetLastError();
}

hipError_t sr_launch_fill_zero(hipStream_t s, void* p, size_t bytes) {
  if (bytes == 0) return hipSuccess;
  size_t n16 = bytes / 16, tail = bytes - n16 * 16;
  int nb = blocks_for((long long)n16, 256 * 4);
  if (nb > 4096) nb = 4096;
  hipLaunchKernelGGL(sr_fill_zero_kernel, dim3(nb), dim3(256), 0, s, (uint4*)p, n16,
                     (unsigned char*)p + n16 * 16, tail);
  return hipGetLastError();
}

hipError_t sr_launch_stage_inputs(hipStream_t s, const SrCtx* ctx, const SrStageNode* nodes, int n_nodes,
                                  int max_elems, int bf16) {
  if (n_nodes == 0) return hipSuccess;
  int nb = blocks_for(max_elems, 256 * 4);
  if (nb > 2048) nb = 2048;
  if (bf16) hipLaunchKernelGGL(sr_stage_inputs_kernel<uint16_t>, dim3(nb, n_nodes), dim3(256), 0, s, ctx, nodes);
  else hipLaunchKernelGGL(sr_stage_inputs_kernel<float>, dim3(nb, n_nodes), dim3(256), 0, s, ctx, nodes);
  return hipGetLastError();
}

hipError_t sr_launch_pack(hipStream_t s, void* dst, const void* src, int px, int C, int Cp, int bf16, int unpack) {
  long long total = (long long)px * (unpack ? C : Cp);
  if (total == 0) return hipSuccess;
  int nb = blocks_for(total, 256 * 4);
  if (nb > 2048) nb = 2048;
  if (bf16) hipLaunchKernelGGL(sr_pack_kernel<uint16_t>, dim3(nb), dim3(256), 0, s, (uint16_t*)dst, (const uint16_t*)src, px, C, Cp, unpack);
  else hipLaunchKernelGGL(sr_pack_kernel<float>, dim3(nb), dim3(256), 0, s, (float*)dst, (const float*)src, px, C, Cp, unpack);
  return hipGetLastError();
}

hipError_t sr_launch_record_output(hipStream_t s, const SrCtx* ctx, const void* state0, const void* state1,
                                   int px, int C, int Cp, int bf16) {
  long long total = (long long)px * C;
  int nb = blocks_for(total, 256 * 4);
  if (nb > 1024) nb = 1024;
  if (bf16) hipLaunchKernelGGL(sr_record_output_kernel<uint16_t>, dim3(nb), dim3(256), 0, s, ctx, (const uint16_t*)state0, (const uint16_t*)state1, px, C, Cp);
  else hipLaunchKernelGGL(sr_record_output_kernel<float>, dim3(nb), dim3(256), 0, s, ctx, (const float*)state0, (const float*)state1, px, C, Cp);
  return hipGetLastError();
}

hipError_t sr_launch_direct(hipStream_t s, const SrCtx* ctx, const SrDirectNode* nodes, const SrDirectEdge* edges,
                            const SrDirectBlock* blocks, int n_blocks, int bf16, int batch) {
  if (n_blocks == 0) return hipSuccess;
  if (bf16) hipLaunchKernelGGL(sr_direct_kernel<uint16_t>, dim3(n_blocks), dim3(256), 0, s, ctx, nodes, edges, blocks, batch);
  else hipLaunchKernelGGL(sr_direct_kernel<float>, dim3(n_blocks), dim3(256), 0, s, ctx, nodes, edges, blocks, batch);
  return hipGetLastError();
}

hipError_t sr_launch_mfma(hipStream_t s, const SrCtx* ctx, const SrMfmaNode* nodes, const SrMfmaEdge* edges,
                          const SrMfmaTile* tiles, int n_tiles, int lds_bytes) {
  if (n_tiles == 0) return hipSuccess;
  hipLaunchKernelGGL(sr_mfma_kernel, dim3(n_tiles), dim3(256), lds_bytes, s, ctx, nodes, edges, tiles);
  return hipGetLastError();
}

hipError_t sr_launch_head(hipStream_t s, const SrCtx* ctx, const SrHead* heads, int n_heads, int max_B,
                          int max_splits, int max_cin, int bf16) {
  if (n_heads == 0) return hipSuccess;
  if (bf16) {
    hipLaunchKernelGGL(sr_gap_partial_kernel<uint16_t>, dim3(max_splits, max_B, n_heads), dim3(256), 0, s, ctx, heads);
    hipLaunchKernelGGL(sr_head_dense_kernel<uint16_t>, dim3(max_B, n_heads), dim3(256), max_cin * sizeof(float), s, ctx, heads);
  } else {
    hipLaunchKernelGGL(sr_gap_partial_kernel<float>, dim3(max_splits, max_B, n_heads), dim3(256), 0, s, ctx, heads);
    hipLaunchKernelGGL(sr_head_dense_kernel<float>, dim3(max_B, n_heads), dim3(256), max_cin * sizeof(float), s, ctx, heads);
  }
  return hipGetLastError();
}

int sr_mfma_max_lds_bytes() { return 64 * 1024; }
