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
#include <atomic>
#include "sr_internal.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4_t;

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
#define SR_GLOBAL __attribute__((address_space(1)))
// load / store: ordinary accesses.  aload / astore: agent-scope accesses (a store goes through to
// memory, a load does not take a stale line from this XCD's L2) for node states, which in a
// dependency-driven launch are produced and consumed by workgroups on different XCDs.
template <> struct Store<float> {
  static __device__ __forceinline__ float aload(const float* p) {
    return __uint_as_float(__hip_atomic_load((const unsigned*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  }
  static __device__ __forceinline__ void astore(float* p, float v) {
    __hip_atomic_store((unsigned*)p, __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ float gload(const SR_GLOBAL float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Store<uint16_t> {
  static __device__ __forceinline__ float aload(const uint16_t* p) {
    return bf16_bits_to_float(__hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  }
  static __device__ __forceinline__ void astore(uint16_t* p, float v) {
    __hip_atomic_store(p, float_to_bf16_bits(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  static __device__ __forceinline__ float load(const uint16_t* p) { return bf16_bits_to_float(*p); }
  static __device__ __forceinline__ float gload(const SR_GLOBAL uint16_t* p) { return bf16_bits_to_float(*p); }
  static __device__ __forceinline__ void store(uint16_t* p, float v) { *p = float_to_bf16_bits(v); }
};

// ---------------------------------------------------------------------------
// bookkeeping kernels
// ---------------------------------------------------------------------------
__global__ void sr_set_ctx_kernel(SrCtx* ctx, SrCtx v, int set_frame) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    const int frame = ctx->frame, timeouts = ctx->dep_timeouts;
    *ctx = v;
    if (!set_frame) {   // a reset clears both; any other call keeps them
      ctx->frame = frame;
      ctx->dep_timeouts = timeouts;
    }
  }
}

__global__ void sr_tick_kernel(SrCtx* ctx) {
  if (threadIdx.x == 0 && blockIdx.x == 0) ctx->frame = ctx->frame + 1;
}

// Called by every workgroup of the last launch of a frame once its work is stored: the workgroup
// that arrives last advances the frame counter by the frames the launch covers (all others have
// read it long before).
__device__ __forceinline__ void sr_block_done(SrCtx* ctx, int n_blocks, int frames) {
  // no fence: the counter only orders "everyone has read the frame counter" (done at kernel start)
  // before its update, and the next launch sees the update through the kernel boundary
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = __hip_atomic_fetch_add(&ctx->done, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (old == n_blocks - 1) {
      ctx->done = 0;
      ctx->frame = ctx->frame + frames;
    }
  }
}

// Dependency-driven launches: wait until every node this work item depends on has completed the
// frames it needs.  The first wave polls, one dependency per lane, sleeping between polls; the other
// waves wait at the barrier.  Counters wrap, so they are compared by signed difference.  The wait is
// bounded: past the spin limit it gives up and reports itself (results are then undefined, the
// launch still ends).
struct SrDepPoll {   // a dependency wait whose first poll is in flight
  const int* counter;
  int need, first, count;
};

// first poll goes out (the caller has other things to do before it needs the answer)
__device__ __forceinline__ SrDepPoll sr_deps_begin(const SrFlow& flow, int begin, int count, int frame) {
  SrDepPoll w;
  w.counter = flow.done;
  w.need = 0;
  w.first = 0;
  w.count = (flow.deps == nullptr) ? 0 : count;
  if (w.count > 0 && threadIdx.x < (unsigned)w.count) {
    const SrDep d = flow.deps[begin + threadIdx.x];
    w.counter = flow.done + d.node * SR_DONE_STRIDE;
    w.need = d.units * (frame - d.lag);
    w.first = __hip_atomic_load(w.counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  return w;
}

// ... and the wait itself
__device__ __forceinline__ void sr_deps_finish(const SrFlow& flow, const SrDepPoll& w, SrCtx* ctx) {
  if (w.count == 0) return;
  if (threadIdx.x < 64) {
    const int lane = threadIdx.x;
    int seen = w.first;
    int spins = 0;
    for (;;) {
      const int ok = (lane >= w.count) || (seen - w.need) >= 0;
      if (__builtin_amdgcn_ballot_w64(!ok) == 0) break;
      // give up at the spin limit -- or at once if any wait of this graph has given up before, so that
      // a broken dependency costs one limit, not one per work item
      int failed = 0;
      if ((spins & 63) == 63) failed = __hip_atomic_load(&ctx->dep_timeouts, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (++spins > flow.spin_limit || failed > 0) {
        if (lane == 0) __hip_atomic_fetch_add(&ctx->dep_timeouts, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        break;
      }
      // back off: the counters are shared by every waiting workgroup of the chip
      if (spins < 16) __builtin_amdgcn_s_sleep(8);
      else if (spins < 64) __builtin_amdgcn_s_sleep(32);
      else __builtin_amdgcn_s_sleep(127);
      if (lane < w.count) seen = __hip_atomic_load(w.counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __syncthreads();
}

__device__ __forceinline__ void sr_wait_deps(const SrFlow& flow, int begin, int count, int frame, SrCtx* ctx) {
  const SrDepPoll w = sr_deps_begin(flow, begin, count, frame);
  sr_deps_finish(flow, w, ctx);
}

// ... and tell the dependants: this work item's results are in memory (its stores were agent-scope
// and have completed when each thread's wait for them ends; the barrier collects the workgroup's).
__device__ __forceinline__ void sr_signal_done(const SrFlow& flow, int gnode) {
  if (flow.deps == nullptr) return;
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0)
    __hip_atomic_fetch_add(flow.done + gnode * SR_DONE_STRIDE, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void sr_fill_zero_kernel(uint4* p, size_t n16, unsigned char* tail, size_t ntail) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) p[i] = make_uint4(0, 0, 0, 0);
  if (blockIdx.x == 0 && threadIdx.x < ntail) tail[threadIdx.x] = 0;
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

// 16-byte agent-scope store of node-state data (see Store<T>::astore)
__device__ __forceinline__ void sr_store16_agent(void* p, u32x4_t v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"((__attribute__((address_space(1))) u32x4_t*)(unsigned long long)p), "v"(v) : "memory");
}

// ---------------------------------------------------------------------------
// auxiliary work items that ride along in a level's launch
// ---------------------------------------------------------------------------
// input staging: state[frame & 1] of an input node := this frame's input, channel pitch C -> Cp;
// one item covers SR_STAGE_CHUNK pixels, one pixel per thread and pass, 16-byte stores when the
// stored pixel is a whole number of them
// `ahead` = 1 stages the NEXT frame's input (into the copy that frame will be read from) while the
// current frame's last launch runs: a pattern whose input edges do not bridge needs frame t's input
// in place before frame t's first launch.  Frames the caller has given no input for are skipped
// (the item still counts as completed for its dependants).
template <typename T>
__device__ __forceinline__ void sr_stage_item(SrCtx* __restrict__ ctx, const SrStageNode& nd, int chunk, int ahead,
                                              int frame_now, const SrFlow& flow) {
  const int frame = frame_now + ahead;
  const char* base = (const char*)ctx->in_ptr[nd.input_slot];
  // the copy written was last read two frames ago (one frame ago, by bridging edges): wait for those readers
  sr_wait_deps(flow, nd.dep_begin, nd.dep_count, frame, ctx);
  if (base != nullptr && frame <= ctx->in_last) {
    const T* in = (const T*)(base + (int64_t)(frame - ctx->in_base) * ctx->in_stride[nd.input_slot]);
    T* out = (T*)nd.state[frame & 1];
    const int end = min(nd.elems_px, (chunk + 1) * SR_STAGE_CHUNK);
    constexpr int V = 16 / sizeof(T);
    if ((nd.Cp == V || nd.Cp == 2 * V) && nd.C <= V && SR_AUX_THREADS * 4 == SR_STAGE_CHUNK) {
      // few channels (an image): one 16-byte piece of data per pixel (and one of zeros if the pitch is two),
      // four pixels per thread, all loads first
      const int p0 = chunk * SR_STAGE_CHUNK + threadIdx.x;
      T v[4][V];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int p = min(p0 + j * SR_AUX_THREADS, nd.elems_px - 1);
        const T* ip = in + (size_t)p * nd.C;
#pragma unroll
        for (int i = 0; i < V; ++i) v[j][i] = (i < nd.C) ? ip[i] : (T)0;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int p = p0 + j * SR_AUX_THREADS;
        if (p < end) {
          sr_store16_agent(out + (size_t)p * nd.Cp, *(const u32x4_t*)v[j]);
          if (nd.Cp == 2 * V) sr_store16_agent(out + (size_t)p * nd.Cp + V, u32x4_t{0u, 0u, 0u, 0u});
        }
      }
    } else if ((nd.Cp % V) == 0) {
      for (int p = chunk * SR_STAGE_CHUNK + threadIdx.x; p < end; p += SR_AUX_THREADS) {
        const T* ip = in + (size_t)p * nd.C;
        for (int c0 = 0; c0 < nd.Cp; c0 += V) {
          T v[V];
#pragma unroll
          for (int i = 0; i < V; ++i) v[i] = (c0 + i < nd.C) ? ip[c0 + i] : (T)0;
          sr_store16_agent(out + (size_t)p * nd.Cp + c0, *(const u32x4_t*)v);
        }
      }
    } else {
      for (int p = chunk * SR_STAGE_CHUNK + threadIdx.x; p < end; p += SR_AUX_THREADS)
        for (int c = 0; c < nd.Cp; ++c)
          Store<T>::astore(out + (size_t)p * nd.Cp + c, (c < nd.C) ? Store<T>::load(in + (size_t)p * nd.C + c) : 0.f);
    }
  }
  sr_signal_done(flow, nd.gnode);
}

// Head node (App. A2: fully connected layers, optionally after global average pooling): a 1x1 node
// whose incoming edges are all dense or GAP+dense.  One item per image (and, for a single pooled
// edge over many pixels, per pixel slab: the slab sums go to `partial` and the item that finishes
// last for an image adds them in slab order).  For every edge the input vector (pooled means or the
// flattened source) is put into LDS, then each of the 4 waves multiplies a quarter of it into up to
// 256 outputs (with at most 64 outputs: 256 / CO slices of it into CO = 16, 32 or 64 output columns);
// the parts are added in a fixed order, then bias, activation, store and, if this node is being
// recorded, the rollout output.  smem: SR_HEAD_MAX_K floats, one int, 4*64*4 floats.
template <typename T>
__device__ __forceinline__ bool sr_head_body(const SrCtx* __restrict__ ctx, const SrHead& h,
                                             const SrHeadEdge* __restrict__ head_edges, int b, int split,
                                             float* smem, int vec_floats, int frame) {
  const int cur = frame & 1;
  int* flag = (int*)(smem + vec_floats);
  float* red = smem + vec_floats + 4;
  const int lane = threadIdx.x & 63, part = threadIdx.x >> 6;
  float acc[4] = {0.f, 0.f, 0.f, 0.f};     // outputs lane, lane+64, lane+128, lane+192: this wave's share
  // up to 64 outputs: CO = 16, 32 or 64 output columns, 256 / CO slices of the input vector
  const bool narrow = h.Cout <= 64;
  const int CO = h.Cout <= 16 ? 16 : (h.Cout <= 32 ? 32 : 64);
  const int n_slices = 256 / CO;
  const int co_n = threadIdx.x & (CO - 1), slice = threadIdx.x / CO;
  for (int ei = 0; ei < h.edge_count; ++ei) {
    const SrHeadEdge e = head_edges[h.edge_begin + ei];
    const T* src = (const T*)((e.bridge ? (cur ^ 1) : cur) ? e.src[1] : e.src[0]) + (size_t)b * e.HW * e.Csp;
    int K;
    __syncthreads();   // the previous edge's vector is no longer needed
    if (e.pooled) {
      K = e.Cin;
      const int per = (e.HW + h.splits - 1) / h.splits;
      const int p0 = split * per, p1 = min(e.HW, p0 + per);
      const float inv = 1.0f / (float)e.HW;
      for (int c = threadIdx.x; c < e.Cin; c += SR_AUX_THREADS) {
        float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
        int p = p0;
        for (; p + 12 <= p1; p += 12) {   // twelve loads in flight
          float v[12];
#pragma unroll
          for (int u = 0; u < 12; ++u) v[u] = Store<T>::aload(src + (size_t)(p + u) * e.Csp + c);
          s0 += (v[0] + v[4]) + v[8];
          s1 += (v[1] + v[5]) + v[9];
          s2 += (v[2] + v[6]) + v[10];
          s3 += (v[3] + v[7]) + v[11];
        }
        for (; p + 4 <= p1; p += 4) {
          s0 += Store<T>::aload(src + (size_t)p * e.Csp + c);
          s1 += Store<T>::aload(src + (size_t)(p + 1) * e.Csp + c);
          s2 += Store<T>::aload(src + (size_t)(p + 2) * e.Csp + c);
          s3 += Store<T>::aload(src + (size_t)(p + 3) * e.Csp + c);
        }
        for (; p < p1; ++p) s0 += Store<T>::aload(src + (size_t)p * e.Csp + c);
        const float sum = (s0 + s1) + (s2 + s3);
        if (h.splits == 1) smem[c] = sum * inv;
        else   // device-coherent (write-through) store, read back below by whichever slab finishes last
          __hip_atomic_store(&h.partial[((size_t)b * h.splits + split) * e.Cin + c], sum, __ATOMIC_RELAXED,
                             __HIP_MEMORY_SCOPE_AGENT);
      }
      if (h.splits > 1) {   // only single-edge heads are cut into slabs
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (threadIdx.x == 0) {
          const int old = __hip_atomic_fetch_add(&h.counters[b], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
          *flag = (old == h.splits - 1);
          if (old == h.splits - 1) h.counters[b] = 0;
        }
        __syncthreads();
        if (!*flag) return false;
        for (int c = threadIdx.x; c < e.Cin; c += SR_AUX_THREADS) {
          float sum = 0.f;
          for (int s = 0; s < h.splits; ++s)
            sum += __hip_atomic_load(&h.partial[((size_t)b * h.splits + s) * e.Cin + c], __ATOMIC_RELAXED,
                                     __HIP_MEMORY_SCOPE_AGENT);
          smem[c] = sum * inv;
        }
      }
    } else {
      K = e.HW * e.Cin;
      for (int k = threadIdx.x; k < K; k += SR_AUX_THREADS) {
        const int p = k / e.Cin, c = k - p * e.Cin;
        smem[k] = Store<T>::aload(src + (size_t)p * e.Csp + c);
      }
    }
    __syncthreads();
    if (narrow) {
      // few outputs: the threads are arranged (slice of the vector) x (output)
      const int kper = (K + n_slices - 1) / n_slices;
      const int k_lo = slice * kper, k_hi = min(K, k_lo + kper);
      if (co_n < h.Cout) {
        // sixteen independent chains keep sixteen weight loads in flight
        float a[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) a[u] = 0.f;
        int k = k_lo;
        for (; k + 16 <= k_hi; k += 16) {
          float wv[16];
#pragma unroll
          for (int u = 0; u < 16; ++u) wv[u] = e.w[(size_t)(k + u) * h.Cout + co_n];
#pragma unroll
          for (int u = 0; u < 16; ++u) a[u] += smem[k + u] * wv[u];
        }
        for (; k < k_hi; ++k) a[0] += smem[k] * e.w[(size_t)k * h.Cout + co_n];
        const float a0 = (a[0] + a[1]) + (a[2] + a[3]), a1 = (a[4] + a[5]) + (a[6] + a[7]);
        const float a2 = (a[8] + a[9]) + (a[10] + a[11]), a3 = (a[12] + a[13]) + (a[14] + a[15]);
        acc[0] += (a0 + a1) + (a2 + a3);
      }
    } else {
      const int kper = (K + 3) / 4;
      const int k_lo = part * kper, k_hi = min(K, k_lo + kper);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int co = lane + 64 * j;
        if (co < h.Cout) {
          float p8[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // eight weight loads in flight
          int k = k_lo;
          for (; k + 8 <= k_hi; k += 8) {
            float wv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) wv[u] = e.w[(size_t)(k + u) * h.Cout + co];
#pragma unroll
            for (int u = 0; u < 8; ++u) p8[u] += smem[k + u] * wv[u];
          }
          for (; k < k_hi; ++k) p8[0] += smem[k] * e.w[(size_t)k * h.Cout + co];
          acc[j] += ((p8[0] + p8[1]) + (p8[2] + p8[3])) + ((p8[4] + p8[5]) + (p8[6] + p8[7]));
        }
      }
    }
  }
  char* rec = h.record ? (char*)ctx->out_ptr : nullptr;
  T* recp = rec ? (T*)(rec + (int64_t)(frame - ctx->out_base) * ctx->out_stride) : nullptr;
  if (narrow) {
    red[slice * CO + co_n] = acc[0];
    __syncthreads();
    for (int co = threadIdx.x; co < h.Cout; co += SR_AUX_THREADS) {
      float v = 0.f;
      for (int sl = 0; sl < n_slices; ++sl) v += red[sl * CO + co];   // slice order: deterministic
      v += h.bias[co];
      if (h.act == 1) v = fmaxf(v, 0.f);
      Store<T>::astore((T*)h.out[cur] + (size_t)b * h.Cp + co, v);
      if (recp) Store<T>::store(recp + (size_t)b * h.Cout + co, v);
    }
    return true;
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) red[(part * 4 + j) * 64 + lane] = acc[j];
  __syncthreads();
  for (int co = threadIdx.x; co < h.Cout; co += SR_AUX_THREADS) {
    const int j = co >> 6, l = co & 63;
    float v = h.bias[co] + ((red[(0 * 4 + j) * 64 + l] + red[(1 * 4 + j) * 64 + l]) +
                            (red[(2 * 4 + j) * 64 + l] + red[(3 * 4 + j) * 64 + l]));
    if (h.act == 1) v = fmaxf(v, 0.f);
    Store<T>::astore((T*)h.out[cur] + (size_t)b * h.Cp + co, v);
    if (recp) Store<T>::store(recp + (size_t)b * h.Cout + co, v);
  }
  return true;
}

// ... as a work item: wait for the source nodes (and for the readers of the copy about to be
// overwritten), compute, and count the image as done once its outputs are in memory
template <typename T>
__device__ __forceinline__ void sr_head_item(SrCtx* __restrict__ ctx, const SrHead& h,
                                             const SrHeadEdge* __restrict__ head_edges, int b, int split,
                                             float* smem, int vec_floats, int frame, const SrFlow& flow) {
  sr_wait_deps(flow, h.dep_begin, h.dep_count, frame, ctx);
  const bool wrote = sr_head_body<T>(ctx, h, head_edges, b, split, smem, vec_floats, frame);
  if (wrote) sr_signal_done(flow, h.gnode);
}


template <typename T>
__device__ __forceinline__ void sr_aux_item(SrCtx* __restrict__ ctx, const SrAux& it,
                                            const SrHead* __restrict__ heads,
                                            const SrHeadEdge* __restrict__ head_edges,
                                            const SrStageNode* __restrict__ stage_nodes, float* smem, int vec_floats,
                                            int frame, const SrFlow& flow) {
  if (it.kind == SR_AUX_HEAD) sr_head_item<T>(ctx, heads[it.a], head_edges, it.b, it.c, smem, vec_floats, frame, flow);
  else if (it.kind == SR_AUX_STAGE) sr_stage_item<T>(ctx, stage_nodes[it.a], it.b, it.c, frame, flow);
}

// ---------------------------------------------------------------------------
// direct path
// ---------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ void sr_direct_block(const SrCtx* __restrict__ ctx, const SrDirectNode& nd,
                                                const SrDirectEdge* __restrict__ edges, int first, int batch) {
  const int cur = ctx->frame & 1;
  const int idx = first + threadIdx.x;
  const int HW = nd.H * nd.W;
  if (idx >= batch * HW * nd.C) return;
  const int m = idx / nd.C, co = idx - m * nd.C;
  const int b = m / HW, r = m - b * HW;
  const int oy = r / nd.W, ox = r - oy * nd.W;
  float acc = nd.bias[co];
  for (int ei = 0; ei < nd.edge_count; ++ei) {
    const SrDirectEdge e = edges[nd.edge_begin + ei];
    // global (not generic) pointers: plain global loads; the copy is picked by a select, not by a dynamic
    // index into the by-value descriptor (which would put the whole descriptor into scratch memory)
    const SR_GLOBAL T* src = (const SR_GLOBAL T*)(unsigned long long)((e.bridge ? (cur ^ 1) : cur) ? e.src[1] : e.src[0]);
    const SR_GLOBAL float* wts = (const SR_GLOBAL float*)(unsigned long long)e.w;
    if (e.kind == 0) {
      const int sy = (oy / e.up) * e.stride - e.pad;
      const int sx = (ox / e.up) * e.stride - e.pad;
      // branch-free: taps outside the source read a clamped (valid) pixel and are replaced by zero, so the
      // loads of several taps and channels can be in flight together; the sum keeps the order
      // (tap row, tap column, channel)
      for (int i = 0; i < e.kh; ++i) {
        const int iy = sy + i;
        const bool row_ok = iy >= 0 && iy < e.Hs;
        const int iyc = min(max(iy, 0), e.Hs - 1);
#pragma unroll 4
        for (int j = 0; j < e.kw; ++j) {
          const int ix = sx + j;
          const bool keep = row_ok && ix >= 0 && ix < e.Ws;
          const int ixc = min(max(ix, 0), e.Ws - 1);
          const SR_GLOBAL T* px = src + ((size_t)(b * e.Hs + iyc) * e.Ws + ixc) * e.Csp;
          const SR_GLOBAL float* w = wts + (size_t)(i * e.kw + j) * e.Cin * nd.C + co;
#pragma unroll 4
          for (int ci = 0; ci < e.Cin; ++ci) {
            const float v = Store<T>::gload(px + ci);
            acc += (keep ? v : 0.f) * w[(size_t)ci * nd.C];
          }
        }
      }
    } else {  // mean over (h,w), then dense
      const int n = e.Hs * e.Ws;
      const float inv = 1.0f / (float)n;
      const SR_GLOBAL T* img = src + (size_t)b * n * e.Csp;
      for (int ci = 0; ci < e.Cin; ++ci) {
        float s = 0.f;
        for (int p = 0; p < n; ++p) s += Store<T>::gload(img + (size_t)p * e.Csp + ci);
        acc += (s * inv) * wts[(size_t)ci * nd.C + co];
      }
    }
  }
  if (nd.act == 1) acc = fmaxf(acc, 0.f);
  Store<T>::store((T*)nd.out[cur] + (size_t)m * nd.Cp + co, acc);
}

template <typename T>
__global__ __launch_bounds__(256) void sr_direct_kernel(SrCtx* __restrict__ ctx, const SrDirectNode* __restrict__ nodes,
                                                        const SrDirectEdge* __restrict__ edges,
                                                        const SrDirectBlock* __restrict__ blocks, int n_blocks,
                                                        int batch, const SrAux* __restrict__ aux,
                                                        const SrHead* __restrict__ heads,
                                                        const SrHeadEdge* __restrict__ head_edges,
                                                        const SrStageNode* __restrict__ stage_nodes, int vec_floats,
                                                        int is_last) {
  extern __shared__ float sr_aux_smem[];
  if ((int)blockIdx.x < n_blocks) {
    const SrDirectBlock blk = blocks[blockIdx.x];
    sr_direct_block<T>(ctx, nodes[blk.node], edges, blk.first, batch);
  } else {
    sr_aux_item<T>(ctx, aux[blockIdx.x - n_blocks], heads, head_edges, stage_nodes, sr_aux_smem, vec_floats, ctx->frame,
                   SrFlow{nullptr, nullptr, 0, 0, nullptr});
  }
  if (is_last) sr_block_done(ctx, gridDim.x, 1);
}

// ---------------------------------------------------------------------------
// MFMA path
// ---------------------------------------------------------------------------
// Workgroup = 4 wave64 arranged waves_m x waves_n; each wave owns 128 pixels x (32*WN) channels:
// 4 x WN accumulator tiles of v_mfma_f32_32x32x16_bf16.  Operand layout of that instruction: lane l
// supplies row (A) / column (B) l % 32 and 8 consecutive k values selected by l / 32.
//
// A operand (pixels x channels of the source): the source patch that the tile's pixels touch is
// staged once per KC channels in LDS and re-read for every tap.  It is written by direct-to-LDS
// loads (no registers in between), all issued back to back, so a stage costs one memory latency;
// a second workgroup on the same CU computes meanwhile.  LDS slot of padded source pixel
// (row q relative to the tile's first row, column px), column-phase major for strided edges so
// that consecutive output pixels read consecutive slots:
//     byte = q*RPB + ((px % stride)*PWs + px / stride)*SP,   SP = KC*2 + 16 bytes per slot.
// The spare 16-byte piece of every slot (and a row pitch RPB chosen to match) makes sixteen
// consecutive pixels fall into sixteen different 16-byte columns of the 256-byte LDS row, which
// is what a conflict-free ds_read_b128 needs.
//
// B operand (weights): pre-packed on the host in exactly the per-lane order of the instruction,
// [tap][k16 block][32-channel tile][lane][8], so a wave's fragment is one coalesced 1 KiB load
// straight into registers, prefetched a few k-steps ahead through a small ring.
#define SR_RING 5   // depth of the weight-fragment ring
#define SR_UNROLL 5 // k-steps per loop body: a multiple of the ring depth

typedef const __attribute__((address_space(1))) bf16x8_t* sr_gfrag_ptr;   // global memory
#define SR_UNIFORM(x) __builtin_amdgcn_readfirstlane(x)

// Wave-uniform copy of an edge descriptor, read through the constant address space so that it
// lives in scalar registers and all per-step address arithmetic stays on the scalar unit.
struct SrEdgeK {
  const unsigned char* src;
  sr_gfrag_ptr wpk;
  int lgRS, lgup, lgK16, nchunk, PHr, RPB, imgB, rowB, r0B, wstride8, src_bytes;
};

typedef int sr_i32x16 __attribute__((ext_vector_type(16)));
__device__ __forceinline__ SrEdgeK sr_load_edge(const __attribute__((address_space(4))) SrPlane4* planes, int index, int cur) {
  // one 64-byte scalar load; everything the kernel derives from it is register arithmetic
  const sr_i32x16 v = *(const __attribute__((address_space(4))) sr_i32x16*)(planes + index);
  SrEdgeK k;
  const int flags = v[6];
  const int pick = (flags & 1) ? (cur ^ 1) : cur;
  const unsigned lo = pick ? (unsigned)v[2] : (unsigned)v[0], hi = pick ? (unsigned)v[3] : (unsigned)v[1];
  k.src = (const unsigned char*)(((unsigned long long)hi << 32) | lo);
  k.wpk = (sr_gfrag_ptr)(((unsigned long long)(unsigned)v[5] << 32) | (unsigned)v[4]);
  k.lgRS = (flags >> 8) & 0xff;
  k.lgup = (flags >> 16) & 0xff;
  k.lgK16 = (flags >> 24) & 0xff;
  k.nchunk = v[7];
  k.PHr = v[8];
  k.RPB = v[9];
  k.imgB = v[10]; k.rowB = v[11]; k.r0B = v[12];
  k.wstride8 = v[13];
  k.src_bytes = v[14];
  return k;
}

// what the tile needs of a plane ahead of its descriptor (SrPlanRef, scalar registers)
struct SrRefK { int plan_at, n_pos, tap_begin, ntaps; };
__device__ __forceinline__ SrRefK sr_load_ref(const __attribute__((address_space(4))) int* refs, int index) {
  SrRefK r;
  r.plan_at = refs[index * 4];
  r.n_pos = refs[index * 4 + 1];
  r.tap_begin = refs[index * 4 + 2];
  r.ntaps = refs[index * 4 + 3];
  return r;
}

// Direct-to-LDS staging.  The LDS patch is an array of 16-byte positions: row q (padded source
// row relative to the tile's first one) starts at q*RPB, slot c of a row at c*SP, piece p of a
// slot at p*16; the last piece of a slot is the spare one.  Which source bytes a position holds
// does not depend on the channel chunk, so the host tabulates it once per (tile, edge) --
// identical tables are shared -- as a byte offset from the tile's first source row, or ZERO for
// padding.  Positions that are never read (spare pieces, row pitch, the tail of the last
// kilobyte) repeat their predecessor's entry, so that every lane of every instruction loads and a
// stage's issue is four instructions per load: no lane masks, no address selects.  ZERO becomes
// the offset of the zero bytes that follow every state (far enough behind it for any chunk's
// offset to stay inside them).  A thread keeps its entries in registers for the whole edge; a
// stage only adds the chunk's offset to the (scalar) base.
#define SR_DMA_ITEMS 20        // positions per thread: 80 KiB of LDS / 16 bytes / 256 threads
#define SR_DMA_ZERO (-1)

__device__ __forceinline__ const unsigned char* sr_uniform_ptr(const unsigned char* p) {
  const unsigned long long v = (unsigned long long)p;
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return (const unsigned char*)(((unsigned long long)hi << 32) | lo);
}

__device__ __forceinline__ void sr_dma_plan(const __attribute__((address_space(1))) int* __restrict__ table,
                                            int n_pos, int tid, int (&off)[SR_DMA_ITEMS]) {
#pragma unroll
  for (int it = 0; it < SR_DMA_ITEMS; ++it) {
    int v = 0;
    if (it * 256 < n_pos) v = table[tid + it * 256];   // tables are padded to 256 entries
    off[it] = v;                                        // SR_DMA_ZERO entries are resolved by the plane's set-up
  }
}

__device__ __forceinline__ void sr_stage_dma(const unsigned char* __restrict__ base, unsigned char* lds,
                                             int n_pos, int tid, int (&off)[SR_DMA_ITEMS]) {
  const int wave_pos = SR_UNIFORM(tid & ~63);
  base = sr_uniform_ptr(base);
#pragma unroll
  for (int it = 0; it < SR_DMA_ITEMS; ++it) {
    const int P0 = wave_pos + it * 256;     // first position of this wave's 1 KiB piece
    if (P0 < n_pos) {
      asm volatile("" : "+v"(off[it]));   // keeps the offset 32-bit: scalar base + 32-bit lane offset addressing
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + (unsigned)off[it]),
                                       (__attribute__((address_space(3))) void*)(lds + (size_t)P0 * 16), 16, 0,
                                       16 /* sc1: agent scope, the state may have been written on another XCD */);
    }
  }
}

// k-step st of a stage = (tap, 16-channel block k inside the chunk).  The per-tap parts of the
// offsets -- LDS byte offset of the tap's A fragments relative to tap (0,0), index of the tap's
// first weight fragment -- are tabulated on the host per plane and held with one tap per lane
// (SrTaps); a step then costs a shift, a mask and a lane read instead of a division and five multiplies.  This matters
// when a wave has its SIMD to itself: a wave's own non-MFMA instructions do not overlap with its
// MFMAs (only another wave's do), so every instruction of the step's bookkeeping costs MFMA time.
struct SrTaps { int a; int b; };   // one tap per lane
__device__ __forceinline__ SrTaps sr_tap_table(const SrRefK& r, const __attribute__((address_space(1))) SrTap* table,
                                               int lane) {
  const __attribute__((address_space(1))) SrTap* p = table + r.tap_begin + min(lane, r.ntaps - 1);
  SrTaps t;
  t.a = p->a;
  t.b = p->b;
  return t;
}
__device__ __forceinline__ int sr_step_aoff(const SrEdgeK& e, const SrTaps& t, int st) {
  const int tap = st >> e.lgK16;
  return __builtin_amdgcn_readlane(t.a, tap) + ((st - (tap << e.lgK16)) << 5);
}
__device__ __forceinline__ int sr_step_boff(const SrEdgeK& e, const SrTaps& t, int st) {
  const int tap = st >> e.lgK16;
  return __builtin_amdgcn_readlane(t.b, tap) + (st - (tap << e.lgK16)) * e.wstride8;
}

// One k-step: 4 x WN MFMAs.  Each A fragment is reloaded for the next step right after its last
// use, which leaves the other rows' MFMAs to cover the LDS latency; the weight fragments of ring
// slot `b` are replaced, once used, by those of step st + SR_RING (the ring is deep enough to cover
// the L2 latency even when the workgroup has the compute unit to itself).  The loads are
// unconditional (past the end of the stage they repeat its last step) so that the loop body is
// branch-free and the hardware wait counters can be tracked exactly.
template <int WN>
__device__ __forceinline__ void sr_step(const SrEdgeK& e, const SrTaps& taps, const unsigned char* lds,
                                        const int (&abase)[4], sr_gfrag_ptr wchunk, bf16x8_t (&a)[4],
                                        bf16x8_t (&b)[WN], f32x16_t (&acc)[4][WN], int st, int NS) {
  const int aoff = sr_step_aoff(e, taps, min(st + 1, NS - 1));
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
    for (int nj = 0; nj < WN; ++nj)
      acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[nj], a[mi], acc[mi][nj], 0, 0, 0);
    a[mi] = *(const bf16x8_t*)(lds + abase[mi] + aoff);
  }
  const int boff = sr_step_boff(e, taps, min(st + SR_RING, NS - 1));
#pragma unroll
  for (int nj = 0; nj < WN; ++nj) b[nj] = wchunk[boff + nj * 64];
  // issue order: lane read of the next A offset; then, four times, WN MFMAs followed by the address
  // add and the LDS read of the row they have just released; then the lane read and address of the
  // weight fragments and their loads
  __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);      // VALU (lane read)
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    __builtin_amdgcn_sched_group_barrier(0x008, WN, 0);   // MFMA
    __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);    // VALU (address)
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);    // DS read
  }
  __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);      // VALU (lane read, pointer)
  __builtin_amdgcn_sched_group_barrier(0x020, WN, 0);     // VMEM read
}

// One stage of the contraction: NS = taps * KC/16 k-steps over the patch in LDS.
template <int WN>
__device__ __forceinline__ void sr_stage_compute(const SrEdgeK& e, const SrTaps& taps, const unsigned char* lds,
                                                 const int (&abase)[4], sr_gfrag_ptr wchunk, bf16x8_t (&bq)[SR_RING][WN],
                                                 f32x16_t (&acc)[4][WN], int NS) {
  bf16x8_t a[4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) a[mi] = *(const bf16x8_t*)(lds + abase[mi]);
  int st0 = 0;
  for (; st0 + SR_UNROLL <= NS; st0 += SR_UNROLL) {
#pragma unroll
    for (int u = 0; u < SR_UNROLL; ++u) sr_step<WN>(e, taps, lds, abase, wchunk, a, bq[u % SR_RING], acc, st0 + u, NS);
  }
  // remaining 0..SR_UNROLL-1 steps (their weight fragments are already in ring slots 0, 1, ...)
#pragma unroll
  for (int u = 0; u < SR_UNROLL - 1; ++u)
    if (st0 + u < NS) sr_step<WN>(e, taps, lds, abase, wchunk, a, bq[u % SR_RING], acc, st0 + u, NS);
}

// K-split hand-off between the workgroups that share a tile.  Every part stores its accumulators to
// its slab, [register pair][thread]; the part whose increment of the tile's counter finds all others
// done adds the slabs up in part order and returns true (the others return false and leave).
// The slabs are written and read with agent-scope accesses (write-through stores, loads that do not
// take a stale line from this XCD's L2), so they may live in any device memory; a thread's stores
// have completed when its wait for them ends, the barrier collects the workgroup's, and only then is
// the counter raised.  The last part resets the counter for the next launch.
template <int WN, int THREADS>
__device__ __forceinline__ bool sr_split_reduce(f32x16_t (&acc)[4][WN], const SrSplitScratch& split, int split_slot,
                                                int part_info, int slab_floats, int tid, int* flag) {
  const int n_parts = part_info >> 16;
  unsigned long long* mine =
      (unsigned long long*)(split.slabs + (size_t)(split_slot + (part_info & 0xffff)) * slab_floats) + tid;
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int nj = 0; nj < WN; ++nj)
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const unsigned long long v = (unsigned long long)__float_as_uint(acc[mi][nj][2 * q]) |
                                     ((unsigned long long)__float_as_uint(acc[mi][nj][2 * q + 1]) << 32);
        __hip_atomic_store(mine + ((mi * WN + nj) * 8 + q) * THREADS, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's partial sums have reached memory
  __syncthreads();
  if (tid == 0) {
    int* counter = split.counters + split_slot;
    const int old = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *flag = (old == n_parts - 1);
    if (old == n_parts - 1) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();
  if (!*flag) return false;
  // part by part (so that all of a part's loads are in flight together), every element summed in
  // part order
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int nj = 0; nj < WN; ++nj)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][nj][r] = 0.f;
  const unsigned long long* all = (const unsigned long long*)(split.slabs + (size_t)split_slot * slab_floats) + tid;
  for (int p = 0; p < n_parts; ++p) {
    const unsigned long long* part = all + (size_t)p * (slab_floats / 2);
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int nj = 0; nj < WN; ++nj)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          const unsigned long long v = __hip_atomic_load(part + ((mi * WN + nj) * 8 + q) * THREADS, __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT);
          acc[mi][nj][2 * q] += __uint_as_float((unsigned)v);
          acc[mi][nj][2 * q + 1] += __uint_as_float((unsigned)(v >> 32));
        }
  }
  return true;
}

// A tile record as the kernel holds it (scalar registers)
struct SrTileK {
  int node, m0, n0, ref_base, p_first, p_last, c_first, c_end, split_slot, part, wn_tiles, b_first, b_last, oy_first, oy_last;
  SrRefK ref0;
};

__device__ __forceinline__ SrTileK sr_load_tile(const SrTile4* tiles, int index) {
  const sr_i32x16 v = *(const __attribute__((address_space(4))) sr_i32x16*)(unsigned long long)(tiles + index);
  SrTileK t;
  t.node = v[0]; t.m0 = v[1]; t.n0 = v[2]; t.ref_base = v[3];
  t.p_first = v[4]; t.p_last = v[5];
  t.c_first = v[6] & 0xffff; t.c_end = (unsigned)v[6] >> 16;
  t.split_slot = v[7]; t.part = v[8];
  t.wn_tiles = v[9] & 0xff;
  t.b_first = v[10]; t.b_last = v[10] + ((unsigned)v[9] >> 8);
  t.oy_first = v[11] & 0xffff; t.oy_last = (unsigned)v[11] >> 16;
  t.ref0.plan_at = v[12]; t.ref0.n_pos = v[13]; t.ref0.tap_begin = v[14]; t.ref0.ntaps = v[15];
  return t;
}

template <int WN>
__device__ __forceinline__ void sr_mfma_tile(SrCtx* __restrict__ ctx, const SrTables4& tb, const SrTileK& t,
                                             unsigned char* lds, const SrSplitScratch& split, int frame,
                                             const SrFlow& flow) {
  // the node's record: one scalar load, in flight together with the frame counter and the first plane's
  // plan, taps and descriptor (the tile record names them all)
  const sr_i32x16 nv = *(const __attribute__((address_space(4))) sr_i32x16*)(unsigned long long)(tb.nodes + t.node);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = SR_UNIFORM(tid >> 6);
  const int cur = frame & 1;
  const int M = nv[6], Wo = nv[8], HoWo = nv[7] * nv[8];
  const int Cp = nv[9], act = nv[10];
  const int waves_n = nv[12];
  const int wm = (waves_n == 4) ? 0 : (waves_n == 2 ? (wave >> 1) : wave);
  const int wn = wave - wm * waves_n;
  const int tile_m0 = t.m0, tile_n0 = t.n0;
  const int wave_m0 = tile_m0 + wm * 128;
  const int wave_n0 = tile_n0 + wn * (32 * WN);
  const int ntile0 = wave_n0 >> 5;
  const int b_first = t.b_first, oy_first = t.oy_first, b_last = t.b_last, oy_last = t.oy_last;
  const int split_slot = t.split_slot, part_info = t.part;
  const __attribute__((address_space(4))) int* refs =
      (const __attribute__((address_space(4))) int*)(unsigned long long)tb.refs + (long long)t.ref_base * 4;
  const __attribute__((address_space(1))) int* plan_tables =
      (const __attribute__((address_space(1))) int*)(unsigned long long)tb.plan_tables;
  const __attribute__((address_space(1))) SrTap* tap_table =
      (const __attribute__((address_space(1))) SrTap*)(unsigned long long)tb.tap_table;
  const __attribute__((address_space(4))) SrPlane4* planes =
      (const __attribute__((address_space(4))) SrPlane4*)(unsigned long long)tb.planes;
  // dependency-driven launch: what the tile reads (first nv[14] & 0xff entries of its node's list) is
  // polled now and waited for before the first patch load; what it overwrites (the next nv[14] >> 8
  // entries: the readers of the copy this frame replaces) before the epilogue's stores
  const SrDepPoll dep_read = sr_deps_begin(flow, nv[13], nv[14] & 0xff, frame);

  // Everything a plane's first stage needs goes out at once: plan and taps (vector loads, located by the
  // plan reference that the tile record, or the previous plane, has fetched) and the descriptor (one
  // scalar load).  For the first plane that is here, ahead of the tile's own set-up.
  int p = t.p_first;
  SrRefK ref = t.ref0;
  int dma_off[SR_DMA_ITEMS];
  sr_dma_plan(plan_tables + ref.plan_at, ref.n_pos, tid, dma_off);
  SrTaps taps = sr_tap_table(ref, tap_table, lane);
  SrEdgeK e = sr_load_edge(planes, p, cur);

  // pixel coordinates of this lane's 4 rows, packed: ox | oy << 12 | (image - first image) << 24;
  // rows past the end repeat the last pixel
  int pix[4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    const int m = min(wave_m0 + mi * 32 + (lane & 31), M - 1);
    const int b = m / HoWo;
    const int r = m - b * HoWo;
    const int oy = r / Wo;
    pix[mi] = (r - oy * Wo) | (oy << 12) | ((b - b_first) << 24);
  }

  f32x16_t acc[4][WN];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int nj = 0; nj < WN; ++nj)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][nj][r] = 0.f;

  // dependency-driven launch: before the first patch is read the node's sources must have completed
  // the frames this tile reads, and the node itself its previous frame (its K-split scratch is free then)
  sr_deps_finish(flow, dep_read, ctx);

  // The tile walks the planes p_first..p_last of the plane table; a plane's plan reference (where its
  // plan and taps are) is fetched during the previous plane, so that at the top of a plane its plan,
  // taps and descriptor all go out together.
  for (;;) {
    const bool more = p < t.p_last;
    SrRefK ref_n = ref;
    if (more) ref_n = sr_load_ref(refs, p + 1);   // in flight during this plane's stages
    const int chunk_lo = (p == t.p_first) ? t.c_first : 0;
    const int chunk_hi = (p == t.p_last) ? t.c_end : e.nchunk;
    const int row_first = (oy_first >> e.lgup) << e.lgRS;         // first patch row of the tile, in its image
    const int n_pos = ref.n_pos;
    const int NS = ref.ntaps << e.lgK16;
    // plan offsets count from the source row that patch row row_first stands for, in image b_first;
    // padding positions read the zero bytes behind the state
    const long long base_off = (long long)b_first * e.imgB + (long long)row_first * e.rowB + e.r0B;
    const unsigned char* dma_base = e.src + base_off;
    // LDS byte address of the tap (0,0), k = 0 fragment of this lane's 4 rows
    const int SP = (32 << e.lgK16) + 16;
    int abase[4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
      const int ox = pix[mi] & 0xfff, oy = (pix[mi] >> 12) & 0xfff, db = pix[mi] >> 24;
      abase[mi] = (db * e.PHr + ((oy >> e.lgup) << e.lgRS) - row_first) * e.RPB + (ox >> e.lgup) * SP + (lane >> 5) * 16;
      asm volatile("" : "+v"(abase[mi]));   // keep it in a register: one add per k-step, not a re-derivation
    }
    {
      const int zero_off = (int)((long long)e.src_bytes - base_off);
#pragma unroll
      for (int it = 0; it < SR_DMA_ITEMS; ++it) dma_off[it] = (dma_off[it] == SR_DMA_ZERO) ? zero_off : dma_off[it];
    }
    const sr_gfrag_ptr wlane = e.wpk + ntile0 * 64 + lane;
    for (int chunk = chunk_lo; chunk < chunk_hi; ++chunk) {
      const sr_gfrag_ptr wchunk = wlane + (size_t)(chunk << e.lgK16) * e.wstride8;
      __syncthreads();   // everyone has finished reading the previous patch
      // the first weight fragments go out ahead of the patch so that both are in flight together
      bf16x8_t bq[SR_RING][WN];
#pragma unroll
      for (int d = 0; d < SR_RING; ++d) {
        const int boff = sr_step_boff(e, taps, min(d, NS - 1));
#pragma unroll
        for (int nj = 0; nj < WN; ++nj) bq[d][nj] = wchunk[boff + nj * 64];
      }
      sr_stage_dma(dma_base + (size_t)(chunk << e.lgK16) * 32, lds, n_pos, tid, dma_off);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's direct-to-LDS loads have landed
      __syncthreads();                                     // ... and everybody else's
      __builtin_amdgcn_s_setprio(3);   // k-steps go ahead of the other workgroup's set-up and issue on this SIMD
      sr_stage_compute<WN>(e, taps, lds, abase, wchunk, bq, acc, NS);
      __builtin_amdgcn_s_setprio(0);
    }
    if (!more) break;
    ref = ref_n;
    ++p;
    sr_dma_plan(plan_tables + ref.plan_at, ref.n_pos, tid, dma_off);
    taps = sr_tap_table(ref, tap_table, lane);
    e = sr_load_edge(planes, p, cur);
  }

  // ---- K-split tiles: leave the accumulators in scratch; the part that arrives last adds all parts
  // in part order (so the result does not depend on which part that is) and goes on to the epilogue.
  if ((part_info >> 16) > 1 &&
      !sr_split_reduce<WN, 256>(acc, split, split_slot, part_info, SR_SPLIT_FLOATS, tid, (int*)lds))
    return;

  sr_wait_deps(flow, nv[13] + (nv[14] & 0xff), nv[14] >> 8, frame, ctx);

  // ---- epilogue: bias, activation, round to bf16, NHWC store.
  // The weights are the MFMA's row operand, so register r of lane l holds channel
  // 8*(r/4) + 4*(l/32) + r%4 of pixel l%32: four consecutive channels per register quad.  Each
  // wave transposes its tile through its own LDS region (64 pixels at a time, rows of 32*WN
  // channels + 16 spare bytes) so that global stores are 16 bytes per lane and whole pixel rows.
  __attribute__((address_space(1))) unsigned char* out = (__attribute__((address_space(1))) unsigned char*)(
      ((unsigned long long)(unsigned)(cur ? nv[3] : nv[1]) << 32) | (unsigned)(cur ? nv[2] : nv[0]));
  const __attribute__((address_space(1))) float* biasp = (const __attribute__((address_space(1))) float*)(
      ((unsigned long long)(unsigned)nv[5] << 32) | (unsigned)nv[4]);
  constexpr int EP = 32 * WN * 2 + 16;          // bytes per pixel row in LDS
  constexpr int PIECES = 32 * WN * 2 / 16;      // 16-byte pieces per pixel row
  unsigned char* my = lds + wave * (64 * EP);
  float bias[WN][4][4];
#pragma unroll
  for (int nj = 0; nj < WN; ++nj)
#pragma unroll
    for (int gq = 0; gq < 4; ++gq)
#pragma unroll
      for (int i = 0; i < 4; ++i) bias[nj][gq][i] = biasp[wave_n0 + nj * 32 + 8 * gq + 4 * (lane >> 5) + i];
  __syncthreads();   // every wave has finished reading the last patch
#pragma unroll
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int mh = 0; mh < 2; ++mh) {
      const int mi = half * 2 + mh;
#pragma unroll
      for (int nj = 0; nj < WN; ++nj)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          bf16x4_t h;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float v = acc[mi][nj][gq * 4 + i] + bias[nj][gq][i];
            if (act == 1) v = fmaxf(v, 0.f);
            h[i] = (__bf16)v;      // round to nearest even
          }
          *(bf16x4_t*)(my + (mh * 32 + (lane & 31)) * EP + (nj * 32 + 8 * gq + 4 * (lane >> 5)) * 2) = h;
        }
    }
    // same wave reads what it wrote: LDS operations of one wave complete in order
#pragma unroll
    for (int it = 0; it < PIECES; ++it) {
      const int p = it * 64 + lane;
      const int row = p / PIECES, piece = p - row * PIECES;
      const int m = wave_m0 + half * 64 + row;
      const u32x4_t v = *(const u32x4_t*)(my + row * EP + piece * 16);
      // agent-scope store (the consumers may run on other XCDs, within this launch) of the pieces that
      // exist: a node whose channel count is no multiple of 32 has fewer than the tile's
      if (m < M && wave_n0 + piece * 8 < Cp)
        asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"((__attribute__((address_space(1))) u32x4_t*)(
                         out + ((size_t)m * Cp + wave_n0) * 2 + piece * 16)), "v"(v) : "memory");
    }
  }
  sr_signal_done(flow, nv[15]);
}

__global__ __launch_bounds__(256, 2) void sr_mfma_kernel(SrCtx* __restrict__ ctx, SrTables4 tb, SrFlow flow,
                                                         const SrTile4* __restrict__ tiles, int n_tiles,
                                                         const SrAux* __restrict__ aux, int n_aux, int aux_at,
                                                         const SrHead* __restrict__ heads,
                                                         const SrHeadEdge* __restrict__ head_edges,
                                                         const SrStageNode* __restrict__ stage_nodes, int vec_floats,
                                                         int is_last, SrSplitScratch split) {
  extern __shared__ __align__(16) unsigned char sr_lds[];
  // work list: tiles in decreasing cost; the auxiliary items are spliced in at position aux_at so
  // that neither the longest tiles start late nor the launch ends on an auxiliary item
  // A launch covers gridDim.y frames (more than one only when dependency-driven); the hardware hands
  // workgroups out in the order x, then y: frame by frame.
  int item = blockIdx.x, frame = ctx->frame + (int)blockIdx.y;
  int n_blocks = gridDim.x * gridDim.y, n_frames = gridDim.y;
  if (flow.order) {
    const int e = ((const __attribute__((address_space(4))) int*)(unsigned long long)flow.order)[blockIdx.x];
    item = e & 0xffffff;
    frame = ctx->frame + (int)((unsigned)e >> 24);
    n_blocks = gridDim.x;
    n_frames = flow.frames;
  }
  const bool is_aux = item >= aux_at && item < aux_at + n_aux;
  if (!is_aux) {
    const SrTileK t = sr_load_tile(tiles, item < aux_at ? item : item - n_aux);
    if (t.node <= -2) {
      // an auxiliary item placed in the list itself (dependency-driven launches order all items of a frame)
      sr_aux_item<uint16_t>(ctx, aux[-2 - t.node], heads, head_edges, stage_nodes, (float*)sr_lds, vec_floats, frame, flow);
    } else if (t.node < 0) {
      // empty slot
    } else if (t.wn_tiles == 2)
      sr_mfma_tile<2>(ctx, tb, t, sr_lds, split, frame, flow);
    else
      sr_mfma_tile<1>(ctx, tb, t, sr_lds, split, frame, flow);
  } else {
    sr_aux_item<uint16_t>(ctx, aux[item - aux_at], heads, head_edges, stage_nodes, (float*)sr_lds, vec_floats, frame, flow);
  }
  if (is_last) sr_block_done(ctx, n_blocks, n_frames);
}

// ---------------------------------------------------------------------------
// 8-wave tile kernel
// ---------------------------------------------------------------------------
// One workgroup of 8 wave64 per compute unit (two waves per SIMD, 256 registers each); the waves are
// arranged waves_m x waves_n and each owns 128 pixels x (32*WN) channels as in the 4-wave kernel.
// Differences:
//  * BOTH operands of a stage come from LDS: the source patch (A) and the stage's slab of packed
//    weights (B) are brought in by direct-to-LDS loads.  No load returns to registers inside the
//    k-loop, so the loads of the NEXT stage can be issued ahead of the current one's k-steps
//    without ever being waited for there (vector-memory results return in order: a register load
//    behind a long direct-to-LDS load would stall on it).
//  * LDS holds two stage buffers; a stage computes out of one while the other is being filled.
//    One barrier per stage.
//  * A stage is one 16*K16-channel chunk of one ROW PHASE of one edge: a stride-s edge is cut into
//    s row phases (source rows q = phase mod s with the taps ti = phase mod s), which keeps the
//    patch of a strided edge as small as that of a stride-1 edge.
//  * Patch slots are KC*2 bytes without padding (sixteen consecutive pixels of a 32-byte slot then
//    hit every LDS column twice; measured, the 2-way conflict costs nothing here).
// LDS layout of a stage buffer: [A: NQr rows x RPB bytes, rounded up to 1 KiB][B: NS x NBT
// fragments of 1 KiB], NS = taps of the phase x K16 k-steps, NBT = BN/32 column tiles; B fragment
// (st, nt) is the packed fragment of tap(st), 16-channel block k(st), column tile n0/32 + nt.
#define SR8_PLAN_ITEMS 10   // direct-to-LDS instructions of a stage: 80 KiB / 8 KiB

struct SrEdge8 {   // wave-uniform copy of an edge descriptor (scalar registers)
  const unsigned char* src;
  const unsigned char* wpk;
  int Hs, Ws, Csp, kw, kh, stride, lgs, lgup, pad, KC, lgK16, PH, PWs, RPB, magicKW, wstride8, k16_total, plan_slot;
  int src_bytes;
};

__device__ __forceinline__ SrEdge8 sr8_load_edge(const SrMfmaEdge* edges, int index, int cur) {
  const __attribute__((address_space(4))) SrMfmaEdge* p =
      (const __attribute__((address_space(4))) SrMfmaEdge*)(unsigned long long)(edges + index);
  SrEdge8 k;
  const int bridge = p->bridge;
  k.src = (const unsigned char*)p->src[bridge ? (cur ^ 1) : cur];
  k.wpk = (const unsigned char*)p->wpk;
  k.Hs = p->Hs; k.Ws = p->Ws; k.Csp = p->Csp;
  k.kw = p->kw; k.kh = p->kh;
  k.stride = p->stride; k.lgs = (k.stride == 1) ? 0 : (k.stride == 2 ? 1 : 2);
  const int up = p->up;
  k.lgup = (up == 1) ? 0 : (up == 2 ? 1 : 2);
  k.pad = p->pad;
  k.KC = p->KC; k.lgK16 = (k.KC == 16) ? 0 : (k.KC == 32 ? 1 : (k.KC == 64 ? 2 : 3));
  k.PH = p->PH; k.PWs = p->PWs; k.RPB = p->RPB;
  k.magicKW = p->magicKW; k.wstride8 = p->wstride8;
  k.k16_total = k.Csp >> 4;
  k.plan_slot = p->plan_slot;
  k.src_bytes = p->src_bytes;
  return k;
}

// What the direct-to-LDS loads of one stage need (wave-uniform).  The buffer is an array of 16-byte
// positions, A's first (rounded up to a multiple of 64) and B's behind them; instruction `it` of a
// stage moves 512 consecutive positions, 64 per wave, so one wave's instruction is all A or all B.
// Every thread holds, per instruction, the byte offset of its position's source from a_base (A) or
// b_base (B); positions that are never read repeat a neighbour's offset (no lane masks).
struct SrProd8 {
  const unsigned char* a_base;   // source state: the byte that offset 0 stands for, this chunk
  const unsigned char* b_base;   // packed weights: this chunk's first 16-channel block, tile's first column tile
  int a_step, b_step;            // bytes from one chunk to the next
  int n_posA, n_pos;             // A positions (rounded); all positions
  int a_bytes;                   // LDS bytes of A; B follows
  int NS;                        // k-steps of the stage
  int lgK16;
};

// all of this wave's loads of a stage: per load a compare and branch, a base select, the LDS address, the load
__device__ __forceinline__ void sr8_issue_stage(const SrProd8& P, unsigned char* buf, int wave,
                                                const int (&plan)[SR8_PLAN_ITEMS]) {
  const unsigned char* a_base = sr_uniform_ptr(P.a_base);
  const unsigned char* b_base = sr_uniform_ptr(P.b_base);
#pragma unroll
  for (int it = 0; it < SR8_PLAN_ITEMS; ++it) {
    const int pos = it * 512 + wave * 64;
    if (pos < P.n_pos) {
      const unsigned char* base = (pos < P.n_posA) ? a_base : b_base;
      __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(base + (unsigned)plan[it]),
                                       (__attribute__((address_space(3))) void*)(buf + pos * 16), 16, 0, 0);
    }
  }
}

// One k-step: 4 x WN MFMAs.  Each A fragment is reloaded for the next step right after its last
// use; the B fragments of the next step go into the other B buffer.
template <int WN>
__device__ __forceinline__ void sr8_step(const unsigned char* rd, const int (&abase)[4], int bbase, int tapA, int lgK16,
                                         int nbt1024, bf16x8_t (&a)[4], const bf16x8_t (&b)[WN], bf16x8_t (&bn)[WN],
                                         f32x16_t (&acc)[4][WN], int st, int NS) {
  const int sn = min(st + 1, NS - 1);
  const int tap = sn >> lgK16;
  const int aoff = __builtin_amdgcn_readlane(tapA, tap) + ((sn - (tap << lgK16)) << 5);
  const int boff = sn * nbt1024;
#pragma unroll
  for (int nj = 0; nj < WN; ++nj) bn[nj] = *(const bf16x8_t*)(rd + bbase + boff + nj * 1024);
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
    for (int nj = 0; nj < WN; ++nj)
      acc[mi][nj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[nj], a[mi], acc[mi][nj], 0, 0, 0);
    a[mi] = *(const bf16x8_t*)(rd + abase[mi] + aoff);
  }
  // issue order: lane read of the next A offset; WN MFMAs, then the address add and the LDS read of
  // the row they released, four times; the reads of the next B fragments go behind the first group
  // (a wait for "all LDS reads" at the top of the step then only covers reads of the step before)
  __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);      // VALU (lane read)
  __builtin_amdgcn_sched_group_barrier(0x008, WN, 0);     // MFMA
  __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);      // VALU (address)
  __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);      // DS read (A)
  __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);      // VALU (B address)
  __builtin_amdgcn_sched_group_barrier(0x100, WN, 0);     // DS read (B)
#pragma unroll
  for (int mi = 1; mi < 4; ++mi) {
    __builtin_amdgcn_sched_group_barrier(0x008, WN, 0);   // MFMA
    __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);    // VALU (address)
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);    // DS read (A)
  }
}

template <int WN>
__device__ __forceinline__ void sr_mfma8_tile(const SrCtx* __restrict__ ctx, const SrMfmaNode* __restrict__ nodes,
                                              const SrMfmaEdge* __restrict__ edges, int node_index, int tile_m0,
                                              int tile_n0, int plan_begin, int stage_begin, int stage_end,
                                              int split_slot, int part_info, unsigned char* lds,
                                              const SrSplitScratch& split) {
  const __attribute__((address_space(4))) SrMfmaNode* nd =
      (const __attribute__((address_space(4))) SrMfmaNode*)(unsigned long long)(nodes + node_index);
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = SR_UNIFORM(tid >> 6);
  const int waves_n = nd->waves_n;
  const int wm = (waves_n == 4) ? (wave >> 2) : (waves_n == 2 ? (wave >> 1) : wave);
  const int wn = wave - wm * waves_n;
  const int cur = ctx->frame & 1;
  const int M = nd->M, Wo = nd->Wo, HoWo = nd->Ho * Wo;
  const int BM = 128 * nd->waves_m;
  const int m_first = tile_m0;
  const int m_last = min(tile_m0 + BM, M) - 1;
  const int wave_m0 = tile_m0 + wm * 128;
  const int wave_n0 = tile_n0 + wn * (32 * WN);
  const int NBT = WN * waves_n;                         // column tiles of the workgroup
  const int lgNBT64 = (NBT == 1) ? 6 : (NBT == 2 ? 7 : 8);
  const int b_first = m_first / HoWo, oy_first = (m_first - b_first * HoWo) / Wo;
  const int b_last = m_last / HoWo, oy_last = (m_last - b_last * HoWo) / Wo;
  const __attribute__((address_space(4))) int* plan_index =
      (const __attribute__((address_space(4))) int*)(unsigned long long)nd->plan_index + plan_begin;
  const __attribute__((address_space(1))) int* plan_tables =
      (const __attribute__((address_space(1))) int*)(unsigned long long)nd->plan_tables;
  const __attribute__((address_space(4))) SrStage8* stages =
      (const __attribute__((address_space(4))) SrStage8*)(unsigned long long)nd->stage_table + nd->stage0;

  int pix[4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    const int m = min(wave_m0 + mi * 32 + (lane & 31), M - 1);
    const int b = m / HoWo;
    const int r = m - b * HoWo;
    const int oy = r / Wo;
    pix[mi] = (r - oy * Wo) | (oy << 12) | ((b - b_first) << 24);
  }

  f32x16_t acc[4][WN];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int nj = 0; nj < WN; ++nj)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[mi][nj][r] = 0.f;

  // ---- producer state (the stage whose loads are being issued) and what the consumer inherits
  SrProd8 P;
  int plan[SR8_PLAN_ITEMS];
  int tapA_n = 0, abase_n[4] = {0, 0, 0, 0};
  int p_chunk = 0, p_nchunk = 0;
  // prepares P (and the consumer's next tap table / fragment addresses) for stage index sidx
  auto prepare = [&](int sidx) {
    if (p_chunk + 1 < p_nchunk) {   // the stage list runs edge by edge, phase by phase, chunk by chunk
      p_chunk += 1;
      P.a_base += P.a_step;
      P.b_base += P.b_step;
      return;
    }
    const int s_edge = stages[sidx].edge, s_phase = stages[sidx].phase, s_chunk = stages[sidx].chunk;
    const SrEdge8 e = sr8_load_edge(edges, s_edge, cur);
    p_chunk = s_chunk;
    p_nchunk = e.Csp >> (4 + e.lgK16);
    const int cnt = (e.kh - s_phase + e.stride - 1) >> e.lgs;         // tap rows of this phase
    const int ntaps = cnt * e.kw;
    const int row_first = (oy_first >> e.lgup) << e.lgs;              // first padded source row, in its image
    const int Q0 = b_first * e.PH + row_first;
    const int Q1 = b_last * e.PH + ((oy_last >> e.lgup) << e.lgs) + e.kh - 1;
    const int NQr = (Q1 - Q0 + 1 - s_phase + e.stride - 1) >> e.lgs;  // patch rows of this phase
    P.n_posA = (NQr * (e.RPB >> 4) + 63) & ~63;
    P.NS = ntaps << e.lgK16;
    P.lgK16 = e.lgK16;
    P.a_bytes = P.n_posA << 4;
    P.n_pos = P.n_posA + (P.NS << lgNBT64);
    P.a_step = e.KC * 2;
    P.b_step = (e.wstride8 << e.lgK16) * 16;
    const long long base_off = ((long long)(b_first * e.Hs + row_first - e.pad) * e.Ws) * e.Csp * 2;
    P.a_base = e.src + base_off + (size_t)s_chunk * P.a_step;
    P.b_base = e.wpk + (size_t)(tile_n0 >> 5) * 1024 + (size_t)s_chunk * P.b_step;
    // offsets of this thread's positions.  A: from the plan table; padding pixels are read from the
    // zero bytes behind the source state (far enough behind for every chunk's offset)
    const int zero_off = (int)((long long)e.src_bytes - base_off);
    const __attribute__((address_space(1))) int* table = plan_tables + plan_index[e.plan_slot + s_phase];
#pragma unroll
    for (int it = 0; it < SR8_PLAN_ITEMS; ++it) {
      int v = 0;
      if (it * 512 < P.n_pos) v = table[tid + it * 512];   // A then B entries, padded to 512 at the end
      plan[it] = (v == SR_DMA_ZERO) ? zero_off : v;
    }
    // A tap table of the phase, one tap per lane: t-th tap = (ti, tj) = (phase + (t / kw) * stride, t % kw)
    {
      const int t = min(lane, ntaps - 1);
      const int q = (t * e.magicKW) >> 16;
      const int tj = t - q * e.kw;
      tapA_n = q * e.RPB + ((tj & (e.stride - 1)) * e.PWs + (tj >> e.lgs)) * (e.KC * 2);
    }
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
      const int ox = pix[mi] & 0xfff, oy = (pix[mi] >> 12) & 0xfff, db = pix[mi] >> 24;
      abase_n[mi] = ((db * e.PH + ((oy >> e.lgup) << e.lgs) - row_first) >> e.lgs) * e.RPB +
                    (ox >> e.lgup) * (e.KC * 2) + (lane >> 5) * 16;
    }
  };

  unsigned char* buf0 = lds;
  unsigned char* buf1 = lds + SR8_BUF_BYTES;
  // first stage: all its loads at once
  prepare(stage_begin);
  sr8_issue_stage(P, buf0, wave, plan);

  int par = 0;
  for (int c = stage_begin; c < stage_end; ++c) {
    // the consumer takes over what was prepared for this stage
    const int NS = P.NS, lgK16 = P.lgK16, a_bytes = P.a_bytes;
    const int tapA = tapA_n;
    int abase[4];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) abase[mi] = abase_n[mi];
    // the producer moves on to the next stage (its plan loads overlap the wait below)
    const bool more = c + 1 < stage_end;
    if (more) prepare(c + 1);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's loads of stage c have landed
    __syncthreads();                                     // ... everybody's; and stage c-1 has been read by all
    const unsigned char* rd = par ? buf1 : buf0;
    unsigned char* wr = par ? buf0 : buf1;
    const int bbase = a_bytes + ((wn * WN) * 64 + lane) * 16;
    const int nbt1024 = NBT * 1024;
    bf16x8_t a[4], b[2][WN];
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) a[mi] = *(const bf16x8_t*)(rd + abase[mi]);
#pragma unroll
    for (int nj = 0; nj < WN; ++nj) b[0][nj] = *(const bf16x8_t*)(rd + bbase + nj * 1024);
    // The loads of the next stage are issued inside this stage's k-steps, one wave at a time: the
    // vector-memory unit takes a direct-to-LDS instruction every ~30 cycles and a wave issuing into a
    // full queue waits, which then costs the issuing wave only while the other wave of its SIMD
    // keeps the matrix pipe busy.  Wave w takes its turn before k-step w*NSI/8 (rounded down to an
    // even step), NSI = the stage's steps less the last three, which leave the loads time to land.
    // (Preparing the next stage there as well, instead of ahead of the barrier, measured slower.)
    const int my_step = more ? ((wave * max(NS - 3, 1)) >> 3) & ~1 : -1;
    for (int st = 0; st < NS; st += 2) {
      if (st == my_step) sr8_issue_stage(P, wr, wave, plan);
      sr8_step<WN>(rd, abase, bbase, tapA, lgK16, nbt1024, a, b[0], b[1], acc, st, NS);
      if (st + 1 < NS) sr8_step<WN>(rd, abase, bbase, tapA, lgK16, nbt1024, a, b[1], b[0], acc, st + 1, NS);
    }
    par ^= 1;
  }

  // ---- K-split tiles: as in the 4-wave kernel, with 512 threads
  if ((part_info >> 16) > 1 &&
      !sr_split_reduce<WN, 512>(acc, split, split_slot, part_info, SR8_SPLIT_FLOATS, tid, (int*)lds))
    return;

  // ---- epilogue: as in the 4-wave kernel (each wave transposes its tile through its own LDS region)
  __attribute__((address_space(1))) unsigned char* out =
      (__attribute__((address_space(1))) unsigned char*)(unsigned long long)nd->out[cur];
  const __attribute__((address_space(1))) float* biasp =
      (const __attribute__((address_space(1))) float*)(unsigned long long)nd->bias;
  const int Cp = nd->Cp, act = nd->act;
  constexpr int EP = 32 * WN * 2 + 16;          // bytes per pixel row in LDS
  constexpr int PIECES = 32 * WN * 2 / 16;      // 16-byte pieces per pixel row
  unsigned char* my = lds + wave * (64 * EP);
  float bias[WN][4][4];
#pragma unroll
  for (int nj = 0; nj < WN; ++nj)
#pragma unroll
    for (int gq = 0; gq < 4; ++gq)
#pragma unroll
      for (int i = 0; i < 4; ++i) bias[nj][gq][i] = biasp[wave_n0 + nj * 32 + 8 * gq + 4 * (lane >> 5) + i];
  __syncthreads();   // every wave has finished reading the last stage
#pragma unroll
  for (int half = 0; half < 2; ++half) {
#pragma unroll
    for (int mh = 0; mh < 2; ++mh) {
      const int mi = half * 2 + mh;
#pragma unroll
      for (int nj = 0; nj < WN; ++nj)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
          bf16x4_t h;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            float v = acc[mi][nj][gq * 4 + i] + bias[nj][gq][i];
            if (act == 1) v = fmaxf(v, 0.f);
            h[i] = (__bf16)v;      // round to nearest even
          }
          *(bf16x4_t*)(my + (mh * 32 + (lane & 31)) * EP + (nj * 32 + 8 * gq + 4 * (lane >> 5)) * 2) = h;
        }
    }
#pragma unroll
    for (int it = 0; it < PIECES; ++it) {
      const int p = it * 64 + lane;
      const int row = p / PIECES, piece = p - row * PIECES;
      const int m = wave_m0 + half * 64 + row;
      const u32x4_t v = *(const u32x4_t*)(my + row * EP + piece * 16);
      if (m < M && wave_n0 + piece * 8 < Cp)
        *(__attribute__((address_space(1))) u32x4_t*)(out + ((size_t)m * Cp + wave_n0) * 2 + piece * 16) = v;
    }
  }
}

__global__ __launch_bounds__(512) void sr_mfma8_kernel(SrCtx* __restrict__ ctx, const SrMfmaNode* __restrict__ nodes,
                                                       const SrMfmaEdge* __restrict__ edges,
                                                       const SrMfmaTile* __restrict__ tiles, int n_tiles,
                                                       const SrAux* __restrict__ aux, int n_aux, int aux_at,
                                                       const SrHead* __restrict__ heads,
                                                       const SrHeadEdge* __restrict__ head_edges,
                                                       const SrStageNode* __restrict__ stage_nodes, int vec_floats,
                                                       int is_last, SrSplitScratch split) {
  extern __shared__ __align__(16) unsigned char sr_lds8[];
  // work list as in the 4-wave kernel: the auxiliary items are spliced in at position aux_at.  An
  // auxiliary item is written for 256 threads: the upper four waves of the workgroup leave (a
  // barrier only waits for the waves that are still there).
  const int item = blockIdx.x;
  if (item >= aux_at && item < aux_at + n_aux) {
    if (threadIdx.x >= SR_AUX_THREADS) return;
    sr_aux_item<uint16_t>(ctx, aux[item - aux_at], heads, head_edges, stage_nodes, (float*)sr_lds8, vec_floats, ctx->frame,
                          SrFlow{nullptr, nullptr, 0, 0, nullptr});
    if (is_last) sr_block_done(ctx, gridDim.x, 1);
    return;
  }
  const SrMfmaTile t = tiles[item < aux_at ? item : item - n_aux];
  const int node_index = SR_UNIFORM(t.node);
  if (node_index < 0) {
    // empty slot
  } else if (nodes[node_index].wn_tiles == 2)
    sr_mfma8_tile<2>(ctx, nodes, edges, node_index, SR_UNIFORM(t.m0), SR_UNIFORM(t.n0), SR_UNIFORM(t.plan_begin),
                     SR_UNIFORM(t.stage_begin), SR_UNIFORM(t.stage_end), SR_UNIFORM(t.split_slot), SR_UNIFORM(t.part),
                     sr_lds8, split);
  else
    sr_mfma8_tile<1>(ctx, nodes, edges, node_index, SR_UNIFORM(t.m0), SR_UNIFORM(t.n0), SR_UNIFORM(t.plan_begin),
                     SR_UNIFORM(t.stage_begin), SR_UNIFORM(t.stage_end), SR_UNIFORM(t.split_slot), SR_UNIFORM(t.part),
                     sr_lds8, split);
  if (is_last) sr_block_done(ctx, gridDim.x, 1);
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

template <typename T>
__global__ void sr_aux_kernel(SrCtx* __restrict__ ctx, const SrAux* __restrict__ aux, const SrHead* __restrict__ heads,
                              const SrHeadEdge* __restrict__ head_edges, const SrStageNode* __restrict__ stage_nodes,
                              int vec_floats, int is_last) {
  extern __shared__ float sr_aux_smem2[];
  sr_aux_item<T>(ctx, aux[blockIdx.x], heads, head_edges, stage_nodes, sr_aux_smem2, vec_floats, ctx->frame,
                 SrFlow{nullptr, nullptr, 0, 0, nullptr});
  if (is_last) sr_block_done(ctx, gridDim.x, 1);
}

// smem_bytes of the aux items: vector floats + 16 bytes + 4 KiB of partial outputs
static inline int sr_vec_floats(int smem_bytes) { return (smem_bytes - 16 - 4096) / 4; }

hipError_t sr_launch_aux(hipStream_t s, SrCtx* ctx, const SrAux* aux, int n_aux, const SrHead* heads,
                         const SrHeadEdge* head_edges, const SrStageNode* stage_nodes, int smem_bytes, int bf16,
                         int is_last) {
  if (n_aux == 0) return hipSuccess;
  const int vf = sr_vec_floats(smem_bytes);
  if (bf16) hipLaunchKernelGGL(sr_aux_kernel<uint16_t>, dim3(n_aux), dim3(256), smem_bytes, s, ctx, aux, heads, head_edges, stage_nodes, vf, is_last);
  else hipLaunchKernelGGL(sr_aux_kernel<float>, dim3(n_aux), dim3(256), smem_bytes, s, ctx, aux, heads, head_edges, stage_nodes, vf, is_last);
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

hipError_t sr_launch_direct(hipStream_t s, SrCtx* ctx, const SrDirectNode* nodes, const SrDirectEdge* edges,
                            const SrDirectBlock* blocks, int n_blocks, int bf16, int batch, const SrAux* aux, int n_aux,
                            const SrHead* heads, const SrHeadEdge* head_edges, const SrStageNode* stage_nodes,
                            int smem_bytes, int is_last) {
  if (n_blocks + n_aux == 0) return hipSuccess;
  const int vf = sr_vec_floats(smem_bytes);
  if (bf16) hipLaunchKernelGGL(sr_direct_kernel<uint16_t>, dim3(n_blocks + n_aux), dim3(256), smem_bytes, s, ctx, nodes, edges, blocks, n_blocks, batch, aux, heads, head_edges, stage_nodes, vf, is_last);
  else hipLaunchKernelGGL(sr_direct_kernel<float>, dim3(n_blocks + n_aux), dim3(256), smem_bytes, s, ctx, nodes, edges, blocks, n_blocks, batch, aux, heads, head_edges, stage_nodes, vf, is_last);
  return hipGetLastError();
}

// hipFuncAttributeMaxDynamicSharedMemorySize of tile kernel `which`, set once on every device that
// launches it (thread-safe; a failed attempt is tried again by the next launch)
static hipError_t sr_request_lds(const void* kernel, int bytes, int which) {
  constexpr int kMaxDevices = 64;
  static std::atomic<int> done[2][kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev >= 0 && dev < kMaxDevices && done[which][dev].load(std::memory_order_acquire)) return hipSuccess;
  e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (e == hipSuccess && dev >= 0 && dev < kMaxDevices) done[which][dev].store(1, std::memory_order_release);
  return e;
}

hipError_t sr_launch_mfma(hipStream_t s, SrCtx* ctx, SrTables4 tables, SrFlow flow, int frames, int n_order,
                          const SrTile4* tiles,
                          int n_tiles, int lds_bytes, const SrAux* aux, int n_aux, const SrHead* heads,
                          const SrHeadEdge* head_edges, const SrStageNode* stage_nodes, int aux_smem_bytes, int is_last,
                          SrSplitScratch split) {
  if (n_tiles + n_aux == 0) return hipSuccess;
  {   // dynamic LDS above 64 KiB has to be requested once per device
    hipError_t e = sr_request_lds((const void*)sr_mfma_kernel, sr_mfma_max_lds_bytes(), 0);
    if (e != hipSuccess) return e;
  }
  const dim3 grid = flow.order ? dim3(n_order) : dim3(n_tiles + n_aux, frames);
  hipLaunchKernelGGL(sr_mfma_kernel, grid, dim3(256), lds_bytes, s, ctx, tables, flow, tiles,
                     n_tiles, aux, n_aux, n_tiles / 2, heads, head_edges, stage_nodes, sr_vec_floats(aux_smem_bytes), is_last,
                     split);
  return hipGetLastError();
}

hipError_t sr_launch_mfma8(hipStream_t s, SrCtx* ctx, const SrMfmaNode* nodes, const SrMfmaEdge* edges,
                           const SrMfmaTile* tiles, int n_tiles, const SrAux* aux, int n_aux, const SrHead* heads,
                           const SrHeadEdge* head_edges, const SrStageNode* stage_nodes, int aux_smem_bytes, int is_last,
                           SrSplitScratch split) {
  if (n_tiles + n_aux == 0) return hipSuccess;
  {
    hipError_t e = sr_request_lds((const void*)sr_mfma8_kernel, 2 * SR8_BUF_BYTES, 1);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(sr_mfma8_kernel, dim3(n_tiles + n_aux), dim3(512), 2 * SR8_BUF_BYTES, s, ctx, nodes, edges, tiles, n_tiles,
                     aux, n_aux, n_tiles / 2, heads, head_edges, stage_nodes, sr_vec_floats(aux_smem_bytes), is_last, split);
  return hipGetLastError();
}

// Scratch for callers that may not allocate: one array per GPU, held from the moment the library is
// loaded there until the process ends.  In host code the array's name is only a handle; its device
// address on the current device comes from hipGetSymbolAddress, once per device.
static __device__ __align__(256) unsigned char sr_static_scratch_array[SR_STATIC_SCRATCH_BYTES];

hipError_t sr_static_scratch(void** ptr) {
  constexpr int kMaxDevices = 64;
  static std::atomic<void*> addr[kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  void* p = addr[dev].load(std::memory_order_acquire);
  if (!p) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(sr_static_scratch_array));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    addr[dev].store(p, std::memory_order_release);
  }
  *ptr = p;
  return hipSuccess;
}

int sr_mfma_max_lds_bytes() { return 80 * 1024; }   // two workgroups per CU share 160 KiB
