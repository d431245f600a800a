// Host side of one training window (Sec. 3: rollout window of size W; Sec. 2: backpropagation through
// the rolled-out network; App. A2: loss): drives the frame path forward, keeps every frame's states,
// and runs the reverse sweep with the kernels of sr_train.hip.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/sr.h"
#include "sr_internal.h"
#include "sr_train.h"
#include "sr_graph.h"

// what a graph keeps for its training windows between calls
struct SrTrainState {
  // one arena: the states of the frames 0..W, two gradient copies (frames i and i-1 of the reverse sweep) and
  // the scratch of the gradient kernels
  float* arena = nullptr;
  size_t arena_floats = 0;
  std::vector<float*> rms_w, rms_b;   // RMSprop's running mean of the squared gradient, per edge / node (on first use)
  // side streams (nodes of one update step of the forward pass; bias and weight gradients of the reverse sweep
  // beside the chain of state gradients) and the events that order them against the graph's stream
  static constexpr int kSides = 3;
  struct Events {
    hipEvent_t main = nullptr, side[kSides] = {nullptr, nullptr, nullptr};
  };
  hipStream_t side[kSides] = {nullptr, nullptr, nullptr};
  Events ev;
};

void sr_train_state_release(SrTrainState* t) {
  if (!t) return;
  auto drop_events = [](SrTrainState::Events& e) {
    if (e.main) hipEventDestroy(e.main);
    for (int k = 0; k < SrTrainState::kSides; ++k)
      if (e.side[k]) hipEventDestroy(e.side[k]);
  };
  drop_events(t->ev);
  for (int k = 0; k < SrTrainState::kSides; ++k)
    if (t->side[k]) { hipStreamSynchronize(t->side[k]); hipStreamDestroy(t->side[k]); }
  if (t->arena) hipFree(t->arena);
  delete t;
}

namespace {

SrTrainState& train_state(sr_graph* g) {
  if (!g->train) g->train = new SrTrainState();
  return *g->train;
}

sr_status make_events(sr_graph* g, SrTrainState::Events* e) {
  if (!e->main) SR_HIP(g, hipEventCreateWithFlags(&e->main, hipEventDisableTiming));
  for (int k = 0; k < SrTrainState::kSides; ++k)
    if (!e->side[k]) SR_HIP(g, hipEventCreateWithFlags(&e->side[k], hipEventDisableTiming));
  return SR_OK;
}

}  // namespace

extern "C" {

sr_status sr_window_gradients(sr_graph* g, int32_t W, const void* const* inputs, const float* const* masks,
                              const int32_t* labels, int32_t out_node, float* loss, float* const* dtheta,
                              float* const* dbias) {
  if (!g || !inputs || !labels || !loss || !dtheta || W < 1)
    return sr_gfail(g, SR_ERR_ARG, "bad argument to sr_window_gradients");
  if (g->dtype != SR_F32) return sr_gfail(g, SR_ERR_ARG, "sr_window_gradients: training windows take SR_F32 graphs only");
  if (out_node < 0 || out_node >= g->n_nodes || g->an.is_input[out_node] || g->nodes[out_node].d.height != 1 ||
      g->nodes[out_node].d.width != 1)
    return sr_gfail(g, SR_ERR_ARG, "sr_window_gradients: out_node must be a 1x1 node with incoming edges (the logits)");
  for (int e = 0; e < g->n_edges; ++e)
    if (!dtheta[e]) return sr_gfail(g, SR_ERR_ARG, "sr_window_gradients: dtheta[" + std::to_string(e) + "] is null");
  for (size_t i = 0; i < g->inputs.size(); ++i)
    if (!inputs[i]) return sr_gfail(g, SR_ERR_ARG, "input " + std::to_string(i) + " is null");
  for (int e = 0; e < g->n_edges; ++e)
    if (!g->edges[e].has_w) return sr_gfail(g, SR_ERR_STATE, "edge " + std::to_string(e) + " has no weights");
  if (W > 4096) return sr_gfail(g, SR_ERR_ARG, "sr_window_gradients: window size above 4096");
  SrTrainState& T = train_state(g);
  const int B = g->batch, N = g->n_nodes;
  auto node_floats = [&](int v) {
    const sr_node_desc& d = g->nodes[v].d;
    return (size_t)B * d.height * d.width * d.channels;
  };
  auto geom_of = [&](const EdgeRt& e) {
    const sr_node_desc& s = g->nodes[e.d.src].d;
    const sr_node_desc& d = g->nodes[e.d.dst].d;
    SrConvGeom q{};
    q.B = B; q.Cin = s.channels; q.Cout = d.channels; q.tall_from = g->train_tall_from;
    if (e.d.kind == SR_EDGE_CONV) {
      q.H = s.height; q.W = s.width; q.kh = e.kh; q.kw = e.kw; q.stride = e.d.stride; q.pad = e.d.pad;
      q.Ho = d.height / e.d.upsample; q.Wo = d.width / e.d.upsample;
    } else if (e.d.kind == SR_EDGE_DENSE) {
      // a 1x1 map on a 1x1 image whose channels are all the source's elements: x[b][h][w][ci] and
      // theta[h][w][ci][co] lie in memory as x[b][(h, w, ci)] and theta[(h, w, ci)][co]
      q.Cin = s.height * s.width * s.channels;
      q.H = 1; q.W = 1; q.kh = 1; q.kw = 1; q.stride = 1; q.pad = 0; q.Ho = 1; q.Wo = 1;
    } else {                                   // GAP + dense: a 1x1 map on the per-image channel means
      q.H = 1; q.W = 1; q.kh = 1; q.kw = 1; q.stride = 1; q.pad = 0; q.Ho = 1; q.Wo = 1;
    }
    return q;
  };
  // arena layout
  size_t at = 0;
  auto take = [&](size_t n) { size_t r = at; at += (n + 63) / 64 * 64; return r; };
  // states frame by frame, inside a frame node by node (frame 0, the zero state, is then one stretch), and the two
  // gradient copies laid out like a frame each (a copy is cleared by one fill)
  std::vector<size_t> in_frame(N, 0);
  size_t frame_floats = 0;
  for (int v = 0; v < N; ++v) {
    if (g->an.is_input[v]) continue;
    in_frame[v] = frame_floats;
    frame_floats += (node_floats(v) + 63) / 64 * 64;
  }
  const size_t x_base = take(frame_floats * (size_t)(W + 1));
  const size_t dx_base[2] = {take(frame_floats), take(frame_floats)};
  auto x_of = [&](int v, int frame) { return x_base + (size_t)frame * frame_floats + in_frame[v]; };
  auto dx_of = [&](int c, int v) { return dx_base[c] + in_frame[v]; };
  size_t pooled_n = 0, mean_n = 0, part_n = 0;
  for (const EdgeRt& e : g->edges) {
    const SrConvGeom q = geom_of(e);
    part_n = std::max(part_n, (size_t)sr_train_wgrad_slices(q) * e.w_count);
    part_n = std::max(part_n, (size_t)SR_TRAIN_MAX_SLICES * g->nodes[e.d.dst].d.channels);   // bias gradient slices
    if (e.d.kind == SR_EDGE_CONV && e.d.upsample > 1) pooled_n = std::max(pooled_n, (size_t)B * q.Ho * q.Wo * q.Cout);
    if (e.d.kind == SR_EDGE_GAP_DENSE) mean_n = std::max(mean_n, (size_t)B * q.Cin);
  }
  // scratch: copy 0 belongs to the graph's stream, copy 1 + k to side stream k
  constexpr int NS = SrTrainState::kSides;
  size_t pooled_at[1 + NS], mean_at[1 + NS], part_at[1 + NS];
  for (int k = 0; k <= NS; ++k) {
    pooled_at[k] = take(pooled_n);
    mean_at[k] = take(mean_n);
    part_at[k] = take(k == 0 ? 0 : part_n);   // partial sums of bias and weight gradients: side streams only
  }
  const size_t dmean_at = take(mean_n);
  const size_t terms_at = take((size_t)W * B);
  if (at > T.arena_floats) {
    SR_HIP(g, hipStreamSynchronize(g->stream));
    if (T.arena) SR_HIP(g, hipFree(T.arena));
    T.arena = nullptr;
    T.arena_floats = 0;
    void* p = nullptr;
    SR_HIP(g, hipMalloc(&p, at * sizeof(float)));
    T.arena = (float*)p;
    T.arena_floats = at;
  }
  float* A = T.arena;
  hipStream_t s = g->stream;
  for (int k = 0; k < NS; ++k)
    if (!T.side[k]) SR_HIP(g, hipStreamCreateWithFlags(&T.side[k], hipStreamNonBlocking));
  SrTrainState::Events* ev = &T.ev;
  if (make_events(g, ev) != SR_OK) return SR_ERR_DEVICE;
  // stream 0 is the graph's, 1 + k side stream k; fork: the side streams take up after what the graph's stream
  // holds so far; join: the graph's stream takes up after all of them
  auto stream_of = [&](int k) { return k == 0 ? s : T.side[k - 1]; };
  // fork(lanes): the side streams in the bit set take up after what the graph's stream holds so far (bit 1 + k:
  // side stream k); join(): the graph's stream takes up after every side stream forked since the last join
  unsigned forked = 0;
  auto fork = [&](unsigned lanes) -> sr_status {
    lanes &= ~1u;
    if (!lanes) return SR_OK;
    SR_HIP(g, hipEventRecord(ev->main, s));
    for (int k = 0; k < NS; ++k)
      if (lanes & (2u << k)) SR_HIP(g, hipStreamWaitEvent(T.side[k], ev->main, 0));
    forked |= lanes;
    return SR_OK;
  };
  auto join = [&]() -> sr_status {
    for (int k = 0; k < NS; ++k)
      if (forked & (2u << k)) {
        SR_HIP(g, hipEventRecord(ev->side[k], T.side[k]));
        SR_HIP(g, hipStreamWaitEvent(s, ev->side[k], 0));
      }
    forked = 0;
    return SR_OK;
  };
  // forward over the window from the zero state, every frame's states written straight into the arena:
  // frames 1..W, inside a frame the update steps of the tableau in order (Eq. 5), per node the sum of its
  // edges' results (the first edge overwrites, the others add), then bias and activation in place
  std::vector<size_t> in_stride(g->inputs.size());
  for (size_t k = 0; k < g->inputs.size(); ++k) in_stride[k] = node_floats(g->inputs[k]);
  std::vector<int> slot_of(N, -1);
  for (size_t k = 0; k < g->inputs.size(); ++k) slot_of[g->inputs[k]] = (int)k;
  std::vector<int> order;
  for (int v = 0; v < N; ++v)
    if (!g->an.is_input[v]) order.push_back(v);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return g->an.level[a] < g->an.level[b]; });
  auto state_of = [&](int u, int frame) -> const float* {
    return g->an.is_input[u] ? (const float*)inputs[slot_of[u]] + (size_t)frame * in_stride[slot_of[u]]
                             : A + x_of(u, frame);
  };
  // Two ways to the same states: when some edge is large enough for the tiled matrix-core kernel the window
  // runs its own forward pass below; a graph of small edges only is better served by the frame path
  // (sr_reset + W x sr_frame_step, each frame's states copied into the arena), whose kernels take a whole
  // update step per launch
  bool own_forward = false;
  for (const EdgeRt& e : g->edges) own_forward |= sr_train_fwd_is_tiled(geom_of(e)) != 0;
  // dropout multipliers of node v at frame i (null: none); the frame path knows no dropout
  auto mask_of = [&](int v, int frame) -> const float* {
    return (masks && masks[v] && !g->an.is_input[v]) ? masks[v] + (size_t)frame * node_floats(v) : nullptr;
  };
  for (int v = 0; masks && v < N; ++v) own_forward |= (masks[v] != nullptr && !g->an.is_input[v]);

  // every launch of the window
  auto enqueue = [&]() -> sr_status {
  SR_HIP(g, sr_launch_fill_zero(s, A + x_base, frame_floats * sizeof(float)));   // frame 0
  if (!own_forward) {
    std::vector<const void*> ptrs(g->inputs.size());
    for (size_t k = 0; k < g->inputs.size(); ++k) ptrs[k] = inputs[k];
    sr_status st = sr_reset(g, ptrs.data());
    if (st != SR_OK) return st;
    for (int i = 1; i <= W; ++i) {
      for (size_t k = 0; k < g->inputs.size(); ++k) ptrs[k] = (const float*)inputs[k] + (size_t)i * in_stride[k];
      st = sr_frame_step(g, ptrs.data());
      if (st != SR_OK) return st;
      for (int v : order)
        SR_HIP(g, hipMemcpyAsync(A + x_of(v, i), g->nodes[v].state[g->host_frame & 1],
                                 node_floats(v) * sizeof(float), hipMemcpyDeviceToDevice, s));
    }
  }
  // the nodes of one update step do not depend on each other: they go round the streams, forked before the step
  // and joined after it
  for (int i = 1; own_forward && i <= W; ++i)
    for (size_t o = 0; o < order.size();) {
      size_t o_end = o;
      while (o_end < order.size() && g->an.level[order[o_end]] == g->an.level[order[o]]) ++o_end;
      const bool wide = o_end - o > 1;
      if (wide && fork((1u << std::min<size_t>(o_end - o, 1 + NS)) - 1u) != SR_OK) return SR_ERR_DEVICE;
      for (size_t k = o; k < o_end; ++k) {
        const int v = order[k];
        const int lane = wide ? (int)((k - o) % (1 + NS)) : 0;
        hipStream_t st = stream_of(lane);
        float* pooled = A + pooled_at[lane];
        float* mean = A + mean_at[lane];
        const sr_node_desc& d = g->nodes[v].d;
        float* dst = A + x_of(v, i);
        int seen = 0;
        for (int ei = 0; ei < g->n_edges; ++ei) {
          const EdgeRt& e = g->edges[ei];
          if (e.d.dst != v) continue;
          const float* xsrc = state_of(e.d.src, i - (int)e.d.bridge);
          const SrConvGeom q = geom_of(e);
          if (e.d.kind == SR_EDGE_GAP_DENSE) {
            const sr_node_desc& sd = g->nodes[e.d.src].d;
            SR_HIP(g, sr_train_gap_mean(st, xsrc, B, sd.height * sd.width, sd.channels, mean));
            SR_HIP(g, sr_train_fwd(st, q, mean, e.w_dev, dst, seen));
          } else if (e.d.kind == SR_EDGE_CONV && e.d.upsample > 1) {
            SR_HIP(g, sr_train_fwd(st, q, xsrc, e.w_dev, pooled, 0));
            SR_HIP(g, sr_train_upsample_add(st, pooled, B, d.height, d.width, d.channels, e.d.upsample, dst, seen));
          } else {
            SR_HIP(g, sr_train_fwd(st, q, xsrc, e.w_dev, dst, seen));
          }
          seen = 1;
        }
        SR_HIP(g, sr_train_bias_act(st, dst, g->nodes[v].bias_dev, mask_of(v, i), d.channels, node_floats(v), d.act));
      }
      if (wide && join() != SR_OK) return SR_ERR_DEVICE;
      o = o_end;
    }

  // reverse sweep: frames W..1, inside a frame the update steps in reverse (Eq. 5), so every
  // (frame, node) has the gradient of all its readers before it is processed.  The chain of state gradients
  // (loss, activation gradient, one state gradient per edge) runs on the graph's stream; what hangs off it (a
  // node's bias gradient and its edges' weight gradients, which nothing later in the sweep reads) runs on the side
  // streams, started per node once the node's gradient is final and joined at the end of each frame, before the
  // gradient copy they read is cleared.  A node's bias and an edge's weights always go to the same side stream, so
  // their sums over the frames keep their order; every side stream has its own scratch.
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return g->an.level[a] > g->an.level[b]; });
  for (int c = 0; c < 2; ++c) SR_HIP(g, sr_launch_fill_zero(s, A + dx_base[c], frame_floats * sizeof(float)));
  auto side_of_edge = [&](int ei) { return 1 + ei % NS; };
  auto side_of_node = [&](int v) { return 1 + v % NS; };
  if (fork(~0u) != SR_OK) return SR_ERR_DEVICE;   // the forward pass is done with the scratch
  for (int e = 0; e < g->n_edges; ++e)
    SR_HIP(g, sr_launch_fill_zero(stream_of(side_of_edge(e)), dtheta[e], g->edges[e].w_count * sizeof(float)));
  if (dbias)
    for (int v : order)
      if (dbias[v])
        SR_HIP(g, sr_launch_fill_zero(stream_of(side_of_node(v)), dbias[v], (size_t)g->nodes[v].d.channels * sizeof(float)));
  const int classes = g->nodes[out_node].d.channels;
  const float scale = 1.0f / ((float)B * (float)W);
  for (int i = W; i >= 1; --i) {
    const int cur = i & 1;
    SR_HIP(g, sr_train_ce(s, A + x_of(out_node, i), labels, B, classes, scale,
                          A + terms_at + (size_t)(i - 1) * B, A + dx_of(cur, out_node)));
    for (int v : order) {
      const sr_node_desc& d = g->nodes[v].d;
      float* da = A + dx_of(cur, v);
      SR_HIP(g, sr_train_act_grad(s, da, A + x_of(v, i), mask_of(v, i), node_floats(v), d.act));
      // da is final: its writers (readers of v in this frame and the next) came earlier in the sweep
      unsigned lanes = (dbias && dbias[v]) ? 1u << side_of_node(v) : 0u;
      for (int ei = 0; ei < g->n_edges; ++ei)
        if (g->edges[ei].d.dst == v) lanes |= 1u << side_of_edge(ei);
      if (fork(lanes) != SR_OK) return SR_ERR_DEVICE;
      if (dbias && dbias[v])
        SR_HIP(g, sr_train_bias_grad(stream_of(side_of_node(v)), da, B * d.height * d.width, d.channels,
                                     A + part_at[side_of_node(v)], dbias[v]));
      for (int ei = 0; ei < g->n_edges; ++ei) {
        const EdgeRt& e = g->edges[ei];
        if (e.d.dst != v) continue;
        const int u = e.d.src, fi = i - (int)e.d.bridge;
        const float* xsrc = state_of(u, fi);
        // frame 0 and the input nodes are given: no gradient is kept for them
        float* dxsrc = (g->an.is_input[u] || fi == 0) ? nullptr : A + dx_of(fi & 1, u);
        const SrConvGeom q = geom_of(e);
        const int lane = side_of_edge(ei);
        hipStream_t w = stream_of(lane);
        if (e.d.kind == SR_EDGE_GAP_DENSE) {
          const sr_node_desc& sd = g->nodes[u].d;
          SR_HIP(g, sr_train_gap_mean(w, xsrc, B, sd.height * sd.width, sd.channels, A + mean_at[lane]));
          SR_HIP(g, sr_train_wgrad(w, q, A + mean_at[lane], da, A + part_at[lane], dtheta[ei]));
          if (dxsrc) {
            SR_HIP(g, sr_train_dgrad(s, q, e.w_dev, da, A + dmean_at, 0));
            SR_HIP(g, sr_train_gap_spread(s, A + dmean_at, B, sd.height * sd.width, sd.channels, dxsrc));
          }
          continue;
        }
        const float* dy = da;
        const float* dy_side = da;
        if (e.d.kind == SR_EDGE_CONV && e.d.upsample > 1) {
          SR_HIP(g, sr_train_pool_sum(w, da, B, q.Ho, q.Wo, q.Cout, e.d.upsample, A + pooled_at[lane]));
          dy_side = A + pooled_at[lane];
          if (dxsrc) SR_HIP(g, sr_train_pool_sum(s, da, B, q.Ho, q.Wo, q.Cout, e.d.upsample, A + pooled_at[0]));
          dy = A + pooled_at[0];
        }
        SR_HIP(g, sr_train_wgrad(w, q, xsrc, dy_side, A + part_at[lane], dtheta[ei]));
        if (dxsrc) SR_HIP(g, sr_train_dgrad(s, q, e.w_dev, dy, dxsrc, 1));
      }
    }
    // the side streams have read this frame's gradients: the copy can be cleared; it next holds frame i - 2
    if (join() != SR_OK) return SR_ERR_DEVICE;
    SR_HIP(g, sr_launch_fill_zero(s, A + dx_base[cur], frame_floats * sizeof(float)));
  }
  SR_HIP(g, sr_train_sum_terms(s, A + terms_at, W * B, scale, loss));
  return SR_OK;
  };

  // Plain launches.  (Capturing a window's launches into a graph bought large windows nothing, the time being
  // inside the kernels, and capture across the four streams ended in segmentation faults inside the runtime.)
  return enqueue();
}

sr_status sr_rmsprop_step(sr_graph* g, float lr, float rho, float eps, const float* const* dtheta,
                          const float* const* dbias) {
  if (!g || !dtheta || !(lr >= 0.f) || !(rho >= 0.f && rho <= 1.f) || !(eps > 0.f))
    return sr_gfail(g, SR_ERR_ARG, "bad argument to sr_rmsprop_step");
  if (g->dtype != SR_F32) return sr_gfail(g, SR_ERR_ARG, "sr_rmsprop_step: SR_F32 graphs only");
  for (int e = 0; e < g->n_edges; ++e) {
    if (!dtheta[e]) return sr_gfail(g, SR_ERR_ARG, "sr_rmsprop_step: dtheta[" + std::to_string(e) + "] is null");
    if (!g->edges[e].has_w) return sr_gfail(g, SR_ERR_STATE, "edge " + std::to_string(e) + " has no weights");
  }
  SrTrainState& T = train_state(g);
  if (T.rms_w.empty()) {
    T.rms_w.assign(g->n_edges, nullptr);
    T.rms_b.assign(g->n_nodes, nullptr);
  }
  auto running = [&](float** slot, size_t n) -> sr_status {
    if (*slot) return SR_OK;
    void* p = nullptr;
    SR_HIP(g, hipMalloc(&p, std::max<size_t>(n, 4) * sizeof(float)));
    g->dev_allocs.push_back(p);
    *slot = (float*)p;
    SR_HIP(g, sr_launch_fill_zero(g->stream, p, n * sizeof(float)));
    return SR_OK;
  };
  for (int e = 0; e < g->n_edges; ++e) {
    sr_status st = running(&T.rms_w[e], g->edges[e].w_count);
    if (st != SR_OK) return st;
    SR_HIP(g, sr_train_rmsprop(g->stream, g->edges[e].w_dev, T.rms_w[e], dtheta[e], g->edges[e].w_count, lr, rho, eps));
  }
  if (dbias)
    for (int v = 0; v < g->n_nodes; ++v) {
      if (g->an.is_input[v] || !dbias[v]) continue;
      const size_t n = (size_t)g->nodes[v].d.channels;
      sr_status st = running(&T.rms_b[v], n);
      if (st != SR_OK) return st;
      SR_HIP(g, sr_train_rmsprop(g->stream, g->nodes[v].bias_dev, T.rms_b[v], dbias[v], n, lr, rho, eps));
    }
  return SR_OK;
}

sr_status sr_graph_get_weights(sr_graph* g, int32_t edge, float* host_w, size_t count) {
  if (!g || !host_w || edge < 0 || edge >= g->n_edges) return sr_gfail(g, SR_ERR_ARG, "bad argument to sr_graph_get_weights");
  const EdgeRt& e = g->edges[edge];
  if (count != e.w_count) return sr_gfail(g, SR_ERR_ARG, "edge " + std::to_string(edge) + ": expected " + std::to_string(e.w_count) + " weights");
  if (!e.has_w) return sr_gfail(g, SR_ERR_STATE, "edge " + std::to_string(edge) + " has no weights");
  SR_HIP(g, hipStreamSynchronize(g->stream));
  SR_HIP(g, hipMemcpy(host_w, e.w_dev, count * sizeof(float), hipMemcpyDeviceToHost));
  return SR_OK;
}

sr_status sr_graph_get_bias(sr_graph* g, int32_t node, float* host_b, size_t count) {
  if (!g || !host_b || node < 0 || node >= g->n_nodes) return sr_gfail(g, SR_ERR_ARG, "bad argument to sr_graph_get_bias");
  if (count != (size_t)g->nodes[node].d.channels) return sr_gfail(g, SR_ERR_ARG, "bias length differs from the node's channels");
  SR_HIP(g, hipStreamSynchronize(g->stream));
  SR_HIP(g, hipMemcpy(host_b, g->nodes[node].bias_dev, count * sizeof(float), hipMemcpyDeviceToHost));
  return SR_OK;
}

}  // extern "C"
