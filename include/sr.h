/*
 * libsr -- streaming-rollout frame update on one AMD MI355X (gfx950).
 *
 * A network is a directed graph whose nodes are layers and whose edges are
 * transformations (Sec. 3 of "The streaming rollout of deep networks").  A
 * rollout pattern R gives every edge a bridging bit: R(e) = 1 means the edge
 * reads its source at frame t-1, R(e) = 0 at frame t (Sec. 3, definition of
 * rollout pattern and window, Eq. 2).  One frame update computes, for every
 * node v that has incoming edges,
 *
 *     x_v(t) = sigma_v( b_v + sum_{e=(u,v)} f_e(theta_e, x_u(t - R(e))) )     (App. A1.2)
 *
 * With R == 1 everywhere (the streaming rollout) all nodes of a frame are
 * independent and are computed by one launch; otherwise a frame takes F(R)
 * dependent launches, one per value of the inference tableau (Eq. 5, Eq. 6).
 * Inference chains windows of size W = 1: the frame just computed is frame 0 of
 * the next window (Sec. 4, Sec. 5), so the library keeps two copies of every
 * state and alternates between them.
 *
 * General conventions
 *  - plain C ABI; every call returns an sr_status and never throws or aborts;
 *    output arguments are written only when SR_OK is returned.
 *  - "host" pointers are ordinary CPU memory, read during the call only.
 *    "device" pointers are HIP device memory owned by the caller, which must
 *    stay valid until the work enqueued by the call has finished on the
 *    graph's stream.
 *  - all tensors at the boundary are dense NHWC, [B][H][W][C], in the graph's
 *    dtype (float for SR_F32, bfloat16 bit patterns for SR_BF16).
 *  - the library owns the graph object, both copies of every node state, the
 *    packed weights and its HIP graph objects; sr_graph_destroy frees them.
 *  - all device work is enqueued on the HIP stream given at creation and is
 *    asynchronous with respect to the host unless stated otherwise.
 *  - node and edge ids are 0-based indices into the arrays given at creation;
 *    nodes need not be listed in any particular order.
 *  - calls on one graph object must not overlap in time (no internal locking).
 */
#ifndef SR_H_
#define SR_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sr_graph sr_graph; /* opaque */

typedef enum {
  SR_OK = 0,
  SR_ERR_ARG = 1,     /* null pointer, negative size, unknown enum value, R(e) not in {0,1} */
  SR_ERR_GRAPH = 2,   /* not a network: no edges, bad node id, or a node not reachable from the input set */
  SR_ERR_ROLLOUT = 3, /* invalid pattern: the edges with R(e)=0 contain a cycle (a self-edge with R=0 is one) */
  SR_ERR_SHAPE = 4,   /* an edge's result does not have the shape of its target node */
  SR_ERR_STATE = 5,   /* call order: weights missing, stepping before sr_reset, ... */
  SR_ERR_OOM = 6,     /* host or device allocation failed */
  SR_ERR_DEVICE = 7   /* a HIP call failed (no device, launch error); see sr_last_error */
} sr_status;

typedef enum { SR_F32 = 0, SR_BF16 = 1 } sr_dtype;
typedef enum { SR_ACT_IDENTITY = 0, SR_ACT_RELU = 1 } sr_act;

typedef enum {
  SR_EDGE_CONV = 0,     /* cross-correlation kh x kw, stride, zero padding pad, then nearest upsampling by `upsample` */
  SR_EDGE_DENSE = 1,    /* dense map over the flattened (h,w,c) source; target is 1x1; kh,kw = source H,W */
  SR_EDGE_GAP_DENSE = 2 /* mean over (h,w) of the source, then a dense map over channels; target is 1x1 */
} sr_edge_kind;

/* A node (layer): state x_v of shape [B][height][width][channels]; `act` is sigma_v.
 * Nodes without incoming edges are the network's inputs (Eq. 1); their `act` is ignored. */
typedef struct {
  int32_t channels, height, width;
  int32_t act; /* sr_act */
} sr_node_desc;

/* An edge (transformation) f_e from node src to node dst (App. A1.2).
 * conv:  y[b,ho,wo,co] = sum_{i,j,ci} theta[i,j,ci,co] * x[b, ho*stride+i-pad, wo*stride+j-pad, ci]
 *        (zero outside the source), then y_up[b,h,w,c] = y[b, h/upsample, w/upsample, c].
 * bridge is R(e): 1 reads the source at frame t-1, 0 at frame t. */
typedef struct {
  int32_t src, dst;
  int32_t kind; /* sr_edge_kind */
  int32_t kh, kw, stride, pad, upsample;
  uint8_t bridge;
} sr_edge_desc;

/* Option keys for sr_graph_configure. */
typedef enum {
  SR_OPT_USE_HIPGRAPH = 0,  /* 1 (default): frames are replayed from a captured HIP graph; 0: plain launches */
  SR_OPT_FORCE_DIRECT = 1,  /* 1: every node is computed by the plain one-thread-per-output kernel (no MFMA); default 0 */
  SR_OPT_FRAMES_PER_GRAPH = 2, /* number of frames captured into one HIP graph for sr_rollout (default 8, >= 1) */
  SR_OPT_K_SPLIT = 3,          /* 1 (default): long tiles are cut along the contraction and reduced by the last part; 0: never */
  SR_OPT_TILE_KERNEL = 4,      /* tile kernel of bf16 graphs: 1 = 4 waves per workgroup, weights from registers;
                                  2 = 8 waves, both operands through LDS, next stage loaded during the current one;
                                  0 (default) = 1 unless some node has an edge that fits its LDS budget neither whole nor cut into phase
                                  planes, then 2 */
  SR_OPT_DATAFLOW = 5,         /* dependency-driven execution of graphs whose nodes all run on the 4-wave tile kernel or as
                                  head items: one launch covers every update step of a frame, and of several frames in
                                  sr_rollout; a work item starts when the nodes it reads have completed the frame it
                                  reads (Eq. 2: frame t - R(e) of the edge's source), not when a whole update step or
                                  frame has -- consecutive frames overlap like the stages of a pipeline.
                                  2 (default): for patterns with more than one update step per frame (F(R) > 1, Eq. 6);
                                  1: whenever possible, also for the streaming pattern; 0: never (one launch per
                                  update step) */
  SR_OPT_DEP_SPIN_LIMIT = 6,   /* polls (with back-off) before a dependency wait of a dependency-driven graph gives up
                                  (default 2^18, about 0.3 s; 0..2^24).  A wait that gives up lets its work item go
                                  on with whatever is in memory and is counted by sr_graph_health; every kernel
                                  still ends normally.  For tests of that path. */
  SR_OPT_FLOW_ORDER = 7,       /* dependency-driven launches that cover several frames (sr_rollout):
                                  1 (default): the work items of all their frames are dispatched in the order of
                                  their depth in the rollout window of those frames (the inference tableau of Eq. 5
                                  taken over update steps of all the frames), so that update steps of consecutive
                                  frames that do not depend on one another run side by side;
                                  0: frame after frame */
  SR_OPT_TRAIN_TALL_TILES_FROM = 8
                               /* training window (sr_window_gradients): a contraction takes the taller of its two
                                  tile shapes when that launch has at least this many workgroups, else the shorter
                                  one (default 2048; 0: always the taller, 2^30: never).  Same results either way
                                  up to the order of no sum; for tests of both shapes and for tuning. */
} sr_option;

/* ---------------------------------------------------------------------------
 * Host-only analysis (Sec. 3).  Touches no device.
 * Validates that (nodes, edges) is a network and that the bridging bits form a
 * valid rollout pattern, and returns
 *   levels[v]          (host, n_nodes ints, may be NULL): value of the inference tableau of the
 *                      size-1 window at (1, v): the update step of a frame at which v is computed;
 *                      0 for input nodes (Eq. 5)
 *   inference_factor   (host, may be NULL): F(R) = max_v levels[v] (Eq. 6); 1 iff the pattern is
 *                      equally model-parallel to the streaming rollout (Theorem 1)
 * Errors: SR_ERR_ARG, SR_ERR_GRAPH, SR_ERR_ROLLOUT.  Shapes are not checked here
 * (n_nodes is enough; node descriptors are not needed). */
sr_status sr_analyze(int32_t n_nodes, const sr_edge_desc* edges, int32_t n_edges,
                     int32_t* levels, int32_t* inference_factor);

/* Number of valid rollout patterns of a network by exhaustive enumeration (Lemma 1
 * bounds this number); n_edges <= 24.  The bridge fields of `edges` are ignored.
 * count (host) receives the number.  Errors: SR_ERR_ARG, SR_ERR_GRAPH. */
sr_status sr_count_valid_patterns(int32_t n_nodes, const sr_edge_desc* edges, int32_t n_edges,
                                  uint64_t* count);

/* Inference tableau of the rollout window of size W (Eq. 5): tableau[i * n_nodes + v], frames
 * i = 0..W, is the number of update steps (Eq. 3, 4) after which node v of frame i has been
 * computed, starting from the initial state (frame 0 and all input nodes given): the length of
 * the longest path of the window ending in (i, v) that does not start with an edge into frame 0.
 * tableau: host, (W + 1) * n_nodes ints.  W >= 1.  The maximum over the window of size 1 is the
 * inference factor (Eq. 6).  Errors: SR_ERR_ARG, SR_ERR_GRAPH, SR_ERR_ROLLOUT. */
sr_status sr_tableau(int32_t n_nodes, const sr_edge_desc* edges, int32_t n_edges, int32_t W, int32_t* tableau);

/* Are two rollout patterns of one network equally model-parallel (Sec. 3), i.e. equal on every
 * edge that does not leave an input node?  bridge_a, bridge_b: host, n_edges values in {0, 1}
 * (the bridge fields of `edges` are ignored); neither needs to be valid.  equal (host) receives
 * 1 or 0.  Errors: SR_ERR_ARG, SR_ERR_GRAPH. */
sr_status sr_equally_model_parallel(int32_t n_nodes, const sr_edge_desc* edges, int32_t n_edges,
                                    const uint8_t* bridge_a, const uint8_t* bridge_b, int32_t* equal);

/* Bounds of Lemma 1 on the number n of valid rollout patterns:
 *   lower_forward = 2^|E_forward|         (edges on no cycle),
 *   lower_cycles  = max over sets C of pairwise edge-disjoint minimal cycles of prod (2^|p| - 1),
 *   upper         = 2^(|E| - |E_rec|)     (E_rec: self-connecting edges),
 * lower_forward <= n, lower_cycles <= n <= upper.  Exhaustive over the minimal cycles: networks
 * with more than 24 edges or more than 20 minimal cycles are refused.  Any output may be NULL.
 * The bridge fields of `edges` are ignored.  Errors: SR_ERR_ARG, SR_ERR_GRAPH. */
sr_status sr_pattern_count_bounds(int32_t n_nodes, const sr_edge_desc* edges, int32_t n_edges,
                                  uint64_t* lower_forward, uint64_t* lower_cycles, uint64_t* upper);

/* ---------------------------------------------------------------------------
 * Create the device-side representation of a network and its rollout pattern
 * (Sec. 3: network, rollout pattern; App. A1.2: node and edge maps).
 *   nodes, edges   host arrays, copied
 *   batch          B >= 1
 *   dtype          storage/arithmetic type: SR_F32 (float everywhere) or SR_BF16 (states and
 *                  weights bfloat16, products accumulated in float, bias float, result rounded to
 *                  nearest-even bfloat16 after sigma)
 *   hip_stream     a hipStream_t (NULL = the default stream); all work goes there
 *   out            receives the graph handle
 * Allocates both state copies (zero-filled), biases (zero) and weight storage on the current
 * device.  Errors: SR_ERR_ARG, SR_ERR_GRAPH, SR_ERR_ROLLOUT, SR_ERR_SHAPE (checked in this order,
 * all before any device call), SR_ERR_OOM, SR_ERR_DEVICE. */
sr_status sr_graph_create(const sr_node_desc* nodes, int32_t n_nodes,
                          const sr_edge_desc* edges, int32_t n_edges,
                          int32_t batch, sr_dtype dtype, void* hip_stream, sr_graph** out);

/* theta_e of one edge, host float array [kh][kw][Cin][Cout] (dense: [Hsrc][Wsrc][Cin][Cout];
 * GAP+dense: [Cin][Cout]); count must equal the product.  The library rounds to the graph's dtype
 * (nearest even) and repacks; synchronous with respect to the host copy. Every edge needs weights
 * before the first frame.  Errors: SR_ERR_ARG, SR_ERR_OOM, SR_ERR_DEVICE. */
sr_status sr_graph_set_weights(sr_graph* g, int32_t edge, const float* host_w, size_t count);

/* Channel-wise bias b_v of a node, host float [C]; default 0; kept in float. */
sr_status sr_graph_set_bias(sr_graph* g, int32_t node, const float* host_b, size_t count);

/* Options (see sr_option); must be called before the first sr_reset. */
sr_status sr_graph_configure(sr_graph* g, int32_t option, int64_t value);

/* Inference factor and tableau of the graph's pattern (as sr_analyze), plus the number of
 * kernel launches one frame takes (launches_per_frame, may be NULL): F(R) launches, one per update
 * step, or 1 for a dependency-driven graph (SR_OPT_DATAFLOW), whose update steps are ordered by
 * per-node completion counters inside the launch; sr_rollout then covers several frames per launch. */
sr_status sr_graph_info(const sr_graph* g, int32_t* inference_factor, int32_t* levels,
                        int32_t* launches_per_frame);

/* Frame 0 (initial state of Sec. 3; zero initial state per App. A2, training details):
 * every node with incoming edges is set to zero; input node i (i-th node without incoming
 * edges, in node order) is set to input_frame0[i] (device, NHWC, graph dtype), or to zero if that
 * pointer or the whole array is NULL.  The frame counter becomes 0. */
sr_status sr_reset(sr_graph* g, const void* const* input_frame0);

/* Advance one frame (one window of size 1 chained to the previous one, Sec. 4):
 * inputs_t[i] (device, NHWC, graph dtype) is the state of the i-th input node at the new frame t;
 * every other node is updated by the node map above.  Asynchronous.
 * Errors: SR_ERR_ARG, SR_ERR_STATE (no sr_reset yet, weights missing), SR_ERR_DEVICE. */
sr_status sr_frame_step(sr_graph* g, const void* const* inputs_t);

/* sr_frame_step for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result (bit for bit)
 * as sr_frame_step, but
 *  - it calls no hipMalloc / hipFree and no allocating library routine; every kernel of the frame is
 *    a plain launch on the graph's stream (nothing is captured or instantiated, no memset node), so
 *    the call may itself be captured by the caller;
 *  - the partial sums and arrival counters of tiles that are cut along their contraction (the only
 *    device memory a frame needs beyond the graph's states and tables) live in a static device
 *    array of the library, 64 MiB on every GPU the library is loaded on, instead of the graph's own
 *    arena: room for 1024 parts' counters and 64 MiB - 4 KiB of partial sums (128 KiB per part with
 *    the 4-wave tile kernel, 256 KiB with the 8-wave one; the 256x256 high-resolution benchmark graph
 *    needs about 38 MiB).  A graph that needs more is refused
 *    with SR_ERR_ARG and sr_last_error names both sizes; sr_frame_step still serves it.
 *  - the graph must have been planned and reset before (sr_reset does both and is where the graph's
 *    tables are allocated): otherwise SR_ERR_STATE.
 * All graphs on one GPU share the array, which keeps what the last call left (the counters are
 * cleared by the call): calls that overlap in time on one GPU -- two graphs on two streams -- race
 * on it and must be serialised by the caller.  Asynchronous.
 * Errors: SR_ERR_ARG, SR_ERR_STATE, SR_ERR_DEVICE. */
sr_status sr_frame_step_static(sr_graph* g, const void* const* inputs_t);

/* sr_reset(frame 0) followed by T calls of sr_frame_step(frame t), t = 1..T, without returning to
 * the host in between.
 *   inputs[i]   device pointer to [T+1][B][H][W][C] of the i-th input node, frame 0 first
 *   out_node    node whose state is recorded after every frame (ignored if outputs is NULL)
 *   outputs     device [T][B][H][W][C] of out_node (frames 1..T), or NULL
 * Asynchronous.  Errors as sr_frame_step. */
sr_status sr_rollout(sr_graph* g, const void* const* inputs, int32_t T, int32_t out_node, void* outputs);

/* Copy the current frame's state of a node to / from dense NHWC device memory of `bytes` bytes
 * (must equal B*H*W*C*sizeof(dtype)); enqueued on the graph's stream.  Together with the frame
 * counter these states are all the memory the stream has (Sec. 5), so get/set of every node is a
 * checkpoint.  sr_set_state on an input node is overwritten by the next frame's input. */
sr_status sr_get_state(const sr_graph* g, int32_t node, void* dst_device, size_t bytes);
sr_status sr_set_state(sr_graph* g, int32_t node, const void* src_device, size_t bytes);

/* Number of frames computed since the last sr_reset (host value). */
sr_status sr_frame_index(const sr_graph* g, int64_t* frame);

/* Run one frame with plain launches, bracketing every kernel of the frame with HIP events on
 * the graph's stream, and wait for it.  kernel_ms (host, capacity `cap`) receives the
 * duration of each launch in launch order, kernel_kind (host, may be NULL) a tag per launch:
 * 0 input staging, 1 MFMA convolution tiles, 2 direct (one thread per output) nodes, 3 GAP+dense
 * head, 4 bookkeeping; n_launches the number written.  Synchronous. */
sr_status sr_frame_step_timed(sr_graph* g, const void* const* inputs_t, float* kernel_ms,
                              int32_t* kernel_kind, int32_t cap, int32_t* n_launches);

/* Work of one frame as the library counts it: nominal multiply-adds * 2 over all edges
 * (padding taps counted, channel padding not), number of MFMA tiles, and bytes of both state
 * copies plus packed weights resident on the device.  Any pointer may be NULL. */
sr_status sr_graph_work(const sr_graph* g, double* flops_per_frame, int64_t* mfma_tiles,
                        int64_t* device_bytes);

/* Bytes one frame moves, by class, as the planner counts them (no cache is modelled; for setting the
 * HBM counters of a profile against): bytes6 (host, 6 doubles) =
 *   [0] every state that some edge reads, once        [1] every edge reading its whole source once
 *   [2] what the tiles of the 4-wave kernel load into LDS: per (tile, plane) the distinct source positions
 *       of its patch, all channel chunks -- [1] plus the halo rows and columns that neighbouring tiles share
 *       (0 for graphs on other kernels)
 *   [3] every weight once                              [4] the weights as the tiles read them (per tile the
 *       packed weights of its channel range; served by the L2 of the tile's XCD after the first tile)
 *   [5] every computed state written once.
 * The frame update of App. A1.2 needs [0] + [3] + [5] at least.  Plans the graph if needed. */
sr_status sr_graph_traffic_model(const sr_graph* g, double* bytes6);

/* Which tile kernel the graph's MFMA nodes run on (what SR_OPT_TILE_KERNEL = 0 chose, Eq. 2 hot
 * path): 1 = 4 waves per workgroup, 2 = 8 waves; 0 if the graph has no MFMA node (fp32 graphs,
 * SR_OPT_FORCE_DIRECT).  Plans the graph if that has not happened yet, as sr_graph_work does. */
sr_status sr_graph_tile_kernel(const sr_graph* g, int32_t* tile_kernel);

/* Health of a graph's device side.  dependency_driven (host, may be NULL): 1 if the graph runs
 * dependency-driven (plans the graph if needed).  dependency_timeouts (host, may be NULL): waits
 * for a node's completion counter that gave up at their spin limit since the last sr_reset; 0
 * unless something is broken (results are undefined otherwise); synchronises with the stream.
 * The waits implement the time index of Eq. 2 inside a launch. */
sr_status sr_graph_health(sr_graph* g, int64_t* dependency_timeouts, int32_t* dependency_driven);

/* Which kernel the planner gave each node of the frame update (App. A1.2 node map; plans the graph if
 * that has not happened yet): kinds[v] (host, n_nodes ints) =
 *   0 input node (its state is staged from the caller's frame),
 *   1 matrix-core tile kernel with 4 waves per workgroup, 2 matrix-core tile kernel with 8 waves,
 *   3 one-thread-per-output kernel (fp32 graphs; nodes neither tile kernel takes: an edge with stride
 *     or upsampling outside {1,2,4}, a source patch larger than the LDS budget),
 *   4 head item (1x1 node fed by dense / GAP+dense edges only).
 * Errors: SR_ERR_ARG, and what planning can return (SR_ERR_STATE: weights missing, SR_ERR_OOM, SR_ERR_DEVICE). */
sr_status sr_graph_node_kernels(const sr_graph* g, int32_t* kinds);

/* ---------------------------------------------------------------------------
 * One training window (Sec. 3: rollout window of size W >= 1 of the graph's pattern; Sec. 2: trained
 * by backpropagation through the rolled-out network; App. A2, training details: zero initial state,
 * loss = mean over the window's frames of the single-frame prediction losses, cross-entropy).
 * Runs frames 1..W from the zero state (the node map of App. A1.2 in fp32, every frame's states kept;
 * the graph's own frame state and frame counter are unspecified afterwards: sr_reset before stepping
 * frames again), then the reverse sweep over the window: frames W..1, inside a frame the update steps of
 * the inference tableau in reverse (Eq. 5).  With z(i) = state of out_node at frame i,
 *     loss = 1/(W*B) * sum_{i=1..W} sum_b -log softmax(z_b(i))[labels[b]]
 * and the gradients of that loss with respect to every theta_e and b_v are returned; the W copies
 * of an edge share their weights, so their gradients are summed.
 *   g         an SR_F32 graph with all weights set (SR_BF16 graphs: SR_ERR_ARG)
 *   inputs    host array, one device pointer per input node: float [W+1][B][H][W][C], frame 0 first
 *             (frame 0 is read by the bridging edges that leave an input node)
 *   masks     dropout (App. A2, training details: rates 0.25 and 0.5): NULL, or a host array of n_nodes device
 *             pointers, masks[v] NULL or float [W+1][B][H][W][C] multipliers of node v's state,
 *             x_v(i) = masks[v][i] * sigma_v(a_v(i)); the caller draws them (0 with the dropout rate,
 *             1/(1 - rate) otherwise, afresh for every frame and node); frame 0 and input nodes are ignored
 *   labels    device, B int32 class indices in [0, channels of out_node); values outside are clamped
 *   out_node  a 1x1 node with incoming edges whose channels are the class scores
 *   loss      device, 1 float
 *   dtheta    host array of n_edges device pointers; dtheta[e]: floats laid out like the weights given
 *             to sr_graph_set_weights for edge e ([kh][kw][Cin][Cout]); overwritten
 *   dbias     host array of n_nodes device pointers or NULL; dbias[v]: [C] floats, overwritten; entries
 *             of input nodes are ignored, a NULL entry skips that node
 * fp32 arithmetic; every sum is taken in a fixed order (no floating-point atomics): the same call
 * gives the same bits.  Device memory for the window's states and
 * gradients (about (W + 3) x the graph's node states, plus scratch) is allocated by the call, kept by
 * the graph and reused by later calls.  Asynchronous: the results are complete in the order of the
 * graph's stream (inside the call three more streams of the library's own, of default priority, run
 * work that does not depend on each other; they are joined to the graph's stream before the call's
 * last kernel); the host arrays are consumed before the call returns.  Every kernel is launched by the
 * call itself (SR_OPT_USE_HIPGRAPH concerns the frame path only).  No optimiser step is taken.
 * Errors: SR_ERR_ARG, SR_ERR_STATE (weights missing), SR_ERR_OOM, SR_ERR_DEVICE. */
sr_status sr_window_gradients(sr_graph* g, int32_t W, const void* const* inputs, const float* const* masks,
                              const int32_t* labels, int32_t out_node, float* loss, float* const* dtheta,
                              float* const* dbias);

/* One RMSprop update of every weight and bias of an SR_F32 graph, in place on the device (App. A2,
 * training details: RMSprop; Tieleman & Hinton 2012):
 *     a <- rho * a + (1 - rho) * g^2,     theta <- theta - lr * g / (sqrt(a) + eps)
 * with g the gradients as sr_window_gradients returns them (dtheta: n_edges device pointers; dbias:
 * n_nodes device pointers or NULL, NULL entries and input nodes skipped) and a the running mean of
 * the squared gradient, kept by the graph per parameter and zero before the first update.  The paper
 * gives lr = 1e-4 with a decay of 1e-6 per update (the caller passes the current lr); rho and eps are
 * not stated there (0.9 and 1e-7 are the defaults of the authors' framework).  The next frame or
 * window uses the new parameters; sr_graph_set_weights / sr_graph_set_bias overwrite them but leave a.
 * Asynchronous.  Errors: SR_ERR_ARG (bf16 graph, null gradient, lr < 0, rho outside [0,1], eps <= 0),
 * SR_ERR_STATE (weights missing), SR_ERR_OOM, SR_ERR_DEVICE. */
sr_status sr_rmsprop_step(sr_graph* g, float lr, float rho, float eps, const float* const* dtheta,
                          const float* const* dbias);

/* Current theta_e / b_v of the graph as the device holds them (after updates), into host float arrays
 * laid out as for sr_graph_set_weights / sr_graph_set_bias; count must match.  For bf16 graphs these are
 * the bf16-rounded values as floats.  Synchronises with the graph's stream.
 * Errors: SR_ERR_ARG, SR_ERR_STATE (no weights set), SR_ERR_DEVICE. */
sr_status sr_graph_get_weights(sr_graph* g, int32_t edge, float* host_w, size_t count);
sr_status sr_graph_get_bias(sr_graph* g, int32_t node, float* host_b, size_t count);

void sr_graph_destroy(sr_graph* g);

const char* sr_status_str(sr_status s);
/* Human-readable detail of the last error on this graph (or of the last failed
 * sr_graph_create / sr_analyze on this thread if g is NULL). */
const char* sr_last_error(const sr_graph* g);

#ifdef __cplusplus
}
#endif
#endif /* SR_H_ */
