// The graph object behind the opaque sr_graph handle of include/sr.h, shared by the host sources of the
// library (frame path: sr_host.cpp; training window: sr_train_host.cpp).
#ifndef SR_GRAPH_H_
#define SR_GRAPH_H_

#include <hip/hip_runtime_api.h>

#include <string>
#include <vector>

#include "../../include/sr.h"
#include "sr_internal.h"

// rollout analysis (host only)
struct Analysis {
  std::vector<int> is_input;   // node has no incoming edge (Eq. 1)
  std::vector<int> level;      // tableau value of (1, v) in the size-1 window (Eq. 5)
  int factor = 0;              // F(R), Eq. 6
};

// ---------------------------------------------------------------------------
// the graph object
// ---------------------------------------------------------------------------
struct NodeRt {
  sr_node_desc d{};
  int Cp = 0;                 // channel pitch of the stored state
  size_t state_bytes = 0;
  void* state[2] = {nullptr, nullptr};
  float* bias_dev = nullptr;  // [Cp] float
  std::vector<float> bias;
  int kind = 0;               // 0 input, 1 mfma, 2 direct, 3 head
  int input_slot = -1;
};

struct EdgeRt {
  sr_edge_desc d{};
  int kh = 0, kw = 0;              // effective kernel (dense: source H, W; GAP: 1)
  size_t w_count = 0;
  bool has_w = false;
  std::vector<float> w_host;       // rounded to the graph dtype, [kh][kw][Cin][Cout]
  float* w_dev = nullptr;          // same, float, for the direct and head kernels
  void* wpk_dev = nullptr;         // packed bf16 for the MFMA kernel
};

struct LevelPlan {
  int tile_begin = 0, n_tiles = 0;
  int block_begin = 0, n_blocks = 0;
  int head_begin = 0, n_heads = 0;
  int aux_begin = 0, n_aux = 0;     // head and input-staging items that ride along in this level's launch
};

struct sr_graph {
  int n_nodes = 0, n_edges = 0, batch = 0;
  sr_dtype dtype = SR_F32;
  hipStream_t stream = nullptr;
  std::vector<NodeRt> nodes;
  std::vector<EdgeRt> edges;
  Analysis an;
  std::vector<int> inputs;    // node ids of the input set, in node order
  std::string err;

  // options
  bool use_hipgraph = true, force_direct = false;
  int frames_per_graph = 8;

  // plan
  bool finalized = false, was_reset = false;
  int64_t host_frame = 0;
  std::vector<LevelPlan> levels;
  std::vector<void*> dev_allocs;     // everything to free
  SrCtx* ctx = nullptr;
  SrStageNode* stage_nodes = nullptr;
  SrAux* aux = nullptr;
  // input staging: 0 rides in level 1's launch (no R=0 edge leaves an input: nothing reads the new
  // input before the next frame); 1 staged one frame ahead: the next frame's input rides in this
  // frame's last launch, the first frame's is staged by the call; 2 a launch of its own ahead of
  // level 1 (an input also feeds a node of the last level over a bridging edge, which still reads
  // the copy the next input would overwrite)
  int stage_mode = 0;
  int stage_aux_begin = 0, n_stage_aux = 0;
  int aux_smem_bytes = 0;
  std::vector<int> head_node;   // node id of each head, in head order
  std::vector<SrHead> heads_host;
  SrDirectNode* d_nodes = nullptr;
  SrDirectEdge* d_edges = nullptr;
  SrDirectBlock* d_blocks = nullptr;
  SrMfmaNode* m_nodes = nullptr;
  SrMfmaEdge* m_edges = nullptr;
  SrMfmaTile* m_tiles = nullptr;
  SrStage8* stage8 = nullptr;
  int32_t* plan_index = nullptr;
  int32_t* plan_tables = nullptr;
  SrTap* tap_table = nullptr;
  SrPlane4* planes4 = nullptr;
  SrNode4* nodes4 = nullptr;
  SrTile4* tiles4 = nullptr;
  // dependency-driven execution (see SrDep): one launch covers all update steps of several frames
  int dataflow_option = 2;   // 0 never, 1 whenever possible, 2 (default) when a frame has more than one update step
  bool dataflow = false;
  int dep_spin_limit = 1 << 18;   // polls before a dependency wait gives up: ~0.3 s
  SrDep* deps = nullptr;
  int32_t* done_counters = nullptr;   // one per graph node
  SrTile4* flow_items = nullptr;      // a frame's work items in dependency order: tiles, and aux items as node = -2 - index
  int n_flow_items = 0;
  int32_t* flow_order = nullptr;      // (frame, item) pairs of a launch of flow_order_frames frames, by depth (see SrFlow)
  int n_flow_order = 0, flow_order_frames = 0;
  bool flow_depth_order = true;       // SR_OPT_FLOW_ORDER
  std::vector<int> flow_dep_begin, flow_dep_count;
  float* split_scratch = nullptr;
  size_t split_scratch_bytes = 0;
  int32_t* split_counters = nullptr;
  int n_split_slots = 0;
  bool allow_split = true;
  int tile_version = 0;       // 1: 4-wave tile kernel, 2: 8-wave tile kernel (both operands through LDS); 0: choose
  SrHead* heads = nullptr;
  SrHeadEdge* head_edges = nullptr;
  int lds_bytes = 0;
  int64_t n_mfma_tiles = 0;
  double flops = 0;
  double traffic[6] = {0, 0, 0, 0, 0, 0};   // see sr_graph_traffic_model
  int64_t device_bytes = 0;
  int launches_per_frame = 0;

  // rollout output recording (set per call)
  int rec_node = -1;

  // what the training window keeps between calls (arena, side streams, captured graph, RMSprop's running means):
  // made on first use and released by sr_train_state_release, both in sr_train_host.cpp
  struct SrTrainState* train = nullptr;
  int train_tall_from = 2048;   // SR_OPT_TRAIN_TALL_TILES_FROM

  hipGraph_t graph1 = nullptr, graphN = nullptr;
  hipGraphExec_t exec1 = nullptr, execN = nullptr;
  int graph_rec_node = -2;   // out_node the captured graphs record
};

void sr_train_state_release(struct SrTrainState* t);

// records the message in the graph (sr_last_error) and returns st
sr_status sr_gfail(sr_graph* g, sr_status st, const std::string& msg);

#define SR_HIP(g, call)                                                                              \
  do {                                                                                               \
    hipError_t e_ = (call);                                                                          \
    if (e_ != hipSuccess)                                                                            \
      return sr_gfail((g), e_ == hipErrorOutOfMemory ? SR_ERR_OOM : SR_ERR_DEVICE,                      \
                   std::string(#call) + ": " + hipGetErrorString(e_));                               \
  } while (0)

#endif  // SR_GRAPH_H_
