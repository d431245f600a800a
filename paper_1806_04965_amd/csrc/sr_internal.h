// Shared between the host planner (sr_host.cpp) and the kernels (sr_kernels.hip):
// device-resident descriptor tables and the launch wrappers.
#pragma once
#include <hip/hip_runtime_api.h>
#include <stdint.h>

#define SR_MAX_INPUTS 16
#define SR_SPLIT_FLOATS (128 * 256)   // accumulator floats one part leaves in scratch
#define SR_XCDS 8          // accelerator complex dies of an MI355X; workgroup i of a launch runs on XCD i % 8
#define SR_CUS 256         // compute units of an MI355X

// One per graph, in device memory.  Kernels read the frame counter from here, so
// the same captured HIP graph serves every frame: the buffer written at frame t
// is t & 1, the buffer holding frame t-1 is the other one.
struct SrCtx {
  int32_t frame;      // index of the frame being computed (>= 1)
  int32_t in_base;    // input frame read = in_ptr[i] + (frame - in_base) * in_stride[i]
  int32_t out_base;   // output slot = frame - out_base
  int32_t done;       // workgroups of the frame's last launch that have finished (returns to 0)
  int32_t in_last;    // last frame for which the caller has given input; staging of a later frame is skipped
  int32_t dep_timeouts;   // dependency waits that gave up at their spin limit (stays 0 unless something is broken)
  const void* in_ptr[SR_MAX_INPUTS];
  int64_t in_stride[SR_MAX_INPUTS];   // bytes between consecutive frames (0: always the same buffer)
  void* out_ptr;                      // may be null
  int64_t out_stride;                 // bytes per recorded frame
};

// ---------------------------------------------------------------------------
// Dependency-driven execution.  In a streaming rollout a node's update at frame t needs nothing but
// its source nodes' states of frame t-1 (an edge with R(e) = 0: of frame t, computed at an earlier
// update step).  A launch in this mode covers several frames and all update steps of each: every
// work item (tile, head item, input-staging item) first waits until the nodes it depends on have
// completed the frames it needs, and adds one to its own node's counter when its results are in
// memory.  Work items are ordered so that every wait refers to items with a smaller workgroup index
// (earlier frame, or earlier update step of the same frame), which the hardware has dispatched
// before; waits are bounded by a spin limit all the same.
struct SrDep {
  int32_t node;    // graph node whose counter is read
  int32_t units;   // work items of that node per frame
  int32_t lag;     // the item at frame t needs units * (t - lag) completions (all of frame t - lag)
  int32_t pad_;
};

#define SR_DONE_STRIDE 64
struct SrFlow {
  const SrDep* deps;   // null: no dependency tracking (one launch per update step, ordered by the stream)
  int32_t* done;       // per graph node, SR_DONE_STRIDE ints apart (a memory line each: they are polled):
                       // work items completed since the last reset (wraps; compared by difference)
  int32_t spin_limit;  // polls before a wait gives up (and counts itself in SrCtx::dep_timeouts)
  int32_t frames;      // with `order`: frames the launch covers
  // null: workgroup (x, y) is work item x of frame y.  Else the launch is one-dimensional and workgroup i is work
  // item order[i] & 0xffffff of frame order[i] >> 24: the (frame, item) pairs of all its frames sorted by their
  // depth in the rollout window of those frames (the inference tableau of Eq. 5 taken over work items), so that
  // update steps of consecutive frames that do not depend on one another run side by side
  const int32_t* order;
};

// ---------------------------------------------------------------------------
// direct path: one thread per output element
// ---------------------------------------------------------------------------
struct SrDirectEdge {
  const void* src[2];   // source state, both copies
  const float* w;       // [kh][kw][Cin][Cout] float (already rounded to the graph dtype)
  int32_t bridge, kind; // kind: 0 conv (dense is a conv as large as its source), 2 GAP+dense
  int32_t Hs, Ws, Cin, Csp;   // source height, width, channels, channel pitch
  int32_t kh, kw, stride, pad, up;
  int32_t pad_;
};

struct SrDirectNode {
  void* out[2];
  const float* bias;    // [C]
  int32_t H, W, C, Cp;  // Cp: channel pitch of the stored state
  int32_t act;
  int32_t edge_begin, edge_count;
  int32_t pad_;
};

struct SrDirectBlock {   // one workgroup of 256 outputs
  int32_t node;
  int32_t first;         // first linear output element (over [B*H*W][C]) of this block
};

// ---------------------------------------------------------------------------
// MFMA path: node-centric implicit-GEMM tiles
// ---------------------------------------------------------------------------
struct SrMfmaEdge {
  const void* src[2];    // bf16 source state [B][Hs][Ws][Csp], both copies
  const void* wpk;       // packed bf16 weights [tap][Cin_p/16][Cout/32][64 lanes][8]
  int32_t bridge;
  int32_t Hs, Ws, Csp;   // source geometry and channel pitch
  int32_t kh, kw, stride, pad, up;
  int32_t KC;            // channels staged per LDS fill (16, 32 or 64)
  int32_t nchunk;        // Csp / KC
  int32_t PH;            // padded source rows per image: Hs + 2*pad
  int32_t PW;            // padded source width: Ws + 2*pad
  int32_t PWs;           // ceil(PW / stride): width of one column-phase plane
  int32_t RP;            // slots per patch row: stride * PWs
  int32_t SP;            // bytes per slot: KC*2 + 16 (one spare 16-byte piece rotates the LDS banks)
  int32_t RPB;           // bytes per patch row in LDS: >= RP*SP, tuned so that row wraps stay conflict-free
  int32_t magicKW;       // ceil(2^16 / kw): tap / kw == (tap * magic) >> 16 for tap < kh*kw (checked on host)
  int32_t wstride8;      // 16-byte units between consecutive k16 blocks in wpk: (Cout/32)*64
  int32_t plan_slot;     // 8-wave kernel: position of this edge's first row phase in a tile's run of plan_index
  int32_t src_bytes;     // bytes of one copy of the source state; SR_ZERO_TAIL zero bytes follow it
  // 4-wave kernel: a strided edge may be cut into phase planes -- the padded source rows q with
  // q % PR == pr and columns px with px % PC == pc, together with the taps (ti, tj) of the same
  // residues -- so that a stage's patch holds whole 128-byte lines of fewer pixels instead of a slice
  // of every pixel.  Every plane is an entry of its own in the edge table, described in patch
  // coordinates (an unsplit edge is the plane PR = PC = 1):
  int32_t lgRS;          // log2 of patch rows per output row: log2(stride) if the rows are not split, else 0
  int32_t PHr;           // patch rows per image
  int32_t ta_max;        // largest tap row offset, in patch rows
  int32_t PRmul, r0;     // source row of patch row r of an image: r * PRmul + r0 (negative or >= Hs: padding)
  int32_t PC, pc;        // column split (1: all columns, column-phase major as described above) and residue
  int32_t ntaps;         // taps of this plane
  int32_t tap_begin;     // first entry of this plane in the node's tap table
  int32_t imgB;          // bytes of one image of the source state: Hs * Ws * Csp * 2
  int32_t rowB;          // source bytes from one patch row to the next: PRmul * Ws * Csp * 2
  int32_t r0B;           // r0 * Ws * Csp * 2 (negative when the first patch row is padding)
  int32_t pad2_;
};

// 4-wave kernel: what the kernel reads of a plane, 16 dwords fetched by one scalar load
struct SrPlane4 {
  const void* src[2];    // source state, both copies
  const void* wpk;       // packed weights of the edge
  int32_t flags;         // bridge | lgRS << 8 | log2(upsample) << 16 | log2(KC / 16) << 24
  int32_t nchunk;
  int32_t PHr, RPB;
  int32_t imgB, rowB, r0B;
  int32_t wstride8;
  int32_t src_bytes;
  int32_t pad_;
};

// 4-wave kernel, per (tile, plane): what is needed to fetch the plane's plan and taps ahead of its descriptor
struct SrPlanRef {
  int32_t plan_at;     // offset of the plan in plan_tables
  int32_t n_pos;       // 16-byte LDS positions of the patch
  int32_t tap_begin;   // the plane's taps in the tap table
  int32_t ntaps;
};

// 4-wave kernel: node and tile records in the form the kernel loads, 16 dwords each (one scalar load)
struct SrNode4 {
  void* out[2];          // bf16 state [M][Cp], both copies
  const float* bias;     // [Cout rounded up to the tile width]
  int32_t M, Ho, Wo, Cp, act;
  int32_t waves_m, waves_n;
  int32_t dep_begin, dep_count;   // what a tile of this node waits for (SrDep table)
  int32_t gnode;                  // graph node id: index of this node's completion counter
};

struct SrTile4 {
  int32_t node;          // < 0: empty slot (pads an XCD's run)
  int32_t m0, n0;        // first output pixel and channel
  int32_t ref_base;      // SrPlanRef of plane p of this tile: refs[ref_base + p]
  int32_t p_first, p_last;   // planes walked (indices into the plane table)
  int32_t chunks;        // first chunk of the first plane | (one past the last chunk of the last plane) << 16
  int32_t split_slot;    // K-split: slot of part 0 in the launch's scratch, -1: not split
  int32_t part;          // part index | number of parts << 16
  int32_t shape;         // 32-channel tiles per wave (1 or 2) | (last image - first image) << 8
  int32_t b_first;       // image of the first pixel
  int32_t rows;          // output row of the first pixel | output row of the last pixel << 16
  SrPlanRef ref0;        // plan reference of plane p_first
};

// per tap of a plane: LDS byte offset of the tap's fragments relative to tap (0, 0) of the plane, and
// the index (in 16-byte units) of the tap's first weight fragment in the packed weights
struct SrTap {
  int32_t a, b;
};

// 8-wave tile kernel: one stage = one channel chunk of one row phase of one edge.  A strided edge
// is cut into `stride` row phases (source rows q with q % stride == phase, taps with
// ti % stride == phase), so that a stage's source patch stays small enough for two stages to be
// resident in LDS.
struct SrStage8 {
  int32_t edge;          // index into the edge table
  int32_t phase;
  int32_t chunk;
  int32_t pad_;
};

struct SrMfmaNode {
  void* out[2];          // bf16 state [M][Cp]
  const float* bias;     // [Cout]
  const int32_t* plan_index;   // [tile.plan_begin + edge]: offset of that (tile, edge) plan in plan_tables
                               // (4-wave kernel: SrPlanRef records, [tile.plan_begin + plane])
  const int32_t* plan_tables;  // per LDS position: source byte offset, or -1: padding (reads the zero tail of the state)
  const SrTap* tap_table;      // 4-wave kernel: taps of every plane of every edge
  const SrPlane4* planes4;     // 4-wave kernel: the edge table in the form the kernel loads (same indices)
  int32_t M;             // B*Ho*Wo
  int32_t Ho, Wo;
  int32_t Cout, Cp;
  int32_t act;
  int32_t edge_begin, edge_count;
  int32_t waves_m, waves_n;   // 4 waves arranged waves_m x waves_n; BM = 128*waves_m
  int32_t wn_tiles;           // 32-wide MFMA column tiles per wave: 1 or 2; BN = 32*wn_tiles*waves_n
  int32_t stage0;             // 8-wave kernel: first entry of this node in the stage table
  const SrStage8* stage_table;
};

struct SrMfmaTile {
  int32_t node;  // < 0: empty slot (pads an XCD's run)
  int32_t m0;    // first output pixel (linear over [B][Ho][Wo])
  int32_t n0;    // first output channel
  int32_t plan_begin;  // first entry of this tile in plan_index (one per incoming edge)
  // K-split: a long tile is cut into parts that each walk a range of the node's stages (a stage =
  // one channel chunk of one edge, counted over the node's edges in order) and leave their
  // accumulators in scratch; the part that finishes last adds them up in part order and stores.
  int32_t stage_begin, stage_end;
  int32_t split_slot;  // index of part 0 of this tile in the launch's scratch / counter arrays (SrSplitScratch), -1: not split
  int32_t part;        // part index | number of parts << 16
  // 4-wave kernel: the same stage range as (plane, chunk) positions in the node's edge table: the
  // tile walks planes e_first..e_last, from chunk c_first of the first one to chunk c_end - 1 of the last
  int32_t e_first, c_first, e_last, c_end;
};

// Where the parts of K-split tiles leave their accumulators during a launch; a kernel argument, so
// that the same tile lists run on the graph's own arena or on the library's static array.
struct SrSplitScratch {
  float* slabs;        // [slot][accumulator registers of a thread][threads of a workgroup] floats
  int32_t* counters;   // [slot] parts finished (returns to 0 when the last part has arrived)
};

// ---------------------------------------------------------------------------
// head nodes: 1x1 nodes all of whose incoming edges are dense or GAP+dense
// ---------------------------------------------------------------------------
struct SrHeadEdge {
  const void* src[2];
  const float* w;        // [K][Cout] float, K = Cin (pooled) or HW*Cin (flattened, (h,w,c) order)
  int32_t bridge;
  int32_t pooled;        // 1: mean over the HW pixels first; 0: the flattened source is the vector
  int32_t HW, Cin, Csp;  // source pixels per image, channels, channel pitch
  int32_t pad_;
};

struct SrHead {
  void* out[2];
  const float* bias;
  float* partial;        // [B][splits][Cin] float scratch (pooled single-edge heads with several slabs)
  int32_t* counters;     // [B] slabs finished per image (return to 0)
  int32_t edge_begin, edge_count;
  int32_t act, B, Cout, Cp;
  int32_t splits, record;   // record: also write the result to the rollout output
  int32_t dep_begin, dep_count, gnode, pad_;   // dependency-driven launches: see SrDep
};

#define SR_HEAD_MAX_K 12288   // longest input vector of a head edge (floats held in LDS)
#define SR_HEAD_MAX_COUT 256

// input staging / state packing
struct SrStageNode {
  void* state[2];
  int32_t elems_px;   // B*H*W
  int32_t C, Cp;
  int32_t input_slot; // index into SrCtx::in_ptr
  int32_t dep_begin, dep_count, gnode, pad_;   // dependency-driven launches: see SrDep
};

// work items other than tiles and direct blocks that ride along in a level's launch
#define SR_AUX_HEAD 1        // a = head index, b = image, c = pixel slab
#define SR_AUX_STAGE 2       // a = input node index (in stage order), b = chunk of SR_STAGE_CHUNK pixels,
                             // c = 0: this frame's input, 1: the next frame's (rides in a frame's last launch)
#define SR_STAGE_CHUNK 1024
#define SR_AUX_THREADS 256   // threads that work on an auxiliary item: a whole workgroup, or the first 256 of an 8-wave one
struct SrAux {
  int32_t kind, a, b, c;
};

// launch wrappers (sr_kernels.hip); each returns the hipError_t of the launch
hipError_t sr_launch_set_ctx(hipStream_t s, SrCtx* ctx, const SrCtx& values, int set_frame);
hipError_t sr_launch_tick(hipStream_t s, SrCtx* ctx);
hipError_t sr_launch_fill_zero(hipStream_t s, void* p, size_t bytes);
hipError_t sr_launch_pack(hipStream_t s, void* dst, const void* src, int px, int C, int Cp, int bf16, int unpack);
hipError_t sr_launch_record_output(hipStream_t s, const SrCtx* ctx, const void* state0, const void* state1,
                                   int px, int C, int Cp, int bf16);
hipError_t sr_launch_aux(hipStream_t s, SrCtx* ctx, const SrAux* aux, int n_aux, const SrHead* heads,
                         const SrHeadEdge* head_edges, const SrStageNode* stage_nodes, int smem_bytes, int bf16,
                         int is_last);
hipError_t sr_launch_direct(hipStream_t s, SrCtx* ctx, const SrDirectNode* nodes, const SrDirectEdge* edges,
                            const SrDirectBlock* blocks, int n_blocks, int bf16, int batch, const SrAux* aux, int n_aux,
                            const SrHead* heads, const SrHeadEdge* head_edges, const SrStageNode* stage_nodes,
                            int smem_bytes, int is_last);
struct SrTables4 {   // 4-wave kernel: the graph's device tables
  const SrNode4* nodes;
  const SrPlane4* planes;
  const SrPlanRef* refs;
  const int32_t* plan_tables;
  const SrTap* tap_table;
};
// frames > 1 or flow.deps != null: dependency-driven launch covering `frames` frames (grid y)
// flow.order != null: one-dimensional launch of n_order workgroups (see SrFlow)
hipError_t sr_launch_mfma(hipStream_t s, SrCtx* ctx, SrTables4 tables, SrFlow flow, int frames, int n_order,
                          const SrTile4* tiles, int n_tiles, int lds_bytes, const SrAux* aux, int n_aux,
                          const SrHead* heads, const SrHeadEdge* head_edges, const SrStageNode* stage_nodes,
                          int aux_smem_bytes, int is_last, SrSplitScratch split);
int sr_mfma_max_lds_bytes();
hipError_t sr_launch_mfma8(hipStream_t s, SrCtx* ctx, const SrMfmaNode* nodes, const SrMfmaEdge* edges,
                           const SrMfmaTile* tiles, int n_tiles, const SrAux* aux, int n_aux, const SrHead* heads,
                           const SrHeadEdge* head_edges, const SrStageNode* stage_nodes, int aux_smem_bytes, int is_last,
                           SrSplitScratch split);
// The library's static scratch: a file-scope device array of SR_STATIC_SCRATCH_BYTES on every GPU the
// library runs on, for the entry point that allocates nothing.  Returns its device address on the
// current device (looked up once per device).  Counters come first, slabs behind them.
#define SR_STATIC_SCRATCH_BYTES (64u << 20)
#define SR_STATIC_MAX_SLOTS 1024            // counters: 4 KiB at the start of the array
hipError_t sr_static_scratch(void** ptr);
// 8-wave kernel: bytes of one of its two stage buffers, and floats of one part's K-split slab
#define SR8_BUF_BYTES (80 * 1024)
#define SR_ZERO_TAIL 2048   // zero bytes behind every state copy: where padding pixels are loaded from
#define SR8_SPLIT_FLOATS (128 * 512)
