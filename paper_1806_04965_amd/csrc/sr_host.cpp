// Host side of libsr: the C ABI of include/sr.h, rollout analysis (Sec. 3), the frame planner
// (levels, tile work-lists, descriptor tables, weight packing) and the HIP-graph frame loop.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/sr.h"
#include "sr_internal.h"
#include "sr_graph.h"

namespace {

thread_local std::string g_last_error;

// ---------------------------------------------------------------------------
// rollout analysis (host only)
// ---------------------------------------------------------------------------

sr_status fail(std::string* err, sr_status st, const std::string& msg) {
  if (err) *err = msg;
  g_last_error = msg;
  return st;
}

// Definition of a network (Sec. 3): at least one edge, valid ids, every node reachable from I_N.
sr_status check_network(int n_nodes, const sr_edge_desc* edges, int n_edges, std::vector<int>* is_input,
                        std::string* err) {
  if (n_nodes <= 0 || n_edges < 0 || (n_edges > 0 && !edges)) return fail(err, SR_ERR_ARG, "bad node/edge arrays");
  if (n_edges == 0) return fail(err, SR_ERR_GRAPH, "a network needs at least one edge");
  for (int e = 0; e < n_edges; ++e) {
    if (edges[e].src < 0 || edges[e].src >= n_nodes || edges[e].dst < 0 || edges[e].dst >= n_nodes)
      return fail(err, SR_ERR_GRAPH, "edge " + std::to_string(e) + " names a node that does not exist");
  }
  is_input->assign(n_nodes, 1);
  for (int e = 0; e < n_edges; ++e) (*is_input)[edges[e].dst] = 0;
  std::vector<int> reached(*is_input), stack;
  for (int v = 0; v < n_nodes; ++v)
    if (reached[v]) stack.push_back(v);
  while (!stack.empty()) {
    int u = stack.back();
    stack.pop_back();
    for (int e = 0; e < n_edges; ++e)
      if (edges[e].src == u && !reached[edges[e].dst]) {
        reached[edges[e].dst] = 1;
        stack.push_back(edges[e].dst);
      }
  }
  for (int v = 0; v < n_nodes; ++v)
    if (!reached[v]) return fail(err, SR_ERR_GRAPH, "node " + std::to_string(v) + " is not reachable from an input node");
  return SR_OK;
}

// Validity (Sec. 3): rollout windows are acyclic iff the edges that stay inside a frame
// (R = 0) contain no cycle, since no window edge points backwards in time.  Levels: longest
// chain of R = 0 edges into v inside frame 1, where a chain may start with any edge whose
// source is already known (an input node, or a frame-0 node reached over an R = 1 edge).
sr_status analyse_pattern(int n_nodes, const sr_edge_desc* edges, int n_edges, const uint8_t* bits,
                          const std::vector<int>& is_input, Analysis* out, std::string* err) {
  std::vector<int> indeg(n_nodes, 0);
  for (int e = 0; e < n_edges; ++e) {
    if (bits[e] > 1) return fail(err, SR_ERR_ARG, "R(e) must be 0 or 1 (edge " + std::to_string(e) + ")");
    if (bits[e] == 0) indeg[edges[e].dst]++;
  }
  // Kahn's algorithm over the R = 0 sub-graph, carrying the longest-path value
  std::vector<int> level(n_nodes, 0), order;
  for (int v = 0; v < n_nodes; ++v) {
    level[v] = is_input[v] ? 0 : 1;   // every non-input node has an incoming edge: path length >= 1
    if (indeg[v] == 0) order.push_back(v);
  }
  for (size_t i = 0; i < order.size(); ++i) {
    int u = order[i];
    for (int e = 0; e < n_edges; ++e) {
      if (bits[e] != 0 || edges[e].src != u) continue;
      int v = edges[e].dst;
      level[v] = std::max(level[v], level[u] + 1);
      if (--indeg[v] == 0) order.push_back(v);
    }
  }
  if ((int)order.size() != n_nodes)
    return fail(err, SR_ERR_ROLLOUT, "the edges with R(e)=0 contain a cycle: rollout windows would be cyclic");
  out->is_input = is_input;
  out->level = level;
  out->factor = *std::max_element(level.begin(), level.end());
  return SR_OK;
}

inline int conv_out(int size, int k, int stride, int pad) { return (size + 2 * pad - k) / stride + 1; }

inline uint16_t f2bf(float f) {
  uint32_t u;
  std::memcpy(&u, &f, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}
inline float bf2f(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  std::memcpy(&f, &u, 4);
  return f;
}

inline uint32_t magic_for(uint32_t d) { return (uint32_t)((((uint64_t)1 << 32) + d - 1) / d); }
// largest x for which umulhi(x, magic_for(d)) == x / d is guaranteed
inline uint64_t magic_range(uint32_t d) {
  uint64_t m = magic_for(d);
  uint64_t e = m * d - ((uint64_t)1 << 32);   // 0 <= e < d
  if (e == 0) return ((uint64_t)1 << 32) - 1;
  return (((uint64_t)1 << 32) / e) - 1;
}

}  // namespace


sr_status sr_gfail(sr_graph* g, sr_status st, const std::string& msg) {
  if (g) g->err = msg;
  g_last_error = msg;
  return st;
}

namespace {

sr_status gfail(sr_graph* g, sr_status st, const std::string& msg) { return sr_gfail(g, st, msg); }


size_t elem_size(const sr_graph* g) { return g->dtype == SR_BF16 ? 2 : 4; }

// Uncached device memory for data that workgroups on different XCDs hand to each other inside one
// launch (K-split partial sums).  Blocks are never given back to the driver: a destroyed graph
// returns its block to this process-wide free list and a later graph reuses it.
struct UncachedBlock { void* ptr; size_t bytes; };
std::vector<UncachedBlock> g_uncached_free;
std::mutex g_uncached_mutex;

// *held receives the size of the block handed out (a reused block may be larger than asked for);
// that size goes back into the list with the block.
hipError_t uncached_alloc(void** p, size_t bytes, size_t* held) {
  std::lock_guard<std::mutex> lock(g_uncached_mutex);
  for (size_t i = 0; i < g_uncached_free.size(); ++i)
    if (g_uncached_free[i].bytes >= bytes) {
      *p = g_uncached_free[i].ptr;
      *held = g_uncached_free[i].bytes;
      g_uncached_free.erase(g_uncached_free.begin() + i);
      return hipSuccess;
    }
  *held = bytes;
  return hipExtMallocWithFlags(p, bytes, hipDeviceMallocUncached);
}

void uncached_release(void* p, size_t bytes) {
  std::lock_guard<std::mutex> lock(g_uncached_mutex);
  g_uncached_free.push_back(UncachedBlock{p, bytes});
}

sr_status dev_alloc(sr_graph* g, void** p, size_t bytes) {
  *p = nullptr;
  if (bytes == 0) bytes = 16;
  SR_HIP(g, hipMalloc(p, bytes));
  g->dev_allocs.push_back(*p);
  g->device_bytes += (int64_t)bytes;
  return SR_OK;
}

template <typename T>
sr_status upload(sr_graph* g, T** dev, const std::vector<T>& host) {
  void* p = nullptr;
  sr_status st = dev_alloc(g, &p, host.size() * sizeof(T));
  if (st != SR_OK) return st;
  if (!host.empty()) SR_HIP(g, hipMemcpy(p, host.data(), host.size() * sizeof(T), hipMemcpyHostToDevice));
  *dev = (T*)p;
  return SR_OK;
}

// shape of f_e's result (App. A1.2: must be summable at the target)
void edge_result_shape(const sr_graph* g, const EdgeRt& e, int* h, int* w) {
  const sr_node_desc& s = g->nodes[e.d.src].d;
  if (e.d.kind == SR_EDGE_CONV) {
    *h = conv_out(s.height, e.d.kh, e.d.stride, e.d.pad) * e.d.upsample;
    *w = conv_out(s.width, e.d.kw, e.d.stride, e.d.pad) * e.d.upsample;
  } else {
    *h = 1;
    *w = 1;
  }
}

// ---------------------------------------------------------------------------
// planner
// ---------------------------------------------------------------------------
struct MfmaChoice {
  int waves_m, waves_n, wn_tiles;
};

bool mfma_eligible(const sr_graph* g, int v) {
  if (g->dtype != SR_BF16 || g->force_direct) return false;
  const NodeRt& n = g->nodes[v];
  bool any = false;
  for (const EdgeRt& e : g->edges) {
    if (e.d.dst != v) continue;
    any = true;
    if (e.d.kind != SR_EDGE_CONV) return false;
    if (e.d.stride != 1 && e.d.stride != 2 && e.d.stride != 4) return false;
    if (e.d.upsample != 1 && e.d.upsample != 2 && e.d.upsample != 4) return false;
  }
  if (n.d.height > 4095 || n.d.width > 4095) return false;
  return any;
}

// Patch geometry of one (tile, edge): padded source rows Q0..Q1 that the tile's pixels touch.
struct PatchRows { int64_t b0, oy0, Q0, Q1; };
PatchRows patch_rows(int64_t m0, int64_t m1, int HoWo, int Wo, int PH, int s, int up, int kh) {
  PatchRows r;
  r.b0 = m0 / HoWo;
  r.oy0 = (m0 % HoWo) / Wo;
  const int64_t b1 = m1 / HoWo, oy1 = (m1 % HoWo) / Wo;
  r.Q0 = r.b0 * PH + (r.oy0 / up) * s;
  r.Q1 = b1 * PH + (oy1 / up) * s + kh - 1;
  return r;
}

int64_t max_patch_rows(const sr_graph* g, int v, const EdgeRt& e, int BM, int PH_override = 0) {
  const sr_node_desc& dn = g->nodes[v].d;
  const sr_node_desc& sn = g->nodes[e.d.src].d;
  const int HoWo = dn.height * dn.width;
  const int64_t M = (int64_t)g->batch * HoWo;
  const int PH = PH_override ? PH_override : sn.height + 2 * e.d.pad;
  int64_t worst = 0;
  for (int64_t m0 = 0; m0 < M; m0 += BM) {
    PatchRows r = patch_rows(m0, std::min<int64_t>(m0 + BM, M) - 1, HoWo, dn.width, PH, e.d.stride, e.d.upsample, e.d.kh);
    worst = std::max(worst, r.Q1 - r.Q0 + 1);
  }
  return worst;
}

// Row pitch of the LDS patch in 16-byte units: at least RP slots of CH1 pieces, and chosen so
// that stepping from the last pixel of an output row to the first pixel of the next one moves
// by the same number of 16-byte columns (mod 16) as stepping to the next pixel inside a row;
// sixteen consecutive pixels then always fall into sixteen different LDS columns.
int row_pitch16(int RP, int CH1, int s, int up, int Wo) {
  const int base = RP * CH1;
  if (up != 1) return base;
  for (int r = base; r < base + 16; ++r)
    if ((s * r) % 16 == (Wo * CH1) % 16) return r;
  return base;
}

// Positions that nothing reads repeat their predecessor's entry (the first one: zero padding): every
// lane of a direct-to-LDS instruction then loads something valid and no lane mask is needed.
void fill_unread_positions(std::vector<int32_t>* out, size_t begin, size_t end) {
  for (size_t i = begin; i < end; ++i)
    if ((*out)[i] == -2) (*out)[i] = (i > begin) ? (*out)[i - 1] : -1;
}

// Direct-to-LDS plan of one (tile, plane): for every 16-byte LDS position the byte offset of its
// source relative to (image b0, the source row that the tile's first patch row stands for), or -1
// (zero padding).  A plane holds the padded source rows q = pr (mod PR) as patch rows (q - pr) / PR
// and, if its columns are split as well, the padded columns px = pc (mod stride) as slots
// (px - pc) / stride; an unsplit row keeps all columns, column-phase major.
void build_plan(std::vector<int32_t>* out, const SrMfmaEdge& m, const PatchRows& r) {
  const int CH1 = m.KC / 8 + 1, CH = CH1 - 1;
  const int RPB16 = m.RPB / 16;
  const int64_t NQ = r.Q1 - r.Q0 + 1;
  const int64_t n_pos = NQ * RPB16;
  const int64_t padded = (n_pos + 255) / 256 * 256;
  out->assign((size_t)padded, -2);
  const int64_t row_first = r.Q0 - r.b0 * m.PHr;                 // patch row of the tile's first row, in its image
  const int64_t iy_first = row_first * m.PRmul + m.r0;
  for (int64_t q = 0; q < NQ; ++q) {
    const int64_t Qg = r.Q0 + q, b = Qg / m.PHr, iy = (Qg % m.PHr) * m.PRmul + m.r0;
    for (int col = 0; col < m.RP; ++col) {
      int px;
      if (m.PC == 1) {
        const int phase = col / m.PWs;
        px = (col % m.PWs) * m.stride + phase;
      } else {
        px = col * m.stride + m.pc;
      }
      if (px >= m.PW) continue;
      const int ix = px - m.pad;
      const bool valid = iy >= 0 && iy < m.Hs && ix >= 0 && ix < m.Ws;
      for (int piece = 0; piece < CH; ++piece) {
        int32_t off = -1;
        if (valid) off = (int32_t)(((((b - r.b0) * m.Hs + iy - iy_first) * m.Ws + ix) * m.Csp) * 2 + piece * 16);
        (*out)[(size_t)(q * RPB16 + col * CH1 + piece)] = off;
      }
    }
  }
  fill_unread_positions(out, 0, out->size());
}

// The planes an edge is cut into for a row split PR and column split PC (each 1 or the stride), and
// what the tile kernel needs to know of each; KC, RPB and the tap table are filled in by the caller.
struct PlaneGeom {
  int pr, pc, PHr, lgRS, ta_max, RP, ntaps;
  std::vector<SrTap> taps;   // here a = tap row offset in patch rows, b = tap slot offset (bytes are formed once RPB and SP are known)
  std::vector<int> tap_id;   // ti * kw + tj of every tap, in the plane's tap order
};
std::vector<PlaneGeom> edge_planes(int kh, int kw, int s, int PH, int PW, int PR, int PC) {
  std::vector<PlaneGeom> planes;
  const int PWs = (PW + s - 1) / s;
  const int lgs = (s == 1) ? 0 : (s == 2 ? 1 : 2);
  for (int pr = 0; pr < PR; ++pr)
    for (int pc = 0; pc < PC; ++pc) {
      PlaneGeom pg;
      pg.pr = pr; pg.pc = pc;
      pg.PHr = (PR == 1) ? PH : (PH - pr + s - 1) / s;
      pg.lgRS = (PR == 1) ? lgs : 0;
      pg.RP = (PC == 1) ? s * PWs : (PW - pc + s - 1) / s;
      pg.ta_max = 0;
      for (int ti = 0; ti < kh; ++ti) {
        if (ti % PR != pr) continue;
        const int ta = (PR == 1) ? ti : (ti - pr) / s;
        for (int tj = 0; tj < kw; ++tj) {
          if (tj % PC != pc) continue;
          const int tb = (PC == 1) ? (tj % s) * PWs + tj / s : (tj - pc) / s;
          pg.taps.push_back(SrTap{ta, tb});
          pg.tap_id.push_back(ti * kw + tj);
          pg.ta_max = std::max(pg.ta_max, ta);
        }
      }
      pg.ntaps = (int)pg.taps.size();
      if (pg.ntaps > 0 && pg.PHr > 0 && pg.RP > 0) planes.push_back(pg);
    }
  return planes;
}

int64_t max_plane_rows(const sr_graph* g, int v, const EdgeRt& e, int BM, const PlaneGeom& pg) {
  const sr_node_desc& dn = g->nodes[v].d;
  const int HoWo = dn.height * dn.width;
  const int64_t M = (int64_t)g->batch * HoWo;
  int64_t worst = 0;
  for (int64_t m0 = 0; m0 < M; m0 += BM) {
    PatchRows r = patch_rows(m0, std::min<int64_t>(m0 + BM, M) - 1, HoWo, dn.width, pg.PHr, 1 << pg.lgRS, e.d.upsample, pg.ta_max + 1);
    worst = std::max(worst, r.Q1 - r.Q0 + 1);
  }
  return worst;
}

// How an edge is staged by the 4-wave kernel: the split (PR, PC) and the channels per stage KC.
// Every stage costs a fixed latency (its loads are issued and waited for in one burst) plus the time
// its patch takes through the compute unit's vector memory path, which moves whole 128-byte lines:
// a stage that takes KC * 2 bytes of a pixel's min(128, Csp * 2) pays for the whole line.  The
// cheapest combination wins (GTSRB-shaped graph: the stride-2 edges from 64-channel 48x48 states go
// from four 16-channel stages that each touch every line to four phase planes of whole lines, 424 ->
// 406 us per frame; the hi-res graph keeps unsplit 32-channel stages, fewer of them).  KC = 0: no
// combination fits the LDS budget.
struct EdgeStaging { int PR = 1, PC = 1, KC = 0; };
EdgeStaging choose_staging(const sr_graph* g, int v, const EdgeRt& e, int BM, int lds_cap) {
  const NodeRt& n = g->nodes[v];
  const NodeRt& sn = g->nodes[e.d.src];
  const int s = e.d.stride, PH = sn.d.height + 2 * e.d.pad, PW = sn.d.width + 2 * e.d.pad;
  constexpr double kStageCycles = 2500.0, kLineBytesPerCycle = 64.0;
  EdgeStaging best;
  double best_cost = 0;
  std::vector<std::pair<int, int>> splits = {{1, 1}};
  if (s > 1) { splits.push_back({s, 1}); splits.push_back({s, s}); }
  for (const auto& sp : splits) {
    const std::vector<PlaneGeom> planes = edge_planes(e.d.kh, e.d.kw, s, PH, PW, sp.first, sp.second);
    for (int cand : {64, 32, 16}) {
      if (sn.Cp % cand != 0) continue;
      bool fits = true;
      double bytes = 0;
      for (const PlaneGeom& pg : planes) {
        const int pitch = row_pitch16(pg.RP, cand / 8 + 1, 1 << pg.lgRS, e.d.upsample, n.d.width);
        const int64_t b = max_plane_rows(g, v, e, BM, pg) * pitch * 16;
        if (b > lds_cap) fits = false;
        bytes += (double)b;
      }
      if (!fits) continue;
      const double eff = std::min(1.0, cand * 2.0 / std::min(128, sn.Cp * 2));
      const int chunks = sn.Cp / cand;
      const double cost = chunks * ((double)planes.size() * kStageCycles + bytes / eff / kLineBytesPerCycle);
      if (best.KC == 0 || cost < best_cost) {
        best_cost = cost;
        best.PR = sp.first; best.PC = sp.second; best.KC = cand;
      }
      break;   // smaller KC of the same split: never better
    }
  }
  return best;
}

// Does the 4-wave tile kernel have a tile shape for node v all of whose edges can be staged (unsplit or
// cut into phase planes) within its LDS budget?  (Decides the default tile kernel: only a graph with a
// node that fails this goes to the 8-wave kernel.  The paper's DSR networks, whose 4x4 node reads 16x16
// states over stride-4 edges, pass since strided edges are staged as phase planes: 16 images' worth of
// every fourth row and column is a few KiB.  On them the 4-wave kernel is as fast or faster per streaming
// frame, 31-51 against 32-61 us, and their sequential pattern runs dependency-driven, 52-137 against
// 82-270 us per frame.)
bool four_wave_kernel_fits(const sr_graph* g, int v, int lds_cap) {
  const NodeRt& n = g->nodes[v];
  const int Cout = (n.d.channels + 31) / 32 * 32;   // channel tiles are 32 wide; the rest of the last one is padding
  for (int wt : {2, 1})
    for (int wn : {4, 2, 1}) {
      if (Cout % (32 * wt * wn) != 0) continue;
      const int BM = 128 * (4 / wn);
      if (BM / ((int64_t)n.d.height * n.d.width) + 2 > 127) continue;
      bool ok = true;
      for (const EdgeRt& e : g->edges) {
        if (e.d.dst != v) continue;
        if (e.d.kh * e.d.kw > 64 || choose_staging(g, v, e, BM, lds_cap).KC == 0) ok = false;
      }
      if (ok) return true;
    }
  return false;
}

// 8-wave kernel: plan of one (tile, edge, row phase): per 16-byte LDS position of a stage buffer the
// byte offset of its source.  First the A positions (patch rows = the source rows q = phase
// (mod stride) of the tile's row range; slots of KC*2 bytes, unpadded; offsets from (image b0,
// source row iy_first); -1 zero padding), rounded up to a multiple of 64; then the B positions
// ((t * K16 + k) * NBT + nt) * 64 + lane: the packed fragment of the phase's t-th tap, 16-channel
// block k of the chunk, column tile nt of the tile (offsets from the chunk's first block and the
// tile's first column tile); the whole padded to a multiple of 512.
void build_plan8(std::vector<int32_t>* out, const SrMfmaEdge& m, const PatchRows& r, int phase, int NBT) {
  const int CH = m.KC / 8;
  const int RPS = m.RP;
  const int64_t NQ = r.Q1 - r.Q0 + 1;
  const int64_t NQr = (NQ - phase + m.stride - 1) / m.stride;
  const int64_t n_pos = NQr * RPS * CH;
  const int64_t padded = (n_pos + 63) / 64 * 64;
  out->assign((size_t)padded, -2);
  const int64_t iy_first = (r.oy0 / m.up) * m.stride - m.pad;
  for (int64_t qr = 0; qr < NQr; ++qr) {
    const int64_t Qg = r.Q0 + qr * m.stride + phase, b = Qg / m.PH, iy = Qg % m.PH - m.pad;
    for (int col = 0; col < m.RP; ++col) {
      const int cphase = col / m.PWs, px = (col % m.PWs) * m.stride + cphase;
      if (px >= m.PW) continue;
      const int ix = px - m.pad;
      const bool valid = iy >= 0 && iy < m.Hs && ix >= 0 && ix < m.Ws;
      for (int piece = 0; piece < CH; ++piece) {
        int32_t off = -1;
        if (valid) off = (int32_t)(((((b - r.b0) * m.Hs + iy - iy_first) * m.Ws + ix) * m.Csp) * 2 + piece * 16);
        (*out)[(size_t)((qr * RPS + col) * CH + piece)] = off;
      }
    }
  }
  const int K16 = m.KC / 16, k16_total = m.Csp / 16;
  const int tap_rows = (m.kh - phase + m.stride - 1) / m.stride;
  const int64_t n_posB = (int64_t)tap_rows * m.kw * K16 * NBT * 64;
  fill_unread_positions(out, 0, out->size());
  const size_t b0 = out->size();
  out->resize((b0 + (size_t)n_posB + 511) / 512 * 512, 0);
  for (int64_t pb = 0; pb < n_posB; ++pb) {
    const int lane = (int)(pb % 64), nt = (int)(pb / 64 % NBT), k = (int)(pb / (64 * NBT) % K16);
    const int t = (int)(pb / (64 * NBT * K16));
    const int tap = (phase + (t / m.kw) * m.stride) * m.kw + t % m.kw;
    (*out)[b0 + (size_t)pb] = (int32_t)((((int64_t)(tap * k16_total + k) * m.wstride8) + nt * 64 + lane) * 16);
  }
}

sr_status finalize(sr_graph* g) {
  if (g->finalized) return SR_OK;
  for (int e = 0; e < g->n_edges; ++e)
    if (!g->edges[e].has_w) return gfail(g, SR_ERR_STATE, "edge " + std::to_string(e) + " has no weights");
  const int B = g->batch;
  const bool bf16 = g->dtype == SR_BF16;
  const int F = g->an.factor;

  // classify nodes
  for (int v = 0; v < g->n_nodes; ++v) {
    NodeRt& n = g->nodes[v];
    if (g->an.is_input[v]) { n.kind = 0; continue; }
    // head: every incoming edge is dense or GAP+dense, with input vectors and outputs that fit the item
    bool head_ok = !g->force_direct && n.d.channels <= SR_HEAD_MAX_COUT;
    for (const EdgeRt& e : g->edges) {
      if (e.d.dst != v) continue;
      const sr_node_desc& sd = g->nodes[e.d.src].d;
      if (e.d.kind == SR_EDGE_CONV) head_ok = false;
      if (e.d.kind == SR_EDGE_DENSE && (int64_t)sd.height * sd.width * sd.channels > SR_HEAD_MAX_K) head_ok = false;
      if (e.d.kind == SR_EDGE_GAP_DENSE && sd.channels > SR_HEAD_MAX_K) head_ok = false;
    }
    if (mfma_eligible(g, v)) n.kind = 1;
    else if (head_ok) n.kind = 3;
    else n.kind = 2;
  }

  // Tile kernel: the 4-wave kernel unless one of its nodes would not fit its LDS budget (patches of
  // edges with a large stride on small images span many images) -- the 8-wave kernel cuts strided
  // edges into row phases and takes those; a node it cannot take either goes the direct way.
  if (g->tile_version == 0) {
    g->tile_version = 1;
    for (int v = 0; v < g->n_nodes; ++v)
      if (g->nodes[v].kind == 1 && !four_wave_kernel_fits(g, v, sr_mfma_max_lds_bytes())) g->tile_version = 2;
  }

  std::vector<SrStageNode> stage;
  for (size_t i = 0; i < g->inputs.size(); ++i) {
    NodeRt& n = g->nodes[g->inputs[i]];
    SrStageNode s{};
    s.state[0] = n.state[0];
    s.state[1] = n.state[1];
    s.elems_px = B * n.d.height * n.d.width;
    s.C = n.d.channels;
    s.Cp = n.Cp;
    s.input_slot = (int)i;
    stage.push_back(s);
  }

  std::vector<SrDirectNode> dn;
  std::vector<SrDirectEdge> de;
  std::vector<SrDirectBlock> db;
  std::vector<SrMfmaNode> mn;
  std::vector<SrMfmaEdge> me;
  std::vector<SrMfmaTile> mt;
  std::vector<SrStage8> stage8;
  std::vector<SrHead> hd;
  std::vector<SrHeadEdge> he;
  std::vector<int32_t> plan_index, plan_tables, plan_tmp;   // per (tile, edge): offset of its plan
  std::vector<SrTap> tap_table;                             // 4-wave kernel: taps of every plane
  size_t tap_mark = 0;
  std::vector<int> node_units(g->n_nodes, 0);               // work items per frame that complete a node (dependency counting)
  std::vector<int> mfma_graph_node;                         // 4-wave kernel: graph node of every entry of the node table
  std::unordered_map<uint64_t, std::vector<int>> plan_seen;
  g->levels.assign(F + 1, LevelPlan());
  const int lds_cap = sr_mfma_max_lds_bytes();
  g->lds_bytes = 0;
  g->flops = 0;
  for (double& t : g->traffic) t = 0;
  for (int v = 0; v < g->n_nodes; ++v) {
    bool read = false;
    for (const EdgeRt& e : g->edges) read |= (e.d.src == v);
    const double bytes = (double)B * g->nodes[v].d.height * g->nodes[v].d.width * g->nodes[v].Cp * elem_size(g);
    if (read) g->traffic[0] += bytes;                       // every state that has a reader, once
    if (!g->an.is_input[v]) g->traffic[5] += bytes;         // every computed state, written once
  }
  for (const EdgeRt& e : g->edges) {
    const NodeRt& sn = g->nodes[e.d.src];
    g->traffic[1] += (double)B * sn.d.height * sn.d.width * sn.Cp * elem_size(g);   // one full read per edge
    g->traffic[3] += (double)e.w_count * elem_size(g);
  }
  g->n_mfma_tiles = 0;

  for (const EdgeRt& e : g->edges) {
    const sr_node_desc& s = g->nodes[e.d.src].d;
    const sr_node_desc& d = g->nodes[e.d.dst].d;
    double macs;
    if (e.d.kind == SR_EDGE_CONV)
      macs = (double)(d.height / e.d.upsample) * (d.width / e.d.upsample) * d.channels * s.channels * e.d.kh * e.d.kw;
    else if (e.d.kind == SR_EDGE_DENSE)
      macs = (double)s.height * s.width * s.channels * d.channels;
    else
      macs = (double)s.channels * d.channels;
    g->flops += 2.0 * B * macs;
  }

  std::vector<SrAux> aux, stage_aux;
  for (size_t i = 0; i < stage.size(); ++i) {
    const int total = stage[i].elems_px;
    for (int c = 0; c * SR_STAGE_CHUNK < total; ++c) stage_aux.push_back(SrAux{SR_AUX_STAGE, (int)i, c, 0});
  }
  g->stage_mode = 0;
  for (const EdgeRt& e : g->edges)
    if (g->an.is_input[e.d.src] && e.d.bridge == 0) g->stage_mode = 1;
  if (g->stage_mode == 1)
    for (const EdgeRt& e : g->edges)
      if (g->an.is_input[e.d.src] && e.d.bridge == 1 && g->an.level[e.d.dst] == F) g->stage_mode = 2;
  if (g->stage_mode != 0) {   // this frame's input as a launch of its own: ahead of level 1, or once per call
    g->stage_aux_begin = 0;
    g->n_stage_aux = (int)stage_aux.size();
    aux = stage_aux;
  }
  for (int L = 1; L <= F; ++L) {
    LevelPlan& lp = g->levels[L];
    lp.tile_begin = (int)mt.size();
    lp.block_begin = (int)db.size();
    lp.head_begin = (int)hd.size();
    struct TileGroup {
      int node_index; double cost; int n_stages; std::vector<SrMfmaTile> tiles;
      std::vector<int> nchunks;   // 4-wave kernel: stages (channel chunks) of every plane of the node, in order
    };
    std::vector<TileGroup> groups;
    std::vector<SrAux> level_aux;
    if (L == 1 && g->stage_mode == 0) level_aux = stage_aux;
    if (L == F && g->stage_mode == 1)
      for (SrAux it : stage_aux) { it.c = 1; level_aux.push_back(it); }

    for (int v = 0; v < g->n_nodes; ++v) {
      NodeRt& n = g->nodes[v];
      if (g->an.level[v] != L || n.kind == 0) continue;
      if (n.kind == 1 && g->tile_version == 2) {
        // ---- 8-wave tile kernel: widest channel tile that divides Cout (at most 128: the weight slab
        // of a stage lives in LDS), 8 waves arranged waves_m x waves_n
        // channel tiles are 32 wide: a node whose channel count is no multiple of 32 gets zero weights and
        // zero bias for the rest of its last tile, and the epilogue stores only the pixel's Cp channels
        const int Cout = (n.d.channels + 31) / 32 * 32;
        const int64_t M = (int64_t)B * n.d.height * n.d.width;
        // shapes (wn_tiles, waves_n), preferred first: the widest channel tile up to 128 (the weight slab
        // of a stage lives in LDS) on the longest pixel tile; then shorter pixel tiles, whose source
        // patches are smaller
        std::vector<std::pair<int, int>> shapes;
        for (const auto& c : {std::pair<int, int>(2, 2), std::pair<int, int>(2, 1), std::pair<int, int>(1, 1),
                              std::pair<int, int>(1, 2), std::pair<int, int>(1, 4)})
          if (Cout % (32 * c.first * c.second) == 0) shapes.push_back(c);
        if (!shapes.empty()) {   // few tiles: shorter pixel tiles of the same channel width first (as in the 4-wave planner)
          const int bn0 = 32 * shapes[0].first * shapes[0].second, bm0 = 128 * (8 / shapes[0].second);
          if ((M + bm0 - 1) / bm0 * (Cout / bn0) < SR_CUS) {
            std::vector<std::pair<int, int>> shorter;
            for (const auto& c : shapes)
              if (32 * c.first * c.second == bn0 && 128 * (8 / c.second) < bm0) shorter.push_back(c);
            shapes.insert(shapes.begin(), shorter.begin(), shorter.end());
          }
        }
        int wt = 0, wn = 0, waves_m = 0, BM = 0, BN = 0, NBT = 0;
        SrMfmaNode node{};
        bool ok = false;
        int plan_slots = 0, n_stages = 0;
        double cyc = 0;
        for (const auto& shape : shapes) {
        wt = shape.first; wn = shape.second;
        waves_m = 8 / wn; BM = 128 * waves_m; BN = 32 * wt * wn; NBT = wt * wn;
        node = SrMfmaNode{};
        node.out[0] = n.state[0];
        node.out[1] = n.state[1];
        node.bias = n.bias_dev;
        node.M = (int)M;
        node.Ho = n.d.height;
        node.Wo = n.d.width;
        node.Cout = Cout;
        node.Cp = n.Cp;
        node.act = n.d.act;
        node.edge_begin = (int)me.size();
        node.waves_m = waves_m;
        node.waves_n = wn;
        node.wn_tiles = wt;
        node.stage0 = (int)stage8.size();
        ok = ((int64_t)BM / ((int64_t)n.d.height * n.d.width) + 2 <= 127);
        plan_slots = 0; n_stages = 0;
        cyc = 8000;
        for (EdgeRt& e : g->edges) {
          if (e.d.dst != v || !ok) continue;
          const NodeRt& sn = g->nodes[e.d.src];
          SrMfmaEdge m{};
          m.src[0] = sn.state[0];
          m.src[1] = sn.state[1];
          m.wpk = e.wpk_dev;
          m.bridge = e.d.bridge;
          m.Hs = sn.d.height;
          m.Ws = sn.d.width;
          m.Csp = sn.Cp;
          m.kh = e.d.kh;
          m.kw = e.d.kw;
          m.stride = e.d.stride;
          m.pad = e.d.pad;
          m.up = e.d.upsample;
          // image pitch in padded rows: a multiple of the stride, so that a row's phase does not
          // depend on the image
          m.PH = (m.Hs + 2 * m.pad + m.stride - 1) / m.stride * m.stride;
          m.PW = m.Ws + 2 * m.pad;
          m.PWs = (m.PW + m.stride - 1) / m.stride;
          m.RP = m.stride * m.PWs;
          m.wstride8 = (Cout / 32) * 64;
          if (sn.state_bytes + SR_ZERO_TAIL + (size_t)(e.d.pad + 1) * sn.d.width * sn.Cp * 2 >= ((size_t)1 << 31) ||
              (size_t)sn.Cp * 2 > SR_ZERO_TAIL) { ok = false; break; }
          m.src_bytes = (int32_t)sn.state_bytes;
          const int nphase = std::min(m.stride, m.kh);
          const int64_t rows = max_patch_rows(g, v, e, BM, m.PH);
          const int64_t rows0 = (rows + m.stride - 1) / m.stride;           // phase 0 has the most rows ...
          const int taps0 = ((m.kh + m.stride - 1) / m.stride) * m.kw;      // ... and the most taps
          int KC = 0;
          for (int cand : {128, 64, 32, 16}) {
            const int64_t a_bytes = (rows0 * m.RP * cand * 2 + 1023) / 1024 * 1024;
            const int64_t b_bytes = (int64_t)taps0 * (cand / 16) * NBT * 1024;
            if (KC == 0 && sn.Cp % cand == 0 && a_bytes + b_bytes <= SR8_BUF_BYTES) KC = cand;
          }
          if (KC == 0) { ok = false; break; }
          m.KC = KC;
          m.nchunk = sn.Cp / KC;
          m.SP = KC * 2;
          m.RPB = m.RP * KC * 2;
          m.magicKW = (int32_t)((65536 + m.kw - 1) / m.kw);
          for (int tap = 0; tap < m.kh * m.kw; ++tap)
            if (((tap * m.magicKW) >> 16) != tap / m.kw) ok = false;
          if (m.kh * m.kw > 64) ok = false;   // one tap per lane in the tap tables
          m.plan_slot = plan_slots;
          plan_slots += nphase;
          for (int ph = 0; ph < nphase; ++ph) {
            const int steps = ((m.kh - ph + m.stride - 1) / m.stride) * m.kw * (KC / 16);
            for (int ch = 0; ch < m.nchunk; ++ch) {
              stage8.push_back(SrStage8{(int)me.size(), ph, ch, 0});
              cyc += 900.0 + steps * 512.0 * wt / 2;
              n_stages += 1;
            }
          }
          me.push_back(m);
        }
        if (ok) break;
        me.resize(node.edge_begin);
        stage8.resize(node.stage0);
        }
        if (!ok) {
          me.resize(node.edge_begin);
          stage8.resize(node.stage0);
          n.kind = 2;
        } else {
          node.edge_count = (int)me.size() - node.edge_begin;
          const int node_index = (int)mn.size();
          mn.push_back(node);
          TileGroup grp;
          grp.node_index = node_index;
          grp.cost = cyc;
          grp.n_stages = n_stages;
          const int n_mt = (int)((M + BM - 1) / BM), n_nt = Cout / BN;
          for (int mi = 0; mi < n_mt; ++mi)
            for (int nt = 0; nt < n_nt; ++nt) {
              SrMfmaTile t{};
              t.node = node_index;
              t.m0 = mi * BM;
              t.n0 = nt * BN;
              t.plan_begin = (int)plan_index.size();
              t.stage_begin = 0;
              t.stage_end = n_stages;
              t.split_slot = -1;
              t.part = 1 << 16;
              for (int ei = 0; ei < node.edge_count; ++ei) {
                const SrMfmaEdge& m = me[node.edge_begin + ei];
                const PatchRows r = patch_rows(t.m0, std::min<int64_t>((int64_t)t.m0 + BM, M) - 1,
                                               n.d.height * n.d.width, n.d.width, m.PH, m.stride, m.up, m.kh);
                for (int ph = 0; ph < std::min(m.stride, m.kh); ++ph) {
                  build_plan8(&plan_tmp, m, r, ph, NBT);
                  uint64_t h = 1469598103934665603ull ^ (uint64_t)((node.edge_begin + ei) * 4 + ph);
                  for (int32_t x : plan_tmp) h = (h ^ (uint32_t)x) * 1099511628211ull;
                  int found = -1;
                  for (int cand : plan_seen[h])
                    if (plan_tables.size() >= (size_t)cand + plan_tmp.size() &&
                        std::equal(plan_tmp.begin(), plan_tmp.end(), plan_tables.begin() + cand)) { found = cand; break; }
                  if (found < 0) {
                    found = (int)plan_tables.size();
                    plan_tables.insert(plan_tables.end(), plan_tmp.begin(), plan_tmp.end());
                    plan_seen[h].push_back(found);
                  }
                  plan_index.push_back(found);
                }
              }
              grp.tiles.push_back(t);
            }
          groups.push_back(std::move(grp));
        }
      }
      if (n.kind == 1 && g->tile_version != 2) {
        // ---- MFMA node: tile shape, per-edge staging depth, tiles
        // channel tiles are 32 wide: a node whose channel count is no multiple of 32 gets zero weights and
        // zero bias for the rest of its last tile, and the epilogue stores only the pixel's Cp channels
        const int Cout = (n.d.channels + 31) / 32 * 32;
        const int64_t M = (int64_t)B * n.d.height * n.d.width;
        // tile shapes to try, preferred first: each wave owns 128 pixels x 32*wn_tiles channels, the 4
        // waves are arranged waves_m x waves_n; a narrower wave tile gives a shorter pixel tile and so a
        // smaller source patch when the preferred shape does not fit the LDS
        struct Shape { int wn_tiles, waves_n; };
        std::vector<Shape> shapes;
        for (int wt : {2, 1})
          for (int wn : {4, 2, 1})
            if (Cout % (32 * wt * wn) == 0) {
              bool dominated = false;   // same pixel tile, narrower channel tile: never better
              for (const Shape& sh : shapes) dominated |= (sh.waves_n == wn);
              if (!dominated) shapes.push_back(Shape{wt, wn});
            }
        if (!shapes.empty()) {
          // a node with fewer tiles than the chip has CUs at its preferred shape tries shorter pixel tiles of
          // the same channel width first: more, shorter tiles (measured: CIFAR-shaped frame 37 -> 29 us,
          // hi-res 160 -> 149 us; the GTSRB-shaped graph has no such node)
          const int bn0 = 32 * shapes[0].wn_tiles * shapes[0].waves_n, bm0 = 128 * (4 / shapes[0].waves_n);
          const int64_t tiles0 = (M + bm0 - 1) / bm0 * (Cout / bn0);
          if (tiles0 < SR_CUS) {
            std::vector<Shape> shorter;
            for (int wn : {4, 2})
              for (int wt : {2, 1})
                if (32 * wt * wn == bn0 && 128 * (4 / wn) < bm0) shorter.push_back(Shape{wt, wn});
            shapes.insert(shapes.begin(), shorter.begin(), shorter.end());
          }
        }
        int wn_tiles = 0, cw = 0, waves_n = 0, waves_m = 0, BM = 0, BN = 0;
        SrMfmaNode node{};
        double ksum = 0;
        bool ok = false;
        for (const Shape& sh : shapes) {
        wn_tiles = sh.wn_tiles;
        cw = 32 * wn_tiles;
        waves_n = sh.waves_n;
        waves_m = 4 / waves_n;
        BM = 128 * waves_m;
        BN = cw * waves_n;
        node = SrMfmaNode{};
        node.out[0] = n.state[0];
        node.out[1] = n.state[1];
        node.bias = n.bias_dev;
        node.M = (int)M;
        node.Ho = n.d.height;
        node.Wo = n.d.width;
        node.Cout = Cout;
        node.Cp = n.Cp;
        node.act = n.d.act;
        node.edge_begin = (int)me.size();
        node.waves_m = waves_m;
        node.waves_n = waves_n;
        node.wn_tiles = wn_tiles;
        ksum = 0;
        ok = true;
        tap_mark = tap_table.size();
        for (EdgeRt& e : g->edges) {
          if (e.d.dst != v) continue;
          const NodeRt& sn = g->nodes[e.d.src];
          SrMfmaEdge m{};
          m.src[0] = sn.state[0];
          m.src[1] = sn.state[1];
          m.wpk = e.wpk_dev;
          m.bridge = e.d.bridge;
          m.Hs = sn.d.height;
          m.Ws = sn.d.width;
          m.Csp = sn.Cp;
          m.kh = e.d.kh;
          m.kw = e.d.kw;
          m.stride = e.d.stride;
          m.pad = e.d.pad;
          m.up = e.d.upsample;
          m.PH = m.Hs + 2 * m.pad;
          m.PW = m.Ws + 2 * m.pad;
          m.PWs = (m.PW + m.stride - 1) / m.stride;
          m.wstride8 = (Cout / 32) * 64;
          // padding positions read the zero bytes behind the source state, at 32-bit offsets
          if (sn.state_bytes + SR_ZERO_TAIL + (size_t)(e.d.pad + 1) * sn.d.width * sn.Cp * 2 >= ((size_t)1 << 31) ||
              (size_t)sn.Cp * 2 > SR_ZERO_TAIL) { ok = false; break; }
          m.src_bytes = (int32_t)sn.state_bytes;
          // the kernel packs (image - first image of the tile) into the top byte of a signed int
          const int64_t imgs_per_tile = BM / ((int64_t)n.d.height * n.d.width) + 2;
          if (imgs_per_tile > 127 || m.kh * m.kw > 64) { ok = false; break; }
          // how the edge is staged: unsplit, or cut into row planes, or into row x column planes
          const EdgeStaging st = choose_staging(g, v, e, BM, lds_cap);
          if (st.KC == 0) { ok = false; break; }
          m.KC = st.KC;
          m.nchunk = sn.Cp / st.KC;
          m.SP = st.KC * 2 + 16;
          m.PC = st.PC;
          m.PRmul = st.PR;
          const int k16_total = sn.Cp / 16;
          for (const PlaneGeom& pg : edge_planes(m.kh, m.kw, m.stride, m.PH, m.PW, st.PR, st.PC)) {
            SrMfmaEdge pm = m;
            pm.pc = pg.pc;
            pm.r0 = pg.pr - m.pad;
            pm.PHr = pg.PHr;
            pm.lgRS = pg.lgRS;
            pm.ta_max = pg.ta_max;
            pm.RP = pg.RP;
            pm.ntaps = pg.ntaps;
            pm.RPB = row_pitch16(pg.RP, st.KC / 8 + 1, 1 << pg.lgRS, m.up, n.d.width) * 16;
            pm.imgB = (int32_t)((int64_t)m.Hs * m.Ws * m.Csp * 2);
            pm.rowB = (int32_t)((int64_t)st.PR * m.Ws * m.Csp * 2);
            pm.r0B = (int32_t)((int64_t)pm.r0 * m.Ws * m.Csp * 2);
            pm.tap_begin = (int32_t)tap_table.size();
            for (int t = 0; t < pg.ntaps; ++t)
              tap_table.push_back(SrTap{pg.taps[t].a * pm.RPB + pg.taps[t].b * pm.SP, pg.tap_id[t] * k16_total * pm.wstride8});
            const int64_t rows = max_plane_rows(g, v, e, BM, pg);
            g->lds_bytes = std::max<int>(g->lds_bytes, (int)((rows * pm.RPB + 1023) / 1024 * 1024));   // whole 1 KiB instructions
            me.push_back(pm);
          }
          g->lds_bytes = std::max<int>(g->lds_bytes, 4 * 64 * (32 * wn_tiles * 2 + 16));
          ksum += (double)sn.Cp * m.kh * m.kw;
        }
        if (ok) break;
        me.resize(node.edge_begin);
        tap_table.resize(tap_mark);
        }
        if (!ok) {   // patch does not fit: this node goes the direct way
          me.resize(node.edge_begin);
          tap_table.resize(tap_mark);
          n.kind = 2;
        } else {
          node.edge_count = (int)me.size() - node.edge_begin;
          const int node_index = (int)mn.size();
          mn.push_back(node);
          TileGroup grp;
          grp.node_index = node_index;
          grp.cost = ksum * BM * BN;
          const int n_mt = (int)((M + BM - 1) / BM), n_nt = Cout / BN;
          node_units[v] = n_mt * n_nt;
          mfma_graph_node.push_back(v);
          // estimated cycles of one tile: k-steps at the MFMA rate of two resident workgroups,
          // plus the staging latency of every stage and a fixed prologue/epilogue
          {
            double cyc = 8000;
            for (int ei = 0; ei < node.edge_count; ++ei) {
              const SrMfmaEdge& m = me[node.edge_begin + ei];   // one plane of an edge
              const double steps = (double)m.ntaps * (m.KC / 16);
              cyc += m.nchunk * (4500.0 + steps * 512.0 * wn_tiles / 2);
            }
            grp.cost = cyc;
          }
          int n_stages = 0;
          for (int ei = 0; ei < node.edge_count; ++ei) {
            n_stages += me[node.edge_begin + ei].nchunk;
            grp.nchunks.push_back(me[node.edge_begin + ei].nchunk);
          }
          grp.n_stages = n_stages;
          // channel tiles of one pixel tile are neighbours in the list (they share the source patch)
          for (int mi = 0; mi < n_mt; ++mi)
            for (int nt = 0; nt < n_nt; ++nt) {
                SrMfmaTile t{};
                t.node = node_index;
                t.m0 = mi * BM;
                t.n0 = nt * BN;
                t.plan_begin = (int)plan_index.size() / 4;   // in SrPlanRef records
                t.stage_begin = 0;
                t.stage_end = n_stages;
                t.split_slot = -1;
                t.part = 1 << 16;
                t.e_first = 0;
                t.c_first = 0;
                t.e_last = node.edge_count - 1;
                t.c_end = me[node.edge_begin + node.edge_count - 1].nchunk;
                for (int ei = 0; ei < node.edge_count; ++ei) {
                  const SrMfmaEdge& m = me[node.edge_begin + ei];
                  const PatchRows r = patch_rows(t.m0, std::min<int64_t>((int64_t)t.m0 + BM, M) - 1,
                                                 n.d.height * n.d.width, n.d.width, m.PHr, 1 << m.lgRS, m.up, m.ta_max + 1);
                  build_plan(&plan_tmp, m, r);
                  {   // traffic model: the plane's distinct source positions, all channel chunks; the tile's weights
                    int64_t pos = 0;
                    for (size_t i = 0; i < plan_tmp.size(); ++i)
                      pos += (plan_tmp[i] >= 0 && (i == 0 || plan_tmp[i] != plan_tmp[i - 1])) ? 1 : 0;
                    g->traffic[2] += (double)pos * 16.0 * m.nchunk;
                    g->traffic[4] += (double)m.ntaps * m.Csp * BN * 2.0;
                  }
                  uint64_t h = 1469598103934665603ull ^ (uint64_t)(node.edge_begin + ei);
                  for (int32_t x : plan_tmp) h = (h ^ (uint32_t)x) * 1099511628211ull;
                  int found = -1;
                  for (int cand : plan_seen[h])
                    if (plan_tables.size() >= (size_t)cand + plan_tmp.size() &&
                        std::equal(plan_tmp.begin(), plan_tmp.end(), plan_tables.begin() + cand)) { found = cand; break; }
                  if (found < 0) {
                    found = (int)plan_tables.size();
                    plan_tables.insert(plan_tables.end(), plan_tmp.begin(), plan_tmp.end());
                    plan_seen[h].push_back(found);
                  }
                  // SrPlanRef of this (tile, plane)
                  plan_index.push_back(found);
                  plan_index.push_back((int32_t)((r.Q1 - r.Q0 + 1) * (m.RPB / 16)));
                  plan_index.push_back(m.tap_begin);
                  plan_index.push_back(m.ntaps);
                }
                grp.tiles.push_back(t);
              }
          groups.push_back(std::move(grp));
        }
      }
      if (n.kind == 3) {
        SrHead h{};
        h.edge_begin = (int)he.size();
        int max_vec = 0, pooled_hw = 0, pooled_cin = 0;
        for (const EdgeRt& e : g->edges) {
          if (e.d.dst != v) continue;
          const NodeRt& sn = g->nodes[e.d.src];
          SrHeadEdge x{};
          x.src[0] = sn.state[0];
          x.src[1] = sn.state[1];
          x.w = e.w_dev;
          x.bridge = e.d.bridge;
          x.pooled = (e.d.kind == SR_EDGE_GAP_DENSE) ? 1 : 0;
          x.HW = sn.d.height * sn.d.width;
          x.Cin = sn.d.channels;
          x.Csp = sn.Cp;
          max_vec = std::max(max_vec, x.pooled ? x.Cin : x.HW * x.Cin);
          if (x.pooled) { pooled_hw = x.HW; pooled_cin = x.Cin; }
          he.push_back(x);
        }
        h.edge_count = (int)he.size() - h.edge_begin;
        h.out[0] = n.state[0];
        h.out[1] = n.state[1];
        h.bias = n.bias_dev;
        h.act = n.d.act;
        h.B = B;
        h.Cout = n.d.channels;
        h.Cp = n.Cp;
        // a single pooled edge over many pixels is cut into slabs of 64 pixels
        h.splits = (h.edge_count == 1 && pooled_hw > 0) ? std::max(1, std::min(64, (pooled_hw + 63) / 64)) : 1;
        h.record = 0;
        void* cnt = nullptr;
        {
          sr_status st2 = dev_alloc(g, &cnt, (size_t)B * sizeof(int32_t));
          if (st2 != SR_OK) return st2;
          SR_HIP(g, sr_launch_fill_zero(g->stream, cnt, (size_t)B * sizeof(int32_t)));
        }
        h.counters = (int32_t*)cnt;
        void* part = nullptr;
        sr_status st = dev_alloc(g, &part, (size_t)B * h.splits * std::max(pooled_cin, 1) * sizeof(float));
        if (st != SR_OK) return st;
        h.partial = (float*)part;
        for (int b = 0; b < B; ++b)
          for (int sp = 0; sp < h.splits; ++sp) level_aux.push_back(SrAux{SR_AUX_HEAD, (int)hd.size(), b, sp});
        g->head_node.push_back(v);
        hd.push_back(h);
        g->aux_smem_bytes = std::max(g->aux_smem_bytes, (int)(max_vec * sizeof(float) + 16 + 4096));
      }
      if (n.kind == 2) {
        SrDirectNode node{};
        node.out[0] = n.state[0];
        node.out[1] = n.state[1];
        node.bias = n.bias_dev;
        node.H = n.d.height;
        node.W = n.d.width;
        node.C = n.d.channels;
        node.Cp = n.Cp;
        node.act = n.d.act;
        node.edge_begin = (int)de.size();
        for (const EdgeRt& e : g->edges) {
          if (e.d.dst != v) continue;
          const NodeRt& sn = g->nodes[e.d.src];
          SrDirectEdge d{};
          d.src[0] = sn.state[0];
          d.src[1] = sn.state[1];
          d.w = e.w_dev;
          d.bridge = e.d.bridge;
          d.kind = (e.d.kind == SR_EDGE_GAP_DENSE) ? 2 : 0;
          d.Hs = sn.d.height;
          d.Ws = sn.d.width;
          d.Cin = sn.d.channels;
          d.Csp = sn.Cp;
          d.kh = e.kh;
          d.kw = e.kw;
          d.stride = (e.d.kind == SR_EDGE_CONV) ? e.d.stride : 1;
          d.pad = (e.d.kind == SR_EDGE_CONV) ? e.d.pad : 0;
          d.up = (e.d.kind == SR_EDGE_CONV) ? e.d.upsample : 1;
          de.push_back(d);
        }
        node.edge_count = (int)de.size() - node.edge_begin;
        const int node_index = (int)dn.size();
        dn.push_back(node);
        const int64_t total = (int64_t)B * node.H * node.W * node.C;
        for (int64_t first = 0; first < total; first += 256) {
          SrDirectBlock blk{node_index, (int)first};
          db.push_back(blk);
        }
      }
    }
    // Work list of the level.  Workgroups are dealt to the 8 XCDs round-robin (workgroup i runs on
    // XCD i % 8) and every XCD has an L2 of its own, so the list is built per XCD and interleaved
    // (XCD x gets positions x, x+8, ...).  XCD x works on the same eighth of the batch-pixel range of
    // every node: what one node's tiles read of a source state, the tiles of the state's other
    // consumers on that XCD read again, and every XCD gets the same mix of nodes, i.e. the same
    // amount of work.  Measured against cutting the cost-sorted list into 8 runs (one or two nodes
    // per XCD at a time): 6 % faster on the GTSRB-shaped graph, 18 % on the hi-res one.  Shorter
    // lists are padded with empty tiles (node -1).
    // K-split: when a node's tiles are long compared with an even share of the level's work (few
    // pixels, deep K) they are cut into parts by stage range, so that the launch does not end on a
    // handful of long tiles while most of the chip idles.
    {
      double level_cost = 0;
      for (const TileGroup& grp : groups) level_cost += grp.cost * grp.tiles.size();
      const double slots = (g->tile_version == 2 ? 1.0 : 2.0) * 256;   // resident workgroups of the chip
      const double share = level_cost / slots;
      for (TileGroup& grp : groups) {
        // only tiles longer than an even share of the level are cut, into parts of about 0.9 of a
        // share but not shorter than ~25 us (a part pays for its own staging and for the reduction:
        // it leaves 128 KiB of partial sums and the last one reads them all).  Measured on the hi-res
        // graph: parts of 0.5 of a share 163 us per frame, 0.65 .. 1.25 of a share 158-160, no cutting 204;
        // shorter parts than 25 us lose on every graph (CIFAR-shaped 33 -> 36 .. 49 us)
        const double part_cost = std::max(0.9 * share, 60000.0);
        int parts = (grp.cost > share) ? (int)std::ceil(grp.cost / part_cost) : 1;
        parts = std::max(1, std::min(std::min(parts, 16), grp.n_stages));
        if (parts <= 1 || !g->allow_split) continue;
        std::vector<SrMfmaTile> cut;
        for (const SrMfmaTile& t : grp.tiles) {
          const int slot = g->n_split_slots;
          g->n_split_slots += parts;
          for (int p = 0; p < parts; ++p) {
            SrMfmaTile tp = t;
            tp.stage_begin = (int)((int64_t)grp.n_stages * p / parts);
            tp.stage_end = (int)((int64_t)grp.n_stages * (p + 1) / parts);
            tp.split_slot = slot;
            tp.part = p | (parts << 16);
            if (!grp.nchunks.empty()) {   // the same range as (plane, chunk) positions
              int base = 0;
              bool first_set = false;
              for (int ei = 0; ei < (int)grp.nchunks.size(); ++ei) {
                const int lo = std::max(tp.stage_begin - base, 0), hi = std::min(tp.stage_end - base, grp.nchunks[ei]);
                if (lo < hi) {
                  if (!first_set) { tp.e_first = ei; tp.c_first = lo; first_set = true; }
                  tp.e_last = ei;
                  tp.c_end = hi;
                }
                base += grp.nchunks[ei];
              }
            }
            cut.push_back(tp);
          }
        }
        grp.tiles.swap(cut);
        grp.cost = grp.cost / parts + 4000.0;
      }
    }
    std::stable_sort(groups.begin(), groups.end(),
                     [](const TileGroup& a, const TileGroup& b) { return a.cost > b.cost; });
    {
      std::vector<std::vector<SrMfmaTile>> per_xcd(SR_XCDS);
      // XCD x takes, of every node, the tiles of the x-th eighth of the node's pixels (batch-major, so
      // of the same images or image rows for all nodes); within an XCD the longest tiles go first
      struct Keyed { double cost; SrMfmaTile t; };
      std::vector<std::vector<Keyed>> keyed(SR_XCDS);
      for (const TileGroup& grp : groups)
        for (const SrMfmaTile& t : grp.tiles) {
          const int x = (int)std::min<int64_t>(SR_XCDS - 1, (int64_t)t.m0 * SR_XCDS / mn[t.node].M);
          keyed[x].push_back(Keyed{grp.cost, t});
          g->n_mfma_tiles += 1;
        }
      for (int x = 0; x < SR_XCDS; ++x) {
        std::stable_sort(keyed[x].begin(), keyed[x].end(), [](const Keyed& a, const Keyed& b) { return a.cost > b.cost; });
        for (const Keyed& k : keyed[x]) per_xcd[x].push_back(k.t);
      }
      size_t longest = 0;
      for (const auto& v : per_xcd) longest = std::max(longest, v.size());
      SrMfmaTile none{};
      none.node = -1;
      for (size_t pos = 0; pos < longest; ++pos)
        for (int x = 0; x < SR_XCDS; ++x) mt.push_back(pos < per_xcd[x].size() ? per_xcd[x][pos] : none);
    }
    lp.n_tiles = (int)mt.size() - lp.tile_begin;
    lp.n_blocks = (int)db.size() - lp.block_begin;
    lp.n_heads = (int)hd.size() - lp.head_begin;
    lp.aux_begin = (int)aux.size();
    aux.insert(aux.end(), level_aux.begin(), level_aux.end());
    lp.n_aux = (int)level_aux.size();
  }

  sr_status st;
  // ---- dependency-driven execution: possible when every node is computed by the 4-wave tile kernel or a
  // head item.  Per node v the list of (node, work items per frame, lag): its sources (lag R(e): the
  // frame read), itself (lag 1: the previous frame's items of v are done, its K-split scratch is free)
  // and its consumers w (lag 1 over a bridging edge, 2 otherwise: the readers of the copy that v is
  // about to overwrite have finished).
  // Measured (CIFAR-shaped graph, batch 64): sequential pattern 113 -> 69 us per frame, hybrid 66 -> 49; under
  // the streaming pattern, where a frame is a single launch anyway, the waits cost more than overlapping
  // consecutive frames gains (30 -> 38 us; GTSRB-shaped 408 -> 414), so it stays one launch per frame.
  g->dataflow = (g->dataflow_option == 1 || (g->dataflow_option == 2 && F > 1)) && bf16 && g->tile_version == 1 &&
                !g->force_direct;
  for (int v = 0; v < g->n_nodes; ++v)
    if (g->nodes[v].kind == 2) g->dataflow = false;
  std::vector<SrDep> deps;
  if (g->dataflow) {
    for (size_t i = 0; i < stage.size(); ++i) node_units[g->inputs[i]] = (stage[i].elems_px + SR_STAGE_CHUNK - 1) / SR_STAGE_CHUNK;
    for (size_t i = 0; i < g->head_node.size(); ++i) node_units[g->head_node[i]] = B;
    std::vector<int> dep_begin(g->n_nodes, 0), dep_count(g->n_nodes, 0);
    for (int v = 0; v < g->n_nodes; ++v) {
      // reads first (sources and the node itself), then what the node's new state overwrites (its readers);
      // a node that is both keeps the stronger requirement among the reads
      std::vector<int> rlag(g->n_nodes, 99), wlag(g->n_nodes, 99);
      rlag[v] = 1;
      for (const EdgeRt& e : g->edges) {
        if (e.d.dst == v) rlag[e.d.src] = std::min(rlag[e.d.src], (int)e.d.bridge);
        if (e.d.src == v) wlag[e.d.dst] = std::min(wlag[e.d.dst], e.d.bridge ? 1 : 2);
      }
      dep_begin[v] = (int)deps.size();
      for (int u = 0; u < g->n_nodes; ++u)
        if (rlag[u] != 99) deps.push_back(SrDep{u, node_units[u], std::min(rlag[u], wlag[u]), 0});
      const int n_read = (int)deps.size() - dep_begin[v];
      for (int u = 0; u < g->n_nodes; ++u)
        if (wlag[u] != 99 && rlag[u] == 99) deps.push_back(SrDep{u, node_units[u], wlag[u], 0});
      const int n_write = (int)deps.size() - dep_begin[v] - n_read;
      dep_count[v] = n_read | (n_write << 8);
      if (n_read + n_write > 64) g->dataflow = false;   // one dependency per lane of the polling wave
    }
    for (size_t i = 0; i < stage.size(); ++i) {
      const int v = g->inputs[i];
      stage[i].dep_begin = dep_begin[v]; stage[i].dep_count = (dep_count[v] & 0xff) + (dep_count[v] >> 8); stage[i].gnode = v;
    }
    for (size_t i = 0; i < hd.size(); ++i) {
      const int v = g->head_node[i];
      hd[i].dep_begin = dep_begin[v]; hd[i].dep_count = (dep_count[v] & 0xff) + (dep_count[v] >> 8); hd[i].gnode = v;
    }
    g->flow_dep_begin = dep_begin;
    g->flow_dep_count = dep_count;
  }
  int flow_stage_begin = 0;
  if (g->dataflow) {   // this frame's staging items, ahead of everything else in the frame
    flow_stage_begin = (int)aux.size();
    aux.insert(aux.end(), stage_aux.begin(), stage_aux.end());
  }
  if ((st = upload(g, &g->stage_nodes, stage)) != SR_OK) return st;
  if ((st = upload(g, &g->d_nodes, dn)) != SR_OK) return st;
  if ((st = upload(g, &g->d_edges, de)) != SR_OK) return st;
  if ((st = upload(g, &g->d_blocks, db)) != SR_OK) return st;
  if ((st = upload(g, &g->plan_index, plan_index)) != SR_OK) return st;
  if ((st = upload(g, &g->plan_tables, plan_tables)) != SR_OK) return st;
  if ((st = upload(g, &g->tap_table, tap_table)) != SR_OK) return st;
  if (g->tile_version != 2) {
    std::vector<SrPlane4> p4(me.size());
    auto lg2 = [](int v) { int l = 0; while ((1 << l) < v) ++l; return l; };
    for (size_t i = 0; i < me.size(); ++i) {
      const SrMfmaEdge& m = me[i];
      SrPlane4& q = p4[i];
      q.src[0] = m.src[0];
      q.src[1] = m.src[1];
      q.wpk = m.wpk;
      q.flags = (m.bridge ? 1 : 0) | (m.lgRS << 8) | (lg2(m.up) << 16) | (lg2(m.KC / 16) << 24);
      q.nchunk = m.nchunk;
      q.PHr = m.PHr;
      q.RPB = m.RPB;
      q.imgB = m.imgB;
      q.rowB = m.rowB;
      q.r0B = m.r0B;
      q.wstride8 = m.wstride8;
      q.src_bytes = m.src_bytes;
      q.pad_ = 0;
    }
    if ((st = upload(g, &g->planes4, p4)) != SR_OK) return st;
    std::vector<SrNode4> n4(mn.size());
    for (size_t i = 0; i < mn.size(); ++i) {
      const SrMfmaNode& a = mn[i];
      SrNode4& q = n4[i];
      q = SrNode4{};
      q.out[0] = a.out[0];
      q.out[1] = a.out[1];
      q.bias = a.bias;
      q.M = a.M; q.Ho = a.Ho; q.Wo = a.Wo; q.Cp = a.Cp; q.act = a.act;
      q.waves_m = a.waves_m; q.waves_n = a.waves_n;
      q.gnode = mfma_graph_node[i];
      if (g->dataflow) {
        const int v = mfma_graph_node[i];
        q.dep_begin = g->flow_dep_begin[v]; q.dep_count = g->flow_dep_count[v];
      }
    }
    if ((st = upload(g, &g->nodes4, n4)) != SR_OK) return st;
    std::vector<SrTile4> t4(mt.size());
    for (size_t i = 0; i < mt.size(); ++i) {
      const SrMfmaTile& a = mt[i];
      SrTile4& q = t4[i];
      q = SrTile4{};
      q.node = a.node;
      if (a.node < 0) continue;
      const SrMfmaNode& nd = mn[a.node];
      const int HoWo = nd.Ho * nd.Wo, BM = 128 * nd.waves_m;
      const int m_last = std::min(a.m0 + BM, nd.M) - 1;
      const int b_first = a.m0 / HoWo, b_last = m_last / HoWo;
      q.m0 = a.m0;
      q.n0 = a.n0;
      q.ref_base = a.plan_begin - nd.edge_begin;
      q.p_first = nd.edge_begin + a.e_first;
      q.p_last = nd.edge_begin + a.e_last;
      q.chunks = a.c_first | (a.c_end << 16);
      q.split_slot = a.split_slot;
      q.part = a.part;
      q.shape = nd.wn_tiles | ((b_last - b_first) << 8);
      q.b_first = b_first;
      q.rows = ((a.m0 % HoWo) / nd.Wo) | (((m_last % HoWo) / nd.Wo) << 16);
      const int32_t* r = &plan_index[(size_t)(a.plan_begin + a.e_first) * 4];
      q.ref0 = SrPlanRef{r[0], r[1], r[2], r[3]};
    }
    if ((st = upload(g, &g->tiles4, t4)) != SR_OK) return st;
    if (g->dataflow) {
      // A frame's work items in an order in which every wait refers to an earlier item: this frame's
      // input staging, then update step by update step the tiles and the head items of the step.
      // Every run is padded to a multiple of 8 so that the tile lists keep their XCD interleaving.
      std::vector<SrTile4> items;
      SrTile4 none{};
      none.node = -1;
      std::vector<int> run_begin;   // the list is a sequence of runs: staging, then per update step its tiles and its head items
      auto pad8 = [&]() { while (items.size() % SR_XCDS) items.push_back(none); };
      auto new_run = [&]() { if (run_begin.empty() || run_begin.back() != (int)items.size()) run_begin.push_back((int)items.size()); };
      auto aux_item = [&](int index) { SrTile4 a{}; a.node = -2 - index; items.push_back(a); };
      new_run();
      for (int k = 0; k < (int)stage_aux.size(); ++k) aux_item(flow_stage_begin + k);
      pad8();
      for (int L = 1; L <= F; ++L) {
        const LevelPlan& lp = g->levels[L];
        // the step's tiles, one run per node (in the order in which the nodes first appear in the step's list:
        // costliest tiles first), every tile on the XCD the step's list gave it: position p of the list runs on XCD p % 8
        {
          std::vector<int> node_order;
          std::vector<std::vector<std::vector<SrTile4>>> lanes;   // [node slot][XCD] -> tiles
          std::vector<int> slot_of_node(mn.size(), -1);
          for (int p = 0; p < lp.n_tiles; ++p) {
            const SrTile4& q = t4[lp.tile_begin + p];
            if (q.node < 0) continue;
            if (slot_of_node[q.node] < 0) {
              slot_of_node[q.node] = (int)node_order.size();
              node_order.push_back(q.node);
              lanes.emplace_back(SR_XCDS);
            }
            lanes[slot_of_node[q.node]][p % SR_XCDS].push_back(q);
          }
          for (size_t sl = 0; sl < node_order.size(); ++sl) {
            new_run();
            size_t longest = 0;
            for (const auto& ln : lanes[sl]) longest = std::max(longest, ln.size());
            for (size_t k = 0; k < longest; ++k)
              for (int x = 0; x < SR_XCDS; ++x) items.push_back(k < lanes[sl][x].size() ? lanes[sl][x][k] : none);
          }
        }
        new_run();
        for (int k = 0; k < lp.n_aux; ++k)
          if (aux[lp.aux_begin + k].kind == SR_AUX_HEAD) aux_item(lp.aux_begin + k);
        pad8();
      }
      g->n_flow_items = (int)items.size();
      // Launches that cover several frames: their (frame, run) pairs in the order of their depth in the rollout
      // window of those frames -- a run's depth is one more than the deepest run it waits for (reads and
      // overwrites alike; what lies before the launch is complete) -- the inference tableau of Eq. 5 taken over
      // runs.  Every wait still refers to an earlier workgroup, and update steps of consecutive frames that do not
      // depend on one another are dispatched side by side instead of frame after frame.
      {
        const int n_frames = g->frames_per_graph;
        run_begin.push_back((int)items.size());
        const int n_runs = (int)run_begin.size() - 1;
        std::vector<std::vector<int>> run_nodes(n_runs);
        std::vector<int> run_of(g->n_nodes, -1);
        for (int r = 0; r < n_runs; ++r)
          for (int i = run_begin[r]; i < run_begin[r + 1]; ++i) {
            const SrTile4& q = items[i];
            int v = -1;
            if (q.node >= 0) v = mfma_graph_node[q.node];
            else if (q.node <= -2) {
              const SrAux& a = aux[-2 - q.node];
              v = (a.kind == SR_AUX_HEAD) ? g->head_node[a.a] : g->inputs[a.a];
            }
            if (v >= 0 && run_of[v] != r) { run_of[v] = r; run_nodes[r].push_back(v); }
          }
        bool ok = n_frames >= 2 && n_frames <= 255 && g->n_flow_items < (1 << 24);
        std::vector<std::vector<int>> depth(n_frames, std::vector<int>(n_runs, 0));
        for (int t = 0; ok && t < n_frames; ++t)
          for (int r = 0; ok && r < n_runs; ++r) {
            int d = 0;
            for (int v : run_nodes[r]) {
              const int cnt = (g->flow_dep_count[v] & 0xff) + (g->flow_dep_count[v] >> 8);
              for (int k = 0; k < cnt; ++k) {
                const SrDep& dp = deps[g->flow_dep_begin[v] + k];
                const int tt = t - dp.lag, rr = run_of[dp.node];
                if (tt < 0 || rr < 0) continue;
                if (dp.lag == 0 && rr >= r) { ok = false; break; }   // cannot be: same-frame sources lie in earlier runs
                d = std::max(d, depth[tt][rr] + 1);
              }
            }
            depth[t][r] = d;
          }
        if (ok) {
          struct Key { int depth, t, r; };
          std::vector<Key> keys;
          for (int t = 0; t < n_frames; ++t)
            for (int r = 0; r < n_runs; ++r) keys.push_back(Key{depth[t][r], t, r});
          std::stable_sort(keys.begin(), keys.end(), [](const Key& a, const Key& b) {
            return a.depth != b.depth ? a.depth < b.depth : (a.t != b.t ? a.t < b.t : a.r < b.r);
          });
          std::vector<int32_t> order;
          order.reserve((size_t)n_frames * items.size());
          for (const Key& k : keys)
            for (int i = run_begin[k.r]; i < run_begin[k.r + 1]; ++i) order.push_back((int32_t)(i | (k.t << 24)));
          g->n_flow_order = (int)order.size();
          g->flow_order_frames = n_frames;
          if ((st = upload(g, &g->flow_order, order)) != SR_OK) return st;
        }
      }
      if ((st = upload(g, &g->flow_items, items)) != SR_OK) return st;
      if ((st = upload(g, &g->deps, deps)) != SR_OK) return st;
      void* dc = nullptr;
      if ((st = dev_alloc(g, &dc, (size_t)g->n_nodes * SR_DONE_STRIDE * sizeof(int32_t))) != SR_OK) return st;
      g->done_counters = (int32_t*)dc;
      SR_HIP(g, sr_launch_fill_zero(g->stream, dc, (size_t)g->n_nodes * SR_DONE_STRIDE * sizeof(int32_t)));
    }
  }
  if ((st = upload(g, &g->stage8, stage8)) != SR_OK) return st;
  if (g->n_split_slots > 0) {
    // arrival counters of the K-split tiles; the slabs themselves are allocated by the first frame
    // that runs on the graph's own scratch (ensure_split_scratch)
    void* sp = nullptr;
    if ((st = dev_alloc(g, &sp, (size_t)g->n_split_slots * sizeof(int32_t))) != SR_OK) return st;
    g->split_counters = (int32_t*)sp;
    SR_HIP(g, sr_launch_fill_zero(g->stream, sp, (size_t)g->n_split_slots * sizeof(int32_t)));
  }
  for (SrMfmaNode& node : mn) {
    node.plan_index = g->plan_index;
    node.plan_tables = g->plan_tables;
    node.tap_table = g->tap_table;
    node.planes4 = g->planes4;
    node.stage_table = g->stage8;
  }
  if ((st = upload(g, &g->m_nodes, mn)) != SR_OK) return st;
  if ((st = upload(g, &g->m_edges, me)) != SR_OK) return st;
  if ((st = upload(g, &g->m_tiles, mt)) != SR_OK) return st;
  if ((st = upload(g, &g->heads, hd)) != SR_OK) return st;
  if ((st = upload(g, &g->head_edges, he)) != SR_OK) return st;
  if ((st = upload(g, &g->aux, aux)) != SR_OK) return st;
  g->heads_host = hd;
  g->lds_bytes = std::max(g->lds_bytes, g->aux_smem_bytes);

  int launches = g->stage_mode == 2 ? 1 : 0;
  for (int L = 1; L <= F; ++L) {
    const LevelPlan& lp = g->levels[L];
    const bool has_tiles = lp.n_tiles > 0, has_blocks = lp.n_blocks > 0;
    const bool aux_ride = has_tiles;   // the tile kernels take the auxiliary items along
    launches += has_tiles + (has_blocks || (!aux_ride && lp.n_aux > 0));
  }
  g->launches_per_frame = g->dataflow ? 1 : launches;
  g->finalized = true;
  return SR_OK;
}

// Enqueue the kernels of one frame.  If `times` is given, every launch is bracketed by events.
struct FrameTimer {
  std::vector<hipEvent_t> ev;
  std::vector<int> kind;
};

// The recorded node's values go out with the head item that computes them; any other recorded node
// needs a copy kernel behind the frame (and then the frame counter a launch of its own).
sr_status set_record_node(sr_graph* g, int node) {
  if (g->rec_node == node) return SR_OK;
  g->rec_node = node;
  bool changed = false;
  for (size_t i = 0; i < g->heads_host.size(); ++i) {
    const int want = (g->head_node[i] == node) ? 1 : 0;
    if (g->heads_host[i].record != want) { g->heads_host[i].record = want; changed = true; }
  }
  if (changed)
    SR_HIP(g, hipMemcpyAsync(g->heads, g->heads_host.data(), g->heads_host.size() * sizeof(SrHead),
                             hipMemcpyHostToDevice, g->stream));
  return SR_OK;
}

bool record_needs_copy(const sr_graph* g) {
  if (g->rec_node < 0) return false;
  for (int v : g->head_node)
    if (v == g->rec_node) return false;
  return true;
}

// Start of a call that computes frames: the per-call values go into the device context, and a graph
// whose input staging runs one frame ahead gets the call's first frame staged here.
sr_status begin_frames(sr_graph* g, const SrCtx& c) {
  SR_HIP(g, sr_launch_set_ctx(g->stream, g->ctx, c, 0));
  if (g->stage_mode == 1 && !g->dataflow)
    SR_HIP(g, sr_launch_aux(g->stream, g->ctx, g->aux + g->stage_aux_begin, g->n_stage_aux, g->heads, g->head_edges,
                            g->stage_nodes, g->aux_smem_bytes, g->dtype == SR_BF16, 0));
  return SR_OK;
}

size_t split_slab_bytes(const sr_graph* g) {
  return (size_t)g->n_split_slots * (g->tile_version == 2 ? SR8_SPLIT_FLOATS : SR_SPLIT_FLOATS) * sizeof(float);
}

// The graph's own K-split slabs: uncached device memory from the process-wide arena, taken by the
// first frame that needs them (a graph that only ever steps on the static scratch never does).
sr_status ensure_split_scratch(sr_graph* g) {
  if (g->n_split_slots == 0 || g->split_scratch) return SR_OK;
  void* sp = nullptr;
  SR_HIP(g, uncached_alloc(&sp, split_slab_bytes(g), &g->split_scratch_bytes));   // split_scratch_bytes: the size held
  g->split_scratch = (float*)sp;
  g->device_bytes += (int64_t)split_slab_bytes(g);
  return SR_OK;
}

// Dependency-driven graphs: `frames` frames, every update step of each, in one launch.
sr_status enqueue_flow(sr_graph* g, int frames, bool advance, SrSplitScratch split) {
  const bool by_depth = g->flow_order && frames == g->flow_order_frames && g->flow_depth_order;
  const SrFlow flow{g->deps, g->done_counters, g->dep_spin_limit, frames, by_depth ? g->flow_order : nullptr};
  SR_HIP(g, sr_launch_mfma(g->stream, g->ctx,
                           SrTables4{g->nodes4, g->planes4, (const SrPlanRef*)g->plan_index, g->plan_tables, g->tap_table},
                           flow, frames, g->n_flow_order, g->flow_items, g->n_flow_items, g->lds_bytes, g->aux, 0, g->heads, g->head_edges,
                           g->stage_nodes, g->aux_smem_bytes, advance ? 1 : 0, split));
  return SR_OK;
}

sr_status enqueue_frame(sr_graph* g, bool record, FrameTimer* ft, SrSplitScratch split) {
  hipStream_t s = g->stream;
  const int bf16 = g->dtype == SR_BF16;
  if (g->dataflow) {
    hipEvent_t e0 = nullptr, e1 = nullptr;
    if (ft) {
      SR_HIP(g, hipEventCreate(&e0));
      SR_HIP(g, hipEventCreate(&e1));
      ft->ev.push_back(e0); ft->kind.push_back(1);
      ft->ev.push_back(e1); ft->kind.push_back(-1);
      SR_HIP(g, hipEventRecord(e0, s));
    }
    const bool copy = record && record_needs_copy(g);
    sr_status st = enqueue_flow(g, 1, !copy, split);
    if (st != SR_OK) return st;
    if (copy) {
      const NodeRt& n = g->nodes[g->rec_node];
      SR_HIP(g, sr_launch_record_output(s, g->ctx, n.state[0], n.state[1], g->batch * n.d.height * n.d.width,
                                        n.d.channels, n.Cp, bf16));
      SR_HIP(g, sr_launch_tick(s, g->ctx));
    }
    if (ft) SR_HIP(g, hipEventRecord(e1, s));
    return SR_OK;
  }
  auto mark = [&](int kind) -> hipError_t {
    if (!ft) return hipSuccess;
    hipEvent_t e;
    hipError_t r = hipEventCreate(&e);
    if (r != hipSuccess) return r;
    r = hipEventRecord(e, s);
    ft->ev.push_back(e);
    ft->kind.push_back(kind);
    return r;
  };
  const bool copy_out = record && record_needs_copy(g);
  // which launch is the frame's last one (it advances the frame counter)
  int last_level = 0, last_is_direct = 0;
  for (int L = 1; L <= g->an.factor; ++L) {
    const LevelPlan& lp = g->levels[L];
    const bool has_tiles = lp.n_tiles > 0;
    const bool aux_ride = has_tiles;
    const bool direct_launch = lp.n_blocks > 0 || (!aux_ride && lp.n_aux > 0);
    if (has_tiles || direct_launch) { last_level = L; last_is_direct = direct_launch; }
  }
  if (g->stage_mode == 2) {
    SR_HIP(g, mark(0));
    SR_HIP(g, sr_launch_aux(s, g->ctx, g->aux + g->stage_aux_begin, g->n_stage_aux, g->heads, g->head_edges, g->stage_nodes,
                            g->aux_smem_bytes, bf16, 0));
  }
  for (int L = 1; L <= g->an.factor; ++L) {
    const LevelPlan& lp = g->levels[L];
    const bool has_tiles = lp.n_tiles > 0;
    const bool aux_ride = has_tiles;
    const bool direct_launch = lp.n_blocks > 0 || (!aux_ride && lp.n_aux > 0);
    if (has_tiles) {
      const int is_last = (!copy_out && L == last_level && !last_is_direct) ? 1 : 0;
      SR_HIP(g, mark(1));
      if (g->tile_version == 2)
        SR_HIP(g, sr_launch_mfma8(s, g->ctx, g->m_nodes, g->m_edges, g->m_tiles + lp.tile_begin, lp.n_tiles,
                                  g->aux + lp.aux_begin, lp.n_aux, g->heads, g->head_edges, g->stage_nodes,
                                  g->aux_smem_bytes, is_last, split));
      else
        SR_HIP(g, sr_launch_mfma(s, g->ctx,
                                 SrTables4{g->nodes4, g->planes4, (const SrPlanRef*)g->plan_index, g->plan_tables, g->tap_table},
                                 SrFlow{nullptr, nullptr, 0, 0, nullptr}, 1, 0, g->tiles4 + lp.tile_begin, lp.n_tiles, g->lds_bytes,
                                 g->aux + lp.aux_begin, lp.n_aux, g->heads, g->head_edges, g->stage_nodes,
                                 g->aux_smem_bytes, is_last, split));
    }
    if (direct_launch) {
      const int is_last = (!copy_out && L == last_level) ? 1 : 0;
      const int n_aux = aux_ride ? 0 : lp.n_aux;   // aux items already went with the tiles
      SR_HIP(g, mark(2));
      if (lp.n_blocks == 0)   // auxiliary items only
        SR_HIP(g, sr_launch_aux(s, g->ctx, g->aux + lp.aux_begin, n_aux, g->heads, g->head_edges, g->stage_nodes,
                                g->aux_smem_bytes, bf16, is_last));
      else
        SR_HIP(g, sr_launch_direct(s, g->ctx, g->d_nodes, g->d_edges, g->d_blocks + lp.block_begin, lp.n_blocks, bf16,
                                   g->batch, g->aux + lp.aux_begin, n_aux, g->heads, g->head_edges, g->stage_nodes,
                                   g->aux_smem_bytes, is_last));
    }
  }
  if (copy_out) {
    SR_HIP(g, mark(4));
    const NodeRt& n = g->nodes[g->rec_node];
    SR_HIP(g, sr_launch_record_output(s, g->ctx, n.state[0], n.state[1], g->batch * n.d.height * n.d.width,
                                      n.d.channels, n.Cp, bf16));
    SR_HIP(g, sr_launch_tick(s, g->ctx));
  }
  SR_HIP(g, mark(-1));
  return SR_OK;
}

void drop_graphs(sr_graph* g) {
  if (g->exec1) hipGraphExecDestroy(g->exec1);
  if (g->execN) hipGraphExecDestroy(g->execN);
  if (g->graph1) hipGraphDestroy(g->graph1);
  if (g->graphN) hipGraphDestroy(g->graphN);
  g->exec1 = g->execN = nullptr;
  g->graph1 = g->graphN = nullptr;
  g->graph_rec_node = -2;
}

sr_status capture(sr_graph* g, int frames, hipGraph_t* graph, hipGraphExec_t* exec) {
  SR_HIP(g, hipStreamBeginCapture(g->stream, hipStreamCaptureModeThreadLocal));
  sr_status st = SR_OK;
  const SrSplitScratch own{g->split_scratch, g->split_counters};
  if (g->dataflow && !record_needs_copy(g))
    st = enqueue_flow(g, frames, true, own);   // all the frames in one launch
  else
    for (int f = 0; f < frames && st == SR_OK; ++f) st = enqueue_frame(g, true, nullptr, own);
  hipError_t e = hipStreamEndCapture(g->stream, graph);
  if (st != SR_OK) return st;
  SR_HIP(g, e);
  SR_HIP(g, hipGraphInstantiate(exec, *graph, nullptr, nullptr, 0));
  return SR_OK;
}

sr_status ensure_graphs(sr_graph* g) {
  if (g->exec1 && g->graph_rec_node == g->rec_node) return SR_OK;
  drop_graphs(g);
  sr_status st = capture(g, 1, &g->graph1, &g->exec1);
  if (st != SR_OK) return st;
  if (g->frames_per_graph > 1) {
    st = capture(g, g->frames_per_graph, &g->graphN, &g->execN);
    if (st != SR_OK) return st;
  }
  g->graph_rec_node = g->rec_node;
  return SR_OK;
}

sr_status run_frames(sr_graph* g, int64_t frames) {
  {
    sr_status st = ensure_split_scratch(g);
    if (st != SR_OK) return st;
  }
  if (!g->use_hipgraph) {
    const SrSplitScratch own{g->split_scratch, g->split_counters};
    if (g->dataflow && !record_needs_copy(g)) {
      for (int64_t left = frames; left > 0;) {
        const int n = (int)std::min<int64_t>(left, g->frames_per_graph);
        sr_status st = enqueue_flow(g, n, true, own);
        if (st != SR_OK) return st;
        left -= n;
      }
    } else {
      for (int64_t f = 0; f < frames; ++f) {
        sr_status st = enqueue_frame(g, true, nullptr, own);
        if (st != SR_OK) return st;
      }
    }
  } else {
    sr_status st = ensure_graphs(g);
    if (st != SR_OK) return st;
    int64_t left = frames;
    while (g->execN && left >= g->frames_per_graph) {
      SR_HIP(g, hipGraphLaunch(g->execN, g->stream));
      left -= g->frames_per_graph;
    }
    for (; left > 0; --left) SR_HIP(g, hipGraphLaunch(g->exec1, g->stream));
  }
  g->host_frame += frames;
  return SR_OK;
}

sr_status do_reset(sr_graph* g, const void* const* input_frame0) {
  sr_status st = finalize(g);
  if (st != SR_OK) return st;
  const int bf16 = g->dtype == SR_BF16;
  for (int v = 0; v < g->n_nodes; ++v) {
    NodeRt& n = g->nodes[v];
    int slot = n.input_slot;
    const void* src = (slot >= 0 && input_frame0) ? input_frame0[slot] : nullptr;
    if (src)
      SR_HIP(g, sr_launch_pack(g->stream, n.state[0], src, g->batch * n.d.height * n.d.width, n.d.channels, n.Cp, bf16, 0));
    else
      SR_HIP(g, sr_launch_fill_zero(g->stream, n.state[0], n.state_bytes));
  }
  if (g->done_counters)   // frames are counted from the reset: so are the nodes' completed work items
    SR_HIP(g, sr_launch_fill_zero(g->stream, g->done_counters, (size_t)g->n_nodes * SR_DONE_STRIDE * sizeof(int32_t)));
  SrCtx c{};
  c.frame = 1;
  SR_HIP(g, sr_launch_set_ctx(g->stream, g->ctx, c, 1));
  g->host_frame = 0;
  g->was_reset = true;
  return SR_OK;
}

}  // namespace

// ---------------------------------------------------------------------------
// C ABI
// ---------------------------------------------------------------------------
extern "C" {

const char* sr_status_str(sr_status s) {
  switch (s) {
    case SR_OK: return "SR_OK";
    case SR_ERR_ARG: return "SR_ERR_ARG";
    case SR_ERR_GRAPH: return "SR_ERR_GRAPH";
    case SR_ERR_ROLLOUT: return "SR_ERR_ROLLOUT";
    case SR_ERR_SHAPE: return "SR_ERR_SHAPE";
    case SR_ERR_STATE: return "SR_ERR_STATE";
    case SR_ERR_OOM: return "SR_ERR_OOM";
    case SR_ERR_DEVICE: return "SR_ERR_DEVICE";
  }
  return "SR_ERR_?";
}

const char* sr_last_error(const sr_graph* g) { return g ? g->err.c_str() : g_last_error.c_str(); }

sr_status sr_analyze(int32_t n_nodes, const sr_edge_desc* edges, int32_t n_edges, int32_t* levels,
                     int32_t* inference_factor) {
  std::vector<int> is_input;
  std::string err;
  sr_status st = check_network(n_nodes, edges, n_edges, &is_input, &err);
  if (st != SR_OK) return st;
  std::vector<uint8_t> bits(n_edges);
  for (int e = 0; e < n_edges; ++e) bits[e] = edges[e].bridge;
  Analysis an;
  st = analyse_pattern(n_nodes, edges, n_edges, bits.data(), is_input, &an, &err);
  if (st != SR_OK) return st;
  if (levels)
    for (int v = 0; v < n_nodes; ++v) levels[v] = an.level[v];
  if (inference_factor) *inference_factor = an.factor;
  return SR_OK;
}

sr_status sr_count_valid_patterns(int32_t n_nodes, const sr_edge_desc* edges, int32_t n_edges, uint64_t* count) {
  if (!count) return fail(nullptr, SR_ERR_ARG, "count is null");
  std::vector<int> is_input;
  sr_status st = check_network(n_nodes, edges, n_edges, &is_input, nullptr);
  if (st != SR_OK) return st;
  if (n_edges > 24) return fail(nullptr, SR_ERR_ARG, "enumeration is limited to 24 edges");
  uint64_t valid = 0;
  std::vector<uint8_t> bits(n_edges);
  Analysis an;
  for (uint64_t mask = 0; mask < ((uint64_t)1 << n_edges); ++mask) {
    for (int e = 0; e < n_edges; ++e) bits[e] = (uint8_t)((mask >> e) & 1);
    if (analyse_pattern(n_nodes, edges, n_edges, bits.data(), is_input, &an, nullptr) == SR_OK) ++valid;
  }
  *count = valid;
  return SR_OK;
}

sr_status sr_tableau(int32_t n_nodes, const sr_edge_desc* edges, int32_t n_edges, int32_t W, int32_t* tableau) {
  if (!tableau || W < 1) return fail(nullptr, SR_ERR_ARG, "tableau is null or W < 1");
  std::vector<int> is_input;
  sr_status st = check_network(n_nodes, edges, n_edges, &is_input, nullptr);
  if (st != SR_OK) return st;
  std::vector<uint8_t> bits(n_edges);
  for (int e = 0; e < n_edges; ++e) bits[e] = edges[e].bridge;
  Analysis an;
  st = analyse_pattern(n_nodes, edges, n_edges, bits.data(), is_input, &an, nullptr);
  if (st != SR_OK) return st;
  // nodes of one frame in an order in which every R = 0 edge points forward: by their level in the
  // size-1 window (an R = 0 edge raises the level by at least one)
  std::vector<int> order(n_nodes);
  for (int v = 0; v < n_nodes; ++v) order[v] = v;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return an.level[a] < an.level[b]; });
  // frame 0 is given: no path may start with an edge into it, so its values are 0; in a later frame
  // the longest path into (i, v) extends the longest path into the source of one of v's edges, in
  // frame i (R = 0) or i - 1 (R = 1)
  for (int v = 0; v < n_nodes; ++v) tableau[v] = 0;
  for (int i = 1; i <= W; ++i) {
    int32_t* row = tableau + (size_t)i * n_nodes;
    const int32_t* prev = row - n_nodes;
    for (int v = 0; v < n_nodes; ++v) row[v] = 0;
    for (int v : order)
      for (int e = 0; e < n_edges; ++e) {
        if (edges[e].dst != v) continue;
        const int32_t from = bits[e] ? prev[edges[e].src] : row[edges[e].src];
        row[v] = std::max(row[v], from + 1);
      }
  }
  return SR_OK;
}

sr_status sr_equally_model_parallel(int32_t n_nodes, const sr_edge_desc* edges, int32_t n_edges,
                                    const uint8_t* bridge_a, const uint8_t* bridge_b, int32_t* equal) {
  if (!bridge_a || !bridge_b || !equal) return fail(nullptr, SR_ERR_ARG, "null argument");
  std::vector<int> is_input;
  sr_status st = check_network(n_nodes, edges, n_edges, &is_input, nullptr);
  if (st != SR_OK) return st;
  int same = 1;
  for (int e = 0; e < n_edges; ++e) {
    if (bridge_a[e] > 1 || bridge_b[e] > 1) return fail(nullptr, SR_ERR_ARG, "R(e) must be 0 or 1");
    if (!is_input[edges[e].src] && bridge_a[e] != bridge_b[e]) same = 0;
  }
  *equal = same;
  return SR_OK;
}

namespace {
// minimal (simple) cycles as bit masks over the edges; a cycle is found from its smallest node
void cycles_from(int start, int node, uint32_t path, uint32_t seen_nodes_lo, std::vector<char>& seen, int n_edges,
                 const sr_edge_desc* edges, std::vector<uint32_t>* out) {
  (void)seen_nodes_lo;
  for (int e = 0; e < n_edges; ++e) {
    if (edges[e].src != node) continue;
    const int t = edges[e].dst;
    if (t == start) {
      out->push_back(path | (1u << e));
    } else if (t > start && !seen[t]) {
      seen[t] = 1;
      cycles_from(start, t, path | (1u << e), 0, seen, n_edges, edges, out);
      seen[t] = 0;
    }
  }
}

uint64_t best_disjoint_product(const std::vector<uint32_t>& cycles, size_t i, uint32_t used) {
  if (i == cycles.size()) return 1;
  uint64_t best = best_disjoint_product(cycles, i + 1, used);   // without cycle i
  if ((cycles[i] & used) == 0) {
    const int len = __builtin_popcount(cycles[i]);
    best = std::max(best, (((uint64_t)1 << len) - 1) * best_disjoint_product(cycles, i + 1, used | cycles[i]));
  }
  return best;
}
}  // namespace

sr_status sr_pattern_count_bounds(int32_t n_nodes, const sr_edge_desc* edges, int32_t n_edges,
                                  uint64_t* lower_forward, uint64_t* lower_cycles, uint64_t* upper) {
  std::vector<int> is_input;
  sr_status st = check_network(n_nodes, edges, n_edges, &is_input, nullptr);
  if (st != SR_OK) return st;
  if (n_edges > 24) return fail(nullptr, SR_ERR_ARG, "the bounds are computed exhaustively: at most 24 edges");
  std::vector<uint32_t> cycles;
  std::vector<char> seen(n_nodes, 0);
  for (int v = 0; v < n_nodes; ++v) {
    seen[v] = 1;
    cycles_from(v, v, 0, 0, seen, n_edges, edges, &cycles);
    seen[v] = 0;
    if (cycles.size() > 20) return fail(nullptr, SR_ERR_ARG, "more than 20 minimal cycles");
  }
  uint32_t on_cycle = 0;
  for (uint32_t c : cycles) on_cycle |= c;
  int n_rec = 0;
  for (int e = 0; e < n_edges; ++e) n_rec += edges[e].src == edges[e].dst;
  if (lower_forward) *lower_forward = (uint64_t)1 << (n_edges - __builtin_popcount(on_cycle));
  if (lower_cycles) *lower_cycles = best_disjoint_product(cycles, 0, 0);
  if (upper) *upper = (uint64_t)1 << (n_edges - n_rec);
  return SR_OK;
}

sr_status sr_graph_create(const sr_node_desc* nodes, int32_t n_nodes, const sr_edge_desc* edges, int32_t n_edges,
                          int32_t batch, sr_dtype dtype, void* hip_stream, sr_graph** out) {
  if (!out || !nodes || n_nodes <= 0 || batch <= 0 || (dtype != SR_F32 && dtype != SR_BF16))
    return fail(nullptr, SR_ERR_ARG, "bad argument to sr_graph_create");
  for (int v = 0; v < n_nodes; ++v) {
    if (nodes[v].channels <= 0 || nodes[v].height <= 0 || nodes[v].width <= 0 ||
        (nodes[v].act != SR_ACT_IDENTITY && nodes[v].act != SR_ACT_RELU))
      return fail(nullptr, SR_ERR_ARG, "node " + std::to_string(v) + ": bad shape or activation");
  }
  std::vector<int> is_input;
  std::string err;
  sr_status st = check_network(n_nodes, edges, n_edges, &is_input, &err);
  if (st != SR_OK) return st;
  for (int e = 0; e < n_edges; ++e) {
    const sr_edge_desc& d = edges[e];
    if (d.kind != SR_EDGE_CONV && d.kind != SR_EDGE_DENSE && d.kind != SR_EDGE_GAP_DENSE)
      return fail(nullptr, SR_ERR_ARG, "edge " + std::to_string(e) + ": unknown kind");
    if (d.kind == SR_EDGE_CONV && (d.kh <= 0 || d.kw <= 0 || d.stride <= 0 || d.pad < 0 || d.upsample <= 0))
      return fail(nullptr, SR_ERR_ARG, "edge " + std::to_string(e) + ": bad convolution geometry");
  }
  std::vector<uint8_t> bits(n_edges);
  for (int e = 0; e < n_edges; ++e) bits[e] = edges[e].bridge;
  Analysis an;
  st = analyse_pattern(n_nodes, edges, n_edges, bits.data(), is_input, &an, &err);
  if (st != SR_OK) return st;

  sr_graph* g = new (std::nothrow) sr_graph();
  if (!g) return fail(nullptr, SR_ERR_OOM, "out of host memory");
  g->n_nodes = n_nodes;
  g->n_edges = n_edges;
  g->batch = batch;
  g->dtype = dtype;
  g->stream = (hipStream_t)hip_stream;
  if (!hip_stream) g->use_hipgraph = false;   // the legacy default stream cannot be captured
  g->an = an;
  g->nodes.resize(n_nodes);
  g->edges.resize(n_edges);
  for (int v = 0; v < n_nodes; ++v) {
    NodeRt& n = g->nodes[v];
    n.d = nodes[v];
    n.Cp = (dtype == SR_BF16) ? ((n.d.channels + 15) / 16) * 16 : n.d.channels;
    n.state_bytes = (size_t)batch * n.d.height * n.d.width * n.Cp * elem_size(g);
    n.bias.assign((n.d.channels + 31) / 32 * 32, 0.f);   // as long as whole 32-channel tiles
    if (is_input[v]) {
      n.input_slot = (int)g->inputs.size();
      g->inputs.push_back(v);
    }
  }
  if ((int)g->inputs.size() > SR_MAX_INPUTS) {
    delete g;
    return fail(nullptr, SR_ERR_ARG, "more than 16 input nodes");
  }
  // shapes (App. A1.2: results of incoming transformations must be summable)
  for (int e = 0; e < n_edges; ++e) {
    EdgeRt& er = g->edges[e];
    er.d = edges[e];
    const sr_node_desc& s = g->nodes[er.d.src].d;
    const sr_node_desc& d = g->nodes[er.d.dst].d;
    if (er.d.kind == SR_EDGE_CONV) { er.kh = er.d.kh; er.kw = er.d.kw; }
    else if (er.d.kind == SR_EDGE_DENSE) { er.kh = s.height; er.kw = s.width; }
    else { er.kh = 1; er.kw = 1; }
    er.w_count = (size_t)er.kh * er.kw * s.channels * d.channels;
    int h, w;
    edge_result_shape(g, er, &h, &w);
    if (h != d.height || w != d.width) {
      std::string msg = "edge " + std::to_string(e) + ": result " + std::to_string(h) + "x" + std::to_string(w) +
                        " does not match node " + std::to_string(er.d.dst) + " (" + std::to_string(d.height) + "x" +
                        std::to_string(d.width) + ")";
      delete g;
      return fail(nullptr, SR_ERR_SHAPE, msg);
    }
  }
  // device memory
  auto bail = [&](sr_status s2) {
    std::string m = g->err;
    sr_graph_destroy(g);
    g_last_error = m;
    return s2;
  };
  for (int v = 0; v < n_nodes; ++v) {
    NodeRt& n = g->nodes[v];
    for (int p = 0; p < 2; ++p) {
      // a zero tail follows every copy (the tile kernels' direct-to-LDS loads read padding pixels from there)
      if ((st = dev_alloc(g, &n.state[p], n.state_bytes + SR_ZERO_TAIL)) != SR_OK) return bail(st);
      hipError_t he = sr_launch_fill_zero(g->stream, n.state[p], n.state_bytes + SR_ZERO_TAIL);
      if (he != hipSuccess) { g->err = hipGetErrorString(he); return bail(SR_ERR_DEVICE); }
    }
    void* b = nullptr;
    if ((st = dev_alloc(g, &b, n.bias.size() * sizeof(float))) != SR_OK) return bail(st);
    n.bias_dev = (float*)b;
    hipError_t he = sr_launch_fill_zero(g->stream, b, n.bias.size() * sizeof(float));
    if (he != hipSuccess) { g->err = hipGetErrorString(he); return bail(SR_ERR_DEVICE); }
  }
  void* c = nullptr;
  if ((st = dev_alloc(g, &c, sizeof(SrCtx))) != SR_OK) return bail(st);
  g->ctx = (SrCtx*)c;
  {
    hipError_t he = sr_launch_fill_zero(g->stream, c, sizeof(SrCtx));
    if (he == hipSuccess) he = hipStreamSynchronize(g->stream);
    if (he != hipSuccess) { g->err = hipGetErrorString(he); return bail(SR_ERR_DEVICE); }
  }
  *out = g;
  return SR_OK;
}

sr_status sr_graph_set_weights(sr_graph* g, int32_t edge, const float* host_w, size_t count) {
  if (!g || !host_w || edge < 0 || edge >= g->n_edges) return gfail(g, SR_ERR_ARG, "bad argument to sr_graph_set_weights");
  EdgeRt& e = g->edges[edge];
  if (count != e.w_count)
    return gfail(g, SR_ERR_ARG, "edge " + std::to_string(edge) + ": expected " + std::to_string(e.w_count) + " weights");
  const bool bf16 = g->dtype == SR_BF16;
  e.w_host.assign(host_w, host_w + count);
  if (bf16)
    for (float& x : e.w_host) x = bf2f(f2bf(x));
  if (!e.w_dev) {
    void* p = nullptr;
    sr_status st = dev_alloc(g, &p, count * sizeof(float));
    if (st != SR_OK) return st;
    e.w_dev = (float*)p;
  }
  // frames still in flight on the graph's stream read the old weights: let them finish first
  SR_HIP(g, hipStreamSynchronize(g->stream));
  SR_HIP(g, hipMemcpy(e.w_dev, e.w_host.data(), count * sizeof(float), hipMemcpyHostToDevice));
  if (bf16 && e.d.kind == SR_EDGE_CONV) {
    // B operand of the tile kernel: [tap][Cin_p/16][Cout/32][lane 0..63][8]; lane l of a
    // (tap, k16 block, channel tile) holds channel tile*32 + l%32 and input channels
    // block*16 + (l/32)*8 + 0..7
    const int Cin = g->nodes[e.d.src].d.channels, Cinp = g->nodes[e.d.src].Cp;
    const int Cout = g->nodes[e.d.dst].d.channels;
    const int taps = e.kh * e.kw, kb = Cinp / 16, nt = (Cout + 31) / 32;   // the last tile's spare columns stay zero
    std::vector<uint16_t> pk((size_t)taps * kb * nt * 512, 0);
    for (int t = 0; t < taps; ++t)
      for (int k = 0; k < kb; ++k)
        for (int n = 0; n < nt; ++n)
          for (int l = 0; l < 64; ++l)
            for (int i = 0; i < 8; ++i) {
              const int ci = k * 16 + (l / 32) * 8 + i, co = n * 32 + (l % 32);
              if (ci < Cin && co < Cout)
                pk[((((size_t)t * kb + k) * nt + n) * 64 + l) * 8 + i] = f2bf(host_w[((size_t)t * Cin + ci) * Cout + co]);
            }
    if (!e.wpk_dev) {
      sr_status st = dev_alloc(g, &e.wpk_dev, pk.size() * 2);
      if (st != SR_OK) return st;
    }
    SR_HIP(g, hipMemcpy(e.wpk_dev, pk.data(), pk.size() * 2, hipMemcpyHostToDevice));
  }
  e.has_w = true;
  return SR_OK;
}

sr_status sr_graph_set_bias(sr_graph* g, int32_t node, const float* host_b, size_t count) {
  if (!g || !host_b || node < 0 || node >= g->n_nodes) return gfail(g, SR_ERR_ARG, "bad argument to sr_graph_set_bias");
  NodeRt& n = g->nodes[node];
  if (count != (size_t)n.d.channels) return gfail(g, SR_ERR_ARG, "bias length differs from the node's channels");
  std::copy(host_b, host_b + count, n.bias.begin());
  SR_HIP(g, hipStreamSynchronize(g->stream));   // frames in flight read the old bias
  SR_HIP(g, hipMemcpy(n.bias_dev, n.bias.data(), n.bias.size() * sizeof(float), hipMemcpyHostToDevice));
  return SR_OK;
}

sr_status sr_graph_configure(sr_graph* g, int32_t option, int64_t value) {
  if (!g) return fail(nullptr, SR_ERR_ARG, "null graph");
  if (g->finalized) return gfail(g, SR_ERR_STATE, "options must be set before the first sr_reset");
  switch (option) {
    case SR_OPT_USE_HIPGRAPH: g->use_hipgraph = value != 0; return SR_OK;
    case SR_OPT_FORCE_DIRECT: g->force_direct = value != 0; return SR_OK;
    case SR_OPT_K_SPLIT: g->allow_split = value != 0; return SR_OK;
    case SR_OPT_DATAFLOW:
      if (value < 0 || value > 2) return gfail(g, SR_ERR_ARG, "dependency-driven execution: 0 (off), 1 (on) or 2 (default)");
      g->dataflow_option = (int)value;
      return SR_OK;
    case SR_OPT_FLOW_ORDER:
      g->flow_depth_order = value != 0;
      return SR_OK;
    case SR_OPT_TRAIN_TALL_TILES_FROM:
      if (value < 0 || value > (1 << 30)) return gfail(g, SR_ERR_ARG, "tall-tile threshold must be in 0..2^30");
      g->train_tall_from = (int)value;
      return SR_OK;
    case SR_OPT_DEP_SPIN_LIMIT:
      if (value < 0 || value > (1 << 24)) return gfail(g, SR_ERR_ARG, "spin limit of dependency waits must be in 0..2^24");
      g->dep_spin_limit = (int)value;
      return SR_OK;
    case SR_OPT_TILE_KERNEL:
      if (value < 0 || value > 2) return gfail(g, SR_ERR_ARG, "tile kernel must be 0 (choose), 1 or 2");
      g->tile_version = (int)value;
      return SR_OK;
    case SR_OPT_FRAMES_PER_GRAPH:
      if (value < 1 || value > 1024) return gfail(g, SR_ERR_ARG, "frames per graph must be in 1..1024");
      g->frames_per_graph = (int)value;
      return SR_OK;
  }
  return gfail(g, SR_ERR_ARG, "unknown option");
}

sr_status sr_graph_info(const sr_graph* g, int32_t* inference_factor, int32_t* levels, int32_t* launches_per_frame) {
  if (!g) return fail(nullptr, SR_ERR_ARG, "null graph");
  if (inference_factor) *inference_factor = g->an.factor;
  if (levels)
    for (int v = 0; v < g->n_nodes; ++v) levels[v] = g->an.level[v];
  if (launches_per_frame) {
    sr_status st = finalize(const_cast<sr_graph*>(g));
    if (st != SR_OK) return st;
    *launches_per_frame = g->launches_per_frame;
  }
  return SR_OK;
}

sr_status sr_reset(sr_graph* g, const void* const* input_frame0) {
  if (!g) return fail(nullptr, SR_ERR_ARG, "null graph");
  return do_reset(g, input_frame0);
}

sr_status sr_frame_step(sr_graph* g, const void* const* inputs_t) {
  if (!g || !inputs_t) return gfail(g, SR_ERR_ARG, "bad argument to sr_frame_step");
  if (!g->was_reset) return gfail(g, SR_ERR_STATE, "sr_frame_step before sr_reset");
  SrCtx c{};
  for (size_t i = 0; i < g->inputs.size(); ++i) {
    if (!inputs_t[i]) return gfail(g, SR_ERR_ARG, "input " + std::to_string(i) + " is null");
    c.in_ptr[i] = inputs_t[i];
    c.in_stride[i] = 0;
  }
  c.out_ptr = nullptr;
  c.in_last = (int32_t)(g->host_frame + 1);   // the frame computed now is the last one with input
  {
    sr_status st = begin_frames(g, c);
    if (st != SR_OK) return st;
  }
  return run_frames(g, 1);
}

sr_status sr_frame_step_static(sr_graph* g, const void* const* inputs_t) {
  if (!g || !inputs_t) return gfail(g, SR_ERR_ARG, "bad argument to sr_frame_step_static");
  if (!g->finalized || !g->was_reset)
    return gfail(g, SR_ERR_STATE, "sr_frame_step_static before sr_reset (which plans the graph and allocates its tables)");
  const size_t slabs = split_slab_bytes(g);
  const size_t counters = (size_t)SR_STATIC_MAX_SLOTS * sizeof(int32_t);
  if (g->n_split_slots > SR_STATIC_MAX_SLOTS || counters + slabs > SR_STATIC_SCRATCH_BYTES)
    return gfail(g, SR_ERR_ARG, "sr_frame_step_static: this graph's K-split tiles need " + std::to_string(g->n_split_slots) +
                                    " slots and " + std::to_string(slabs) + " bytes of partial sums; the static scratch holds " +
                                    std::to_string(SR_STATIC_MAX_SLOTS) + " slots and " +
                                    std::to_string(SR_STATIC_SCRATCH_BYTES - counters) + " bytes");
  SrCtx c{};
  for (size_t i = 0; i < g->inputs.size(); ++i) {
    if (!inputs_t[i]) return gfail(g, SR_ERR_ARG, "input " + std::to_string(i) + " is null");
    c.in_ptr[i] = inputs_t[i];
    c.in_stride[i] = 0;
  }
  c.out_ptr = nullptr;
  c.in_last = (int32_t)(g->host_frame + 1);
  SrSplitScratch split{nullptr, nullptr};
  if (g->n_split_slots > 0) {
    void* base = nullptr;
    SR_HIP(g, sr_static_scratch(&base));
    split.counters = (int32_t*)base;
    split.slabs = (float*)((unsigned char*)base + counters);
    // the array keeps what the last call (of any graph) left: the counters must start at zero
    // (a fill kernel, not a memset: the caller may be capturing the stream)
    SR_HIP(g, sr_launch_fill_zero(g->stream, split.counters, (size_t)g->n_split_slots * sizeof(int32_t)));
  }
  sr_status st = begin_frames(g, c);
  if (st != SR_OK) return st;
  st = enqueue_frame(g, true, nullptr, split);   // plain launches: nothing is captured or instantiated
  if (st != SR_OK) return st;
  g->host_frame += 1;
  return SR_OK;
}

sr_status sr_rollout(sr_graph* g, const void* const* inputs, int32_t T, int32_t out_node, void* outputs) {
  if (!g || !inputs || T < 0) return gfail(g, SR_ERR_ARG, "bad argument to sr_rollout");
  if (outputs && (out_node < 0 || out_node >= g->n_nodes)) return gfail(g, SR_ERR_ARG, "bad out_node");
  const void* frame0[SR_MAX_INPUTS] = {nullptr};
  for (size_t i = 0; i < g->inputs.size(); ++i) {
    if (!inputs[i]) return gfail(g, SR_ERR_ARG, "input " + std::to_string(i) + " is null");
    frame0[i] = inputs[i];
  }
  sr_status st = do_reset(g, frame0);
  if (st != SR_OK) return st;
  SrCtx c{};
  for (size_t i = 0; i < g->inputs.size(); ++i) {
    const sr_node_desc& d = g->nodes[g->inputs[i]].d;
    c.in_ptr[i] = inputs[i];
    c.in_stride[i] = (int64_t)g->batch * d.height * d.width * d.channels * (int64_t)elem_size(g);
  }
  c.in_base = 0;    // frame t reads inputs[t]
  c.in_last = T;
  c.out_base = 1;   // frame t is recorded in slot t-1
  {
    sr_status st2 = set_record_node(g, outputs ? out_node : -1);
    if (st2 != SR_OK) return st2;
  }
  if (outputs) {
    const sr_node_desc& d = g->nodes[out_node].d;
    c.out_ptr = outputs;
    c.out_stride = (int64_t)g->batch * d.height * d.width * d.channels * (int64_t)elem_size(g);
  }
  st = begin_frames(g, c);
  if (st != SR_OK) return st;
  return run_frames(g, T);
}

sr_status sr_get_state(const sr_graph* g, int32_t node, void* dst_device, size_t bytes) {
  if (!g || !dst_device || node < 0 || node >= g->n_nodes) return fail(nullptr, SR_ERR_ARG, "bad argument to sr_get_state");
  sr_graph* gm = const_cast<sr_graph*>(g);
  const NodeRt& n = g->nodes[node];
  const size_t want = (size_t)g->batch * n.d.height * n.d.width * n.d.channels * elem_size(g);
  if (bytes != want) return gfail(gm, SR_ERR_ARG, "sr_get_state: expected " + std::to_string(want) + " bytes");
  SR_HIP(gm, sr_launch_pack(g->stream, dst_device, n.state[g->host_frame & 1], g->batch * n.d.height * n.d.width,
                            n.d.channels, n.Cp, g->dtype == SR_BF16, 1));
  return SR_OK;
}

sr_status sr_set_state(sr_graph* g, int32_t node, const void* src_device, size_t bytes) {
  if (!g || !src_device || node < 0 || node >= g->n_nodes) return gfail(g, SR_ERR_ARG, "bad argument to sr_set_state");
  const NodeRt& n = g->nodes[node];
  const size_t want = (size_t)g->batch * n.d.height * n.d.width * n.d.channels * elem_size(g);
  if (bytes != want) return gfail(g, SR_ERR_ARG, "sr_set_state: expected " + std::to_string(want) + " bytes");
  SR_HIP(g, sr_launch_pack(g->stream, n.state[g->host_frame & 1], src_device, g->batch * n.d.height * n.d.width,
                           n.d.channels, n.Cp, g->dtype == SR_BF16, 0));
  return SR_OK;
}

sr_status sr_frame_index(const sr_graph* g, int64_t* frame) {
  if (!g || !frame) return fail(nullptr, SR_ERR_ARG, "bad argument to sr_frame_index");
  *frame = g->host_frame;
  return SR_OK;
}

sr_status sr_frame_step_timed(sr_graph* g, const void* const* inputs_t, float* kernel_ms, int32_t* kernel_kind,
                              int32_t cap, int32_t* n_launches) {
  if (!g || !inputs_t || !kernel_ms || !n_launches || cap <= 0) return gfail(g, SR_ERR_ARG, "bad argument to sr_frame_step_timed");
  if (!g->was_reset) return gfail(g, SR_ERR_STATE, "sr_frame_step_timed before sr_reset");
  SrCtx c{};
  for (size_t i = 0; i < g->inputs.size(); ++i) {
    if (!inputs_t[i]) return gfail(g, SR_ERR_ARG, "input " + std::to_string(i) + " is null");
    c.in_ptr[i] = inputs_t[i];
  }
  c.in_last = (int32_t)(g->host_frame + 1);
  sr_status st = begin_frames(g, c);
  if (st != SR_OK) return st;
  FrameTimer ft;
  st = ensure_split_scratch(g);
  if (st != SR_OK) return st;
  st = enqueue_frame(g, false, &ft, SrSplitScratch{g->split_scratch, g->split_counters});
  hipError_t he = hipStreamSynchronize(g->stream);
  int n = 0;
  if (st == SR_OK && he == hipSuccess) {
    for (size_t i = 0; i + 1 < ft.ev.size() && n < cap; ++i, ++n) {
      float ms = 0.f;
      hipEventElapsedTime(&ms, ft.ev[i], ft.ev[i + 1]);
      kernel_ms[n] = ms;
      if (kernel_kind) kernel_kind[n] = ft.kind[i];
    }
  }
  for (hipEvent_t e : ft.ev) hipEventDestroy(e);
  if (st != SR_OK) return st;
  SR_HIP(g, he);
  g->host_frame += 1;
  *n_launches = n;
  return SR_OK;
}

sr_status sr_graph_work(const sr_graph* g, double* flops_per_frame, int64_t* mfma_tiles, int64_t* device_bytes) {
  if (!g) return fail(nullptr, SR_ERR_ARG, "null graph");
  sr_status st = finalize(const_cast<sr_graph*>(g));
  if (st != SR_OK) return st;
  if (flops_per_frame) *flops_per_frame = g->flops;
  if (mfma_tiles) *mfma_tiles = g->n_mfma_tiles;
  if (device_bytes) *device_bytes = g->device_bytes;
  return SR_OK;
}

sr_status sr_graph_traffic_model(const sr_graph* g, double* bytes6) {
  if (!g || !bytes6) return fail(nullptr, SR_ERR_ARG, "bad argument to sr_graph_traffic_model");
  sr_status st = finalize(const_cast<sr_graph*>(g));
  if (st != SR_OK) return st;
  for (int i = 0; i < 6; ++i) bytes6[i] = g->traffic[i];
  return SR_OK;
}

sr_status sr_graph_tile_kernel(const sr_graph* g, int32_t* tile_kernel) {
  if (!g || !tile_kernel) return fail(nullptr, SR_ERR_ARG, "null argument");
  sr_status st = finalize(const_cast<sr_graph*>(g));
  if (st != SR_OK) return st;
  *tile_kernel = g->n_mfma_tiles > 0 ? g->tile_version : 0;
  return SR_OK;
}

sr_status sr_graph_health(sr_graph* g, int64_t* dependency_timeouts, int32_t* dependency_driven) {
  if (!g) return fail(nullptr, SR_ERR_ARG, "null graph");
  if (dependency_driven) {
    sr_status st = finalize(g);
    if (st != SR_OK) return st;
    *dependency_driven = g->dataflow ? 1 : 0;
  }
  if (dependency_timeouts) {
    SrCtx c{};
    SR_HIP(g, hipStreamSynchronize(g->stream));
    SR_HIP(g, hipMemcpy(&c, g->ctx, sizeof(SrCtx), hipMemcpyDeviceToHost));
    *dependency_timeouts = c.dep_timeouts;
  }
  return SR_OK;
}

sr_status sr_graph_node_kernels(const sr_graph* g, int32_t* kinds) {
  if (!g || !kinds) return fail(nullptr, SR_ERR_ARG, "null argument");
  sr_status st = finalize(const_cast<sr_graph*>(g));
  if (st != SR_OK) return st;
  for (int v = 0; v < g->n_nodes; ++v) {
    const int k = g->nodes[v].kind;   // 0 input, 1 tile kernel, 2 direct, 3 head
    kinds[v] = (k == 0) ? 0 : (k == 1 ? (g->tile_version == 2 ? 2 : 1) : (k == 2 ? 3 : 4));
  }
  return SR_OK;
}

void sr_graph_destroy(sr_graph* g) {
  if (!g) return;
  if (g->stream || !g->dev_allocs.empty()) hipStreamSynchronize(g->stream);
  drop_graphs(g);
  for (void* p : g->dev_allocs) hipFree(p);
  if (g->split_scratch) uncached_release(g->split_scratch, g->split_scratch_bytes);
  sr_train_state_release(g->train);
  delete g;
}

}  // extern "C"
