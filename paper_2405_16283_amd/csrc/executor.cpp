// Event-driven execution of a memgraph on one GPU.
//
// Section 5 and Appendix A: a central loop launches any vertex whose memgraph dependencies have
// completed and for which a resource (a stream) is free, learns of completions, frees the
// resources and looks for more work; it never calls an allocator, because every tensor's GPU
// location was fixed by the compile.  Offloads take a slot of a pinned host arena, reloads give
// it back.
//
// Differences from the paper's engine, chosen for this hardware: completions are observed by
// polling one HIP event per stream from the loop thread (no callback thread); a stream carries
// one *group* at a time, where a group is up to `max_batch` ready vertices of the same kernel
// family served by a single grouped launch (a 512x512 tile cannot fill 256 compute units on its
// own, and a launch costs more than such a tile's run time); the operand tables the kernels read
// are built once at creation, since locations never change.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <array>
#include <chrono>
#include <cmath>
#include <cstring>
#include <deque>
#include <map>
#include <unordered_map>
#include <set>

#include "graph.h"
#include "kernels.h"

namespace tn {
namespace {

using Clock = std::chrono::steady_clock;
constexpr int kMaxQueueDepth = 8;  // groups in flight per compute stream, at most
constexpr int64_t kMaxProfEvents = (1 << 17) + 1;  // timing events per executor: 65536 timed launches per run

struct VInfo {
  int8_t cls = -1;  // LaunchClass, or -1 for non-kernel vertices
  int8_t dtype = 0;
  int16_t head_dim = 0;
  int8_t depth = 0;    // tile products: class of the summed depth K (see the GEMM case of tn_executor_create)
  int16_t group = -1;  // index of its (cls, dtype, head_dim, depth) combination: vertices of one group can share a launch
  int32_t desc = -1;
  int32_t nblocks = 0;
  int64_t lock = -1;  // increments: the vertex whose output they add to; one of them runs at a time
  double flops = 0, bytes = 0;
};

struct Slot {  // one stream and the group it carries
  hipStream_t stream = nullptr;
  hipEvent_t done = nullptr;
  bool busy = false, event_seen = false;
  int family = 0;  // 0 gemm, 1 attention, 2 elementwise, 3 h2d, 4 d2h
  Clock::time_point release;
  std::vector<int64_t> verts;
  int prof = -1;  // index of the (start, stop) event pair when profiling
  double flops = 0, bytes = 0;
};

constexpr int64_t kSmallGemmTiles = 128;
// Offloads moved by the chip's copy engines (TN_COPY_KERNEL_IN) are first gathered, by a copy inside GPU
// memory, into one of these staging slots, so that a whole group leaves with a single large copy.
constexpr uint64_t kStageBytes = 16ull << 20;
constexpr int kStageGatherWorkgroups = 64;  // see the launch of tile products in run_memgraph

struct Group {  // one grouped kernel launch in flight on a compute stream
  std::vector<int64_t> verts;
  hipEvent_t done = nullptr;
  int family = 0, prof = -1;
};

struct XGroup {  // one group of copies in flight on a copy stream
  std::vector<int64_t> verts;
  hipEvent_t done = nullptr;
  int prof = -1;
  bool event_seen = false;
  Clock::time_point release;
};

struct ArenaBlock {
  uint64_t size;
  bool used;
};

inline uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

// Ready vertices of one kind, handed out in the order the policy asks for: oldest first, newest
// first, at random, or smallest position in the serial order first (a binary heap).
struct ReadyQueue {
  int policy = TN_POLICY_FIFO;
  const int64_t* key = nullptr;  // TN_POLICY_BY_ORDER: position of every vertex in the serial order
  std::deque<int64_t> q;         // FIFO / LIFO
  std::vector<int64_t> v;        // RANDOM (unordered) / BY_ORDER (heap)
  size_t sel = 0;                // RANDOM: index chosen by peek()

  bool heap_less(int64_t a, int64_t b) const { return key[a] > key[b]; }  // min-heap through std::*_heap
  size_t size() const { return policy == TN_POLICY_FIFO || policy == TN_POLICY_LIFO ? q.size() : v.size(); }
  bool empty() const { return size() == 0; }
  void clear() { q.clear(); v.clear(); }
  void push(int64_t m) {
    if (policy == TN_POLICY_FIFO || policy == TN_POLICY_LIFO) {
      q.push_back(m);
    } else {
      v.push_back(m);
      if (policy == TN_POLICY_BY_ORDER)
        std::push_heap(v.begin(), v.end(), [this](int64_t a, int64_t b) { return heap_less(a, b); });
    }
  }
  // the vertex pop() would remove; rng is advanced by the random policy only
  int64_t peek(uint64_t& rng) {
    switch (policy) {
      case TN_POLICY_FIFO: return q.front();
      case TN_POLICY_LIFO: return q.back();
      case TN_POLICY_RANDOM: rng = mix64(rng); sel = (size_t)(rng % v.size()); return v[sel];
      default: return v.front();
    }
  }
  void pop() {
    switch (policy) {
      case TN_POLICY_FIFO: q.pop_front(); break;
      case TN_POLICY_LIFO: q.pop_back(); break;
      case TN_POLICY_RANDOM: v[sel] = v.back(); v.pop_back(); break;
      default:
        std::pop_heap(v.begin(), v.end(), [this](int64_t a, int64_t b) { return heap_less(a, b); });
        v.pop_back();
    }
  }
};


}  // namespace
}  // namespace tn

using namespace tn;

struct tn_executor {
  const MemGraph* mg = nullptr;
  char* dbase = nullptr;
  uint64_t dbytes = 0;
  char* arena = nullptr;
  char* stage = nullptr;  // kMaxQueueDepth staging slots of kStageBytes in GPU memory, for GPU -> host copies
  uint64_t arena_bytes = 0;
  bool own_arena = false, poisoned = false;
  int n_compute = 0;
  std::vector<Slot> slots;  // compute streams, then h2d, then d2h
  std::vector<std::vector<hipEvent_t>> cevents;  // per compute stream: ring of completion events
  hipEvent_t xevents[2][kMaxQueueDepth] = {};    // per copy direction: ring of completion events
  std::vector<std::deque<Group>> cqueue;         // per compute stream: groups in flight, oldest first
  std::vector<int64_t> pred_start, pred;         // CSR of predecessors
  // The operand tables the kernels read, as one image: descriptors, operand addresses, auxiliary
  // integers, rotary angles, each section 256-byte aligned.  h_image is pinned host memory (the
  // source of every upload), d_image the copy in GPU memory that tn_execute's kernels read.
  char* h_image = nullptr;
  char* d_image = nullptr;
  size_t image_bytes = 0, image_off[4] = {0, 0, 0, 0};
  DeviceTables tables{};
  std::vector<VInfo> info;
  // dependency structure (CSR of successors)
  std::vector<int64_t> succ_start, succ, indeg;
  // kernel vertices, host-to-device transfers and device-to-host transfers, each in the serial
  // order the memgraph was compiled for (TN_POLICY_IN_ORDER dispatches along these)
  std::vector<int64_t> serial[3];
  std::vector<int64_t> order_key;  // position of every vertex in that order
  std::vector<VInfo> groups;       // one representative per launch group (cls, dtype, head_dim)
  // per run
  std::vector<int64_t> remaining, last_order, arena_off;
  std::map<uint64_t, ArenaBlock> arena_map;
  std::map<uint64_t, std::set<uint64_t>> arena_free;  // size -> offsets of the free blocks of that size
  std::vector<hipEvent_t> prof_events;
  struct ProfRec { int32_t family, prof, n_vertices; int64_t work; double amount; };  // one timed launch of the last run
  std::vector<ProfRec> prof_recs;
  std::vector<tn_launch_record> launch_log;  // the same with its times, filled when the run ends
  // host buffers already found to be GPU-addressable pinned memory (start, end)
  std::vector<std::pair<const char*, const char*>> pinned_ranges;
  std::vector<std::pair<const char*, const char*>> device_ranges;  // callers' buffers in GPU memory
  bool arena_device_visible = false;
};

namespace {

#define TN_HIP(call)                                                                     \
  do {                                                                                   \
    hipError_t e_ = (call);                                                              \
    if (e_ != hipSuccess) return fail(TN_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

// (query, key) pairs of an attention block that the causal mask lets through: the work its
// products are accounted with (the masked part of a block on the diagonal is not work)
double visible_pairs(int q_rows, int kv_rows, const tn_op_params& p) {
  if (!p.causal) return (double)q_rows * kv_rows;
  double n = 0;
  for (int q = 0; q < q_rows; ++q) n += std::min<int64_t>(kv_rows, std::max<int64_t>(0, (int64_t)p.q_pos0 + q - p.k_pos0 + 1));
  return n;
}

// the table pointers for a copy of the image that starts at `base`
DeviceTables tables_at(const tn_executor& ex, const char* base) {
  return {(const OpDesc*)(base + ex.image_off[0]), (void* const*)(base + ex.image_off[1]),
          (const int32_t*)(base + ex.image_off[2]), (const double*)(base + ex.image_off[3])};
}

tn_status build_tables(tn_executor& ex) {
  const MemGraph& mg = *ex.mg;
  const int64_t nv = (int64_t)mg.v.size();
  std::vector<OpDesc> descs;
  std::vector<void*> ptrs;
  std::vector<int32_t> aux;
  std::vector<double> theta;
  std::map<std::pair<int32_t, uint32_t>, int32_t> theta_at;
  ex.info.assign(nv, VInfo{});
  auto addr = [&](int64_t m, uint64_t need, void** out) -> tn_status {
    const MVertex& o = mg.v[m];
    if (o.offset < 0 || (uint64_t)o.offset + need > ex.dbytes || need > o.bytes)
      return fail(TN_ERR_INVALID, "operand vertex %lld lies outside the device buffer", (long long)m);
    *out = ex.dbase + o.offset;
    return TN_OK;
  };
  for (int64_t m = 0; m < nv; ++m) {
    const MVertex& x = mg.v[m];
    if (x.offset >= 0 && (uint64_t)x.offset + x.bytes > ex.dbytes)
      return fail(TN_ERR_INVALID, "vertex %lld lies outside the device buffer", (long long)m);
    if (x.kind != TN_MG_OP) continue;
    OpDesc d{};
    d.out = ex.dbase + x.offset;
    d.ptr0 = (uint32_t)ptrs.size();
    d.aux0 = (uint32_t)aux.size();
    d.rows = x.desc.rows;
    d.cols = x.desc.cols;
    d.n_in = (int32_t)x.operands.size();
    d.p = x.p;
    d.trans_b = x.p.trans_b;
    d.dtype = x.operands.empty() ? x.desc.dtype : mg.v[x.operands[0]].desc.dtype;
    for (int64_t o : x.operands) {
      void* p = nullptr;
      tn_status s = addr(o, tensor_bytes(mg.v[o].desc), &p);
      if (s != TN_OK) return s;
      ptrs.push_back(p);
    }
    VInfo& vi = ex.info[m];
    vi.dtype = (int8_t)d.dtype;
    auto odesc = [&](int i) -> const tn_tensor_desc& { return mg.v[x.operands[i]].desc; };
    switch (x.op_kind) {
      case TN_OP_GEMM: {
        if (x.p.trans_c) std::swap(d.rows, d.cols);  // the kernels work on the logical [rows, cols] product
        bool mfma = d.dtype == TN_BF16 && d.trans_b && !x.p.trans_a, k32 = true;
        double K = 0;
        for (int k = 0; k < x.p.nk; ++k) {
          const int32_t kk = x.p.trans_a ? odesc(k).rows : odesc(k).cols;
          aux.push_back(kk);
          K += kk;
          if (kk % 8) mfma = false;
          if (kk % 32) k32 = false;
        }
        const bool big = k32 && d.rows >= 256 && d.cols >= 256;
        // the fused forms (mode 1: + residual, mode 2: gated pair) exist in the 256-tile kernel, which clamps its
        // loads and guards its stores for any shape, and in the generic one, which the thinnest products take
        const bool fused_mfma = x.p.mode != 0 && k32 && d.rows >= 64;
        vi.cls = !mfma ? LC_GEMM_F32 : (big || fused_mfma) ? LC_GEMM_BF16_NT256 : x.p.mode != 0 ? LC_GEMM_F32 : LC_GEMM_BF16_NT;
        vi.flops = (x.p.mode == 2 ? 4.0 : 2.0) * d.rows * d.cols * K;
        // Products of very different depth do not share a launch.  The workgroups of a launch that run at the same
        // time read the same operand panels at the same moment only as long as they walk along K in step, and that
        // sharing in the L2s is what feeds them: 22016-deep products started one by one between 4096-deep ones
        // run at 390 TFLOP/s, in a launch of their own at 1000.
        vi.depth = K <= 6144 ? 0 : K <= 12288 ? 1 : 2;
        break;
      }
      case TN_OP_RMS_STAT:
        for (int i = 0; i < d.n_in; ++i) aux.push_back(odesc(i).cols);
        vi.cls = LC_RMS_STAT;
        vi.bytes = (double)d.rows * x.p.d * elem_bytes(d.dtype) + d.rows * 4.0;
        break;
      case TN_OP_RMS_APPLY:
        vi.cls = LC_RMS_APPLY;
        vi.bytes = 2.0 * x.bytes + d.rows * 4.0 + d.cols * (double)elem_bytes(d.dtype);
        break;
      case TN_OP_ROPE: {
        vi.cls = LC_ROPE;
        vi.bytes = 2.0 * x.bytes;
        uint32_t bits;
        memcpy(&bits, &x.p.rope_base, 4);
        auto key = std::make_pair(x.p.head_dim, bits);
        auto it = theta_at.find(key);
        if (it == theta_at.end()) {
          it = theta_at.emplace(key, (int32_t)theta.size()).first;
          for (int i = 0; i < x.p.head_dim / 2; ++i)
            theta.push_back(std::pow((double)x.p.rope_base, -2.0 * i / x.p.head_dim));
        }
        d.aux0 = (uint32_t)it->second;
        break;
      }
      case TN_OP_ATTN_BLOCK: {
        const int nq = x.p.n_q_tiles, nkv = x.p.n_kv_tiles, nc = x.p.n_col_tiles, hd = x.p.head_dim;
        const int tq = odesc(0).rows, tk = odesc(nq * nc).rows, tc = odesc(0).cols;
        int q_rows = 0, kv_rows = 0;
        // the kernels address tiles as a uniform grid: equal tiles except a shorter last row tile
        for (int r = 0; r < nq; ++r) {
          q_rows += odesc(r * nc).rows;
          if ((r + 1 < nq && odesc(r * nc).rows != tq) || odesc(r * nc).rows > tq)
            return fail(TN_ERR_SHAPE, "attn_block %lld: Q row tiles are not uniform", (long long)m);
        }
        for (int r = 0; r < nkv; ++r) {
          kv_rows += odesc(nq * nc + r * nc).rows;
          if ((r + 1 < nkv && odesc(nq * nc + r * nc).rows != tk) || odesc(nq * nc + r * nc).rows > tk)
            return fail(TN_ERR_SHAPE, "attn_block %lld: K/V row tiles are not uniform", (long long)m);
        }
        for (int c = 0; c < nc; ++c)
          if (odesc(c).cols != tc) return fail(TN_ERR_SHAPE, "attn_block %lld: column tiles are not uniform", (long long)m);
        if (hd != 64 && hd != 128) return fail(TN_ERR_SHAPE, "attn_block %lld: head_dim must be 64 or 128", (long long)m);
        aux.insert(aux.end(), {tq, tk, tc, q_rows, kv_rows});
        // the MFMA kernel wants V^T tiles, whole heads inside one column tile, 64-key chunks inside
        // one row tile, 16-byte chunks that do not straddle anything, and a positive scale (it takes
        // the row maximum before scaling)
        vi.cls = (d.dtype == TN_BF16 && x.p.v_trans && tc % hd == 0 && tk % 64 == 0 && kv_rows % 8 == 0 && x.p.scale > 0.f)
                     ? LC_ATTN_BF16 : LC_ATTN_F32;
        vi.head_dim = (int16_t)hd;
        vi.flops = 4.0 * visible_pairs(q_rows, kv_rows, x.p) * (double)(nc * tc);
        break;
      }
      case TN_OP_ATTN_COMBINE:
        vi.cls = LC_ATTN_COMBINE;
        d.dtype = x.desc.dtype;
        vi.dtype = (int8_t)d.dtype;
        vi.bytes = x.bytes + d.n_in * ((double)d.rows * d.cols * 4.0);
        break;
      case TN_OP_SILU_MUL:
      case TN_OP_ADD:
        vi.cls = x.op_kind == TN_OP_ADD ? LC_ADD : LC_SILU_MUL;
        vi.bytes = 3.0 * x.bytes;
        break;
      case TN_OP_TRANSPOSE:
        vi.cls = LC_TRANSPOSE;
        vi.bytes = 2.0 * x.bytes;
        break;
      case TN_OP_SOFTMAX_STAT:
        for (int i = 0; i < d.n_in; ++i) {
          aux.push_back(odesc(i).cols);
          vi.bytes += (double)d.rows * odesc(i).cols * elem_bytes(d.dtype);
        }
        vi.cls = LC_SOFTMAX_STAT;
        break;
      case TN_OP_SOFTMAX_APPLY:
        vi.cls = LC_SOFTMAX_APPLY;
        vi.bytes = 2.0 * x.bytes + d.rows * 8.0;
        break;
      case TN_OP_ZERO:
        vi.cls = LC_ZERO;
        vi.bytes = (double)x.bytes;
        break;
      case TN_OP_SUM_INTO:  // output = operand 0 + operand 1, written where operand 1 lies
        if (x.operands.size() != 2 || mg.v[x.operands[1]].offset != x.offset)
          return fail(TN_ERR_INVALID, "increment %lld does not name the output it adds to", (long long)m);
        vi.cls = LC_ADD;
        vi.bytes = 3.0 * x.bytes;
        vi.lock = x.operands[1];
        break;
      case TN_OP_SILU_MUL_BWD:
        vi.cls = LC_SILU_BWD;
        vi.bytes = 4.0 * x.bytes;
        break;
      case TN_OP_RMS_BWD_STAT:
        for (int i = 0; i < x.p.nk; ++i) aux.push_back(odesc(i).cols);
        vi.cls = LC_RMS_BWD_STAT;
        for (int i = 0; i < x.p.nk; ++i) vi.bytes += 2.0 * d.rows * odesc(i).cols * elem_bytes(d.dtype);
        break;
      case TN_OP_RMS_BWD_APPLY:
        vi.cls = LC_RMS_BWD_APPLY;
        vi.bytes = (d.n_in == 6 ? 4.0 : 3.0) * x.bytes + d.rows * 8.0;
        break;
      case TN_OP_ATTN_BWD: {
        const int nq = x.p.n_q_tiles, nkv = x.p.n_kv_tiles, nc = x.p.n_col_tiles, hd = x.p.head_dim;
        const int tq = odesc(0).rows, tk = odesc(nq * nc).rows, tc = odesc(0).cols;
        int q_rows = 0, kv_rows = 0;
        for (int r = 0; r < nq; ++r) {
          q_rows += odesc(r * nc).rows;
          if ((r + 1 < nq && odesc(r * nc).rows != tq) || odesc(r * nc).rows > tq)
            return fail(TN_ERR_SHAPE, "attn_bwd %lld: Q row tiles are not uniform", (long long)m);
        }
        for (int r = 0; r < nkv; ++r) {
          kv_rows += odesc(nq * nc + r * nc).rows;
          if ((r + 1 < nkv && odesc(nq * nc + r * nc).rows != tk) || odesc(nq * nc + r * nc).rows > tk)
            return fail(TN_ERR_SHAPE, "attn_bwd %lld: K/V row tiles are not uniform", (long long)m);
        }
        for (int c = 0; c < nc; ++c)
          if (odesc(c).cols != tc) return fail(TN_ERR_SHAPE, "attn_bwd %lld: column tiles are not uniform", (long long)m);
        if (hd != 64 && hd != 128) return fail(TN_ERR_SHAPE, "attn_bwd %lld: head_dim must be 64 or 128", (long long)m);
        aux.insert(aux.end(), {tq, tk, tc, q_rows, kv_rows});
        // the MFMA kernel wants plain V tiles, the transposed grid (except for the statistics), whole
        // heads inside one column tile, 64-row chunks inside one row tile, 8-row groups that
        // straddle nothing, and a positive scale (the row maximum is taken before scaling)
        vi.cls = (d.dtype == TN_BF16 && !x.p.v_trans && x.p.scale > 0.f && (x.p.mode == 0 || x.p.trans_a) && tc % hd == 0 && tq % 64 == 0 &&
                  tk % 64 == 0 && q_rows % 8 == 0 && kv_rows % 8 == 0 && q_rows >= 8 && kv_rows >= 8)
                     ? (int8_t)(LC_ATTN_BWD_BF16 + x.p.mode) : (int8_t)LC_ATTN_BWD;
        vi.head_dim = (int16_t)hd;
        vi.flops = (x.p.mode == 3 ? 4.0 : 6.0) * visible_pairs(q_rows, kv_rows, x.p) * (double)(nc * tc);
        break;
      }
      default: return fail(TN_ERR_INVALID, "vertex %lld has an unknown kind", (long long)m);
    }
    d.nblocks = blocks_for(vi.cls, d, aux.data());
    vi.nblocks = d.nblocks;
    vi.desc = (int32_t)descs.size();
    descs.push_back(d);
  }
  const size_t sizes[4] = {descs.size() * sizeof(OpDesc), ptrs.size() * sizeof(void*), aux.size() * 4, theta.size() * 8};
  const void* src[4] = {descs.data(), ptrs.data(), aux.data(), theta.data()};
  size_t at = 0;
  for (int k = 0; k < 4; ++k) {
    ex.image_off[k] = at;
    at += (std::max<size_t>(sizes[k], 16) + 255) / 256 * 256;
  }
  ex.image_bytes = at;
  TN_HIP(hipHostMalloc((void**)&ex.h_image, at, hipHostMallocDefault));
  memset(ex.h_image, 0, at);
  for (int k = 0; k < 4; ++k)
    if (sizes[k]) memcpy(ex.h_image + ex.image_off[k], src[k], sizes[k]);
  TN_HIP(hipMalloc((void**)&ex.d_image, at));
  TN_HIP(hipMemcpy(ex.d_image, ex.h_image, at, hipMemcpyHostToDevice));
  ex.tables = tables_at(ex, ex.d_image);
  return TN_OK;
}

// host arena with coalescing; offsets are 256-byte aligned.  Free blocks are indexed by size, so
// that an allocation takes the lowest free block of the smallest sufficient size in O(log n): a
// run that offloads tens of thousands of tensors cannot afford to walk over the used ones.
void arena_index_add(tn_executor& ex, uint64_t off, uint64_t size) { ex.arena_free[size].insert(off); }
void arena_index_del(tn_executor& ex, uint64_t off, uint64_t size) {
  auto it = ex.arena_free.find(size);
  it->second.erase(off);
  if (it->second.empty()) ex.arena_free.erase(it);
}

bool arena_alloc(tn_executor& ex, uint64_t size, uint64_t* off) {
  size = (size + 255) / 256 * 256;
  auto f = ex.arena_free.lower_bound(size);
  if (f == ex.arena_free.end()) return false;
  const uint64_t o = *f->second.begin(), have = f->first;
  arena_index_del(ex, o, have);
  ex.arena_map[o] = {size, true};
  if (have > size) {
    ex.arena_map[o + size] = {have - size, false};
    arena_index_add(ex, o + size, have - size);
  }
  *off = o;
  return true;
}

// Largest free block: what a run of adjacent slots can take at most.
uint64_t arena_largest_free(const tn_executor& ex) { return ex.arena_free.empty() ? 0 : ex.arena_free.rbegin()->first; }

// Adjacent slots for n tensors (sizes rounded up to 256 bytes), each of which can be freed on its own.
bool arena_alloc_run(tn_executor& ex, const uint64_t* sizes, int n, uint64_t* first) {
  uint64_t total = 0;
  for (int i = 0; i < n; ++i) total += (sizes[i] + 255) / 256 * 256;
  if (!arena_alloc(ex, total, first)) return false;
  ex.arena_map.erase(*first);
  uint64_t at = *first;
  for (int i = 0; i < n; ++i) {
    const uint64_t sz = (sizes[i] + 255) / 256 * 256;
    ex.arena_map[at] = {sz, true};
    at += sz;
  }
  return true;
}

void arena_free(tn_executor& ex, uint64_t off) {
  auto it = ex.arena_map.find(off);
  it->second.used = false;
  auto nx = std::next(it);
  if (nx != ex.arena_map.end() && !nx->second.used) {
    arena_index_del(ex, nx->first, nx->second.size);
    it->second.size += nx->second.size;
    ex.arena_map.erase(nx);
  }
  if (it != ex.arena_map.begin()) {
    auto pv = std::prev(it);
    if (!pv->second.used) {
      arena_index_del(ex, pv->first, pv->second.size);
      pv->second.size += it->second.size;
      ex.arena_map.erase(it);
      it = pv;
    }
  }
  arena_index_add(ex, it->first, it->second.size);
}

// True if [p, p+bytes) is memory that kernels can address: pinned host memory, or memory of the
// GPU itself (a caller's buffer for results that stay on the GPU; *on_device is then set).
// Ranges found once are remembered, so that a repeated call with the same buffers costs a few
// comparisons.
bool device_visible_host(tn_executor& ex, const void* p, uint64_t bytes, bool* on_device = nullptr) {
  const char* a = (const char*)p;
  for (auto& r : ex.device_ranges)
    if (a >= r.first && a + bytes <= r.second) {
      if (on_device) *on_device = true;
      return true;
    }
  for (auto& r : ex.pinned_ranges)
    if (a >= r.first && a + bytes <= r.second) return true;
  hipPointerAttribute_t at{};
  if (hipPointerGetAttributes(&at, p) != hipSuccess) {
    (void)hipGetLastError();  // pageable memory is reported as an error: not ours to keep
    return false;
  }
  if (at.type == hipMemoryTypeDevice) {
    void* base = nullptr;
    size_t size = 0;
    if (hipMemGetAddressRange((hipDeviceptr_t*)&base, &size, (hipDeviceptr_t)p) != hipSuccess || !base ||
        a < (const char*)base || a + bytes > (const char*)base + size) {
      (void)hipGetLastError();
      return false;
    }
    ex.device_ranges.emplace_back((const char*)base, (const char*)base + size);
    if (on_device) *on_device = true;
    return true;
  }
  if (at.type != hipMemoryTypeHost || !at.devicePointer) return false;
  void* base = nullptr;
  size_t size = 0;
  if (hipMemGetAddressRange((hipDeviceptr_t*)&base, &size, (hipDeviceptr_t)at.devicePointer) == hipSuccess && base && size) {
    // identity-mapped pinned allocation: remember the whole of it
    if (at.devicePointer == p && (const char*)base <= a && a + bytes <= (const char*)base + size) {
      ex.pinned_ranges.emplace_back((const char*)base, (const char*)base + size);
      return true;
    }
  } else {
    (void)hipGetLastError();
  }
  if (at.devicePointer != p) return false;
  ex.pinned_ranges.emplace_back(a, a + bytes);
  return true;
}

int family_of(int cls) {
  switch (cls) {
    case LC_GEMM_F32:
    case LC_GEMM_BF16_NT:
    case LC_GEMM_BF16_NT256: return 0;
    case LC_ATTN_F32:
    case LC_ATTN_BF16:
    case LC_ATTN_BWD:
    case LC_ATTN_BWD_BF16:
    case LC_ATTN_BWD_BF16_DQ:
    case LC_ATTN_BWD_BF16_DK:
    case LC_ATTN_BWD_BF16_DV: return 1;
    default: return 2;
  }
}

}  // namespace

extern "C" {

tn_status tn_executor_create(const tn_memgraph* mg, void* device_base, uint64_t device_bytes, void* pinned_arena,
                             uint64_t arena_bytes, void* const* compute_streams, int32_t n_compute,
                             void* h2d_stream, void* d2h_stream, tn_executor** out) {
  if (!mg || !device_base || !compute_streams || n_compute < 1 || n_compute > 64 || !out)
    return fail(TN_ERR_INVALID, "NULL argument or bad stream count");
  if ((uintptr_t)device_base % 256) return fail(TN_ERR_INVALID, "device_base must be 256-byte aligned");
  if (device_bytes < mg->stats.high_water)
    return fail(TN_ERR_INVALID, "device buffer of %llu bytes is smaller than the memgraph's high-water mark %llu",
                (unsigned long long)device_bytes, (unsigned long long)mg->stats.high_water);
  auto* ex = new (std::nothrow) tn_executor();
  if (!ex) return fail(TN_ERR_INVALID, "out of host memory");
  ex->mg = mg;
  ex->dbase = (char*)device_base;
  ex->dbytes = device_bytes;
  ex->n_compute = n_compute;
  ex->slots.resize(n_compute + 2);
  for (int i = 0; i < n_compute; ++i) ex->slots[i].stream = (hipStream_t)compute_streams[i];
  ex->slots[n_compute].stream = (hipStream_t)h2d_stream;
  ex->slots[n_compute + 1].stream = (hipStream_t)d2h_stream;
  auto bail = [&](tn_status s) {
    tn_executor_destroy(ex);
    return s;
  };
  for (auto& sl : ex->slots) {
    hipError_t e = hipEventCreateWithFlags(&sl.done, hipEventDisableTiming);
    if (e != hipSuccess) return bail(fail(TN_ERR_HIP, "hipEventCreateWithFlags: %s", hipGetErrorString(e)));
  }
  if (arena_bytes == 0) arena_bytes = mg->stats.host_arena_bytes;
  ex->arena_bytes = arena_bytes / 256 * 256;
  if (pinned_arena) {
    ex->arena = (char*)pinned_arena;
  } else if (ex->arena_bytes) {
    hipError_t e = hipHostMalloc((void**)&ex->arena, ex->arena_bytes, hipHostMallocDefault);
    if (e != hipSuccess) return bail(fail(TN_ERR_HIP, "hipHostMalloc(%llu): %s", (unsigned long long)ex->arena_bytes, hipGetErrorString(e)));
    ex->own_arena = true;
  }
  if (ex->arena && ex->arena_bytes) ex->arena_device_visible = device_visible_host(*ex, ex->arena, ex->arena_bytes);
  if (mg->stats.n_offload + mg->stats.n_store > 0) {
    hipError_t e = hipMalloc((void**)&ex->stage, kStageBytes * kMaxQueueDepth);
    if (e != hipSuccess) return bail(fail(TN_ERR_HIP, "hipMalloc of the offload staging slots: %s", hipGetErrorString(e)));
  }
  // dependency structure
  const int64_t nv = (int64_t)mg->v.size();
  ex->indeg.assign(nv, 0);
  ex->succ_start.assign(nv + 1, 0);
  for (const auto& e : mg->edges) {
    ++ex->succ_start[e.from + 1];
    ++ex->indeg[e.to];
  }
  for (int64_t i = 0; i < nv; ++i) ex->succ_start[i + 1] += ex->succ_start[i];
  ex->succ.resize(mg->edges.size());
  {
    std::vector<int64_t> at(ex->succ_start.begin(), ex->succ_start.end() - 1);
    for (const auto& e : mg->edges) ex->succ[at[e.from]++] = e.to;
  }
  ex->pred_start.assign(nv + 1, 0);
  for (const auto& e : mg->edges) ++ex->pred_start[e.to + 1];
  for (int64_t i = 0; i < nv; ++i) ex->pred_start[i + 1] += ex->pred_start[i];
  ex->pred.resize(mg->edges.size());
  {
    std::vector<int64_t> at(ex->pred_start.begin(), ex->pred_start.end() - 1);
    for (const auto& e : mg->edges) ex->pred[at[e.to]++] = e.from;
  }
  ex->cevents.resize(n_compute);
  ex->cqueue.resize(n_compute);
  for (int i = 0; i < n_compute; ++i)
    for (int k = 0; k < kMaxQueueDepth; ++k) {
      hipEvent_t ev;
      hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
      if (e != hipSuccess) return bail(fail(TN_ERR_HIP, "hipEventCreateWithFlags: %s", hipGetErrorString(e)));
      ex->cevents[i].push_back(ev);
    }
  for (int dir = 0; dir < 2; ++dir)
    for (int k = 0; k < kMaxQueueDepth; ++k) {
      hipError_t e = hipEventCreateWithFlags(&ex->xevents[dir][k], hipEventDisableTiming);
      if (e != hipSuccess) return bail(fail(TN_ERR_HIP, "hipEventCreateWithFlags: %s", hipGetErrorString(e)));
    }
  ex->arena_off.assign(nv, -1);
  {
    // Timing events for profiled runs: a pair per launch, and a launch carries at least one kernel
    // or transfer vertex.  Made here so that a run creates nothing (Section 5: no allocation calls
    // while the memgraph executes).
    int64_t n_work = 0;
    for (const auto& x : mg->v) n_work += x.kind != TN_MG_INPUT && x.kind != TN_MG_DROP && x.kind != TN_MG_JOIN;
    const int64_t pool = std::min<int64_t>(2 * n_work + 1, kMaxProfEvents);
    ex->prof_events.reserve(pool);
    for (int64_t k = 0; k < pool; ++k) {
      hipEvent_t ev;
      hipError_t e = hipEventCreate(&ev);
      if (e != hipSuccess) return bail(fail(TN_ERR_HIP, "hipEventCreate: %s", hipGetErrorString(e)));
      ex->prof_events.push_back(ev);
    }
    ex->prof_recs.reserve((size_t)pool / 2);
    ex->launch_log.reserve((size_t)pool / 2);
  }
  tn_status s = build_tables(*ex);
  if (s != TN_OK) return bail(s);
  {
    ex->order_key.resize(nv);
    std::vector<int64_t> by_pos(nv);
    for (int64_t m = 0; m < nv; ++m) {
      ex->order_key[m] = mg->v[m].order_pos;
      by_pos[m] = m;
    }
    std::stable_sort(by_pos.begin(), by_pos.end(), [&](int64_t a, int64_t b) { return ex->order_key[a] < ex->order_key[b]; });
    for (int64_t m : by_pos) {
      const int32_t k = mg->v[m].kind;
      if (k == TN_MG_OP) ex->serial[0].push_back(m);
      else if (k == TN_MG_LOAD || k == TN_MG_RELOAD) ex->serial[1].push_back(m);
      else if (k == TN_MG_OFFLOAD || k == TN_MG_STORE) ex->serial[2].push_back(m);
    }
    for (int64_t m = 0; m < nv; ++m) {
      VInfo& vi = ex->info[m];
      if (vi.cls < 0) continue;
      size_t g = 0;
      while (g < ex->groups.size() && !(ex->groups[g].cls == vi.cls && ex->groups[g].dtype == vi.dtype &&
                                        ex->groups[g].head_dim == vi.head_dim && ex->groups[g].depth == vi.depth)) ++g;
      if (g == ex->groups.size()) ex->groups.push_back(vi);
      vi.group = (int16_t)g;
    }
  }
  *out = ex;
  return TN_OK;
}

void tn_executor_destroy(tn_executor* ex) {
  if (!ex) return;
  for (auto& sl : ex->slots)
    if (sl.done) (void)hipEventDestroy(sl.done);
  for (auto e : ex->prof_events) (void)hipEventDestroy(e);
  for (auto& ring : ex->cevents)
    for (auto e : ring) (void)hipEventDestroy(e);
  for (auto& ring : ex->xevents)
    for (auto e : ring)
      if (e) (void)hipEventDestroy(e);
  if (ex->d_image) (void)hipFree(ex->d_image);
  if (ex->h_image) (void)hipHostFree(ex->h_image);
  if (ex->own_arena && ex->arena) (void)hipHostFree(ex->arena);
  if (ex->stage) (void)hipFree(ex->stage);
  delete ex;
}

tn_status tn_executor_place_inputs(tn_executor* ex, const void* const* host_inputs) {
  if (!ex || !host_inputs) return fail(TN_ERR_INVALID, "NULL argument");
  if (ex->poisoned) return fail(TN_ERR_HIP, "executor is poisoned by an earlier HIP error");
  const MemGraph& mg = *ex->mg;
  hipStream_t s = ex->slots[ex->n_compute].stream;
  for (int64_t m = 0; m < mg.n_task; ++m) {
    const MVertex& x = mg.v[m];
    if (x.kind != TN_MG_INPUT) continue;
    if (!host_inputs[m]) return fail(TN_ERR_INVALID, "no host buffer for device-resident input %lld", (long long)m);
    // the source may be host memory or (a tensor another kernel left there) GPU memory: let the runtime tell
    TN_HIP(hipMemcpyAsync(ex->dbase + x.offset, host_inputs[m], x.bytes, hipMemcpyDefault, s));
  }
  TN_HIP(hipStreamSynchronize(s));
  return TN_OK;
}

// The engine behind tn_execute and tn_execute_static: `tables` says where the kernels of this run
// find their operand tables.
static tn_status run_memgraph(tn_executor* ex, const void* const* host_inputs, void* const* host_outputs,
                              const tn_exec_opts* opts_in, tn_exec_report* report, const DeviceTables& tables) {
  const MemGraph& mg = *ex->mg;
  const int64_t nv = (int64_t)mg.v.size();
  tn_exec_opts opt{};
  if (opts_in) opt = *opts_in;
  const int max_batch = opt.max_batch > 0 ? std::min<int>(opt.max_batch, kMaxBatch) : 64;
  const int max_xfer = std::min(opt.max_transfers > 0 ? opt.max_transfers : 32, kMaxCopies);
  // queue_depth 1 is the paper's rule: a vertex is launched once its dependencies have completed.
  // With a deeper queue a kernel may be enqueued as soon as the kernels it depends on are
  // enqueued: the stream waits for their events on the device, so the order of execution still
  // respects every dependency while the host no longer sits between two dependent kernels.
  // Anything that depends on a transfer still waits for the host to see that transfer complete.
  const int depth = std::max(1, std::min<int>(opt.queue_depth > 0 ? opt.queue_depth : 1, kMaxQueueDepth));
  const bool ahead = depth > 1;
  // every buffer the run will touch must be there before anything is launched
  for (int64_t m = 0; m < nv; ++m) {
    const MVertex& x = mg.v[m];
    if (x.kind == TN_MG_LOAD && (!host_inputs || !host_inputs[x.src]))
      return fail(TN_ERR_INVALID, "no host buffer for input %d", (int)x.src);
    if (x.kind == TN_MG_STORE && (!host_outputs || !host_outputs[x.output_index]))
      return fail(TN_ERR_INVALID, "no host buffer for output %d", x.output_index);
    // a caller's buffer in GPU memory must not lie inside the buffer the memgraph's locations refer to
    const char* cb = x.kind == TN_MG_LOAD ? (const char*)host_inputs[x.src]
                     : x.kind == TN_MG_STORE ? (const char*)host_outputs[x.output_index] : nullptr;
    if (cb && cb < ex->dbase + mg.cap && cb + x.bytes > ex->dbase)
      return fail(TN_ERR_INVALID, "buffer of %s %d overlaps the executor's device buffer",
                  x.kind == TN_MG_LOAD ? "input" : "output", x.kind == TN_MG_LOAD ? (int)x.src : x.output_index);
  }
  bool kernel_copies = opt.copy_engine != TN_COPY_MEMCPY;
  bool any_on_device = false;  // a caller's buffer lies in GPU memory: hipMemcpyAsync is told to find the direction itself
  {
    bool ok = ex->arena_device_visible || mg.stats.n_offload == 0;
    for (int64_t m = 0; m < nv && ok; ++m) {
      const MVertex& x = mg.v[m];
      if (x.kind == TN_MG_LOAD) ok = device_visible_host(*ex, host_inputs[x.src], x.bytes, &any_on_device);
      else if (x.kind == TN_MG_STORE) ok = device_visible_host(*ex, host_outputs[x.output_index], x.bytes, &any_on_device);
    }
    if (!ok) any_on_device = true;  // not every buffer was looked at (pageable memory ends the scan)
    if (kernel_copies && !ok && (opt.copy_engine == TN_COPY_KERNEL || opt.copy_engine == TN_COPY_KERNEL_IN))
      return fail(TN_ERR_INVALID, "copy_engine KERNEL needs every host buffer to be GPU-addressable pinned memory");
    kernel_copies = kernel_copies && ok;
  }
  ex->remaining = ex->indeg;
  std::vector<int64_t> rem_enq(ex->indeg);           // dependencies not yet enqueued (kernels) or completed
  std::vector<hipEvent_t> ev_of(nv, nullptr);        // event of the group a kernel vertex was enqueued in
  std::vector<int8_t> stream_of(nv, -1), state(nv, 0);  // state: 0 waiting, 1 enqueued, 2 complete
  std::vector<int> ring_next(ex->n_compute, 0);
  for (auto& q : ex->cqueue) q.clear();
  ex->last_order.clear();
  ex->last_order.reserve(nv);
  ex->arena_map.clear();
  ex->arena_free.clear();
  if (ex->arena_bytes) {
    ex->arena_map[0] = {ex->arena_bytes, false};
    ex->arena_free[ex->arena_bytes].insert(0);
  }
  std::fill(ex->arena_off.begin(), ex->arena_off.end(), -1);
  for (auto& sl : ex->slots) {
    sl.busy = false;
    sl.verts.clear();
  }
  tn_exec_report rep{};
  if (opt.policy < TN_POLICY_FIFO || opt.policy > TN_POLICY_IN_ORDER) return fail(TN_ERR_INVALID, "unknown policy %d", opt.policy);
  const bool in_order = opt.policy == TN_POLICY_IN_ORDER;
  // ready vertices: one queue per launch group of kernels, one per transfer direction.  The
  // in-order policy walks the serial lists instead and only needs to know who is ready.
  const size_t n_groups = ex->groups.size();
  std::vector<ReadyQueue> rq(n_groups + 2);
  for (auto& q : rq) {
    q.policy = in_order ? TN_POLICY_FIFO : opt.policy;
    q.key = ex->order_key.data();
  }
  ReadyQueue* const rq_x = rq.data() + n_groups;  // [0] host to device, [1] device to host
  std::vector<char> is_ready(in_order ? nv : 0, 0);
  std::vector<uint64_t> arrival(opt.policy <= TN_POLICY_LIFO ? nv : 0, 0);  // when a vertex became ready
  uint64_t n_arrived = 0;
  int64_t n_ready_k = 0, n_ready_x[2] = {0, 0};
  size_t serial_next[3] = {0, 0, 0};
  std::vector<int64_t> work;
  auto make_ready = [&](int64_t w) {
    const int32_t k = mg.v[w].kind;
    const int which = k == TN_MG_OP ? -1 : (k == TN_MG_LOAD || k == TN_MG_RELOAD) ? 0 : 1;
    if (which < 0) ++n_ready_k; else ++n_ready_x[which];
    if (in_order) {
      is_ready[w] = 1;
      return;
    }
    if (!arrival.empty()) arrival[w] = n_arrived++;
    (which < 0 ? rq[ex->info[w].group] : rq_x[which]).push(w);
  };
  int64_t completed = 0;
  uint64_t rng = mix64(opt.order_seed ^ 0x7475726E6970ull);
  uint64_t arena_used = 0;
  size_t prof_used = 0;
  hipEvent_t prof_base = nullptr;
  tn_status status = TN_OK;

  // timing events come from the pool made at creation; a run with more launches than the pool
  // covers leaves the rest untimed (counted in the report) rather than create events while it runs
  auto prof_pair = [&](int* first) -> bool {
    if (prof_used + 2 > ex->prof_events.size()) {
      ++rep.untimed_launches;
      return false;
    }
    *first = (int)prof_used;
    prof_used += 2;
    return true;
  };

  // Appendix A (resources): the output of a sum is protected by a write lock; an increment takes
  // it when it is launched and gives it back when it has completed, and increments that find it
  // taken wait here, outside the ready lists
  std::vector<char> lock_busy(nv, 0);
  std::unordered_map<int64_t, std::vector<int64_t>> lock_wait;
  // a vertex whose dependencies are all complete joins a ready list; vertices with no work
  // (inputs already in place, drops, joins of sums) complete on the spot
  auto complete = [&](int64_t first) {
    work.push_back(first);
    while (!work.empty()) {
      const int64_t m = work.back();
      work.pop_back();
      ++completed;
      const bool was_enqueued_kernel = ahead && mg.v[m].kind == TN_MG_OP;  // its successors were told at enqueue time
      state[m] = 2;
      if (const int64_t lk = ex->info[m].lock; lk >= 0) {
        lock_busy[lk] = 0;
        auto it = lock_wait.find(lk);
        if (it != lock_wait.end()) {
          for (int64_t w : it->second) make_ready(w);
          lock_wait.erase(it);
        }
      }
      for (int64_t i = ex->succ_start[m]; i < ex->succ_start[m + 1]; ++i) {
        const int64_t w = ex->succ[i];
        const bool all_done = --ex->remaining[w] == 0;
        const int32_t k = mg.v[w].kind;
        if (k == TN_MG_OP) {
          if (ahead) {
            if (!was_enqueued_kernel && --rem_enq[w] == 0) make_ready(w);
          } else if (all_done) {
            make_ready(w);
          }
          continue;
        }
        if (!all_done) continue;
        if (k == TN_MG_INPUT || k == TN_MG_DROP || k == TN_MG_JOIN) {
          ex->last_order.push_back(w);
          work.push_back(w);
        } else {
          make_ready(w);
        }
      }
    }
  };
  for (int64_t m = 0; m < nv; ++m) {
    if (ex->indeg[m] != 0) continue;
    if (mg.v[m].kind == TN_MG_INPUT || mg.v[m].kind == TN_MG_DROP || mg.v[m].kind == TN_MG_JOIN) {
      ex->last_order.push_back(m);
      complete(m);
    } else {
      make_ready(m);
    }
  }

  auto hip_fail = [&](const char* what, hipError_t e) {
    ex->poisoned = true;
    status = fail(TN_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
  };

  if (opt.profile) {
    if (ex->prof_events.empty() || hipEventRecord(prof_base = ex->prof_events[prof_used++], ex->slots[0].stream) != hipSuccess)
      return fail(TN_ERR_HIP, "cannot record the profiling base event");
    ex->prof_recs.clear();
    ex->launch_log.clear();
  }
  const auto t_start = Clock::now();
  Batch batch;
  CopyBatch copies;
  std::deque<XGroup> xq[2];  // copy groups in flight, host to device and device to host
  int xring[2] = {0, 0};
  const int xdepth = std::max(1, std::min<int>(opt.transfer_depth > 0 ? opt.transfer_depth : 3, kMaxQueueDepth));
  std::vector<int64_t> same, xverts, sort_b, stage_verts;
  std::vector<uint64_t> stage_sizes, stage_run, stage_tmp_s;
  std::vector<size_t> stage_ord;
  std::vector<int64_t> stage_tmp_v;
  std::vector<const void*> stage_tmp_src;
  std::vector<std::array<int64_t, 4>> sort_keys;
  std::vector<hipEvent_t> waited;

  while (completed < nv && status == TN_OK) {
    bool progressed = false;
    // ---- launch transfers: per direction a few groups of copies in flight, so that the stream
    // does not run dry while the host looks at the completion of the previous group
    for (int dir = 0; dir < 2 && status == TN_OK; ++dir) {
      Slot& sl = ex->slots[ex->n_compute + dir];
      ReadyQueue& r = rq_x[dir];
      const std::vector<int64_t>& serial = ex->serial[1 + dir];
      if ((int)xq[dir].size() >= xdepth || n_ready_x[dir] == 0) continue;
      std::vector<int64_t>& tv = xverts;
      tv.clear();
      copies.n = 0;
      copies.total_blocks = 0;
      // a group whose copies all stay inside GPU memory is not bound by the host link: it gets a
      // launch as wide as the chip instead of the few workgroups that keep the link busy
      bool inside_gpu = any_on_device;
      auto on_gpu = [&](const void* p) {
        for (auto& r : ex->device_ranges)
          if ((const char*)p >= r.first && (const char*)p < r.second) return true;
        return false;
      };
      hipError_t e = hipSuccess;
      // GPU -> host copies can be left to the copy engines of the chip while host -> GPU copies stay with the
      // copy kernel (TN_COPY_KERNEL_IN); copies into a caller's buffer in GPU memory stay with the kernel
      const bool use_copy_kernel = kernel_copies && !(dir == 1 && (opt.copy_engine == TN_COPY_KERNEL_IN || opt.copy_engine == TN_COPY_AUTO) && !any_on_device);
      // ... and then the offloads of a group are gathered into a staging slot and leave as one copy
      const bool staged = dir == 1 && kernel_copies && !use_copy_kernel && ex->stage;
      char* const slot = staged ? ex->stage + (uint64_t)xring[1] * kStageBytes : nullptr;
      uint64_t stage_used = 0;
      stage_verts.clear();
      stage_sizes.clear();
      // copies handed to the runtime one by one are enqueued as the group is put together: their start stamp
      // has to go first (given back below if the group stays empty)
      int early_prof = -1;
      if (!use_copy_kernel && opt.profile && prof_pair(&early_prof)) e = hipEventRecord(ex->prof_events[early_prof], sl.stream);
      // (copies inside GPU memory need no pipelining against the host link: one group takes all that fit)
      while (n_ready_x[dir] > 0 && (int)tv.size() < (inside_gpu && use_copy_kernel ? kMaxCopies : max_xfer) && e == hipSuccess) {
        int64_t m;
        if (in_order) {  // the next transfer of this direction in the serial order, or none
          m = serial[serial_next[1 + dir]];
          if (!is_ready[m]) break;
        } else {
          m = r.peek(rng);
        }
        const MVertex& x = mg.v[m];
        const void* src;
        void* dst;
        if (x.kind == TN_MG_LOAD) {
          src = host_inputs[x.src];
          dst = ex->dbase + x.offset;
          inside_gpu = inside_gpu && on_gpu(src);
        } else if (x.kind == TN_MG_RELOAD) {
          src = ex->arena + ex->arena_off[x.operands[0]];
          dst = ex->dbase + x.offset;
          inside_gpu = false;
        } else if (x.kind == TN_MG_STORE && !(staged && x.bytes <= kStageBytes)) {
          src = ex->dbase + mg.v[x.operands[0]].offset;
          dst = host_outputs[x.output_index];
          inside_gpu = inside_gpu && on_gpu(dst);
        } else if (x.kind == TN_MG_STORE) {  // store by way of the staging slot
          const uint64_t need = (x.bytes + 255) / 256 * 256;
          if (stage_used + need > kStageBytes || copies.n >= kMaxCopies) break;
          copies.it[copies.n++] = {ex->dbase + mg.v[x.operands[0]].offset, slot + stage_used, (uint32_t)x.bytes,
                                   (uint32_t)copies.total_blocks};
          copies.total_blocks += (int32_t)((x.bytes + kCopyBlockBytes - 1) / kCopyBlockBytes);
          stage_used += need;
          stage_verts.push_back(m);
          stage_sizes.push_back(x.bytes);
          src = dst = nullptr;  // moved after the loop
        } else if (staged && ex->arena && x.bytes <= kStageBytes) {  // offload by way of the staging slot
          inside_gpu = false;
          const uint64_t need = (x.bytes + 255) / 256 * 256;
          if (stage_used + need > kStageBytes || copies.n >= kMaxCopies) break;  // the slot is full: the rest goes with the next group
          if (arena_largest_free(*ex) < stage_used + need) {
            if (!tv.empty() || !xq[1].empty()) break;  // what is queued (and later reloads) will free slots
            if (!xq[0].empty() || n_ready_x[0] > 0) break;
            status = fail(TN_ERR_ARENA, "pinned host arena of %llu bytes is exhausted (offload of %llu bytes)",
                          (unsigned long long)ex->arena_bytes, (unsigned long long)x.bytes);
            break;
          }
          copies.it[copies.n++] = {ex->dbase + mg.v[x.operands[0]].offset, slot + stage_used, (uint32_t)x.bytes,
                                   (uint32_t)copies.total_blocks};
          copies.total_blocks += (int32_t)((x.bytes + kCopyBlockBytes - 1) / kCopyBlockBytes);
          stage_used += need;
          stage_verts.push_back(m);
          stage_sizes.push_back(x.bytes);
          arena_used += need;
          rep.arena_high_water = std::max(rep.arena_high_water, arena_used);
          ++rep.n_offload;
          src = dst = nullptr;  // moved after the loop
        } else {  // offload
          inside_gpu = false;
          uint64_t off;
          if (!ex->arena || !arena_alloc(*ex, x.bytes, &off)) {
            if (!tv.empty() || !xq[1].empty()) break;  // let the copies already queued (and later reloads) free slots
            if (!xq[0].empty() || n_ready_x[0] > 0) break;
            status = fail(TN_ERR_ARENA, "pinned host arena of %llu bytes is exhausted (offload of %llu bytes)",
                          (unsigned long long)ex->arena_bytes, (unsigned long long)x.bytes);
            break;
          }
          ex->arena_off[m] = (int64_t)off;
          arena_used += (x.bytes + 255) / 256 * 256;
          rep.arena_high_water = std::max(rep.arena_high_water, arena_used);
          src = ex->dbase + mg.v[x.operands[0]].offset;
          dst = ex->arena + off;
          ++rep.n_offload;
        }
        if (use_copy_kernel) {
          copies.it[copies.n++] = {src, dst, (uint32_t)x.bytes, (uint32_t)copies.total_blocks};
          copies.total_blocks += (int32_t)((x.bytes + kCopyBlockBytes - 1) / kCopyBlockBytes);
        } else if (src) {
          e = hipMemcpyAsync(dst, src, x.bytes,
                             any_on_device ? hipMemcpyDefault : dir == 0 ? hipMemcpyHostToDevice : hipMemcpyDeviceToHost, sl.stream);
          if (e != hipSuccess) break;
        }
        if (in_order) {
          is_ready[m] = 0;
          ++serial_next[1 + dir];
        } else {
          r.pop();
        }
        --n_ready_x[dir];
        tv.push_back(m);
        (dir == 0 ? rep.h2d_bytes : rep.d2h_bytes) += x.bytes;
        rep.n_reload += x.kind == TN_MG_RELOAD;
        ex->last_order.push_back(m);
      }
      if (status != TN_OK) break;
      if (tv.empty() && e == hipSuccess) {
        if (early_prof >= 0) prof_used -= 2;
        continue;
      }
      XGroup xg;
      xg.done = ex->xevents[dir][xring[dir]];
      xring[dir] = (xring[dir] + 1) % kMaxQueueDepth;
      // the start stamp goes after whatever the stream still carries; the group's copies are
      // queued behind it
      if (early_prof >= 0) xg.prof = early_prof;
      else if (e == hipSuccess && opt.profile && prof_pair(&xg.prof)) e = hipEventRecord(ex->prof_events[xg.prof], sl.stream);
      if (e == hipSuccess && use_copy_kernel) {
        const int wgs = inside_gpu ? kDeviceCopyWorkgroups
                        : (dir == 1 && opt.d2h_workgroups > 0) ? opt.d2h_workgroups : opt.copy_workgroups;
        e = launch_copies(copies, wgs, sl.stream);
      }
      if (e == hipSuccess && !stage_verts.empty()) {
        // adjacent arena slots for the gathered offloads (the largest free block was checked to suffice, and
        // nothing has taken from the arena since), the gather inside GPU memory, then one copy to the host per
        // run of tensors whose places in host memory follow one another as their places in the slot do
        stage_run.clear();
        for (size_t k = 0; k < stage_verts.size(); ++k)
          if (mg.v[stage_verts[k]].kind == TN_MG_OFFLOAD) stage_run.push_back(stage_sizes[k]);
        uint64_t at = 0;
        if (!stage_run.empty() && !arena_alloc_run(*ex, stage_run.data(), (int)stage_run.size(), &at)) {
          status = fail(TN_ERR_ARENA, "pinned host arena: no run of adjacent slots for %zu offloads", stage_run.size());
          break;
        }
        // Stores first sorted by where they go in host memory, so that tiles the caller keeps next to each other
        // leave as one copy: a copy engine moves 512 KiB in 12 us and 4 MiB in 75, and between two copies it rests.
        if (stage_verts.size() > 1) {
          const size_t n = stage_verts.size();
          std::vector<size_t>& ord = stage_ord;
          ord.resize(n);
          for (size_t k = 0; k < n; ++k) ord[k] = k;
          auto key = [&](size_t k) -> uintptr_t {
            const MVertex& x = mg.v[stage_verts[k]];
            return x.kind == TN_MG_OFFLOAD ? 0 : (uintptr_t)host_outputs[x.output_index];
          };
          std::stable_sort(ord.begin(), ord.end(), [&](size_t a, size_t b) { return key(a) < key(b); });
          stage_tmp_v.assign(stage_verts.begin(), stage_verts.end());
          stage_tmp_s.assign(stage_sizes.begin(), stage_sizes.end());
          stage_tmp_src.resize(n);
          for (size_t k = 0; k < n; ++k) stage_tmp_src[k] = copies.it[k].src;
          uint64_t pos = 0;
          int32_t blocks = 0;
          for (size_t k = 0; k < n; ++k) {
            const size_t o = ord[k];
            stage_verts[k] = stage_tmp_v[o];
            stage_sizes[k] = stage_tmp_s[o];
            copies.it[k] = {stage_tmp_src[o], slot + pos, (uint32_t)stage_sizes[k], (uint32_t)blocks};
            blocks += (int32_t)((stage_sizes[k] + kCopyBlockBytes - 1) / kCopyBlockBytes);
            pos += (stage_sizes[k] + 255) / 256 * 256;
          }
        }
        e = launch_copies(copies, kStageGatherWorkgroups, sl.stream);
        // A run may cross the padding behind a tensor (sizes are rounded up to 256 bytes in the slot) only where
        // that padding is the library's own, in the arena: bytes between two of the caller's buffers are not ours.
        char* run_dst = nullptr;
        uint64_t run_src = 0, run_bytes = 0, run_pad = 0, in_slot = 0;
        bool pad_is_ours = true;
        auto flush = [&]() {
          if (run_bytes) e = hipMemcpyAsync(run_dst, slot + run_src, run_bytes - run_pad, hipMemcpyDeviceToHost, sl.stream);
          run_bytes = 0;
        };
        for (size_t k = 0; k < stage_verts.size() && e == hipSuccess; ++k) {
          const MVertex& x = mg.v[stage_verts[k]];
          const uint64_t sz = (stage_sizes[k] + 255) / 256 * 256;
          char* dst;
          if (x.kind == TN_MG_OFFLOAD) {
            ex->arena_off[stage_verts[k]] = (int64_t)at;
            dst = ex->arena + at;
            at += sz;
          } else {
            dst = (char*)host_outputs[x.output_index];
          }
          if (run_bytes && !(dst == run_dst + run_bytes && (run_pad == 0 || pad_is_ours))) flush();
          if (e != hipSuccess) break;
          if (!run_bytes) { run_dst = dst; run_src = in_slot; }
          run_bytes += sz;
          run_pad = sz - stage_sizes[k];
          pad_is_ours = x.kind == TN_MG_OFFLOAD;
          in_slot += sz;
        }
        if (e == hipSuccess) flush();
      }
      if (xg.prof >= 0) xg.done = ex->prof_events[xg.prof + 1];
      if (e == hipSuccess) e = hipEventRecord(xg.done, sl.stream);
      if (e != hipSuccess) { hip_fail("transfer", e); break; }
      if (xg.prof >= 0) {
        int64_t moved = 0;
        for (int64_t m : tv) moved += (int64_t)mg.v[m].bytes;
        ex->prof_recs.push_back({3 + dir, xg.prof, (int32_t)tv.size(), moved, (double)moved});
      }
      xg.verts = tv;
      xq[dir].push_back(std::move(xg));
      ++rep.n_launches;
      progressed = true;
    }
    // ---- launch kernels: one group per compute stream with room in its queue ---------------
    while (status == TN_OK && n_ready_k > 0) {
      int si = -1;
      for (int k = 0; k < ex->n_compute; ++k)
        if ((int)ex->cqueue[k].size() < depth && (si < 0 || ex->cqueue[k].size() < ex->cqueue[si].size())) si = k;
      if (si < 0) break;
      hipStream_t stream = ex->slots[si].stream;
      // GEMM groups that overlap only share the compute units; holding the next one back until a
      // running one ends lets it gather more ready tiles and fill the chip on its own
      bool gemm_ok = true;
      if (opt.max_gemm_inflight > 0 && !in_order) {
        int inflight = 0;
        for (auto& q : ex->cqueue)
          for (auto& g : q) inflight += g.family == 0;
        gemm_ok = inflight < opt.max_gemm_inflight;
      }
      same.clear();
      int gi = -1;  // launch group of the lead vertex
      if (in_order) {
        // the next kernel of the serial order leads; the kernels right behind it join while they
        // are ready and of its launch group
        const std::vector<int64_t>& serial = ex->serial[0];
        size_t at = serial_next[0];
        if (!is_ready[serial[at]]) break;
        if (ex->info[serial[at]].lock >= 0 && lock_busy[ex->info[serial[at]].lock]) break;
        gi = ex->info[serial[at]].group;
        uint32_t lo = (uint32_t)ex->info[serial[at]].desc, hi = lo;
        while (at < serial.size() && (int)same.size() < max_batch && is_ready[serial[at]] &&
               ex->info[serial[at]].group == gi) {
          const uint32_t d = (uint32_t)ex->info[serial[at]].desc;
          if (std::max(hi, d) - std::min(lo, d) > kMaxBatchSpan) break;
          if (const int64_t lk = ex->info[serial[at]].lock; lk >= 0) {
            if (lock_busy[lk]) break;
            lock_busy[lk] = 1;
          }
          lo = std::min(lo, d);
          hi = std::max(hi, d);
          is_ready[serial[at]] = 0;
          same.push_back(serial[at++]);
        }
        serial_next[0] = at;
      } else {
        // lead: what the policy would take first among all ready kernels
        uint64_t total = 0;
        for (size_t g = 0; g < n_groups; ++g) {
          if (rq[g].empty() || (!gemm_ok && family_of(ex->groups[g].cls) == 0)) continue;
          total += rq[g].size();
          if (gi < 0) { gi = (int)g; continue; }
          switch (opt.policy) {
            case TN_POLICY_FIFO: if (arrival[rq[g].q.front()] < arrival[rq[gi].q.front()]) gi = (int)g; break;
            case TN_POLICY_LIFO: if (arrival[rq[g].q.back()] > arrival[rq[gi].q.back()]) gi = (int)g; break;
            case TN_POLICY_BY_ORDER: if (ex->order_key[rq[g].v.front()] < ex->order_key[rq[gi].v.front()]) gi = (int)g; break;
            default: break;
          }
        }
        if (gi < 0) break;  // only GEMMs are ready and enough of them are running
        if (opt.policy == TN_POLICY_RANDOM) {  // a ready kernel drawn uniformly decides the group
          rng = mix64(rng);
          uint64_t pick = rng % total;
          for (size_t g = 0; g < n_groups; ++g) {
            if (rq[g].empty() || (!gemm_ok && family_of(ex->groups[g].cls) == 0)) continue;
            if (pick < rq[g].size()) { gi = (int)g; break; }
            pick -= rq[g].size();
          }
        }
        // the group: ready vertices of the lead's launch group, in the policy's order; a launch
        // names its vertices by 16-bit offsets from the smallest descriptor index
        ReadyQueue& q = rq[gi];
        uint32_t lo = 0, hi = 0;
        while (!q.empty() && (int)same.size() < max_batch) {
          const int64_t m = q.peek(rng);
          const int64_t lk = ex->info[m].lock;
          if (lk >= 0 && lock_busy[lk]) {  // its output is being added to: wait for the lock
            q.pop();
            lock_wait[lk].push_back(m);
            --n_ready_k;
            continue;
          }
          const uint32_t d = (uint32_t)ex->info[m].desc;
          if (same.empty()) lo = hi = d;
          if (std::max(hi, d) - std::min(lo, d) > kMaxBatchSpan) break;
          lo = std::min(lo, d);
          hi = std::max(hi, d);
          q.pop();
          if (lk >= 0) lock_busy[lk] = 1;
          same.push_back(m);
        }
        if (same.empty()) continue;  // everything looked at waits for a lock
      }
      n_ready_k -= (int64_t)same.size();
      const VInfo lead = ex->groups[gi];
      // The workgroups of a launch run in the order of its vertices, and those of one XCD (one L2)
      // take a contiguous run of them.  Arrange the tile products so that vertices next to each
      // other share operands both ways -- blocks of two A row panels by four B column panels --
      // instead of one A panel against every B panel of the launch.
      if (lead.cls == LC_GEMM_BF16_NT256 && same.size() >= 16) {
        auto b0 = [&](int64_t m) { return mg.v[m].operands[mg.v[m].p.nk]; };
        std::vector<int64_t>& bs = sort_b;
        bs.clear();
        for (int64_t m : same) bs.push_back(b0(m));
        std::sort(bs.begin(), bs.end());
        bs.erase(std::unique(bs.begin(), bs.end()), bs.end());
        sort_keys.clear();  // (block of four B panels, A panel, B panel, position in the policy's order)
        for (size_t k = 0; k < same.size(); ++k) {
          const int64_t rb = (int64_t)(std::lower_bound(bs.begin(), bs.end(), b0(same[k])) - bs.begin());
          sort_keys.push_back({rb / 4, mg.v[same[k]].operands[0], rb, (int64_t)k});
        }
        std::sort(sort_keys.begin(), sort_keys.end());
        sort_b.resize(same.size());
        for (size_t k = 0; k < same.size(); ++k) sort_b[k] = same[(size_t)sort_keys[k][3]];
        same.swap(sort_b);
      }
      batch.n = (int32_t)same.size();
      batch.base = (uint32_t)ex->info[same[0]].desc;
      for (int64_t m : same) batch.base = std::min(batch.base, (uint32_t)ex->info[m].desc);
      int32_t max_blocks = 0;
      int64_t n_blocks = 0;
      double flops = 0, bytes = 0;
      for (int k = 0; k < batch.n; ++k) {
        const VInfo& v = ex->info[same[k]];
        batch.idx[k] = (uint16_t)(v.desc - batch.base);
        max_blocks = std::max(max_blocks, v.nblocks);
        n_blocks += v.nblocks;
        flops += v.flops;
        bytes += v.bytes;
      }
      hipError_t e = hipSuccess;
      // device-side waits for kernels this group depends on that are enqueued on other streams
      if (ahead) {
        waited.clear();
        for (int64_t m : same)
          for (int64_t i = ex->pred_start[m]; i < ex->pred_start[m + 1] && e == hipSuccess; ++i) {
            const int64_t pv = ex->pred[i];
            if (state[pv] != 1 || stream_of[pv] == si) continue;
            if (std::find(waited.begin(), waited.end(), ev_of[pv]) != waited.end()) continue;
            waited.push_back(ev_of[pv]);
            e = hipStreamWaitEvent(stream, ev_of[pv], 0);
          }
      }
      Group grp;
      grp.family = family_of(lead.cls);
      grp.done = ex->cevents[si][ring_next[si]];
      ring_next[si] = (ring_next[si] + 1) % kMaxQueueDepth;
      if (e == hipSuccess && opt.profile && prof_pair(&grp.prof)) e = hipEventRecord(ex->prof_events[grp.prof], stream);
      // A group of tile products with at most kSmallGemmTiles 256x256 tiles leaves CUs without work for as long
      // as one tile takes; cut into 128x128 tiles (at most four per 256x256 tile, two workgroups per CU) it is
      // spread over four times as many workgroups that all run at once.  The bits do not depend on the form.
      int launch_cls = lead.cls;
      if (lead.cls == LC_GEMM_BF16_NT256 && n_blocks <= (opt.small_gemm_tiles > 0 ? opt.small_gemm_tiles : opt.small_gemm_tiles < 0 ? 0 : kSmallGemmTiles)) {
        launch_cls = LC_GEMM_BF16_NT256_SMALL;
        max_blocks *= 4;
        n_blocks *= 4;
      }
      if (e == hipSuccess) e = launch_batch(launch_cls, lead.dtype, lead.head_dim, tables, batch, max_blocks, stream);
      // a timed launch completes with its second stamp: one event record less between two kernels
      if (grp.prof >= 0) grp.done = ex->prof_events[grp.prof + 1];
      if (e == hipSuccess) e = hipEventRecord(grp.done, stream);
      if (e != hipSuccess) { hip_fail("kernel launch", e); break; }
      for (int64_t m : same) {
        ex->last_order.push_back(m);
        state[m] = 1;
        ev_of[m] = grp.done;
        stream_of[m] = (int8_t)si;
      }
      if (ahead)  // kernels that only waited for these to be enqueued can follow
        for (int64_t m : same)
          for (int64_t i = ex->succ_start[m]; i < ex->succ_start[m + 1]; ++i) {
            const int64_t w = ex->succ[i];
            if (mg.v[w].kind == TN_MG_OP && --rem_enq[w] == 0) make_ready(w);
          }
      ++rep.n_launches;
      ++rep.n_kernel_launches;
      if (grp.family == 0) { ++rep.gemm_launches; rep.gemm_flops += flops; }
      else if (grp.family == 1) { ++rep.attn_launches; rep.attn_flops += flops; }
      else { ++rep.ewise_launches; rep.ewise_bytes += bytes; }
      if (grp.prof >= 0) ex->prof_recs.push_back({grp.family, grp.prof, batch.n, n_blocks, grp.family == 2 ? bytes : flops});
      grp.verts = same;
      ex->cqueue[si].push_back(std::move(grp));
      progressed = true;
    }
    if (status != TN_OK) break;
    // ---- completions -----------------------------------------------------------------------
    for (int si = 0; si < ex->n_compute && status == TN_OK; ++si) {
      auto& q = ex->cqueue[si];
      while (!q.empty()) {  // a stream finishes its groups in order
        hipError_t e = hipEventQuery(q.front().done);
        if (e == hipErrorNotReady) break;
        if (e != hipSuccess) { hip_fail("hipEventQuery", e); break; }
        Group g = std::move(q.front());
        q.pop_front();
        for (int64_t m : g.verts) complete(m);
        progressed = true;
      }
    }
    for (int dir = 0; dir < 2 && status == TN_OK; ++dir) {
      while (!xq[dir].empty()) {  // a stream finishes its groups in order
        XGroup& g = xq[dir].front();
        if (!g.event_seen) {
          hipError_t e = hipEventQuery(g.done);
          if (e == hipErrorNotReady) break;
          if (e != hipSuccess) { hip_fail("hipEventQuery", e); break; }
          g.event_seen = true;
          g.release = Clock::now();
          if (opt.max_delay_us) {
            // injected transfer delay: the completion is reported late; the copy itself ran normally
            const uint64_t us = mix64(opt.delay_seed ^ (uint64_t)g.verts[0] * 0x9E3779B1ull) % (opt.max_delay_us + 1ull);
            g.release += std::chrono::microseconds(us);
          }
        }
        if (Clock::now() < g.release) break;
        XGroup done = std::move(g);
        xq[dir].pop_front();
        for (int64_t m : done.verts) {
          const MVertex& x = mg.v[m];
          if (x.kind == TN_MG_RELOAD) {
            const int64_t o = x.operands[0];
            arena_free(*ex, (uint64_t)ex->arena_off[o]);
            arena_used -= (mg.v[o].bytes + 255) / 256 * 256;
            ex->arena_off[o] = -1;
          }
          complete(m);
        }
        progressed = true;
      }
    }
    if (!progressed) {
      bool any_busy = false;
      any_busy = !xq[0].empty() || !xq[1].empty();
      for (auto& q : ex->cqueue) any_busy |= !q.empty();
      if (!any_busy && n_ready_k == 0 && n_ready_x[0] == 0 && n_ready_x[1] == 0 && completed < nv) {
        status = fail(TN_ERR_CYCLE, "no vertex is ready and none is running: %lld of %lld completed",
                      (long long)completed, (long long)nv);
        break;
      }
    }
  }
  // drain whatever is still in flight (error paths): every stream the run used is idle on return
  for (int dir = 0; dir < 2; ++dir)
    if (!xq[dir].empty()) {
      (void)hipStreamSynchronize(ex->slots[ex->n_compute + dir].stream);
      xq[dir].clear();
    }
  for (int si = 0; si < ex->n_compute; ++si)
    if (!ex->cqueue[si].empty()) {
      (void)hipStreamSynchronize(ex->slots[si].stream);
      ex->cqueue[si].clear();
    }
  rep.wall_ms = std::chrono::duration<double, std::milli>(Clock::now() - t_start).count();
  rep.n_vertices = completed;
  if (status == TN_OK && opt.profile) {
    // device time per family and the union of kernel intervals
    std::vector<std::pair<float, float>> iv;
    for (const auto& r : ex->prof_recs) {
      const int fam = r.family, p = r.prof;
      float t0 = 0, t1 = 0;
      if (hipEventElapsedTime(&t0, prof_base, ex->prof_events[p]) != hipSuccess ||
          hipEventElapsedTime(&t1, prof_base, ex->prof_events[p + 1]) != hipSuccess)
        continue;
      ex->launch_log.push_back({r.family, r.n_vertices, r.work, r.amount, t0, t1});
      if (fam >= 3) {  // transfers: time per direction, not part of the kernel-busy union
        (fam == 3 ? rep.h2d_ms : rep.d2h_ms) += t1 - t0;
        continue;
      }
      (fam == 0 ? rep.gemm_ms : fam == 1 ? rep.attn_ms : rep.ewise_ms) += t1 - t0;
      iv.emplace_back(t0, t1);
    }
    std::sort(iv.begin(), iv.end());
    float lo = 0, hi = -1, first = 0, last = 0;
    for (size_t k = 0; k < iv.size(); ++k) {
      if (k == 0) { first = iv[0].first; lo = iv[0].first; hi = iv[0].second; }
      else if (iv[k].first <= hi) hi = std::max(hi, iv[k].second);
      else { rep.kernel_busy_ms += hi - lo; lo = iv[k].first; hi = iv[k].second; }
      last = std::max(last, iv[k].second);
    }
    if (!iv.empty()) {
      rep.kernel_busy_ms += hi - lo;
      const double span = std::max<double>(last - first, 1e-9);
      rep.idle_frac = 1.0 - rep.kernel_busy_ms / span;
      rep.idle_frac_wall = std::max(0.0, 1.0 - rep.kernel_busy_ms / std::max(rep.wall_ms, 1e-9));
    }
  }
  if (report) *report = rep;
  return status;
}

tn_status tn_execute(tn_executor* ex, const void* const* host_inputs, void* const* host_outputs,
                     const tn_exec_opts* opts, tn_exec_report* report) {
  if (!ex) return fail(TN_ERR_INVALID, "NULL executor");
  if (ex->poisoned) return fail(TN_ERR_HIP, "executor is poisoned by an earlier HIP error");
  return run_memgraph(ex, host_inputs, host_outputs, opts, report, ex->tables);
}

tn_status tn_execute_static(tn_executor* ex, const void* const* host_inputs, void* const* host_outputs,
                            const tn_exec_opts* opts, tn_exec_report* report) {
  if (!ex) return fail(TN_ERR_INVALID, "NULL executor");
  if (ex->poisoned) return fail(TN_ERR_HIP, "executor is poisoned by an earlier HIP error");
  if (ex->image_bytes > kStaticTableBytes)
    return fail(TN_ERR_INVALID, "the operand tables of this memgraph take %llu bytes; the static table region holds %llu",
                (unsigned long long)ex->image_bytes, (unsigned long long)kStaticTableBytes);
  char* region = nullptr;
  hipError_t e = static_table_region((void**)&region);
  if (e != hipSuccess) return fail(TN_ERR_HIP, "address of the static table region: %s", hipGetErrorString(e));
  // The region keeps whatever the last call on this GPU left there; this call's kernels read only
  // [0, image_bytes), all of which is written here, and nothing else has to start from zero.  The
  // upload is complete before the first kernel is enqueued on any stream.
  hipStream_t s0 = ex->slots[0].stream;
  e = hipMemcpyAsync(region, ex->h_image, ex->image_bytes, hipMemcpyHostToDevice, s0);
  if (e == hipSuccess) e = hipStreamSynchronize(s0);
  if (e != hipSuccess) {
    ex->poisoned = true;
    return fail(TN_ERR_HIP, "upload of the operand tables: %s", hipGetErrorString(e));
  }
  return run_memgraph(ex, host_inputs, host_outputs, opts, report, tables_at(*ex, region));
}

int64_t tn_executor_last_order(const tn_executor* ex, int64_t* out, int64_t cap) {
  if (!ex) return TN_ERR_INVALID;
  const int64_t n = (int64_t)ex->last_order.size();
  for (int64_t i = 0; i < n && i < cap; ++i) out[i] = ex->last_order[i];
  return n;
}

int64_t tn_executor_last_launches(const tn_executor* ex, tn_launch_record* out, int64_t cap) {
  if (!ex) return fail(TN_ERR_INVALID, "NULL executor");
  const int64_t n = (int64_t)ex->launch_log.size();
  for (int64_t i = 0; out && i < cap && i < n; ++i) out[i] = ex->launch_log[(size_t)i];
  return n;
}

}  // extern "C"
