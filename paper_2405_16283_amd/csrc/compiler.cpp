// BuildMemgraph: compile a taskgraph into a memgraph for a given amount of GPU memory.
//
// Section 6 (Algorithms 1 and 2): simulate a serial execution of the taskgraph with a simulated
// malloc/free; two horizons walk the serial order V -- allocHzn (everything before it has a
// location) runs greedily ahead of execHzn (everything before it has been "run"); a failed
// allocation for the vertex that must run next evicts a victim (offload now, reload before its
// next use); a location that is reused gets memory dependencies from every reader of its
// previous occupant.  Section 7: inserted offloads and reloads sit just before the vertex that
// caused them, offloads first, so every edge points forward in the extended serial order.
//
// The paper presents the uniform case (one slot per tensor) and says variably-sized tensors
// only mean that one allocation may evict several victims.  This file is that general case:
// a byte-addressed first-fit allocator over [0, cap), an interval map of the last dead occupant
// of every byte, and victim *windows* of adjacent blocks.
//
// Appendix A (resources): a vertex that sums n tensors runs as n increment kernels into an output
// protected by a write lock.  Here the output gets its location when the first operand has been
// produced (a vertex that clears it; the memory dependencies of the location point there), every
// operand is added by an increment vertex placed right after its producer -- so a partial product
// lives only until it has been added -- and the sum vertex itself is a join that runs after all
// increments and then stands for the tensor.  Until the join the output cannot be evicted: an
// increment that came late in some execution order would otherwise write to a stale location.
#include <algorithm>
#include <climits>
#include <cstring>
#include <map>
#include <set>
#include <unordered_set>

#include "graph.h"

namespace tn {
namespace {

constexpr uint64_t kSmallTensor = 64 * 1024;  // tensors below this size are packed at the top end

struct Block {
  uint64_t size;
  int64_t owner;  // memgraph vertex occupying it, or -1 if free
};

struct Compiler {
  const TaskGraph& tg;
  const tn_compile_opts& opt;
  MemGraph& mg;
  const int64_t n;
  uint64_t align, cap;

  std::vector<tn_vid> V;
  std::vector<int64_t> pos;                 // position of a taskgraph vertex in V
  std::vector<std::vector<int64_t>> cons;   // consumer positions per tensor, ascending
  std::vector<size_t> cons_ptr;             // first entry of cons[t] that is >= execHzn
  std::vector<int64_t> name;                // current GPU incarnation of tensor t, or -1
  std::vector<int64_t> evicted_by;          // offload/drop vertex holding tensor t while it is out
  std::vector<std::vector<int64_t>> readers;  // per memgraph vertex: who has read its output so far
  std::vector<std::vector<size_t>> malloc_edges;  // per memgraph vertex: edges its allocation added
  std::vector<char> edge_dead;
  std::vector<char> counted_ahead;  // per memgraph vertex: its allocation counts as run-ahead
  std::unordered_set<uint64_t> edge_set[3];
  std::map<uint64_t, Block> blocks;                          // offset -> block, covers [0, cap)
  std::map<uint64_t, std::pair<uint64_t, int64_t>> history;  // offset -> (end, last dead occupant)
  // tensors that hold data on the GPU, ordered by their next use: the eviction candidates
  std::set<std::pair<int64_t, tn_vid>> by_use;
  std::vector<int64_t> use_key;  // key under which tensor t is in by_use, or -1
  std::map<uint64_t, uint64_t> free_at;                      // the free blocks alone: offset -> size
  std::map<uint64_t, std::set<uint64_t>> free_by_size;       // size -> offsets of the free blocks of that size
  int64_t execHzn = 0, allocHzn = 0, lookahead_blocked_until = -1, compacted_at = -1;
  uint64_t lookahead_bytes = 0, live_bytes = 0, cursor = 0;
  std::vector<int64_t> step_pre;  // offloads and reloads inserted just before V[execHzn], in the order made
  std::vector<std::vector<tn_vid>> sums_of;     // per tensor: the sum vertices it is an operand of
  std::vector<int64_t> acc_of;                  // per sum vertex: the vertex that clears its output, or -1
  std::vector<std::vector<int64_t>> incs_of;    // per sum vertex: its increments so far
  std::vector<char> open_acc;                   // per memgraph vertex: an output still being summed into
  // The allocations in the order allocHzn takes them: the output of every vertex of V that needs
  // one (entry = the vertex), and right after the first operand of a sum the sum's output
  // (entry = ~sum vertex).  Device-resident inputs are placed before anything else and sums have
  // no allocation of their own, so neither appears.
  std::vector<int64_t> A;
  std::vector<int64_t> apos;        // per taskgraph vertex: index of its own entry in A, or -1
  std::vector<int64_t> apos_acc;    // per sum vertex: index of its output's entry in A
  std::vector<int64_t> owner_pos;   // per entry of A: position in V of the vertex after whose run it is needed
  std::vector<char> zero_placed;    // per sum vertex: its clearing vertex has a place in the extended order

  Compiler(const TaskGraph& t, const tn_compile_opts& o, MemGraph& m)
      : tg(t), opt(o), mg(m), n((int64_t)t.v.size()) {}

  uint64_t aligned(uint64_t b) const { return (b + align - 1) / align * align; }
  uint64_t vbytes(int64_t m) const { return aligned(mg.v[m].bytes); }

  // ---- graph bookkeeping ---------------------------------------------------------------
  int64_t new_vertex(int32_t kind, tn_vid src) {
    MVertex x;
    x.kind = kind;
    x.src = src;
    x.desc = tg.v[src].desc;
    x.bytes = tensor_bytes(x.desc);
    mg.v.push_back(std::move(x));
    readers.emplace_back();
    malloc_edges.emplace_back();
    open_acc.push_back(0);
    counted_ahead.push_back(0);
    return (int64_t)mg.v.size() - 1;
  }

  bool add_edge(int64_t a, int64_t b, int32_t kind, bool from_malloc) {
    if (a == b) return false;
    uint64_t key = ((uint64_t)a << 32) | (uint64_t)b;
    if (!edge_set[kind].insert(key).second) return false;
    mg.edges.push_back({a, b, kind});
    edge_dead.push_back(0);
    if (from_malloc) malloc_edges[b].push_back(mg.edges.size() - 1);
    return true;
  }

  int64_t next_use(tn_vid t) {
    auto& c = cons[t];
    size_t& p = cons_ptr[t];
    while (p < c.size() && c[p] < execHzn) ++p;
    return p < c.size() ? c[p] : LLONG_MAX;
  }

  bool produced(int64_t m) const { return m >= n ? !open_acc[m] : pos[m] < execHzn; }
  bool is_sum(tn_vid v) const { return tg.v[v].kind == TN_OP_SUM; }

  void use_erase(tn_vid t) {
    if (use_key[t] >= 0) by_use.erase({use_key[t], t});
    use_key[t] = -1;
  }
  // (re-)enters tensor t, resident and holding data, under its current next use
  void use_insert(tn_vid t) {
    use_erase(t);
    // tiny tensors (statistics, low-rank activations) are not worth evicting for a tile; they stay
    // out of the candidate list and are only ever moved by the exhaustive search
    if (aligned(tensor_bytes(tg.v[t].desc)) < kSmallTensor) return;
    use_key[t] = next_use(t);
    by_use.insert({use_key[t], t});
  }

  // ---- simulated memory ------------------------------------------------------------------
  void free_add(uint64_t off, uint64_t size) {
    free_at[off] = size;
    free_by_size[size].insert(off);
  }
  void free_del(uint64_t off, uint64_t size) {
    free_at.erase(off);
    auto it = free_by_size.find(size);
    it->second.erase(off);
    if (it->second.empty()) free_by_size.erase(it);
  }

  // `it` has just become free: merge it with free neighbours and enter the result in the index
  void coalesce(std::map<uint64_t, Block>::iterator it) {
    auto nx = std::next(it);
    if (nx != blocks.end() && nx->second.owner < 0) {
      free_del(nx->first, nx->second.size);
      it->second.size += nx->second.size;
      blocks.erase(nx);
    }
    if (it != blocks.begin()) {
      auto pv = std::prev(it);
      if (pv->second.owner < 0) {
        free_del(pv->first, pv->second.size);
        pv->second.size += it->second.size;
        blocks.erase(it);
        it = pv;
      }
    }
    free_add(it->first, it->second.size);
  }

  void history_set(uint64_t a, uint64_t b, int64_t owner) {
    // overwrite [a, b) in the interval map
    auto it = history.lower_bound(a);
    if (it != history.begin()) {
      auto pv = std::prev(it);
      if (pv->second.first > a) {  // straddles a
        auto tail = pv->second;
        pv->second.first = a;
        if (tail.first > b) history[b] = tail;
      }
    }
    it = history.lower_bound(a);
    while (it != history.end() && it->first < b) {
      if (it->second.first > b) {
        history[b] = it->second;
      }
      it = history.erase(it);
    }
    history[a] = {b, owner};
  }

  // place vertex m at [off, off+size) inside the free block `it`; simMalloc's second half: add
  // a memory dependency from every reader of each previous occupant of those bytes
  void place(std::map<uint64_t, Block>::iterator it, uint64_t off, int64_t m) {
    const uint64_t size = vbytes(m), b0 = it->first, bsz = it->second.size;
    blocks.erase(it);
    free_del(b0, bsz);
    if (off > b0) {
      blocks[b0] = {off - b0, -1};
      free_add(b0, off - b0);
    }
    blocks[off] = {size, m};
    if (off + size < b0 + bsz) {
      blocks[off + size] = {b0 + bsz - off - size, -1};
      free_add(off + size, b0 + bsz - off - size);
    }
    mg.v[m].offset = (int64_t)off;
    live_bytes += size;
    mg.stats.peak_live_bytes = std::max(mg.stats.peak_live_bytes, live_bytes);
    mg.stats.high_water = std::max(mg.stats.high_water, off + size);
    auto h = history.upper_bound(off);
    if (h != history.begin()) --h;
    for (; h != history.end() && h->first < off + size; ++h) {
      if (h->second.first <= off) continue;
      const int64_t prev = h->second.second;
      if (readers[prev].empty()) {
        add_edge(prev, m, TN_EDGE_MEM, true);
      } else {
        for (int64_t r : readers[prev]) add_edge(r, m, TN_EDGE_MEM, true);
      }
    }
  }

  // simMalloc: find an open range or fail
  bool sim_malloc(int64_t m) {
    const uint64_t size = vbytes(m);
    // first fit = the lowest (for small tensors: the highest) address among the free blocks that
    // are large enough; free blocks come in few distinct sizes, so the search goes size by size
    auto from = free_by_size.lower_bound(size);
    if (from == free_by_size.end()) return false;
    if (size >= kSmallTensor) {
      uint64_t best = UINT64_MAX;
      if (opt.next_fit) {  // lowest address at or above the cursor, else wrap round
        for (auto it = from; it != free_by_size.end(); ++it) {
          auto lb = it->second.lower_bound(cursor);
          if (lb != it->second.end()) best = std::min(best, *lb);
        }
      }
      if (best == UINT64_MAX)
        for (auto it = from; it != free_by_size.end(); ++it) best = std::min(best, *it->second.begin());
      cursor = best + size;
      place(blocks.find(best), best, m);
    } else {  // at the top end of the highest hole
      uint64_t best = 0, bsz = 0;
      for (auto it = from; it != free_by_size.end(); ++it)
        if (bsz == 0 || *it->second.rbegin() > best) {
          best = *it->second.rbegin();
          bsz = it->first;
        }
      place(blocks.find(best), best + bsz - size, m);
    }
    return true;
  }

  // simFree: the range becomes open and remembers its occupant
  void sim_free(int64_t m) {
    auto it = blocks.find((uint64_t)mg.v[m].offset);
    const uint64_t size = it->second.size;
    it->second.owner = -1;
    live_bytes -= size;
    history_set(it->first, it->first + size, m);
    coalesce(it);
  }

  // take back an allocation whose range was never written: no history is recorded and the
  // memory dependencies the allocation added are withdrawn
  void unplace(int64_t m) {
    auto it = blocks.find((uint64_t)mg.v[m].offset);
    it->second.owner = -1;
    live_bytes -= it->second.size;
    if (counted_ahead[m]) lookahead_bytes -= it->second.size;
    counted_ahead[m] = 0;
    coalesce(it);
    mg.v[m].offset = -1;
    for (size_t e : malloc_edges[m]) {
      edge_dead[e] = 1;
      edge_set[mg.edges[e].kind].erase(((uint64_t)mg.edges[e].from << 32) | (uint64_t)mg.edges[e].to);
    }
    malloc_edges[m].clear();
  }

  // undo the newest run-ahead allocation (Algorithm 1 does not say what to do when memory is
  // full of locations reserved for results that do not exist yet; they cannot be offloaded)
  bool revoke_newest_preallocation() {
    if (allocHzn == 0 || owner_pos[allocHzn - 1] <= execHzn) return false;
    --allocHzn;
    unplace(entry_vertex(allocHzn));
    ++mg.stats.n_revoked;
    lookahead_blocked_until = execHzn + 1;
    return true;
  }

  // the memgraph vertex that owns the allocation A[i]; a sum's clearing vertex is made on first use
  int64_t entry_vertex(int64_t i) {
    if (A[i] >= 0) return A[i];
    const tn_vid s = (tn_vid)~A[i];
    if (acc_of[s] < 0) {
      acc_of[s] = new_vertex(TN_MG_OP, s);
      mg.v[acc_of[s]].op_kind = TN_OP_ZERO;
      open_acc[acc_of[s]] = 1;
    }
    return acc_of[s];
  }

  // Last resort against fragmentation: pinned operands scattered over memory can leave no hole
  // for m although the bytes would suffice.  Empty the memory (offload everything that holds
  // data, take back every reservation), then place the output of the vertex about to run and m
  // into the empty space.  The remaining operands are reloaded by the caller, compactly.
  // Guarantees that cap >= (sum of a vertex's operands + its output) always compiles.
  tn_status compact_and_place(int64_t m) {
    const tn_vid v = V[execHzn];
    while (revoke_newest_preallocation()) {}
    std::vector<int64_t> resident;
    for (auto& b : blocks)
      if (b.second.owner >= 0 && produced(b.second.owner)) resident.push_back(b.second.owner);
    for (int64_t w : resident) evict(w);
    const bool had_output = mg.v[v].offset >= 0;
    if (had_output) unplace(v);
    ++mg.stats.n_compactions;
    if ((had_output || m == v) && !sim_malloc(v)) return TN_ERR_CAP_TOO_SMALL;
    if (m != v && !sim_malloc(m)) return TN_ERR_CAP_TOO_SMALL;
    return TN_OK;
  }

  void evict(int64_t victim) {
    const tn_vid t = mg.v[victim].src;
    const bool clean = opt.drop_clean_inputs && mg.v[victim].kind == TN_MG_LOAD;
    const int64_t off = new_vertex(clean ? TN_MG_DROP : TN_MG_OFFLOAD, t);
    mg.v[off].operands = {victim};
    add_edge(victim, off, TN_EDGE_DATA, false);
    readers[victim].push_back(off);  // the offload reads the range; it precedes whoever takes it
    step_pre.push_back(off);
    sim_free(victim);
    use_erase(t);
    name[t] = -1;
    evicted_by[t] = off;
  }

  // evict more than the allocation at hand needs (tn_compile_opts::evict_ahead_bytes)
  void evict_ahead(const std::vector<int64_t>& pinned) {
    if (!opt.evict_ahead_bytes) return;
    // only what is not needed for a long while: a sixteenth of the serial order, 30000 vertices at most
    const int64_t kFarAhead = std::min<int64_t>(30000, n / 16);
    uint64_t freed = 0;
    std::vector<int64_t> victims;
    for (auto c = by_use.rbegin(); c != by_use.rend() && freed < opt.evict_ahead_bytes; ++c) {
      if (c->first - execHzn < kFarAhead) break;
      const int64_t w = name[c->second];
      if (w < 0 || !produced(w) || std::binary_search(pinned.begin(), pinned.end(), w)) continue;
      victims.push_back(w);
      freed += vbytes(w);
    }
    for (int64_t w : victims) evict(w);
  }

  // simMallocOffld: make room by evicting a window of adjacent blocks, none of them pinned
  tn_status sim_malloc_offld(int64_t m, const std::vector<int64_t>& pinned) {
    const uint64_t size = vbytes(m);
    auto evictable = [&](int64_t o) {
      return produced(o) && !std::binary_search(pinned.begin(), pinned.end(), o);
    };
    for (;;) {
      if (sim_malloc(m)) return TN_OK;
      // best window: furthest minimum next use, then fewest evicted bytes, then lowest address
      bool found = false;
      uint64_t best_start = 0, best_bytes = 0;
      int64_t best_use = -1;
      // Shortcut: instead of trying every window of memory, grow a window around each of the
      // candidates with the furthest next use -- towards the neighbour that is free or, failing
      // that, the evictable neighbour that is needed later -- and keep the best of these.  Only
      // if none of them can be grown to `size` is every window tried.
      int looked = 0;
      for (auto c = by_use.rbegin(); c != by_use.rend() && looked < 64; ++c, ++looked) {
        const int64_t w = name[c->second];
        if (w < 0 || !evictable(w)) continue;
        if (found && c->first <= best_use) break;  // no later candidate can beat the window we have
        auto lo = blocks.find((uint64_t)mg.v[w].offset), hi = lo;  // window = [lo, hi]
        uint64_t total = lo->second.size, ev_bytes = total;
        int64_t min_use = c->first;
        auto usable = [&](std::map<uint64_t, Block>::iterator b, int64_t* use) {
          if (b->second.owner < 0) { *use = LLONG_MAX; return true; }
          if (!evictable(b->second.owner)) return false;
          *use = next_use(mg.v[b->second.owner].src);
          return true;
        };
        int steps = 0;  // a window of many tiny tensors is not worth its transfers: give up on it
        while (total < size && ++steps <= 16) {
          int64_t ul = -1, ur = -1;
          const bool okl = lo != blocks.begin() && usable(std::prev(lo), &ul);
          auto nx = std::next(hi);
          const bool okr = nx != blocks.end() && usable(nx, &ur);
          if (!okl && !okr) break;
          if (okl && (!okr || ul >= ur)) {
            --lo;
            if (lo->second.owner >= 0) ev_bytes += lo->second.size;
            min_use = std::min(min_use, ul);
            total += lo->second.size;
          } else {
            hi = nx;
            if (hi->second.owner >= 0) ev_bytes += hi->second.size;
            min_use = std::min(min_use, ur);
            total += hi->second.size;
          }
        }
        if (total < size) continue;
        // free neighbours below the window belong to the hole that eviction will leave
        if (!found || min_use > best_use || (min_use == best_use && ev_bytes < best_bytes)) {
          found = true;
          best_start = lo->first;
          best_bytes = ev_bytes;
          best_use = min_use;
        }
      }
      const bool shortcut = found;
      for (auto i = blocks.begin(); i != blocks.end() && !shortcut; ++i) {
        uint64_t total = 0, ev_bytes = 0;
        int64_t min_use = LLONG_MAX;
        for (auto j = i; j != blocks.end(); ++j) {
          if (j->second.owner >= 0) {
            if (!evictable(j->second.owner)) break;
            ev_bytes += j->second.size;
            min_use = std::min(min_use, next_use(mg.v[j->second.owner].src));
          }
          total += j->second.size;
          if (total >= size) {
            if (!found || min_use > best_use || (min_use == best_use && ev_bytes < best_bytes)) {
              found = true;
              best_start = i->first;
              best_bytes = ev_bytes;
              best_use = min_use;
            }
            break;
          }
        }
      }
      if (found) {
        std::vector<int64_t> victims;
        uint64_t total = 0;
        for (auto j = blocks.find(best_start); total < size; ++j) {
          if (j->second.owner >= 0) victims.push_back(j->second.owner);
          total += j->second.size;
        }
        for (int64_t w : victims) evict(w);
        auto it = blocks.upper_bound(best_start);
        --it;  // the coalesced free block containing the window
        // small tensors go to the top end of the hole, like sim_malloc does
        uint64_t off = size >= kSmallTensor ? std::max(it->first, best_start)
                                            : it->first + it->second.size - size;
        if (off < it->first || off + size > it->first + it->second.size) off = it->first;
        place(it, off, m);
        evict_ahead(pinned);
        return TN_OK;
      }
      // nothing can be evicted to make room: take back reservations made ahead of the execution,
      // as many as it takes to free `size` bytes, and try again
      uint64_t before = live_bytes;
      bool revoked = false;
      while (revoke_newest_preallocation()) {
        revoked = true;
        if (before - live_bytes >= size) break;
      }
      if (!revoked) {
        if (compacted_at != execHzn) {
          compacted_at = execHzn;
          if (compact_and_place(m) == TN_OK) return TN_OK;
        }
        uint64_t need = 0;
        const tn_vid v = V[execHzn];
        std::vector<tn_vid> d(tg.v[v].in);
        std::sort(d.begin(), d.end());
        d.erase(std::unique(d.begin(), d.end()), d.end());
        for (tn_vid u : d) need += aligned(tensor_bytes(tg.v[u].desc));
        need += aligned(tensor_bytes(tg.v[v].desc));
        return fail(TN_ERR_CAP_TOO_SMALL,
                    "vertex %d needs its %zu operands and its output (%llu bytes) co-resident; cap %llu is "
                    "too small",
                    (int)v, d.size(), (unsigned long long)need, (unsigned long long)cap);
      }
    }
  }

  // ---- Algorithm 1 -----------------------------------------------------------------------
  std::vector<int64_t> pinned_for(tn_vid v) {
    std::vector<int64_t> p;
    for (tn_vid u : tg.v[v].in)
      if (name[u] >= 0) p.push_back(name[u]);
    std::sort(p.begin(), p.end());  // sim_malloc_offld searches it
    return p;
  }

  // brings evicted tensor u back: a reload of what its offload holds (a fresh load after a drop),
  // placed with `pinned` kept where it is; the new vertex joins the transfers of the current step
  tn_status bring_back(tn_vid u, const std::vector<int64_t>& pinned) {
    const int64_t ev = evicted_by[u];
    const int64_t r = new_vertex(mg.v[ev].kind == TN_MG_DROP ? TN_MG_LOAD : TN_MG_RELOAD, u);
    mg.v[r].operands = {ev};
    add_edge(ev, r, TN_EDGE_DATA, false);
    tn_status s = sim_malloc_offld(r, pinned);
    if (s != TN_OK) return s;
    name[u] = r;
    use_insert(u);
    evicted_by[u] = -1;
    step_pre.push_back(r);
    return TN_OK;
  }

  // tensor u, just produced, is added to the output of sum vertex s
  tn_status increment(tn_vid s, tn_vid u) {
    // the output is allocated like any other, ahead of the execution if memory allows; if the
    // run-ahead has not come this far, now is the latest moment (the entries between are outputs
    // of other sums that u is the first operand of)
    while (allocHzn <= apos_acc[s]) {
      tn_status st = sim_malloc_offld(entry_vertex(allocHzn), name[u] >= 0 ? std::vector<int64_t>{name[u]} : std::vector<int64_t>{});
      if (st != TN_OK) return st;
      ++allocHzn;
    }
    // Emptying the memory against fragmentation spares nothing that holds data, u included: it
    // comes back next to the output it is added to (outputs of unfinished sums never move).  If the
    // two do not fit together, the cap is too small for this sum.
    if (name[u] < 0) {
      tn_status st = bring_back(u, {});
      if (st != TN_OK)
        return st != TN_ERR_CAP_TOO_SMALL ? st : fail(TN_ERR_CAP_TOO_SMALL,
                    "adding vertex %d to the sum %d needs the two (%llu bytes each) co-resident next to the outputs of "
                    "unfinished sums; cap %llu is too small", (int)u, (int)s,
                    (unsigned long long)aligned(tensor_bytes(tg.v[u].desc)), (unsigned long long)cap);
    }
    for (int64_t o : step_pre) mg.order.push_back(o);  // what made room comes first
    step_pre.clear();
    if (!zero_placed[s]) {
      const int64_t z0 = acc_of[s];
      zero_placed[s] = 1;
      if (counted_ahead[z0]) lookahead_bytes -= vbytes(z0);
      counted_ahead[z0] = 0;
      mg.order.push_back(z0);
    }
    const int64_t z = acc_of[s];
    const int64_t i = new_vertex(TN_MG_OP, s);
    mg.v[i].op_kind = TN_OP_SUM_INTO;
    mg.v[i].operands = {name[u], z};
    mg.v[i].offset = mg.v[z].offset;
    add_edge(name[u], i, TN_EDGE_DATA, false);
    add_edge(z, i, TN_EDGE_DATA, false);
    readers[name[u]].push_back(i);
    readers[z].push_back(i);
    incs_of[s].push_back(i);
    mg.order.push_back(i);
    ++mg.stats.n_increment;
    return TN_OK;
  }

  tn_status execute_next() {
    const tn_vid v = V[execHzn];
    const Vertex& tv = tg.v[v];
    if (is_sum(v)) {
      // the join: every operand has been added by an increment placed after its producer; the
      // cleared-and-summed output now counts as this vertex's, at the same location
      const int64_t z = acc_of[v];
      mg.v[v].operands = {z};
      for (int64_t i : incs_of[v]) add_edge(i, v, TN_EDGE_DATA, false);
      readers[z].push_back(v);
      blocks.find((uint64_t)mg.v[z].offset)->second.owner = v;
      mg.v[v].offset = mg.v[z].offset;
      open_acc[z] = 0;
    }
    // (1) bring back every evicted operand; operands already here and v's output stay pinned.
    // A compaction in the middle of this may push out operands that were here: go round again.
    for (bool again = !is_sum(v); again;) {
      again = false;
      for (tn_vid u : tv.in) {
        if (name[u] >= 0) continue;
        const int64_t compactions = mg.stats.n_compactions;
        tn_status s = bring_back(u, pinned_for(v));
        if (s != TN_OK) return s;
        if (mg.stats.n_compactions != compactions) again = true;
      }
    }
    // (2) data dependencies, from whatever now stands for each operand
    for (tn_vid u : tv.in) {
      if (is_sum(v)) break;
      mg.v[v].operands.push_back(name[u]);
      add_edge(name[u], v, TN_EDGE_DATA, false);
      if (readers[name[u]].empty() || readers[name[u]].back() != v) readers[name[u]].push_back(v);
    }
    // Section 7: the inserted transfers take place just before v, each offload before the
    // allocation it makes room for
    for (int64_t o : step_pre) mg.order.push_back(o);
    step_pre.clear();
    mg.order.push_back(v);
    name[v] = v;
    if (counted_ahead[v]) lookahead_bytes -= vbytes(v);
    counted_ahead[v] = 0;
    ++execHzn;
    use_insert(v);
    // a wanted result leaves for the caller's buffer right away
    if (tv.output_index >= 0) {
      const int64_t s = new_vertex(TN_MG_STORE, v);
      mg.v[s].operands = {v};
      mg.v[s].output_index = tv.output_index;
      add_edge(v, s, TN_EDGE_DATA, false);
      readers[v].push_back(s);
      mg.order.push_back(s);
    }
    // operands of sums are added to them right away
    for (tn_vid s : sums_of[v]) {
      tn_status st = increment(s, v);
      if (st != TN_OK) return st;
    }
    // (3) free what will not be used again
    std::vector<tn_vid> d(tv.in);
    d.push_back(v);
    std::sort(d.begin(), d.end());
    d.erase(std::unique(d.begin(), d.end()), d.end());
    for (tn_vid u : d) {
      if (name[u] < 0) continue;
      if (next_use(u) == LLONG_MAX) {
        sim_free(name[u]);
        use_erase(u);
        name[u] = -1;
      } else {
        use_insert(u);  // its next use has moved on
      }
    }
    return TN_OK;
  }

  tn_status run() {
    align = opt.alignment ? opt.alignment : 256;
    cap = mg.cap / align * align;
    if (cap == 0) return fail(TN_ERR_CAP_TOO_SMALL, "cap is smaller than one allocation unit");
    blocks[0] = {cap, -1};
    free_add(0, cap);
    pos.assign(n, -1);
    for (int64_t i = 0; i < n; ++i) pos[V[i]] = i;
    cons.assign(n, {});
    sums_of.assign(n, {});
    acc_of.assign(n, -1);
    incs_of.assign(n, {});
    for (int64_t i = 0; i < n; ++i)
      for (tn_vid u : tg.v[V[i]].in) {
        if (is_sum(V[i])) {  // consumed by an increment right after u is produced, not at position i
          sums_of[u].push_back(V[i]);
          continue;
        }
        if (cons[u].empty() || cons[u].back() != i) cons[u].push_back(i);
      }
    cons_ptr.assign(n, 0);
    name.assign(n, -1);
    use_key.assign(n, -1);
    evicted_by.assign(n, -1);
    mg.v.reserve(n + n / 4);
    for (int64_t v = 0; v < n; ++v) {
      const Vertex& tv = tg.v[v];
      int64_t m = new_vertex(tv.kind == TN_OP_INPUT ? (tv.residency == TN_DEVICE ? TN_MG_INPUT : TN_MG_LOAD)
                                                    : TN_MG_OP, (tn_vid)v);
      mg.v[m].op_kind = tv.kind;
      mg.v[m].p = tv.p;
      if (tv.kind == TN_OP_SUM) mg.v[m].kind = TN_MG_JOIN;
    }
    // tensors that are on the GPU before execution starts occupy memory from the beginning
    for (int64_t i = 0; i < n; ++i)
      if (mg.v[V[i]].kind == TN_MG_INPUT && !sim_malloc(V[i]))
        return fail(TN_ERR_CAP_TOO_SMALL, "the device-resident inputs alone exceed the cap of %llu bytes",
                    (unsigned long long)cap);
    apos.assign(n, -1);
    apos_acc.assign(n, -1);
    zero_placed.assign(n, 0);
    for (int64_t i = 0; i < n; ++i) {
      const tn_vid v = V[i];
      if (mg.v[v].kind != TN_MG_INPUT && !is_sum(v)) {
        apos[v] = (int64_t)A.size();
        A.push_back(v);
        owner_pos.push_back(i);
      }
      for (tn_vid s : sums_of[v])
        if (apos_acc[s] < 0) {
          apos_acc[s] = (int64_t)A.size();
          A.push_back(~(int64_t)s);
          owner_pos.push_back(i);
        }
    }
    const int64_t na = (int64_t)A.size();
    while (execHzn < n) {
      const tn_vid v = V[execHzn];
      const bool v_placed = apos[v] < allocHzn;  // also true for vertices without an entry
      if (allocHzn < na) {
        // an entry the next vertex waits for is its own: whatever comes before it in A belongs to
        // vertices that have run
        const int64_t m = entry_vertex(allocHzn);
        const uint64_t sz = vbytes(m);
        const bool ahead_ok = !v_placed || (execHzn >= lookahead_blocked_until && opt.max_lookahead_bytes >= sz &&
                                            lookahead_bytes <= opt.max_lookahead_bytes - sz);
        if (ahead_ok && sim_malloc(m)) {
          if (v_placed) {
            lookahead_bytes += sz;
            counted_ahead[m] = 1;
          }
          ++allocHzn;
          continue;
        }
        if (!v_placed) {
          tn_status s = sim_malloc_offld(m, pinned_for(v));
          if (s != TN_OK) return s;
          ++allocHzn;
          continue;
        }
      }
      tn_status s = execute_next();
      if (s != TN_OK) return s;
    }
    return TN_OK;
  }
};

tn_status serial_order(const TaskGraph& tg, const tn_vid* order, std::vector<tn_vid>& V) {
  const int64_t n = (int64_t)tg.v.size();
  std::vector<tn_vid> given;
  if (order) {
    given.assign(order, order + n);
    std::vector<char> seen(n, 0);
    for (tn_vid v : given) {
      if (v < 0 || v >= n || seen[v]) return fail(TN_ERR_INVALID, "order is not a permutation of the vertex ids");
      seen[v] = 1;
    }
  } else {
    // insertion order; a host-resident input moves to just before its first consumer, so that
    // its load is not scheduled (and its memory not held) long before it is needed
    std::vector<std::vector<tn_vid>> first_for(n);
    std::vector<char> placed(n, 0);
    for (int64_t v = 0; v < n; ++v)
      for (tn_vid u : tg.v[v].in)
        if (tg.v[u].kind == TN_OP_INPUT && tg.v[u].residency == TN_HOST && !placed[u]) {
          placed[u] = 1;
          first_for[v].push_back(u);
        }
    for (int64_t v = 0; v < n; ++v) {
      const bool host_input = tg.v[v].kind == TN_OP_INPUT && tg.v[v].residency == TN_HOST;
      if (host_input && placed[v]) continue;  // emitted with its first consumer
      for (tn_vid u : first_for[v]) given.push_back(u);
      given.push_back((tn_vid)v);
    }
  }
  // device-resident inputs first, in id order
  V.clear();
  for (int64_t v = 0; v < n; ++v)
    if (tg.v[v].kind == TN_OP_INPUT && tg.v[v].residency == TN_DEVICE) V.push_back((tn_vid)v);
  for (tn_vid v : given)
    if (!(tg.v[v].kind == TN_OP_INPUT && tg.v[v].residency == TN_DEVICE)) V.push_back(v);
  std::vector<int64_t> where(n);
  for (int64_t i = 0; i < n; ++i) where[V[i]] = i;
  for (int64_t v = 0; v < n; ++v)
    for (tn_vid u : tg.v[v].in)
      if (where[u] >= where[v])
        return fail(TN_ERR_NOT_TOPOLOGICAL, "vertex %d comes before its operand %d in the given order", (int)v, (int)u);
  return TN_OK;
}

}  // namespace
}  // namespace tn

using namespace tn;

extern "C" tn_status tn_compile(const tn_taskgraph* tg, const tn_vid* order, uint64_t gpu_cap_bytes,
                                const tn_compile_opts* opts, tn_memgraph** out) {
  if (!tg || !out) return fail(TN_ERR_INVALID, "NULL argument");
  if (tg->v.empty()) return fail(TN_ERR_INVALID, "empty taskgraph");
  tn_compile_opts o{};
  o.max_lookahead_bytes = UINT64_MAX;
  o.drop_clean_inputs = 1;
  if (opts) o = *opts;
  if (o.alignment && (o.alignment & (o.alignment - 1))) return fail(TN_ERR_INVALID, "alignment must be a power of two");
  auto* mg = new (std::nothrow) tn_memgraph();
  if (!mg) return fail(TN_ERR_INVALID, "out of host memory");
  mg->n_task = (int64_t)tg->v.size();
  mg->cap = gpu_cap_bytes;
  mg->n_outputs = (int64_t)tg->outputs.size();
  Compiler c(*tg, o, *mg);
  tn_status s = serial_order(*tg, order, c.V);
  if (s == TN_OK) s = c.run();
  if (s != TN_OK) {
    delete mg;
    return s;
  }
  // drop withdrawn edges; optionally the memory dependencies that repeat a data dependency
  std::vector<tn_mg_edge> kept;
  for (size_t e = 0; e < mg->edges.size(); ++e) {
    if (c.edge_dead[e]) continue;
    const auto& ed = mg->edges[e];
    if (o.prune_superfluous && ed.kind == TN_EDGE_MEM &&
        c.edge_set[TN_EDGE_DATA].count(((uint64_t)ed.from << 32) | (uint64_t)ed.to))
      continue;
    kept.push_back(ed);
  }
  mg->edges.swap(kept);
  for (size_t i = 0; i < mg->order.size(); ++i) mg->v[mg->order[i]].order_pos = (int64_t)i;
  if (o.fix_order) {
    // Section 8, item 3: extra dependencies that fix the order of kernels, and of transfers in
    // each direction, to the serial order given to the compiler
    int64_t last[3] = {-1, -1, -1};
    for (int64_t m : mg->order) {
      const int32_t k = mg->v[m].kind;
      if (k == TN_MG_OP && mg->v[m].op_kind == TN_OP_SUM_INTO) continue;  // reductions keep their freedom
      int cls = k == TN_MG_OP ? 0 : (k == TN_MG_LOAD || k == TN_MG_RELOAD) ? 1 : (k == TN_MG_OFFLOAD || k == TN_MG_STORE) ? 2 : -1;
      if (cls < 0) continue;
      if (last[cls] >= 0) c.add_edge(last[cls], m, TN_EDGE_ORDER, false);
      last[cls] = m;
    }
  }
  tn_mg_stats& st = mg->stats;
  st.cap = gpu_cap_bytes;
  st.n_task = mg->n_task;
  st.n_vertices = (int64_t)mg->v.size();
  st.n_edges = (int64_t)mg->edges.size();
  for (const auto& e : mg->edges) st.n_mem_edges += e.kind == TN_EDGE_MEM;
  for (const auto& x : mg->v) {
    switch (x.kind) {
      case TN_MG_OFFLOAD: ++st.n_offload; st.offload_bytes += x.bytes; st.host_arena_bytes += c.aligned(x.bytes); break;
      case TN_MG_RELOAD: ++st.n_reload; st.reload_bytes += x.bytes; break;
      case TN_MG_DROP: ++st.n_drop; break;
      case TN_MG_LOAD: ++st.n_load; st.load_bytes += x.bytes; break;
      case TN_MG_STORE: ++st.n_store; st.store_bytes += x.bytes; break;
      default: break;
    }
  }
  *out = mg;
  return TN_OK;
}
