// Memgraph introspection, JSON export and the CPU dry run.
//
// The dry run is the host-side "null executor": it walks an order, checks it against the
// dependencies, and tracks which tensor every byte range holds, so that a memgraph can be
// validated without a GPU.  It does no arithmetic.
#include <cstdio>
#include <map>

#include "graph.h"

using namespace tn;

extern "C" {

void tn_memgraph_destroy(tn_memgraph* mg) { delete mg; }

int64_t tn_memgraph_num_vertices(const tn_memgraph* mg) { return mg ? (int64_t)mg->v.size() : TN_ERR_INVALID; }
int64_t tn_memgraph_num_edges(const tn_memgraph* mg) { return mg ? (int64_t)mg->edges.size() : TN_ERR_INVALID; }

tn_status tn_memgraph_vertex(const tn_memgraph* mg, int64_t i, tn_mg_vertex* out) {
  if (!mg || !out || i < 0 || i >= (int64_t)mg->v.size()) return fail(TN_ERR_INVALID, "no such memgraph vertex");
  const MVertex& x = mg->v[i];
  out->kind = x.kind;
  out->op_kind = x.op_kind;
  out->src = x.src;
  out->offset = x.offset;
  out->bytes = x.bytes;
  out->n_operands = (int32_t)x.operands.size();
  out->order_pos = x.order_pos;
  return TN_OK;
}

int32_t tn_memgraph_operands(const tn_memgraph* mg, int64_t i, int64_t* out, int32_t cap) {
  if (!mg || i < 0 || i >= (int64_t)mg->v.size()) return fail(TN_ERR_INVALID, "no such memgraph vertex");
  const auto& o = mg->v[i].operands;
  for (int32_t k = 0; k < cap && k < (int32_t)o.size(); ++k) out[k] = o[k];
  return (int32_t)o.size();
}

tn_status tn_memgraph_edge(const tn_memgraph* mg, int64_t i, tn_mg_edge* out) {
  if (!mg || !out || i < 0 || i >= (int64_t)mg->edges.size()) return fail(TN_ERR_INVALID, "no such edge");
  *out = mg->edges[i];
  return TN_OK;
}

tn_status tn_memgraph_stats(const tn_memgraph* mg, tn_mg_stats* out) {
  if (!mg || !out) return fail(TN_ERR_INVALID, "NULL argument");
  *out = mg->stats;
  return TN_OK;
}

tn_status tn_memgraph_dump_json(const tn_memgraph* mg, const char* path) {
  if (!mg || !path) return fail(TN_ERR_INVALID, "NULL argument");
  FILE* f = fopen(path, "w");
  if (!f) return fail(TN_ERR_INVALID, "cannot open %s for writing", path);
  static const char* kinds[] = {"input", "load", "op", "offload", "reload", "drop", "store", "join"};
  static const char* ekinds[] = {"data", "mem", "order"};
  fprintf(f, "{\"n_task\": %lld, \"cap\": %llu,\n \"vertices\": [\n", (long long)mg->n_task, (unsigned long long)mg->cap);
  for (size_t i = 0; i < mg->v.size(); ++i) {
    const MVertex& x = mg->v[i];
    fprintf(f, "  {\"id\": %zu, \"kind\": \"%s\", \"op\": %d, \"src\": %d, \"offset\": %lld, \"bytes\": %llu, \"operands\": [",
            i, kinds[x.kind], x.op_kind, (int)x.src, (long long)x.offset, (unsigned long long)x.bytes);
    for (size_t k = 0; k < x.operands.size(); ++k) fprintf(f, "%s%lld", k ? ", " : "", (long long)x.operands[k]);
    fprintf(f, "]}%s\n", i + 1 < mg->v.size() ? "," : "");
  }
  fprintf(f, " ],\n \"edges\": [\n");
  for (size_t i = 0; i < mg->edges.size(); ++i)
    fprintf(f, "  [%lld, %lld, \"%s\"]%s\n", (long long)mg->edges[i].from, (long long)mg->edges[i].to,
            ekinds[mg->edges[i].kind], i + 1 < mg->edges.size() ? "," : "");
  fprintf(f, " ],\n \"order\": [");
  for (size_t i = 0; i < mg->order.size(); ++i) fprintf(f, "%s%lld", i ? ", " : "", (long long)mg->order[i]);
  fprintf(f, "]\n}\n");
  fclose(f);
  return TN_OK;
}

tn_status tn_memgraph_simulate(const tn_memgraph* mg, const int64_t* order, int64_t n) {
  if (!mg) return fail(TN_ERR_INVALID, "NULL argument");
  const int64_t nv = (int64_t)mg->v.size();
  if (order && n != nv) return fail(TN_ERR_INVALID, "order has %lld entries, the memgraph %lld vertices", (long long)n, (long long)nv);
  std::vector<int64_t> npred(nv, 0), nread(nv, 0);
  std::vector<std::vector<int64_t>> succ(nv);
  for (const auto& e : mg->edges) {
    ++npred[e.to];
    succ[e.from].push_back(e.to);
  }
  for (const auto& x : mg->v)
    for (int64_t o : x.operands) ++nread[o];
  // contents: offset -> (size, memgraph vertex whose output lies there); live: still has readers
  std::map<uint64_t, std::pair<uint64_t, int64_t>> mem;
  std::vector<char> done(nv, 0), on_host(nv, 0);
  auto write = [&](int64_t m) -> tn_status {
    const MVertex& x = mg->v[m];
    if (x.offset < 0 || (uint64_t)x.offset + x.bytes > mg->cap)
      return fail(TN_ERR_INVALID, "vertex %lld writes outside [0, cap)", (long long)m);
    const uint64_t a = (uint64_t)x.offset, b = a + x.bytes;
    auto it = mem.upper_bound(a);
    if (it != mem.begin()) --it;
    while (it != mem.end() && it->first < b) {
      if (it->first + it->second.first > a) {
        if (nread[it->second.second] > 0)
          return fail(TN_ERR_INVALID, "vertex %lld overwrites the output of vertex %lld, which still has readers",
                      (long long)m, (long long)it->second.second);
        it = mem.erase(it);
      } else {
        ++it;
      }
    }
    mem[a] = {x.bytes, m};
    return TN_OK;
  };
  auto read = [&](int64_t reader, int64_t o) -> tn_status {
    const MVertex& x = mg->v[o];
    auto it = mem.find((uint64_t)x.offset);
    if (x.offset < 0 || it == mem.end() || it->second.second != o)
      return fail(TN_ERR_INVALID, "vertex %lld reads the output of vertex %lld, which is not in GPU memory",
                  (long long)reader, (long long)o);
    --nread[o];
    return TN_OK;
  };
  for (int64_t m = 0; m < nv; ++m)
    if (mg->v[m].kind == TN_MG_INPUT) {
      tn_status s = write(m);
      if (s != TN_OK) return s;
    }
  for (int64_t i = 0; i < nv; ++i) {
    const int64_t m = order ? order[i] : mg->order[i];
    if (m < 0 || m >= nv || done[m]) return fail(TN_ERR_INVALID, "order is not a permutation (entry %lld)", (long long)i);
    if (npred[m] != 0) return fail(TN_ERR_NOT_TOPOLOGICAL, "vertex %lld runs before one of its dependencies", (long long)m);
    const MVertex& x = mg->v[m];
    tn_status s = TN_OK;
    switch (x.kind) {
      case TN_MG_INPUT: break;
      case TN_MG_LOAD:
        if (!x.operands.empty() && !on_host[x.operands[0]]) s = fail(TN_ERR_INVALID, "load %lld before its drop", (long long)m);
        if (s == TN_OK) s = write(m);
        break;
      case TN_MG_OP:
        for (int64_t o : x.operands)
          if ((s = read(m, o)) != TN_OK) break;
        if (s == TN_OK && x.op_kind == TN_OP_SUM_INTO) {  // updates its second operand in place, owns nothing
          if (x.operands.size() != 2 || mg->v[x.operands[1]].op_kind != TN_OP_ZERO || mg->v[x.operands[1]].offset != x.offset)
            s = fail(TN_ERR_INVALID, "increment %lld does not name the output it adds to", (long long)m);
          break;
        }
        if (s == TN_OK) s = write(m);
        break;
      case TN_MG_JOIN: {  // the summed output changes its name; every increment has read it by now
        const int64_t z = x.operands.empty() ? -1 : x.operands[0];
        if (z < 0 || mg->v[z].op_kind != TN_OP_ZERO || mg->v[z].offset != x.offset) {
          s = fail(TN_ERR_INVALID, "join %lld has no output to take over", (long long)m);
          break;
        }
        if ((s = read(m, z)) != TN_OK) break;
        if (nread[z] != 0) {
          s = fail(TN_ERR_INVALID, "join %lld runs while increments are outstanding", (long long)m);
          break;
        }
        mem[(uint64_t)x.offset].second = m;
        break;
      }
      case TN_MG_OFFLOAD:
      case TN_MG_STORE:
        s = read(m, x.operands[0]);
        on_host[m] = 1;
        break;
      case TN_MG_DROP:
        --nread[x.operands[0]];
        on_host[m] = 1;
        break;
      case TN_MG_RELOAD:
        if (!on_host[x.operands[0]]) s = fail(TN_ERR_INVALID, "reload %lld before its offload", (long long)m);
        if (s == TN_OK) s = write(m);
        break;
      default: s = fail(TN_ERR_INVALID, "bad vertex kind");
    }
    if (s != TN_OK) return s;
    done[m] = 1;
    for (int64_t w : succ[m]) --npred[w];
  }
  return TN_OK;
}

}  // extern "C"
