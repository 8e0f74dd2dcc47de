// Internal data structures shared by the host-side parts of the library (taskgraph, compiler,
// memgraph introspection, executor).  Nothing here is visible through the C ABI.
#pragma once

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <string>
#include <vector>

#include "turnip.h"

namespace tn {

// Thread-local error text behind tn_last_error().
void set_error(const char* fmt, ...);
tn_status fail(tn_status code, const char* fmt, ...);

inline uint64_t elem_bytes(int32_t dtype) { return dtype == TN_F32 ? 4u : 2u; }
inline uint64_t tensor_bytes(const tn_tensor_desc& d) {
  return (uint64_t)d.rows * (uint64_t)d.cols * elem_bytes(d.dtype);
}

struct Vertex {
  int32_t kind = TN_OP_INPUT;
  int32_t residency = TN_HOST;
  int32_t output_index = -1;
  tn_tensor_desc desc{};
  tn_op_params p{};
  std::vector<tn_vid> in;
};

struct TaskGraph {
  std::vector<Vertex> v;
  std::vector<tn_vid> outputs;
  std::vector<tn_llama_binding> bindings;
};

struct MVertex {
  int32_t kind = TN_MG_OP;
  int32_t op_kind = TN_OP_INPUT;
  tn_vid src = -1;
  int64_t offset = -1;
  uint64_t bytes = 0;
  int64_t order_pos = -1;
  int32_t output_index = -1;
  tn_tensor_desc desc{};
  tn_op_params p{};
  std::vector<int64_t> operands;
};

struct MemGraph {
  int64_t n_task = 0;
  uint64_t cap = 0;
  int64_t n_outputs = 0;
  std::vector<MVertex> v;
  std::vector<tn_mg_edge> edges;
  std::vector<int64_t> order;
  tn_mg_stats stats{};
};

// Shape/type rules of the vertex kinds; returns TN_OK or sets the error text.
tn_status validate_op(const TaskGraph& g, int32_t kind, const tn_op_params& p, const tn_vid* in,
                      int32_t n_in, const tn_tensor_desc& out);

}  // namespace tn

struct tn_taskgraph : tn::TaskGraph {};
struct tn_memgraph : tn::MemGraph {};
