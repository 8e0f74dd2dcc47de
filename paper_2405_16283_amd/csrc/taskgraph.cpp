// Taskgraph container, operand validation, and the tiler that turns a LLaMA-style decoder
// forward pass into a taskgraph.
//
// Section 4, first paragraph: a taskgraph is a dataflow DAG; a vertex without inputs carries an
// input tensor, any other vertex is a kernel call.  The paper leaves the production of the
// taskgraph to an outside framework (Section 4, second paragraph), so the decomposition below is
// this library's own.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>

#include "graph.h"

namespace tn {

static thread_local char g_err[1024] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}

tn_status fail(tn_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

static bool same(const tn_tensor_desc& a, const tn_tensor_desc& b) {
  return a.dtype == b.dtype && a.rows == b.rows && a.cols == b.cols;
}

tn_status validate_op(const TaskGraph& g, int32_t kind, const tn_op_params& p, const tn_vid* in,
                      int32_t n_in, const tn_tensor_desc& out) {
  auto D = [&](int i) -> const tn_tensor_desc& { return g.v[in[i]].desc; };
  if (out.rows <= 0 || out.cols <= 0 || (out.dtype != TN_F32 && out.dtype != TN_BF16))
    return fail(TN_ERR_SHAPE, "output tensor must be non-empty fp32 or bf16");
  switch (kind) {
    case TN_OP_GEMM: {
      if (p.mode < 0 || p.mode > 2) return fail(TN_ERR_SHAPE, "gemm: mode must be 0, 1 or 2");
      const int32_t want = p.mode == 1 ? 2 * p.nk + 1 : p.mode == 2 ? 3 * p.nk : 2 * p.nk;
      if (p.nk < 1 || n_in != want) return fail(TN_ERR_SHAPE, "gemm: needs %d operands for nk %d, mode %d", want, p.nk, p.mode);
      if (p.mode != 0 && (p.trans_a || p.trans_c)) return fail(TN_ERR_SHAPE, "gemm: modes 1 and 2 go with neither trans_a nor trans_c");
      if (p.mode == 1 && !same(D(2 * p.nk), out)) return fail(TN_ERR_SHAPE, "gemm: the residual operand must have the output's shape and type");
      for (int k = 0; p.mode == 2 && k < p.nk; ++k)
        if (!same(D(p.nk + k), D(2 * p.nk + k))) return fail(TN_ERR_SHAPE, "gemm: up tile %d is not shaped like its gate tile", k);
      tn_tensor_desc lo = out;  // logical [rows, cols] of the product
      if (p.trans_c) std::swap(lo.rows, lo.cols);
      for (int k = 0; k < p.nk; ++k) {
        tn_tensor_desc a = D(k);
        const auto& b = D(p.nk + k);
        if (p.trans_a) std::swap(a.rows, a.cols);
        const int32_t bk = p.trans_b ? b.cols : b.rows, bn = p.trans_b ? b.rows : b.cols;
        if (a.rows != lo.rows || bn != lo.cols || a.cols != bk || a.dtype != out.dtype ||
            b.dtype != out.dtype)
          return fail(TN_ERR_SHAPE, "gemm: k tile %d has A [%d,%d] B [%d,%d] for C [%d,%d]", k,
                      a.rows, a.cols, b.rows, b.cols, lo.rows, lo.cols);
      }
      return TN_OK;
    }
    case TN_OP_RMS_STAT: {
      if (n_in < 1 || out.dtype != TN_F32 || out.cols != 1)
        return fail(TN_ERR_SHAPE, "rms_stat: output must be fp32 [rows,1]");
      int64_t cols = 0;
      for (int i = 0; i < n_in; ++i) {
        if (D(i).rows != out.rows || D(i).dtype != D(0).dtype)
          return fail(TN_ERR_SHAPE, "rms_stat: operand %d does not match the row block", i);
        cols += D(i).cols;
      }
      if (cols != p.d) return fail(TN_ERR_SHAPE, "rms_stat: operands cover %lld columns, d = %d",
                                   (long long)cols, p.d);
      return TN_OK;
    }
    case TN_OP_RMS_APPLY: {
      if (n_in != 3) return fail(TN_ERR_SHAPE, "rms_apply: needs x, stat, gain");
      if (!same(D(0), out) || D(1).dtype != TN_F32 || D(1).rows != out.rows || D(1).cols != 1 ||
          D(2).rows != 1 || D(2).cols != out.cols || D(2).dtype != out.dtype)
        return fail(TN_ERR_SHAPE, "rms_apply: operand shapes do not fit");
      return TN_OK;
    }
    case TN_OP_ROPE: {
      if (n_in != 1 || !same(D(0), out)) return fail(TN_ERR_SHAPE, "rope: one operand of the output's shape");
      if ((out.cols & 1) || (p.col0 & 1) || p.head_dim < 2 || (p.head_dim & 1) || p.col0 < 0 ||
          p.pos0 < 0 || !(p.rope_base > 0))
        return fail(TN_ERR_SHAPE, "rope: pairs must not straddle tiles (even cols, col0, head_dim)");
      return TN_OK;
    }
    case TN_OP_ATTN_BLOCK: {
      int nq = p.n_q_tiles, nkv = p.n_kv_tiles, nc = p.n_col_tiles;
      if (nq < 1 || nkv < 1 || nc < 1 || n_in != (nq + 2 * nkv) * nc || p.head_dim < 1)
        return fail(TN_ERR_SHAPE, "attn_block: needs (n_q_tiles + 2 n_kv_tiles) * n_col_tiles operands");
      int64_t gw = 0, qrows = 0;
      for (int c = 0; c < nc; ++c) gw += D(c).cols;
      if (gw % p.head_dim) return fail(TN_ERR_SHAPE, "attn_block: columns are not whole heads");
      int32_t dt = D(0).dtype;
      for (int r = 0; r < nq; ++r) {
        qrows += D(r * nc).rows;
        for (int c = 0; c < nc; ++c)
          if (D(r * nc + c).rows != D(r * nc).rows || D(r * nc + c).cols != D(c).cols ||
              D(r * nc + c).dtype != dt)
            return fail(TN_ERR_SHAPE, "attn_block: Q tile (%d,%d) does not fit the grid", r, c);
      }
      for (int r = 0; r < nkv; ++r)
        for (int c = 0; c < nc; ++c) {
          const auto& k = D(nq * nc + r * nc + c);
          tn_tensor_desc v = D((nq + nkv) * nc + r * nc + c);
          if (p.v_trans) std::swap(v.rows, v.cols);
          if (k.cols != D(c).cols || !same(k, v) || k.rows != D(nq * nc + r * nc).rows || k.dtype != dt)
            return fail(TN_ERR_SHAPE, "attn_block: K/V tile (%d,%d) does not fit the grid", r, c);
        }
      int64_t hpg = gw / p.head_dim;
      if (out.dtype != TN_F32 || out.rows != qrows || out.cols != gw + 2 * hpg)
        return fail(TN_ERR_SHAPE, "attn_block: output must be fp32 [%lld,%lld]", (long long)qrows,
                    (long long)(gw + 2 * hpg));
      return TN_OK;
    }
    case TN_OP_ATTN_COMBINE: {
      if (n_in < 1 || p.hpg < 1 || p.head_dim < 1) return fail(TN_ERR_SHAPE, "attn_combine: needs partials");
      int64_t gw = (int64_t)p.hpg * p.head_dim;
      for (int i = 0; i < n_in; ++i)
        if (D(i).dtype != TN_F32 || D(i).cols != gw + 2 * p.hpg || D(i).rows != D(0).rows)
          return fail(TN_ERR_SHAPE, "attn_combine: operand %d is not a partial of this group", i);
      if (p.row0 < 0 || p.col0 < 0 || p.row0 + out.rows > D(0).rows || p.col0 + out.cols > gw)
        return fail(TN_ERR_SHAPE, "attn_combine: output window leaves the block");
      return TN_OK;
    }
    case TN_OP_SILU_MUL:
    case TN_OP_ADD:
      if (n_in != 2 || !same(D(0), out) || !same(D(1), out))
        return fail(TN_ERR_SHAPE, "elementwise: two operands of the output's shape and type");
      return TN_OK;
    case TN_OP_SILU_MUL_BWD:
      if (n_in != 3 || !same(D(0), out) || !same(D(1), out) || !same(D(2), out) || (p.mode != 0 && p.mode != 1))
        return fail(TN_ERR_SHAPE, "silu_mul_bwd: dact, gate, up of the output's shape and type; mode 0 or 1");
      return TN_OK;
    case TN_OP_RMS_BWD_STAT: {
      if (p.nk < 1 || n_in != 3 * p.nk || out.dtype != TN_F32 || out.cols != 1)
        return fail(TN_ERR_SHAPE, "rms_bwd_stat: 3*nk operands, output fp32 [rows,1]");
      for (int i = 0; i < p.nk; ++i) {
        const auto &dy = D(i), &x = D(p.nk + i), &g = D(2 * p.nk + i);
        if (dy.rows != out.rows || !same(dy, x) || g.rows != 1 || g.cols != dy.cols || g.dtype != dy.dtype ||
            dy.dtype != D(0).dtype)
          return fail(TN_ERR_SHAPE, "rms_bwd_stat: column tile %d does not fit", i);
      }
      return TN_OK;
    }
    case TN_OP_RMS_BWD_APPLY: {
      if (n_in != 5 && n_in != 6) return fail(TN_ERR_SHAPE, "rms_bwd_apply: dy, x, stat, dot, gain[, residual gradient]");
      if (!same(D(0), out) || !same(D(1), out) || D(2).dtype != TN_F32 || D(2).rows != out.rows || D(2).cols != 1 ||
          D(3).dtype != TN_F32 || D(3).rows != out.rows || D(3).cols != 1 || D(4).rows != 1 ||
          D(4).cols != out.cols || D(4).dtype != out.dtype || (n_in == 6 && !same(D(5), out)) || p.d < out.cols)
        return fail(TN_ERR_SHAPE, "rms_bwd_apply: operand shapes do not fit");
      return TN_OK;
    }
    case TN_OP_SOFTMAX_STAT:
      if (out.dtype != TN_F32 || out.cols != 2 || !(p.scale > 0.f))
        return fail(TN_ERR_SHAPE, "softmax_stat: output is fp32 [rows, 2] and scale is positive");
      for (int i = 0; i < n_in; ++i)
        if (D(i).rows != out.rows || D(i).dtype != D(0).dtype)
          return fail(TN_ERR_SHAPE, "softmax_stat: operand %d is not a score tile of this row block", i);
      return TN_OK;
    case TN_OP_SOFTMAX_APPLY:
      if (n_in != 2 || !same(D(0), out) || D(1).dtype != TN_F32 || D(1).rows != out.rows || D(1).cols != 2 ||
          !(p.scale > 0.f))
        return fail(TN_ERR_SHAPE, "softmax_apply: a score tile of the output's shape and type, then fp32 [rows, 2]");
      return TN_OK;
    case TN_OP_SUM:
      for (int i = 0; i < n_in; ++i) {
        if (D(i).rows != out.rows || D(i).cols != out.cols || D(i).dtype != out.dtype)
          return fail(TN_ERR_SHAPE, "sum: operand %d is not of the output's shape and type", i);
        for (int k = 0; k < i; ++k)
          if (in[k] == in[i]) return fail(TN_ERR_INVALID, "sum: operand %d repeats operand %d", i, k);
      }
      return TN_OK;
    case TN_OP_ZERO:
    case TN_OP_SUM_INTO:
      return fail(TN_ERR_INVALID, "vertex kind %d exists in memgraphs only (see TN_OP_SUM)", kind);
    case TN_OP_TRANSPOSE:
      if (n_in != 1 || D(0).rows != out.cols || D(0).cols != out.rows || D(0).dtype != out.dtype)
        return fail(TN_ERR_SHAPE, "transpose: one operand [cols, rows] of the output's type");
      return TN_OK;
    case TN_OP_ATTN_BWD: {
      const int nq = p.n_q_tiles, nkv = p.n_kv_tiles, nc = p.n_col_tiles;
      if (nq < 1 || nkv < 1 || nc < 1 || p.head_dim < 1 || p.mode < 0 || p.mode > 3 ||
          (p.trans_a && (p.mode == 0 || p.v_trans)) ||
          n_in != (2 * nq + 2 * nkv) * nc + (p.mode ? nq : 0) + (p.trans_a ? (p.mode == 1 ? nkv : nq) * nc : 0))
        return fail(TN_ERR_SHAPE, "attn_bwd: needs (2 n_q_tiles + 2 n_kv_tiles) * n_col_tiles operands, plus n_q_tiles "
                                  "statistics unless mode is 0, plus the transposed grid if trans_a is set");
      int64_t gw = 0, qrows = 0, kvrows = 0;
      for (int c = 0; c < nc; ++c) gw += D(c).cols;
      if (gw % p.head_dim) return fail(TN_ERR_SHAPE, "attn_bwd: columns are not whole heads");
      const int64_t hpg = gw / p.head_dim;
      const int32_t dt = D(0).dtype;
      const int d0 = (nq + 2 * nkv) * nc, s0 = d0 + nq * nc;
      for (int r = 0; r < nq; ++r) {
        qrows += D(r * nc).rows;
        for (int c = 0; c < nc; ++c)
          if (D(r * nc + c).rows != D(r * nc).rows || D(r * nc + c).cols != D(c).cols || D(r * nc + c).dtype != dt ||
              !same(D(d0 + r * nc + c), D(r * nc + c)))
            return fail(TN_ERR_SHAPE, "attn_bwd: Q / dO tile (%d,%d) does not fit the grid", r, c);
        if (p.mode && (D(s0 + r).dtype != TN_F32 || D(s0 + r).rows != D(r * nc).rows || D(s0 + r).cols != 2 * hpg))
          return fail(TN_ERR_SHAPE, "attn_bwd: statistics of Q row tile %d must be fp32 [rows, 2*hpg]", r);
      }
      for (int r = 0; r < nkv; ++r) {
        kvrows += D(nq * nc + r * nc).rows;
        for (int c = 0; c < nc; ++c) {
          const auto& k = D(nq * nc + r * nc + c);
          tn_tensor_desc v = D((nq + nkv) * nc + r * nc + c);
          if (p.v_trans) std::swap(v.rows, v.cols);
          if (k.cols != D(c).cols || !same(k, v) || k.rows != D(nq * nc + r * nc).rows || k.dtype != dt)
            return fail(TN_ERR_SHAPE, "attn_bwd: K/V tile (%d,%d) does not fit the grid", r, c);
        }
      }
      if (p.trans_a) {
        const int t0 = s0 + nq, src0 = p.mode == 1 ? nq * nc : p.mode == 2 ? 0 : d0, cnt = (p.mode == 1 ? nkv : nq) * nc;
        for (int i = 0; i < cnt; ++i) {
          tn_tensor_desc tt = D(t0 + i);
          std::swap(tt.rows, tt.cols);
          if (!same(tt, D(src0 + i))) return fail(TN_ERR_SHAPE, "attn_bwd: transposed tile %d does not mirror its tile", i);
        }
      }
      const bool ok = p.mode == 0 ? (out.dtype == TN_F32 && out.rows == qrows && out.cols == 2 * hpg)
                    : p.mode == 1 ? (out.dtype == dt && out.rows == qrows && out.cols == gw)
                                  : (out.dtype == dt && out.rows == kvrows && out.cols == gw);
      if (!ok) return fail(TN_ERR_SHAPE, "attn_bwd: output shape does not fit mode %d", p.mode);
      return TN_OK;
    }
    default:
      return fail(TN_ERR_INVALID, "unknown vertex kind %d", kind);
  }
}

// ---------------------------------------------------------------------------------------------
// LLaMA tiler
// ---------------------------------------------------------------------------------------------

namespace {

struct Range { int32_t a, b; int32_t len() const { return b - a; } };

std::vector<Range> cut(int32_t n, int32_t t) {
  std::vector<Range> r;
  for (int32_t s = 0; s < n; s += t) r.push_back({s, std::min(s + t, n)});
  return r;
}

using Grid = std::vector<std::vector<tn_vid>>;  // [row tile][column tile]

struct Tiler {
  const tn_llama_config& c;
  TaskGraph& g;
  std::vector<Range> dcols, fcols, rows;

  Tiler(const tn_llama_config& cfg, TaskGraph& tg) : c(cfg), g(tg) {
    dcols = cut(c.d_model, c.tile);
    fcols = cut(c.ffn, c.tile);
    rows = cut(c.seq, c.tile);
  }

  tn_vid input(int32_t rws, int32_t cls, int32_t residency, int32_t tensor, int32_t layer, Range rr,
               Range cr) {
    Vertex v;
    v.kind = TN_OP_INPUT;
    v.residency = residency;
    v.desc = {c.dtype, rws, cls};
    g.v.push_back(v);
    tn_vid id = (tn_vid)g.v.size() - 1;
    g.bindings.push_back({id, tensor, layer, rr.a, rr.b, cr.a, cr.b, 0});
    return id;
  }

  tn_vid op(int32_t kind, const tn_op_params& p, std::vector<tn_vid> in, tn_tensor_desc d) {
    Vertex v;
    v.kind = kind;
    v.p = p;
    v.desc = d;
    v.in = std::move(in);
    g.v.push_back(std::move(v));
    return (tn_vid)g.v.size() - 1;
  }

  Grid weight(int32_t tensor, int32_t layer, const std::vector<Range>& rr, const std::vector<Range>& cc) {
    Grid w(rr.size(), std::vector<tn_vid>(cc.size()));
    for (size_t i = 0; i < rr.size(); ++i)
      for (size_t j = 0; j < cc.size(); ++j) {
        if (c.weights_transposed) {
          w[i][j] = input(cc[j].len(), rr[i].len(), c.weights_residency, tensor, layer, rr[i], cc[j]);
          g.bindings.back().transposed = 1;
        } else {
          w[i][j] = input(rr[i].len(), cc[j].len(), c.weights_residency, tensor, layer, rr[i], cc[j]);
        }
      }
    return w;
  }

  std::vector<tn_vid> gain(int32_t tensor, int32_t layer) {
    std::vector<tn_vid> gns;
    for (auto& cr : dcols) gns.push_back(input(1, cr.len(), c.weights_residency, tensor, layer, {0, 1}, cr));
    return gns;
  }

  // one output tile of X(row tile) * W: full K inside one vertex, or (k_split) partial products
  // over runs of K tiles joined by a sum vertex
  // residual >= 0: that tile is added inside the vertex (mode 1); up != nullptr: the gated pair of products (mode 2)
  tn_vid gemm(const std::vector<tn_vid>& xrow, const Grid& w, size_t j, int32_t m, int32_t n,
              bool trans_c = false, tn_vid residual = -1, const Grid* up = nullptr) {
    const size_t nk = xrow.size();
    if (residual >= 0 || up) {
      tn_op_params p{};
      p.nk = (int32_t)nk;
      p.trans_b = c.weights_transposed ? 1 : 0;
      p.mode = up ? 2 : 1;
      std::vector<tn_vid> in(xrow);
      for (size_t k = 0; k < nk; ++k) in.push_back(w[k][j]);
      if (up) for (size_t k = 0; k < nk; ++k) in.push_back((*up)[k][j]);
      else in.push_back(residual);
      return op(TN_OP_GEMM, p, std::move(in), {c.dtype, m, n});
    }
    const size_t per = c.k_split > 1 ? (nk + c.k_split - 1) / c.k_split : nk;
    const tn_tensor_desc d = trans_c ? tn_tensor_desc{c.dtype, n, m} : tn_tensor_desc{c.dtype, m, n};
    std::vector<tn_vid> parts;
    for (size_t k0 = 0; k0 < nk; k0 += per) {
      const size_t k1 = std::min(nk, k0 + per);
      tn_op_params p{};
      p.nk = (int32_t)(k1 - k0);
      p.trans_b = c.weights_transposed ? 1 : 0;
      p.trans_c = trans_c ? 1 : 0;
      std::vector<tn_vid> in(xrow.begin() + k0, xrow.begin() + k1);
      for (size_t k = k0; k < k1; ++k) in.push_back(w[k][j]);
      parts.push_back(op(TN_OP_GEMM, p, std::move(in), d));
    }
    return parts.size() == 1 ? parts[0] : op(TN_OP_SUM, tn_op_params{}, std::move(parts), d);
  }

  std::vector<tn_vid> rmsnorm(const std::vector<tn_vid>& xrow, const std::vector<tn_vid>& gns, int32_t m,
                              tn_vid* stat = nullptr) {
    tn_op_params p{};
    p.d = c.d_model;
    p.eps = c.eps;
    tn_vid st = op(TN_OP_RMS_STAT, p, xrow, {TN_F32, m, 1});
    if (stat) *stat = st;
    std::vector<tn_vid> out;
    for (size_t j = 0; j < xrow.size(); ++j)
      out.push_back(op(TN_OP_RMS_APPLY, tn_op_params{}, {xrow[j], st, gns[j]}, {c.dtype, m, dcols[j].len()}));
    return out;
  }

  tn_vid rope(tn_vid x, int32_t pos0, int32_t col_start, int32_t m, int32_t n, bool inverse = false) {
    tn_op_params p{};
    p.pos0 = pos0;
    p.col0 = col_start % c.head_dim;
    p.head_dim = c.head_dim;
    p.rope_base = c.rope_base;
    p.mode = inverse ? 1 : 0;
    return op(TN_OP_ROPE, p, {x}, {c.dtype, m, n});
  }

  // weight tiles in [in, out] layout, for the reverse pass: grid[i][j] = rows rr[i], columns cc[j]
  Grid natural(int32_t tensor, int32_t layer, const std::vector<Range>& rr, const std::vector<Range>& cc) {
    Grid w(rr.size(), std::vector<tn_vid>(cc.size()));
    for (size_t i = 0; i < rr.size(); ++i)
      for (size_t j = 0; j < cc.size(); ++j)
        w[i][j] = input(rr[i].len(), cc[j].len(), c.weights_residency, tensor, layer, rr[i], cc[j]);
    return w;
  }

  // sum_k A_k B_k with explicit operand lists; B_k stored [cols, K_k] if trans_b, A_k stored [K_k, rows] if trans_a
  tn_vid gemm_list(const std::vector<tn_vid>& a, const std::vector<tn_vid>& b, int32_t m, int32_t n, bool trans_a,
                   bool trans_b, bool trans_c = false) {
    tn_op_params p{};
    p.nk = (int32_t)a.size();
    p.trans_a = trans_a ? 1 : 0;
    p.trans_b = trans_b ? 1 : 0;
    p.trans_c = trans_c ? 1 : 0;
    std::vector<tn_vid> in(a);
    in.insert(in.end(), b.begin(), b.end());
    return op(TN_OP_GEMM, p, std::move(in), trans_c ? tn_tensor_desc{c.dtype, n, m} : tn_tensor_desc{c.dtype, m, n});
  }

  tn_vid add(tn_vid a, tn_vid b, int32_t m, int32_t n) { return op(TN_OP_ADD, tn_op_params{}, {a, b}, {c.dtype, m, n}); }

  void mark_output(tn_vid id, int32_t tensor, int32_t layer, Range rr, Range cr) {
    g.v[id].output_index = (int32_t)g.outputs.size();
    g.outputs.push_back(id);
    g.bindings.push_back({id, tensor, layer, rr.a, rr.b, cr.a, cr.b, 0});
  }
};

}  // namespace
}  // namespace tn

using namespace tn;

extern "C" {

const char* tn_last_error(void) { return g_err; }

tn_status tn_taskgraph_create(tn_taskgraph** out) {
  if (!out) return fail(TN_ERR_INVALID, "out is NULL");
  *out = new (std::nothrow) tn_taskgraph();
  return *out ? TN_OK : fail(TN_ERR_INVALID, "out of host memory");
}

void tn_taskgraph_destroy(tn_taskgraph* tg) { delete tg; }

tn_status tn_taskgraph_add_input(tn_taskgraph* tg, const tn_tensor_desc* desc, int32_t residency, tn_vid* out) {
  if (!tg || !desc || !out) return fail(TN_ERR_INVALID, "NULL argument");
  if (desc->rows <= 0 || desc->cols <= 0 || (desc->dtype != TN_F32 && desc->dtype != TN_BF16))
    return fail(TN_ERR_SHAPE, "input tensor must be non-empty fp32 or bf16");
  if (residency != TN_HOST && residency != TN_DEVICE) return fail(TN_ERR_INVALID, "bad residency");
  Vertex v;
  v.kind = TN_OP_INPUT;
  v.residency = residency;
  v.desc = *desc;
  tg->v.push_back(v);
  *out = (tn_vid)tg->v.size() - 1;
  return TN_OK;
}

tn_status tn_taskgraph_add_op(tn_taskgraph* tg, int32_t kind, const tn_op_params* params, const tn_vid* inputs,
                              int32_t n_inputs, const tn_tensor_desc* out_desc, tn_vid* out) {
  if (!tg || !params || !out_desc || !out || (n_inputs > 0 && !inputs) || n_inputs < 1)
    return fail(TN_ERR_INVALID, "NULL argument or no operands");
  if (kind == TN_OP_INPUT) return fail(TN_ERR_INVALID, "use tn_taskgraph_add_input for inputs");
  for (int i = 0; i < n_inputs; ++i)
    if (inputs[i] < 0 || inputs[i] >= (tn_vid)tg->v.size())
      return fail(TN_ERR_INVALID, "operand %d names vertex %d, which does not exist yet", i, inputs[i]);
  tn_status s = validate_op(*tg, kind, *params, inputs, n_inputs, *out_desc);
  if (s != TN_OK) return s;
  Vertex v;
  v.kind = kind;
  v.p = *params;
  v.desc = *out_desc;
  v.in.assign(inputs, inputs + n_inputs);
  tg->v.push_back(std::move(v));
  *out = (tn_vid)tg->v.size() - 1;
  return TN_OK;
}

tn_status tn_taskgraph_mark_output(tn_taskgraph* tg, tn_vid v) {
  if (!tg || v < 0 || v >= (tn_vid)tg->v.size()) return fail(TN_ERR_INVALID, "no such vertex");
  if (tg->v[v].output_index >= 0) return fail(TN_ERR_INVALID, "vertex %d is already an output", v);
  tg->v[v].output_index = (int32_t)tg->outputs.size();
  tg->outputs.push_back(v);
  return TN_OK;
}

int64_t tn_taskgraph_num_vertices(const tn_taskgraph* tg) { return tg ? (int64_t)tg->v.size() : TN_ERR_INVALID; }
int64_t tn_taskgraph_num_outputs(const tn_taskgraph* tg) { return tg ? (int64_t)tg->outputs.size() : TN_ERR_INVALID; }

tn_status tn_taskgraph_vertex(const tn_taskgraph* tg, tn_vid v, tn_tg_vertex* out) {
  if (!tg || !out || v < 0 || v >= (tn_vid)tg->v.size()) return fail(TN_ERR_INVALID, "no such vertex");
  const Vertex& x = tg->v[v];
  out->kind = x.kind;
  out->residency = x.residency;
  out->n_inputs = (int32_t)x.in.size();
  out->output_index = x.output_index;
  out->desc = x.desc;
  out->params = x.p;
  return TN_OK;
}

int32_t tn_taskgraph_inputs(const tn_taskgraph* tg, tn_vid v, tn_vid* out, int32_t cap) {
  if (!tg || v < 0 || v >= (tn_vid)tg->v.size()) return fail(TN_ERR_INVALID, "no such vertex");
  const auto& in = tg->v[v].in;
  for (int32_t i = 0; i < cap && i < (int32_t)in.size(); ++i) out[i] = in[i];
  return (int32_t)in.size();
}

tn_status tn_taskgraph_level_order(const tn_taskgraph* tg, tn_vid* out, int64_t cap) {
  if (!tg || !out) return fail(TN_ERR_INVALID, "NULL argument");
  const int64_t n = (int64_t)tg->v.size();
  if (cap < n) return fail(TN_ERR_INVALID, "room for %lld vertex ids, the graph has %lld", (long long)cap, (long long)n);
  // keys in half levels: an operation of level l has key 2l, an input read first at level l key 2l - 1
  std::vector<int64_t> key(n, 0);
  for (int64_t v = 0; v < n; ++v) {
    const Vertex& x = tg->v[v];
    if (x.kind == TN_OP_INPUT) continue;
    int64_t lv = 0;
    for (tn_vid u : x.in)
      if (tg->v[u].kind != TN_OP_INPUT) lv = std::max(lv, key[u] / 2);
    key[v] = 2 * (lv + 1);
  }
  for (int64_t v = 0; v < n; ++v) {
    const Vertex& x = tg->v[v];
    if (x.kind == TN_OP_INPUT) continue;
    for (tn_vid u : x.in)
      if (tg->v[u].kind == TN_OP_INPUT && (key[u] == 0 || key[v] - 1 < key[u])) key[u] = key[v] - 1;
  }
  for (int64_t v = 0; v < n; ++v)
    if (tg->v[v].kind == TN_OP_INPUT && key[v] == 0) key[v] = 1;  // an input nobody reads: before the first level
  std::vector<tn_vid> order(n);
  for (int64_t v = 0; v < n; ++v) order[v] = (tn_vid)v;
  std::stable_sort(order.begin(), order.end(), [&](tn_vid a, tn_vid b) { return key[a] < key[b]; });
  std::copy(order.begin(), order.end(), out);
  return TN_OK;
}

tn_status tn_taskgraph_clustered_order(const tn_taskgraph* tg, tn_vid* out, int64_t cap) {
  if (!tg || !out) return fail(TN_ERR_INVALID, "NULL argument");
  const int64_t n = (int64_t)tg->v.size();
  if (cap < n) return fail(TN_ERR_INVALID, "room for %lld vertex ids, the graph has %lld", (long long)cap, (long long)n);
  auto is_input = [&](tn_vid u) { return tg->v[u].kind == TN_OP_INPUT; };
  std::vector<int64_t> lv(n, 0);  // level of a kernel vertex as in the level order; 0 for inputs
  std::vector<std::vector<tn_vid>> readers(n);
  for (int64_t v = 0; v < n; ++v) {
    if (is_input((tn_vid)v)) continue;
    int64_t l = 0;
    for (tn_vid u : tg->v[v].in) {
      if (!is_input(u)) l = std::max(l, lv[u]);
      if (readers[u].empty() || readers[u].back() != (tn_vid)v) readers[u].push_back((tn_vid)v);
    }
    lv[v] = l + 1;
  }
  // Reductions: kernel vertices whose kernel operands all lie one level below and are read by nothing but
  // vertices with this very operand list.  Such a vertex, the vertices that share its operand list and the
  // operands form a cluster that is placed as a whole at the operands' level: operands, then the reductions.
  std::vector<int64_t> cluster(n, -1), role(n, 0);
  std::vector<std::vector<tn_vid>> members;
  for (int64_t c = 0; c < n; ++c) {
    const Vertex& x = tg->v[c];
    if (x.kind == TN_OP_INPUT || cluster[c] >= 0) continue;
    bool ok = false;
    for (tn_vid u : x.in)
      if (!is_input(u)) ok = true;
    for (tn_vid u : x.in) {
      if (!ok) break;
      if (is_input(u)) continue;
      if (lv[u] != lv[c] - 1 || cluster[u] >= 0) ok = false;
      for (tn_vid w : readers[u])
        if (ok && (cluster[w] >= 0 || tg->v[w].in != x.in)) ok = false;
    }
    if (!ok) continue;
    const int64_t id = (int64_t)members.size();
    members.emplace_back();
    for (tn_vid u : x.in)
      if (!is_input(u) && cluster[u] < 0) {
        cluster[u] = id;
        members[id].push_back(u);
      }
    tn_vid first_op = x.in[0];
    for (tn_vid u : x.in)
      if (!is_input(u)) { first_op = u; break; }
    for (tn_vid w : readers[first_op]) {  // every kernel operand has the same readers
      cluster[w] = id;
      role[w] = 1;
      members[id].push_back(w);
    }
  }
  // Units (clusters and single vertices) of one level are ordered by the first input any of their vertices
  // reads -- so that the units that read one weight tile follow one another and the tile is needed once --
  // and then by their numbering.
  auto first_input = [&](tn_vid v) {
    int64_t k = std::numeric_limits<int64_t>::max();
    for (tn_vid u : tg->v[v].in)
      if (is_input(u)) k = std::min<int64_t>(k, u);
    return k;
  };
  struct Unit { int64_t level, input, first; int64_t cluster; tn_vid v; };
  std::vector<Unit> units;
  for (int64_t v = 0; v < n; ++v)
    if (!is_input((tn_vid)v) && cluster[v] < 0) units.push_back({lv[v], first_input((tn_vid)v), v, -1, (tn_vid)v});
  for (size_t id = 0; id < members.size(); ++id) {
    Unit u{0, std::numeric_limits<int64_t>::max(), std::numeric_limits<int64_t>::max(), (int64_t)id, -1};
    for (tn_vid v : members[id]) {
      if (role[v] == 0) u.level = lv[v];
      u.input = std::min(u.input, first_input(v));
      u.first = std::min<int64_t>(u.first, v);
    }
    units.push_back(u);
  }
  std::sort(units.begin(), units.end(), [](const Unit& a, const Unit& b) {
    if (a.level != b.level) return a.level < b.level;
    if (a.input != b.input) return a.input < b.input;
    return a.first < b.first;
  });
  // inputs go right before their first reader; inputs nobody reads come first
  std::vector<char> placed(n, 0);
  int64_t at = 0;
  for (int64_t v = 0; v < n; ++v)
    if (is_input((tn_vid)v) && readers[v].empty()) {
      out[at++] = (tn_vid)v;
      placed[v] = 1;
    }
  auto emit = [&](tn_vid v) {
    for (tn_vid u : tg->v[v].in)
      if (is_input(u) && !placed[u]) {
        out[at++] = u;
        placed[u] = 1;
      }
    out[at++] = v;
  };
  for (const Unit& u : units) {
    if (u.cluster < 0) {
      emit(u.v);
      continue;
    }
    std::vector<tn_vid> ms = members[(size_t)u.cluster];
    std::stable_sort(ms.begin(), ms.end(), [&](tn_vid a, tn_vid b) { return role[a] != role[b] ? role[a] < role[b] : a < b; });
    for (tn_vid v : ms) emit(v);
  }
  if (at != n) return fail(TN_ERR_INVALID, "internal: %lld of %lld vertices ordered", (long long)at, (long long)n);
  return TN_OK;
}

int64_t tn_taskgraph_num_bindings(const tn_taskgraph* tg) { return tg ? (int64_t)tg->bindings.size() : TN_ERR_INVALID; }

tn_status tn_taskgraph_binding(const tn_taskgraph* tg, int64_t i, tn_llama_binding* out) {
  if (!tg || !out || i < 0 || i >= (int64_t)tg->bindings.size()) return fail(TN_ERR_INVALID, "no such binding");
  *out = tg->bindings[i];
  return TN_OK;
}

// The decoder is emitted stripe by stripe: a stripe is one attention block of rows of one
// sequence.  Causal attention of a stripe needs K and V of the stripes before it only, so the
// serial order "layer, sequence, stripe" keeps the live set small: per-stripe activations die
// at the end of the stripe and only K/V of earlier stripes stay.
tn_status tn_build_llama(const tn_llama_config* cfg, tn_taskgraph** out) {
  if (!cfg || !out) return fail(TN_ERR_INVALID, "NULL argument");
  const tn_llama_config& c = *cfg;
  if (c.layers < 1 || c.d_model < 1 || c.n_heads < 1 || c.head_dim < 2 || c.ffn < 1 || c.seq < 1 ||
      c.batch < 1 || c.tile < 2 || c.attn_block < c.tile)
    return fail(TN_ERR_INVALID, "non-positive model dimension");
  if (c.n_heads * c.head_dim != c.d_model) return fail(TN_ERR_SHAPE, "n_heads * head_dim != d_model");
  if (c.attn_block % c.tile) return fail(TN_ERR_SHAPE, "attn_block must be a multiple of tile");
  if ((c.tile % c.head_dim) && (c.head_dim % c.tile))
    return fail(TN_ERR_SHAPE, "tile and head_dim must divide one another");
  if ((c.tile & 1) || (c.head_dim & 1)) return fail(TN_ERR_SHAPE, "tile and head_dim must be even");
  const int32_t gw = std::max(c.tile, c.head_dim);  // columns of a head group
  if (c.d_model % gw) return fail(TN_ERR_SHAPE, "d_model must be a multiple of max(tile, head_dim)");
  if (c.dtype != TN_F32 && c.dtype != TN_BF16) return fail(TN_ERR_INVALID, "bad dtype");
  if (c.lora_rank < 0 || (c.train && c.lora_rank < 1)) return fail(TN_ERR_INVALID, "train needs lora_rank > 0");
  if (c.train && gw != c.tile) return fail(TN_ERR_SHAPE, "train needs head_dim <= tile (one column tile per head group)");
  if (c.train && c.kv_outputs) return fail(TN_ERR_INVALID, "train and kv_outputs do not go together");
  if (c.k_split < 0) return fail(TN_ERR_INVALID, "k_split must not be negative");
  if (c.output_layer_stride < 0) return fail(TN_ERR_INVALID, "output_layer_stride must not be negative");
  if (c.decode_steps < 0) return fail(TN_ERR_INVALID, "decode_steps must not be negative");
  if (c.attn_whole_rows && (c.train || c.materialize_scores))
    return fail(TN_ERR_INVALID, "attn_whole_rows goes with neither train nor materialize_scores");
  if (c.decode_steps > 0 && (c.train || c.materialize_scores || c.batch != 1 || c.lora_rank > 0))
    return fail(TN_ERR_INVALID, "decode_steps needs one sequence, and none of train, lora_rank, materialize_scores");
  if (c.checkpoint && !c.train) return fail(TN_ERR_INVALID, "checkpoint applies to train only");
  if (c.fuse_epilogues < 0 || c.fuse_epilogues > 3 || (c.fuse_epilogues && (c.train || c.k_split > 1)))
    return fail(TN_ERR_INVALID, "fuse_epilogues takes bits 1 and 2 and goes with neither train nor k_split");
  if ((c.recompute_normed || c.recompute_gate_up) && !c.train)
    return fail(TN_ERR_INVALID, "recompute_normed and recompute_gate_up need train");
  if (c.checkpoint_layers < 0 || (c.checkpoint_layers > 0 && !c.checkpoint))
    return fail(TN_ERR_INVALID, "checkpoint_layers needs checkpoint and must not be negative");
  // layers whose forward tensors the reverse pass forms again instead of reading saved ones
  auto recomputed = [&](int l) { return c.checkpoint && (c.checkpoint_layers == 0 || l < c.checkpoint_layers); };
  if (c.materialize_scores && (c.tile != c.head_dim || c.train || c.kv_outputs))
    return fail(TN_ERR_INVALID, "materialize_scores needs tile == head_dim and neither train nor kv_outputs");

  auto* tg = new (std::nothrow) tn_taskgraph();
  if (!tg) return fail(TN_ERR_INVALID, "out of host memory");
  Tiler t(c, *tg);
  const int32_t hpg = gw / c.head_dim, ctg = gw / c.tile, n_groups = c.d_model / gw;
  const auto stripes = cut(c.seq, c.attn_block);
  const size_t nd = t.dcols.size(), nf = t.fcols.size();

  // residual stream, one grid per sequence
  std::vector<Grid> x(c.batch);
  for (int b = 0; b < c.batch; ++b) {
    x[b].assign(t.rows.size(), std::vector<tn_vid>(nd));
    for (size_t i = 0; i < t.rows.size(); ++i)
      for (size_t j = 0; j < nd; ++j) {
        Range rr{b * c.seq + t.rows[i].a, b * c.seq + t.rows[i].b};
        x[b][i][j] = t.input(t.rows[i].len(), t.dcols[j].len(), c.x_residency, TN_T_X, -1, rr, t.dcols[j]);
      }
  }

  // what the reverse pass needs of the forward pass, per layer and sequence, indexed by row tile
  struct Saved {
    Grid xin, a, q, k, v, h1, gate, up;
    std::vector<tn_vid> rstd1, rstd2, tq, tv;
  };
  std::vector<std::vector<Saved>> saved(c.train ? c.layers : 0, std::vector<Saved>(c.batch));
  // with checkpointing only the input of each layer is kept; the rest is formed again in the reverse pass
  std::vector<std::vector<Grid>> layer_in(c.checkpoint ? c.layers : 0, std::vector<Grid>(c.batch));
  struct LayerInputs {
    Grid wq, wk, wv, wo, w1, w3, w2;
    std::vector<tn_vid> g1, g2, aq, bq, av, bv, aqT, bqT, avT, bvT;
  };
  std::vector<LayerInputs> lin(c.train || c.decode_steps ? c.layers : 0);
  std::vector<Grid> kcache(c.decode_steps ? c.layers : 0), vcache(c.decode_steps ? c.layers : 0);  // K, V of the prefill
  const int32_t rk = c.lora_rank;
  const Range rkr{0, rk};

  // which layers' K/V (kv_outputs) and hidden states (hidden_outputs) are outputs
  auto layer_is_output = [&](int l) {
    const int n = c.output_layer_stride;
    return n <= 1 || l % n == 0 || l % n == n - 1 || l + 2 >= c.layers;
  };

  // One layer, one sequence, stripe by stripe.  `sv`: where to note what the reverse pass reads
  // (null: nothing is noted).  `tail`: whether the layer's output is formed (second half of the
  // feed-forward block and the residual); a pass that only restores saved values stops before it.
  auto forward_layer = [&](int l, const LayerInputs& w, int b, Grid& xb, Saved* sv, bool tail) {
    const Grid &wq = w.wq, &wk = w.wk, &wv = w.wv, &wo = w.wo, &w1 = w.w1, &w3 = w.w3, &w2 = w.w2;
    const std::vector<tn_vid>&g1 = w.g1, &g2 = w.g2, &aqT = w.aqT, &bqT = w.bqT, &avT = w.avT, &bvT = w.bvT;
    if (sv) {
      sv->xin = xb;
      for (Grid* gp : {&sv->a, &sv->q, &sv->k, &sv->v, &sv->h1, &sv->gate, &sv->up}) gp->assign(t.rows.size(), {});
      for (auto* vp : {&sv->rstd1, &sv->rstd2, &sv->tq, &sv->tv}) vp->assign(t.rows.size(), -1);
    }
    Grid kk(t.rows.size()), vv(t.rows.size());  // K, V of the stripes done so far
    for (size_t s = 0; s < stripes.size(); ++s) {
      std::vector<size_t> rt;  // row tiles of this stripe
      for (size_t i = 0; i < t.rows.size(); ++i)
        if (t.rows[i].a >= stripes[s].a && t.rows[i].a < stripes[s].b) rt.push_back(i);
      Grid q(t.rows.size());
      for (size_t i : rt) {
        const int32_t m = t.rows[i].len();
        tn_vid st1 = -1, tq = -1, tv = -1;
        auto a = t.rmsnorm(xb[i], g1, m, &st1);
        if (rk > 0) {  // the low-rank activations a Aq and a Av
          tq = t.gemm_list(a, aqT, m, rk, false, true);
          tv = t.gemm_list(a, avT, m, rk, false, true);
        }
        for (size_t j = 0; j < nd; ++j) {
          const int32_t n = t.dcols[j].len();
          tn_vid qj = t.gemm(a, wq, j, m, n), vj = t.gemm(a, wv, j, m, n, c.v_transposed != 0);
          if (rk > 0) {
            qj = t.add(qj, t.gemm_list({tq}, {bqT[j]}, m, n, false, true), m, n);
            const bool vt = c.v_transposed != 0;
            vj = t.op(TN_OP_ADD, tn_op_params{}, {vj, t.gemm_list({tv}, {bvT[j]}, m, n, false, true, vt)},
                      vt ? tn_tensor_desc{c.dtype, n, m} : tn_tensor_desc{c.dtype, m, n});
          }
          q[i].push_back(t.rope(qj, t.rows[i].a, t.dcols[j].a, m, n));
          kk[i].push_back(t.rope(t.gemm(a, wk, j, m, n), t.rows[i].a, t.dcols[j].a, m, n));
          vv[i].push_back(vj);
          if (sv && j + 1 == nd) {
            sv->a[i] = a; sv->q[i] = q[i]; sv->k[i] = kk[i]; sv->v[i] = vv[i];
            sv->rstd1[i] = st1; sv->tq[i] = tq; sv->tv[i] = tv;
          }
          if (c.kv_outputs && layer_is_output(l)) {
            Range rr{b * c.seq + t.rows[i].a, b * c.seq + t.rows[i].b};
            for (int which = 0; which < 2; ++which) {
              tn_vid id = which ? vv[i][j] : kk[i][j];
              tg->v[id].output_index = (int32_t)tg->outputs.size();
              tg->outputs.push_back(id);
              tg->bindings.push_back({id, which ? TN_T_V : TN_T_K, l, rr.a, rr.b, t.dcols[j].a, t.dcols[j].b,
                                      (which && c.v_transposed) ? 1 : 0});
            }
          }
        }
      }
      // attention of this stripe against stripes 0..s, one partial per pair, per head group
      Grid o(t.rows.size(), std::vector<tn_vid>(nd, -1));
      if (c.materialize_scores) {
        // scores and probabilities as tensors: per head (= column tile) and row tile i the score
        // tiles against the row tiles 0..i, the softmax over them in two portions, and P V
        const float scale = 1.0f / std::sqrt((float)c.head_dim);
        for (size_t i : rt)
          for (size_t h = 0; h < nd; ++h) {
            const int32_t m = t.rows[i].len();
            std::vector<tn_vid> sc, pv;
            for (size_t j = 0; j <= i; ++j) {
              tn_op_params p{};
              p.nk = 1;
              p.trans_b = 1;
              sc.push_back(t.op(TN_OP_GEMM, p, {q[i][h], kk[j][h]}, {c.dtype, m, t.rows[j].len()}));
            }
            tn_op_params ps{};
            ps.scale = scale;
            ps.causal = 1;
            ps.q_pos0 = t.rows[i].a;
            ps.k_pos0 = 0;
            const tn_vid st = t.op(TN_OP_SOFTMAX_STAT, ps, sc, {TN_F32, m, 2});
            for (size_t j = 0; j <= i; ++j) {
              ps.k_pos0 = t.rows[j].a;
              pv.push_back(t.op(TN_OP_SOFTMAX_APPLY, ps, {sc[j], st}, {c.dtype, m, t.rows[j].len()}));
            }
            tn_op_params pg{};
            pg.nk = (int32_t)(i + 1);
            pg.trans_b = c.v_transposed ? 1 : 0;
            for (size_t j = 0; j <= i; ++j) pv.push_back(vv[j][h]);
            o[i][h] = t.op(TN_OP_GEMM, pg, std::move(pv), {c.dtype, m, t.dcols[h].len()});
          }
      }
      for (int32_t gi = 0; gi < (c.materialize_scores ? 0 : n_groups); ++gi) {
        std::vector<tn_vid> parts;
        // attn_whole_rows: one vertex per query block over all keys up to the block's own, instead of one per
        // key block (its online softmax runs over the whole range; one partial instead of s + 1)
        for (size_t s2 = c.attn_whole_rows ? s : 0; s2 <= s; ++s2) {
          const int32_t k_from = c.attn_whole_rows ? 0 : stripes[s2].a;
          std::vector<size_t> kt;
          for (size_t i = 0; i < t.rows.size(); ++i)
            if (t.rows[i].a >= k_from && t.rows[i].a < stripes[s2].b) kt.push_back(i);
          std::vector<tn_vid> in;
          for (size_t i : rt) for (int32_t cc = 0; cc < ctg; ++cc) in.push_back(q[i][gi * ctg + cc]);
          for (size_t i : kt) for (int32_t cc = 0; cc < ctg; ++cc) in.push_back(kk[i][gi * ctg + cc]);
          for (size_t i : kt) for (int32_t cc = 0; cc < ctg; ++cc) in.push_back(vv[i][gi * ctg + cc]);
          tn_op_params p{};
          p.n_q_tiles = (int32_t)rt.size();
          p.n_kv_tiles = (int32_t)kt.size();
          p.n_col_tiles = ctg;
          p.head_dim = c.head_dim;
          p.q_pos0 = stripes[s].a;
          p.k_pos0 = k_from;
          p.causal = (s2 == s);
          p.v_trans = c.v_transposed ? 1 : 0;
          p.scale = 1.0f / std::sqrt((float)c.head_dim);
          parts.push_back(t.op(TN_OP_ATTN_BLOCK, p, std::move(in), {TN_F32, stripes[s].len(), gw + 2 * hpg}));
        }
        for (size_t i : rt)
          for (int32_t cc = 0; cc < ctg; ++cc) {
            tn_op_params p{};
            p.row0 = t.rows[i].a - stripes[s].a;
            p.col0 = cc * c.tile;
            p.head_dim = c.head_dim;
            p.hpg = hpg;
            o[i][gi * ctg + cc] = t.op(TN_OP_ATTN_COMBINE, p, parts,
                                      {c.dtype, t.rows[i].len(), t.dcols[gi * ctg + cc].len()});
          }
      }
      // output projection, residual, feed-forward, residual -- row tile by row tile
      for (size_t i : rt) {
        const int32_t m = t.rows[i].len();
        std::vector<tn_vid> h(nd);
        for (size_t j = 0; j < nd; ++j) {
          const int32_t n = t.dcols[j].len();
          h[j] = (c.fuse_epilogues & 1) ? t.gemm(o[i], wo, j, m, n, false, xb[i][j])
                                        : t.op(TN_OP_ADD, tn_op_params{}, {xb[i][j], t.gemm(o[i], wo, j, m, n)}, {c.dtype, m, n});
        }
        tn_vid st2 = -1;
        auto bn = t.rmsnorm(h, g2, m, &st2);
        std::vector<tn_vid> act(nf), gates(nf), ups(nf);
        for (size_t j = 0; j < nf; ++j) {
          const int32_t n = t.fcols[j].len();
          if (c.fuse_epilogues & 2) {  // never with train: nothing is saved
            if (tail) act[j] = t.gemm(bn, w1, j, m, n, false, -1, &w3);
            continue;
          }
          tn_vid gate = t.gemm(bn, w1, j, m, n), up = t.gemm(bn, w3, j, m, n);
          gates[j] = gate;
          ups[j] = up;
          if (tail) act[j] = t.op(TN_OP_SILU_MUL, tn_op_params{}, {gate, up}, {c.dtype, m, n});
        }
        if (sv) {
          sv->h1[i] = h; sv->gate[i] = gates; sv->up[i] = ups; sv->rstd2[i] = st2;
        }
        for (size_t j = 0; tail && j < nd; ++j) {
          const int32_t n = t.dcols[j].len();
          xb[i][j] = (c.fuse_epilogues & 1) ? t.gemm(act, w2, j, m, n, false, h[j])
                                            : t.op(TN_OP_ADD, tn_op_params{}, {h[j], t.gemm(act, w2, j, m, n)}, {c.dtype, m, n});
        }
      }
    }
    if (c.decode_steps) {
      kcache[l] = kk;
      vcache[l] = vv;
    }
  };

  for (int l = 0; l < c.layers; ++l) {
    Grid wq = t.weight(TN_T_WQ, l, t.dcols, t.dcols), wk = t.weight(TN_T_WK, l, t.dcols, t.dcols);
    Grid wv = t.weight(TN_T_WV, l, t.dcols, t.dcols), wo = t.weight(TN_T_WO, l, t.dcols, t.dcols);
    Grid w1 = t.weight(TN_T_W1, l, t.dcols, t.fcols), w3 = t.weight(TN_T_W3, l, t.dcols, t.fcols);
    Grid w2 = t.weight(TN_T_W2, l, t.fcols, t.dcols);
    auto g1 = t.gain(TN_T_G1, l), g2 = t.gain(TN_T_G2, l);
    std::vector<tn_vid> aq, bq, av, bv;  // adapter tiles: A cut along its rows, B along its columns
    if (rk > 0)
      for (size_t j = 0; j < nd; ++j) {
        aq.push_back(t.input(t.dcols[j].len(), rk, c.weights_residency, TN_T_AQ, l, t.dcols[j], rkr));
        bq.push_back(t.input(rk, t.dcols[j].len(), c.weights_residency, TN_T_BQ, l, rkr, t.dcols[j]));
        av.push_back(t.input(t.dcols[j].len(), rk, c.weights_residency, TN_T_AV, l, t.dcols[j], rkr));
        bv.push_back(t.input(rk, t.dcols[j].len(), c.weights_residency, TN_T_BV, l, rkr, t.dcols[j]));
      }
    // transposed copies of the adapter tiles, so that the adapter products are A B^T products like
    // every other projection (the form the MFMA kernels take)
    std::vector<tn_vid> aqT, bqT, avT, bvT;
    for (size_t j = 0; j < aq.size(); ++j) {
      const int32_t n = t.dcols[j].len();
      aqT.push_back(t.op(TN_OP_TRANSPOSE, tn_op_params{}, {aq[j]}, {c.dtype, rk, n}));
      avT.push_back(t.op(TN_OP_TRANSPOSE, tn_op_params{}, {av[j]}, {c.dtype, rk, n}));
      bqT.push_back(t.op(TN_OP_TRANSPOSE, tn_op_params{}, {bq[j]}, {c.dtype, n, rk}));
      bvT.push_back(t.op(TN_OP_TRANSPOSE, tn_op_params{}, {bv[j]}, {c.dtype, n, rk}));
    }
    const LayerInputs w{wq, wk, wv, wo, w1, w3, w2, g1, g2, aq, bq, av, bv, aqT, bqT, avT, bvT};
    if (c.train || c.decode_steps) lin[l] = w;
    for (int b = 0; b < c.batch; ++b) {
      if (recomputed(l)) layer_in[l][b] = x[b];
      forward_layer(l, w, b, x[b], c.train && !recomputed(l) ? &saved[l][b] : nullptr, true);
      if (c.hidden_outputs && layer_is_output(l) && l + 1 < c.layers)  // (the last layer's output is y)
        for (size_t i = 0; i < t.rows.size(); ++i)
          for (size_t j = 0; j < nd; ++j)
            t.mark_output(x[b][i][j], TN_T_H, l, {b * c.seq + t.rows[i].a, b * c.seq + t.rows[i].b}, t.dcols[j]);
    }
  }
  for (int b = 0; b < c.batch; ++b)
    for (size_t i = 0; i < t.rows.size(); ++i)
      for (size_t j = 0; j < nd; ++j) {
        tn_vid id = x[b][i][j];
        tg->v[id].output_index = (int32_t)tg->outputs.size();
        tg->outputs.push_back(id);
        tg->bindings.push_back({id, TN_T_Y, -1, b * c.seq + t.rows[i].a, b * c.seq + t.rows[i].b,
                                t.dcols[j].a, t.dcols[j].b, 0});
      }
  // ---- decode steps, known in number beforehand (Section 9, limitations: the memgraph is compiled
  // for a fixed number of generated tokens).  Step u runs the one row at position seq + u through
  // every layer; its keys and values join the cache as single-row tiles, so the attention block over
  // the generated positions grows by one tile per step, while the blocks over the prefill's stripes
  // read the prefill's tiles.  The row's embedding is an input (there is no vocabulary here), bound
  // as row seq + u of x; its output is row seq + u of y.
  if (c.decode_steps > 0) {
    const int32_t P = c.seq;
    std::vector<std::vector<std::vector<tn_vid>>> kdec(c.layers), vdec(c.layers);  // [layer][step][column tile]
    const float scale = 1.0f / std::sqrt((float)c.head_dim);
    for (int u = 0; u < c.decode_steps; ++u) {
      const Range rr{P + u, P + u + 1};
      std::vector<tn_vid> xr(nd);
      for (size_t j = 0; j < nd; ++j) xr[j] = t.input(1, t.dcols[j].len(), c.x_residency, TN_T_X, -1, rr, t.dcols[j]);
      for (int l = 0; l < c.layers; ++l) {
        const LayerInputs& w = lin[l];
        auto a = t.rmsnorm(xr, w.g1, 1);
        std::vector<tn_vid> q(nd), kr(nd), vr(nd);
        for (size_t j = 0; j < nd; ++j) {
          const int32_t n = t.dcols[j].len();
          q[j] = t.rope(t.gemm(a, w.wq, j, 1, n), P + u, t.dcols[j].a, 1, n);
          kr[j] = t.rope(t.gemm(a, w.wk, j, 1, n), P + u, t.dcols[j].a, 1, n);
          vr[j] = t.gemm(a, w.wv, j, 1, n, c.v_transposed != 0);
          if (c.kv_outputs && layer_is_output(l)) {
            t.mark_output(kr[j], TN_T_K, l, rr, t.dcols[j]);
            t.mark_output(vr[j], TN_T_V, l, rr, t.dcols[j]);
            if (c.v_transposed) tg->bindings.back().transposed = 1;
          }
        }
        kdec[l].push_back(kr);
        vdec[l].push_back(vr);
        std::vector<tn_vid> o(nd);
        for (int32_t gi = 0; gi < n_groups; ++gi) {
          std::vector<tn_vid> parts;
          tn_op_params p{};
          p.n_q_tiles = 1;
          p.n_col_tiles = ctg;
          p.head_dim = c.head_dim;
          p.q_pos0 = P + u;
          p.causal = 0;  // every cached position lies before the row's own
          p.v_trans = c.v_transposed ? 1 : 0;
          p.scale = scale;
          for (size_t s2 = 0; s2 < stripes.size(); ++s2) {  // the prefill's stripes
            std::vector<size_t> kt;
            for (size_t i = 0; i < t.rows.size(); ++i)
              if (t.rows[i].a >= stripes[s2].a && t.rows[i].a < stripes[s2].b) kt.push_back(i);
            std::vector<tn_vid> in;
            for (int32_t cc = 0; cc < ctg; ++cc) in.push_back(q[gi * ctg + cc]);
            for (size_t i : kt) for (int32_t cc = 0; cc < ctg; ++cc) in.push_back(kcache[l][i][gi * ctg + cc]);
            for (size_t i : kt) for (int32_t cc = 0; cc < ctg; ++cc) in.push_back(vcache[l][i][gi * ctg + cc]);
            p.n_kv_tiles = (int32_t)kt.size();
            p.k_pos0 = stripes[s2].a;
            parts.push_back(t.op(TN_OP_ATTN_BLOCK, p, std::move(in), {TN_F32, 1, gw + 2 * hpg}));
          }
          {  // the generated positions so far, this row's included: one single-row tile each
            std::vector<tn_vid> in;
            for (int32_t cc = 0; cc < ctg; ++cc) in.push_back(q[gi * ctg + cc]);
            for (int v = 0; v <= u; ++v) for (int32_t cc = 0; cc < ctg; ++cc) in.push_back(kdec[l][v][gi * ctg + cc]);
            for (int v = 0; v <= u; ++v) for (int32_t cc = 0; cc < ctg; ++cc) in.push_back(vdec[l][v][gi * ctg + cc]);
            p.n_kv_tiles = u + 1;
            p.k_pos0 = P;
            parts.push_back(t.op(TN_OP_ATTN_BLOCK, p, std::move(in), {TN_F32, 1, gw + 2 * hpg}));
          }
          for (int32_t cc = 0; cc < ctg; ++cc) {
            tn_op_params pc{};
            pc.row0 = 0;
            pc.col0 = cc * c.tile;
            pc.head_dim = c.head_dim;
            pc.hpg = hpg;
            o[gi * ctg + cc] = t.op(TN_OP_ATTN_COMBINE, pc, parts, {c.dtype, 1, t.dcols[gi * ctg + cc].len()});
          }
        }
        std::vector<tn_vid> h(nd);
        for (size_t j = 0; j < nd; ++j)
          h[j] = (c.fuse_epilogues & 1) ? t.gemm(o, w.wo, j, 1, t.dcols[j].len(), false, xr[j])
                                        : t.add(xr[j], t.gemm(o, w.wo, j, 1, t.dcols[j].len()), 1, t.dcols[j].len());
        auto bn = t.rmsnorm(h, w.g2, 1);
        std::vector<tn_vid> act(nf);
        for (size_t j = 0; j < nf; ++j) {
          const int32_t n = t.fcols[j].len();
          act[j] = (c.fuse_epilogues & 2)
                       ? t.gemm(bn, w.w1, j, 1, n, false, -1, &w.w3)
                       : t.op(TN_OP_SILU_MUL, tn_op_params{}, {t.gemm(bn, w.w1, j, 1, n), t.gemm(bn, w.w3, j, 1, n)}, {c.dtype, 1, n});
        }
        for (size_t j = 0; j < nd; ++j)
          xr[j] = (c.fuse_epilogues & 1) ? t.gemm(act, w.w2, j, 1, t.dcols[j].len(), false, h[j])
                                         : t.add(h[j], t.gemm(act, w.w2, j, 1, t.dcols[j].len()), 1, t.dcols[j].len());
        if (c.hidden_outputs && layer_is_output(l) && l + 1 < c.layers)
          for (size_t j = 0; j < nd; ++j) t.mark_output(xr[j], TN_T_H, l, rr, t.dcols[j]);
      }
      for (size_t j = 0; j < nd; ++j) t.mark_output(xr[j], TN_T_Y, -1, rr, t.dcols[j]);
    }
  }
  if (c.train) {
    // ---- reverse pass for L = sum(y * probe): dL/dy is the probe itself ------------------------
    const size_t nr = t.rows.size();
    std::vector<Grid> dy(c.batch);
    for (int b = 0; b < c.batch; ++b) {
      dy[b].assign(nr, std::vector<tn_vid>(nd));
      for (size_t i = 0; i < nr; ++i)
        for (size_t j = 0; j < nd; ++j) {
          Range rr{b * c.seq + t.rows[i].a, b * c.seq + t.rows[i].b};
          dy[b][i][j] = t.input(t.rows[i].len(), t.dcols[j].len(), c.x_residency, TN_T_PROBE, -1, rr, t.dcols[j]);
        }
    }
    for (int l = c.layers - 1; l >= 0; --l) {
      const LayerInputs& w = lin[l];
      if (recomputed(l))  // form what the reverse pass reads of this layer again, from the layer's input
        for (int b = 0; b < c.batch; ++b) {
          Grid xin = layer_in[l][b];
          forward_layer(l, w, b, xin, &saved[l][b], false);
        }
      // base weights as [in, out] tiles: the forward pass's own if it uses that layout
      const bool own = c.weights_transposed != 0;
      Grid wqn = own ? t.natural(TN_T_WQ, l, t.dcols, t.dcols) : w.wq, wkn = own ? t.natural(TN_T_WK, l, t.dcols, t.dcols) : w.wk;
      Grid wvn = own ? t.natural(TN_T_WV, l, t.dcols, t.dcols) : w.wv, won = own ? t.natural(TN_T_WO, l, t.dcols, t.dcols) : w.wo;
      Grid w1n = own ? t.natural(TN_T_W1, l, t.dcols, t.fcols) : w.w1, w3n = own ? t.natural(TN_T_W3, l, t.dcols, t.fcols) : w.w3;
      Grid w2n = own ? t.natural(TN_T_W2, l, t.fcols, t.dcols) : w.w2;
      // operands of the adapter gradients, summed over all rows of all sequences
      // (all transposed, so that the sums over the rows are plain A B^T products over K = rows)
      std::vector<tn_vid> all_tq, all_tv, all_dtq, all_dtv;
      std::vector<std::vector<tn_vid>> a_cols(nd), dq_cols(nd), dv_cols(nd);
      for (int b = 0; b < c.batch; ++b) {
        const Saved& sv = saved[l][b];
        Grid dh1(nr, std::vector<tn_vid>(nd)), dO(nr, std::vector<tn_vid>(nd));
        for (size_t i = 0; i < nr; ++i) {
          const int32_t m = t.rows[i].len();
          // feed-forward block: y = h1 + (silu(gate) * up) W2, gate = bn W1, up = bn W3, bn = RMSNorm(h1; g2)
          std::vector<tn_vid> dgate(nf), dup(nf);
          // recompute_gate_up: the gate and up products of this row tile are formed again, from the normalised h1
          // (itself formed again from h1 and its statistic), instead of read from the forward pass
          const bool again = c.recompute_gate_up && !recomputed(l);
          std::vector<tn_vid> bn2;
          if (again)
            for (size_t j = 0; j < nd; ++j)
              bn2.push_back(t.op(TN_OP_RMS_APPLY, tn_op_params{}, {sv.h1[i][j], sv.rstd2[i], w.g2[j]},
                                 {c.dtype, m, t.dcols[j].len()}));
          for (size_t f = 0; f < nf; ++f) {
            const int32_t n = t.fcols[f].len();
            tn_vid dact = t.gemm_list(dy[b][i], w2n[f], m, n, false, true);
            const tn_vid gate = again ? t.gemm(bn2, w.w1, f, m, n) : sv.gate[i][f];
            const tn_vid up = again ? t.gemm(bn2, w.w3, f, m, n) : sv.up[i][f];
            tn_op_params p{};
            dgate[f] = t.op(TN_OP_SILU_MUL_BWD, p, {dact, gate, up}, {c.dtype, m, n});
            p.mode = 1;
            dup[f] = t.op(TN_OP_SILU_MUL_BWD, p, {dact, gate, up}, {c.dtype, m, n});
          }
          std::vector<tn_vid> dbn(nd);
          for (size_t j = 0; j < nd; ++j) {
            std::vector<tn_vid> av(dgate), bv(w1n[j]);
            av.insert(av.end(), dup.begin(), dup.end());
            bv.insert(bv.end(), w3n[j].begin(), w3n[j].end());
            dbn[j] = t.gemm_list(av, bv, m, t.dcols[j].len(), false, true);
          }
          tn_op_params ps{};
          ps.nk = (int32_t)nd;
          std::vector<tn_vid> sin(dbn);
          sin.insert(sin.end(), sv.h1[i].begin(), sv.h1[i].end());
          sin.insert(sin.end(), w.g2.begin(), w.g2.end());
          tn_vid dot2 = t.op(TN_OP_RMS_BWD_STAT, ps, std::move(sin), {TN_F32, m, 1});
          tn_op_params pa{};
          pa.d = c.d_model;
          for (size_t j = 0; j < nd; ++j)
            dh1[i][j] = t.op(TN_OP_RMS_BWD_APPLY, pa, {dbn[j], sv.h1[i][j], sv.rstd2[i], dot2, w.g2[j], dy[b][i][j]},
                             {c.dtype, m, t.dcols[j].len()});
          // output projection: h1 = x + o Wo
          for (size_t j = 0; j < nd; ++j) dO[i][j] = t.gemm_list(dh1[i], won[j], m, t.dcols[j].len(), false, true);
        }
        // attention, one head group (= one column tile) at a time.  The reverse kernels read V as
        // plain tiles and K^T, Q^T, dO^T as row-major tiles of their own.
        auto transposed = [&](tn_vid x, int32_t rws, int32_t cls) {  // x is [rws, cls]
          return t.op(TN_OP_TRANSPOSE, tn_op_params{}, {x}, {c.dtype, cls, rws});
        };
        Grid dq(nr, std::vector<tn_vid>(nd)), dk(nr, std::vector<tn_vid>(nd)), dv(nr, std::vector<tn_vid>(nd));
        for (size_t j = 0; j < nd; ++j) {
          tn_op_params p{};
          p.n_col_tiles = 1;
          p.head_dim = c.head_dim;
          p.causal = 1;
          p.scale = 1.0f / std::sqrt((float)c.head_dim);
          const int32_t n = t.dcols[j].len(), hpg_ = n / c.head_dim;
          std::vector<tn_vid> vn(nr), kT(nr), qT(nr), dOT(nr), stats(nr);
          for (size_t i = 0; i < nr; ++i) {
            const int32_t m = t.rows[i].len();
            vn[i] = c.v_transposed ? transposed(sv.v[i][j], n, m) : sv.v[i][j];
            kT[i] = transposed(sv.k[i][j], m, n);
            qT[i] = transposed(sv.q[i][j], m, n);
            dOT[i] = transposed(dO[i][j], m, n);
          }
          for (size_t i = 0; i < nr; ++i) {  // query tile i against the key tiles 0..i
            std::vector<tn_vid> in{sv.q[i][j]};
            for (size_t r = 0; r <= i; ++r) in.push_back(sv.k[r][j]);
            for (size_t r = 0; r <= i; ++r) in.push_back(vn[r]);
            in.push_back(dO[i][j]);
            p.n_q_tiles = 1;
            p.n_kv_tiles = (int32_t)i + 1;
            p.q_pos0 = t.rows[i].a;
            p.k_pos0 = 0;
            p.mode = 0;
            p.trans_a = 0;
            stats[i] = t.op(TN_OP_ATTN_BWD, p, in, {TN_F32, t.rows[i].len(), 2 * hpg_});
            in.push_back(stats[i]);
            for (size_t r = 0; r <= i; ++r) in.push_back(kT[r]);
            p.mode = 1;
            p.trans_a = 1;
            dq[i][j] = t.op(TN_OP_ATTN_BWD, p, std::move(in), {c.dtype, t.rows[i].len(), n});
          }
          for (size_t r = 0; r < nr; ++r) {  // key tile r against the query tiles r..end
            std::vector<tn_vid> in;
            for (size_t i = r; i < nr; ++i) in.push_back(sv.q[i][j]);
            in.push_back(sv.k[r][j]);
            in.push_back(vn[r]);
            for (size_t i = r; i < nr; ++i) in.push_back(dO[i][j]);
            for (size_t i = r; i < nr; ++i) in.push_back(stats[i]);
            p.n_q_tiles = (int32_t)(nr - r);
            p.n_kv_tiles = 1;
            p.q_pos0 = t.rows[r].a;
            p.k_pos0 = t.rows[r].a;
            p.trans_a = 1;
            std::vector<tn_vid> in_k(in), in_v(in);
            for (size_t i = r; i < nr; ++i) in_k.push_back(qT[i]);
            for (size_t i = r; i < nr; ++i) in_v.push_back(dOT[i]);
            p.mode = 2;
            dk[r][j] = t.op(TN_OP_ATTN_BWD, p, std::move(in_k), {c.dtype, t.rows[r].len(), n});
            p.mode = 3;
            dv[r][j] = t.op(TN_OP_ATTN_BWD, p, std::move(in_v), {c.dtype, t.rows[r].len(), n});
          }
        }
        // projections with adapters, first normalisation, residual
        for (size_t i = 0; i < nr; ++i) {
          const int32_t m = t.rows[i].len();
          std::vector<tn_vid> big;  // dq, dk (before the rotation), dv: operands of the gradient of a
          for (size_t j = 0; j < nd; ++j) {
            dq[i][j] = t.rope(dq[i][j], t.rows[i].a, t.dcols[j].a, m, t.dcols[j].len(), true);
            dk[i][j] = t.rope(dk[i][j], t.rows[i].a, t.dcols[j].a, m, t.dcols[j].len(), true);
          }
          big = dq[i];
          big.insert(big.end(), dk[i].begin(), dk[i].end());
          big.insert(big.end(), dv[i].begin(), dv[i].end());
          // gradients of the low-rank activations: dq Bq^T and dv Bv^T
          tn_vid dtq = t.gemm_list(dq[i], w.bq, m, rk, false, true), dtv = t.gemm_list(dv[i], w.bv, m, rk, false, true);
          std::vector<tn_vid> da(nd);
          for (size_t j = 0; j < nd; ++j) {
            std::vector<tn_vid> bw(wqn[j]);
            bw.insert(bw.end(), wkn[j].begin(), wkn[j].end());
            bw.insert(bw.end(), wvn[j].begin(), wvn[j].end());
            const int32_t n = t.dcols[j].len();
            da[j] = t.add(t.gemm_list(big, bw, m, n, false, true),
                          t.gemm_list({dtq, dtv}, {w.aq[j], w.av[j]}, m, n, false, true), m, n);
          }
          tn_op_params ps{};
          ps.nk = (int32_t)nd;
          std::vector<tn_vid> sin(da);
          sin.insert(sin.end(), sv.xin[i].begin(), sv.xin[i].end());
          sin.insert(sin.end(), w.g1.begin(), w.g1.end());
          tn_vid dot1 = t.op(TN_OP_RMS_BWD_STAT, ps, std::move(sin), {TN_F32, m, 1});
          tn_op_params pa{};
          pa.d = c.d_model;
          for (size_t j = 0; j < nd; ++j)
            dy[b][i][j] = t.op(TN_OP_RMS_BWD_APPLY, pa, {da[j], sv.xin[i][j], sv.rstd1[i], dot1, w.g1[j], dh1[i][j]},
                               {c.dtype, m, t.dcols[j].len()});
          auto tr = [&](tn_vid x, int32_t rws, int32_t cls) {  // x is [rws, cls]
            return t.op(TN_OP_TRANSPOSE, tn_op_params{}, {x}, {c.dtype, cls, rws});
          };
          all_tq.push_back(tr(sv.tq[i], m, rk));
          all_tv.push_back(tr(sv.tv[i], m, rk));
          all_dtq.push_back(tr(dtq, m, rk));
          all_dtv.push_back(tr(dtv, m, rk));
          for (size_t j = 0; j < nd; ++j) {
            const int32_t n = t.dcols[j].len();
            const tn_vid an = c.recompute_normed
                                  ? t.op(TN_OP_RMS_APPLY, tn_op_params{}, {sv.xin[i][j], sv.rstd1[i], w.g1[j]}, {c.dtype, m, n})
                                  : sv.a[i][j];
            a_cols[j].push_back(tr(an, m, n));
            dq_cols[j].push_back(tr(dq[i][j], m, n));
            dv_cols[j].push_back(tr(dv[i][j], m, n));
          }
        }
      }
      // adapter gradients: dA = a^T dt = (a^T)(dt^T)^T, dB = t^T dq = (t^T)(dq^T)^T, summed over every row of
      // every sequence
      for (size_t j = 0; j < nd; ++j) {
        const int32_t n = t.dcols[j].len();
        t.mark_output(t.gemm_list(a_cols[j], all_dtq, n, rk, false, true), TN_T_DAQ, l, t.dcols[j], rkr);
        t.mark_output(t.gemm_list(all_tq, dq_cols[j], rk, n, false, true), TN_T_DBQ, l, rkr, t.dcols[j]);
        t.mark_output(t.gemm_list(a_cols[j], all_dtv, n, rk, false, true), TN_T_DAV, l, t.dcols[j], rkr);
        t.mark_output(t.gemm_list(all_tv, dv_cols[j], rk, n, false, true), TN_T_DBV, l, rkr, t.dcols[j]);
      }
    }
    for (int b = 0; b < c.batch; ++b)
      for (size_t i = 0; i < nr; ++i)
        for (size_t j = 0; j < nd; ++j)
          t.mark_output(dy[b][i][j], TN_T_DX, -1, {b * c.seq + t.rows[i].a, b * c.seq + t.rows[i].b}, t.dcols[j]);
  }
  // every vertex the tiler emitted must satisfy the same rules a caller's would
  for (size_t v = 0; v < tg->v.size(); ++v) {
    const Vertex& x_ = tg->v[v];
    if (x_.kind == TN_OP_INPUT) continue;
    tn_status s = validate_op(*tg, x_.kind, x_.p, x_.in.data(), (int32_t)x_.in.size(), x_.desc);
    if (s != TN_OK) {
      delete tg;
      return s;
    }
  }
  *out = tg;
  return TN_OK;
}

}  // extern "C"
