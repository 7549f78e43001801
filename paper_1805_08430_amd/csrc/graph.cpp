// Static shape inference over a small dataflow graph (paper section 3.4, first
// step of the analyzer): user-annotated input shapes + one shape function per
// node decide which cross-partition tensors have shapes that never change.
#include <cstring>
#include <set>
#include <string>
#include <vector>

#include "planner.h"
#include "rdev.h"

namespace rdev {
rdev_status fail_msg(rdev_status st, const std::string &msg);   // sets the thread's error text (rdev.hip)
}
using rdev::fail_msg;

namespace {

struct Value {
    uint32_t dtype = 0;
    std::vector<int64_t> dims;
    uint32_t partition = 0;
    int32_t node = -1;          // producing node, -1 for inputs
    bool inferred = false;
};

struct Node {
    uint32_t op;
    std::vector<uint32_t> in;
    std::vector<int64_t> attrs;
    uint32_t partition;
    uint32_t out;
};

bool known(int64_t d) { return d >= 0; }

// product of dims if all known
bool count(const std::vector<int64_t> &d, uint64_t *n) {
    uint64_t c = 1;
    for (int64_t x : d) {
        if (!known(x)) return false;
        if (__builtin_mul_overflow(c, (uint64_t)x, &c)) return false;
    }
    *n = c;
    return true;
}

}  // namespace

struct rdev_graph_s {
    std::vector<Value> values;
    std::vector<Node> nodes;
};

namespace {

rdev_status infer_node(rdev_graph_t *g, const Node &n, std::string &why) {
    auto in = [&](size_t i) -> const Value & { return g->values[n.in[i]]; };
    Value &o = g->values[n.out];
    auto need_inputs = [&](size_t lo, size_t hi) {
        if (n.in.size() < lo || n.in.size() > hi) { why = "wrong number of inputs"; return false; }
        return true;
    };
    switch (n.op) {
        case RDEV_OP_UNARY:
            if (!need_inputs(1, 1)) return RDEV_E_INVAL;
            o.dtype = in(0).dtype;
            o.dims = in(0).dims;
            return RDEV_OK;
        case RDEV_OP_CAST:
            if (!need_inputs(1, 1) || n.attrs.size() != 1 || !rdev::dtype_size((uint32_t)n.attrs[0])) { why = "cast needs one input and a valid type"; return RDEV_E_INVAL; }
            o.dtype = (uint32_t)n.attrs[0];
            o.dims = in(0).dims;
            return RDEV_OK;
        case RDEV_OP_BINARY: {
            if (!need_inputs(2, 2)) return RDEV_E_INVAL;
            if (in(0).dtype != in(1).dtype) { why = "element types differ"; return RDEV_E_INVAL; }
            const auto &a = in(0).dims, &b = in(1).dims;
            const size_t r = std::max(a.size(), b.size());
            std::vector<int64_t> d(r);
            for (size_t k = 0; k < r; ++k) {              // k counts from the last dim
                const int64_t x = k < a.size() ? a[a.size() - 1 - k] : 1;
                const int64_t y = k < b.size() ? b[b.size() - 1 - k] : 1;
                int64_t z;
                if (x == 1) z = y;
                else if (y == 1) z = x;
                else if (!known(x)) z = y;               // unknown against a known size > 1: must equal it
                else if (!known(y)) z = x;
                else if (x == y) z = x;
                else { why = "shapes do not broadcast"; return RDEV_E_INVAL; }
                d[r - 1 - k] = z;
            }
            o.dtype = in(0).dtype;
            o.dims = d;
            return RDEV_OK;
        }
        case RDEV_OP_MATMUL: {
            if (!need_inputs(2, 2) || n.attrs.size() != 2) { why = "matmul needs 2 inputs and 2 attrs"; return RDEV_E_INVAL; }
            if (in(0).dtype != in(1).dtype) { why = "element types differ"; return RDEV_E_INVAL; }
            std::vector<int64_t> a = in(0).dims, b = in(1).dims;
            if (a.size() < 2 || b.size() != 2) { why = "matmul takes [.., m, k] x [k, n]"; return RDEV_E_INVAL; }
            if (n.attrs[0]) std::swap(a[a.size() - 1], a[a.size() - 2]);
            if (n.attrs[1]) std::swap(b[0], b[1]);
            const int64_t k1 = a.back(), k2 = b[0];
            if (known(k1) && known(k2) && k1 != k2) { why = "inner dims differ"; return RDEV_E_INVAL; }
            a.back() = b[1];
            o.dtype = in(0).dtype;
            o.dims = a;
            return RDEV_OK;
        }
        case RDEV_OP_TRANSPOSE: {
            if (!need_inputs(1, 1)) return RDEV_E_INVAL;
            const auto &a = in(0).dims;
            if (n.attrs.size() != a.size()) { why = "permutation length differs from the rank"; return RDEV_E_INVAL; }
            std::vector<int64_t> d(a.size());
            std::set<int64_t> seen;
            for (size_t k = 0; k < a.size(); ++k) {
                if (n.attrs[k] < 0 || (size_t)n.attrs[k] >= a.size() || !seen.insert(n.attrs[k]).second) { why = "not a permutation"; return RDEV_E_INVAL; }
                d[k] = a[n.attrs[k]];
            }
            o.dtype = in(0).dtype;
            o.dims = d;
            return RDEV_OK;
        }
        case RDEV_OP_RESHAPE: {
            if (!need_inputs(1, 1)) return RDEV_E_INVAL;
            std::vector<int64_t> d(n.attrs.begin(), n.attrs.end());
            int hole = -1;
            uint64_t prod = 1;
            for (size_t k = 0; k < d.size(); ++k) {
                if (d[k] == -1) { if (hole >= 0) { why = "more than one -1 in reshape"; return RDEV_E_INVAL; } hole = (int)k; }
                else if (d[k] < 0) { why = "negative dim"; return RDEV_E_INVAL; }
                else prod *= (uint64_t)d[k];
            }
            uint64_t total;
            if (count(in(0).dims, &total)) {
                if (hole >= 0) {
                    if (prod == 0 || total % prod) { why = "element count does not divide"; return RDEV_E_INVAL; }
                    d[hole] = (int64_t)(total / prod);
                } else if (prod != total) { why = "element count changes"; return RDEV_E_INVAL; }
            }
            o.dtype = in(0).dtype;
            o.dims = d;
            return RDEV_OK;
        }
        case RDEV_OP_CONCAT: {
            if (n.in.empty() || n.attrs.size() != 1) { why = "concat needs inputs and an axis"; return RDEV_E_INVAL; }
            std::vector<int64_t> d = in(0).dims;
            const int64_t ax = n.attrs[0];
            if (ax < 0 || (size_t)ax >= d.size()) { why = "axis out of range"; return RDEV_E_INVAL; }
            for (size_t i = 1; i < n.in.size(); ++i) {
                const auto &b = in(i).dims;
                if (b.size() != d.size() || in(i).dtype != in(0).dtype) { why = "ranks or types differ"; return RDEV_E_INVAL; }
                for (size_t k = 0; k < d.size(); ++k) {
                    if ((int64_t)k == ax) d[k] = (known(d[k]) && known(b[k])) ? d[k] + b[k] : -1;
                    else if (known(d[k]) && known(b[k]) && d[k] != b[k]) { why = "non-axis dims differ"; return RDEV_E_INVAL; }
                    else if (!known(d[k])) d[k] = b[k];
                }
            }
            o.dtype = in(0).dtype;
            o.dims = d;
            return RDEV_OK;
        }
        case RDEV_OP_REDUCE: {
            if (!need_inputs(1, 1) || n.attrs.empty()) { why = "reduce needs keepdims and axes"; return RDEV_E_INVAL; }
            const auto &a = in(0).dims;
            std::set<int64_t> axes;
            for (size_t k = 1; k < n.attrs.size(); ++k) {
                if (n.attrs[k] < 0 || (size_t)n.attrs[k] >= a.size() || !axes.insert(n.attrs[k]).second) { why = "bad axis"; return RDEV_E_INVAL; }
            }
            std::vector<int64_t> d;
            for (size_t k = 0; k < a.size(); ++k) {
                if (!axes.count((int64_t)k)) d.push_back(a[k]);
                else if (n.attrs[0]) d.push_back(1);
            }
            o.dtype = in(0).dtype;
            o.dims = d;
            return RDEV_OK;
        }
        case RDEV_OP_GATHER: {
            if (!need_inputs(2, 2)) return RDEV_E_INVAL;
            const auto &p = in(0).dims, &ids = in(1).dims;
            if (p.empty()) { why = "gather from a scalar"; return RDEV_E_INVAL; }
            std::vector<int64_t> d(ids);
            d.insert(d.end(), p.begin() + 1, p.end());
            o.dtype = in(0).dtype;
            o.dims = d;
            return RDEV_OK;
        }
        case RDEV_OP_UNIQUE:
            if (!need_inputs(1, 1)) return RDEV_E_INVAL;
            o.dtype = in(0).dtype;
            o.dims = {-1};
            return RDEV_OK;
        case RDEV_OP_CONV2D: {
            if (!need_inputs(2, 2) || n.attrs.size() != 3) { why = "conv2d needs 2 inputs and 3 attrs"; return RDEV_E_INVAL; }
            const auto &x = in(0).dims, &f = in(1).dims;
            if (x.size() != 4 || f.size() != 4 || n.attrs[0] < 1 || n.attrs[1] < 1) { why = "conv2d takes NHWC x HWIO with strides >= 1"; return RDEV_E_INVAL; }
            if (known(x[3]) && known(f[2]) && x[3] != f[2]) { why = "channel counts differ"; return RDEV_E_INVAL; }
            auto out_dim = [&](int64_t i, int64_t k, int64_t s) -> int64_t {
                if (!known(i) || !known(k)) return -1;
                if (n.attrs[2]) return (i + s - 1) / s;                 // same
                return i >= k ? (i - k) / s + 1 : 0;                      // valid
            };
            o.dtype = in(0).dtype;
            o.dims = {x[0], out_dim(x[1], f[0], n.attrs[0]), out_dim(x[2], f[1], n.attrs[1]), f[3]};
            return RDEV_OK;
        }
        case RDEV_OP_GRAD:
            if (n.in.empty()) { why = "grad needs the value it differentiates against"; return RDEV_E_INVAL; }
            o.dtype = in(n.in.size() - 1).dtype;
            o.dims = in(n.in.size() - 1).dims;
            return RDEV_OK;
        default:
            why = "unknown op";
            return RDEV_E_INVAL;
    }
}

}  // namespace

extern "C" {

rdev_status rdev_graph_open(rdev_graph_t **out) {
    if (!out) return fail_msg(RDEV_E_INVAL, "NULL argument");
    *out = new rdev_graph_t();
    return RDEV_OK;
}

rdev_status rdev_graph_close(rdev_graph_t *g) {
    if (!g) return fail_msg(RDEV_E_INVAL, "NULL argument");
    delete g;
    return RDEV_OK;
}

rdev_status rdev_graph_input(rdev_graph_t *g, uint32_t dtype, uint32_t ndims, const int64_t *dims, uint32_t partition,
                             uint32_t *value_out) {
    if (!g || !value_out || (!dims && ndims)) return fail_msg(RDEV_E_INVAL, "NULL argument");
    if (!rdev::dtype_size(dtype)) return fail_msg(RDEV_E_INVAL, "unknown element type");
    if (ndims > RDEV_MAX_DIMS) return fail_msg(RDEV_E_INVAL, "rank exceeds RDEV_MAX_DIMS");
    Value v;
    v.dtype = dtype;
    for (uint32_t i = 0; i < ndims; ++i) {
        if (dims[i] < -1) return fail_msg(RDEV_E_INVAL, "negative dim");
        v.dims.push_back(dims[i]);
    }
    v.partition = partition;
    v.inferred = true;
    g->values.push_back(v);
    *value_out = (uint32_t)g->values.size() - 1;
    return RDEV_OK;
}

rdev_status rdev_graph_node(rdev_graph_t *g, uint32_t op, const uint32_t *inputs, uint32_t n_inputs,
                            const int64_t *attrs, uint32_t n_attrs, uint32_t partition, uint32_t *value_out) {
    if (!g || !value_out || (!inputs && n_inputs) || (!attrs && n_attrs)) return fail_msg(RDEV_E_INVAL, "NULL argument");
    if (op > RDEV_OP_CAST) return fail_msg(RDEV_E_INVAL, "unknown op");
    Node n;
    n.op = op;
    for (uint32_t i = 0; i < n_inputs; ++i) {
        if (inputs[i] >= g->values.size()) return fail_msg(RDEV_E_INVAL, "input value does not exist yet");
        n.in.push_back(inputs[i]);
    }
    n.attrs.assign(attrs, attrs + n_attrs);
    n.partition = partition;
    Value v;
    v.partition = partition;
    v.node = (int32_t)g->nodes.size();
    g->values.push_back(v);
    n.out = (uint32_t)g->values.size() - 1;
    g->nodes.push_back(n);
    *value_out = n.out;
    return RDEV_OK;
}

rdev_status rdev_graph_infer(rdev_graph_t *g) {
    if (!g) return fail_msg(RDEV_E_INVAL, "NULL argument");
    for (size_t k = 0; k < g->nodes.size(); ++k) {
        std::string why;
        rdev_status st = infer_node(g, g->nodes[k], why);
        if (st != RDEV_OK) return fail_msg(st, "node " + std::to_string(k) + " (op " + std::to_string(g->nodes[k].op) + "): " + why);
        Value &o = g->values[g->nodes[k].out];
        if (o.dims.size() > RDEV_MAX_DIMS) return fail_msg(RDEV_E_INVAL, "node " + std::to_string(k) + ": rank exceeds RDEV_MAX_DIMS");
        o.inferred = true;
    }
    return RDEV_OK;
}

rdev_status rdev_graph_value(const rdev_graph_t *g, uint32_t value, rdev_tensor_desc *out) {
    if (!g || !out) return fail_msg(RDEV_E_INVAL, "NULL argument");
    if (value >= g->values.size()) return fail_msg(RDEV_E_INVAL, "unknown value");
    const Value &v = g->values[value];
    if (!v.inferred) return fail_msg(RDEV_E_STATE, "shapes have not been inferred");
    std::memset(out, 0, sizeof(*out));
    out->tensor_id = value;
    out->dtype = v.dtype;
    out->ndims = (uint32_t)v.dims.size();
    out->dst_arena = v.partition;
    for (size_t i = 0; i < v.dims.size(); ++i) out->dims[i] = v.dims[i];
    return RDEV_OK;
}

rdev_status rdev_graph_transfers(const rdev_graph_t *g, const uint32_t *partition_to_arena, uint32_t n_partitions,
                                 rdev_tensor_desc *out, uint32_t *values_out, uint32_t *dst_partitions_out,
                                 uint32_t cap, uint32_t *n_out) {
    if (!g || !n_out || !partition_to_arena || (!out && cap)) return fail_msg(RDEV_E_INVAL, "NULL argument");
    std::set<std::pair<uint32_t, uint32_t>> edges;           // (value, consumer partition)
    for (const Node &n : g->nodes)
        for (uint32_t v : n.in)
            if (g->values[v].partition != n.partition) edges.insert({v, n.partition});
    uint32_t i = 0;
    for (const auto &e : edges) {
        const Value &v = g->values[e.first];
        if (!v.inferred) return fail_msg(RDEV_E_STATE, "shapes have not been inferred");
        if (e.second >= n_partitions) return fail_msg(RDEV_E_INVAL, "partition without an arena");
        if (i < cap) {
            std::memset(&out[i], 0, sizeof(out[i]));
            out[i].tensor_id = i;
            out[i].dtype = v.dtype;
            out[i].ndims = (uint32_t)v.dims.size();
            out[i].dst_arena = partition_to_arena[e.second];
            for (size_t k = 0; k < v.dims.size(); ++k) out[i].dims[k] = v.dims[k];
            if (values_out) values_out[i] = e.first;
            if (dst_partitions_out) dst_partitions_out[i] = e.second;
        }
        ++i;
    }
    *n_out = i;
    if (i > cap) return fail_msg(RDEV_E_NOMEM, "output arrays too small for " + std::to_string(i) + " transfers");
    return RDEV_OK;
}

}  // extern "C"
