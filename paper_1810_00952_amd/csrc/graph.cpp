// Typing rules and fusion-group legality (host only).
#include "graph.h"
#include "kernels.h"

#include <algorithm>
#include <set>
#include <sstream>

namespace rl {

static const char *kOpNames[RL_OP_KIND_COUNT] = {
    "dense", "conv2d", "bias_add", "add", "sub", "mul", "div", "neg", "sq", "relu", "sigmoid", "tanh",
    "maxpool2d", "global_avgpool", "flatten", "lstm_gates", "cast", "concat", "layout_transform",
    "dense_grad_x", "dense_grad_w", "conv2d_grad_x", "conv2d_grad_w"};

const char *op_name(int kind) { return (kind >= 0 && kind < RL_OP_KIND_COUNT) ? kOpNames[kind] : "?"; }
bool is_anchor(int kind) { return kind == RL_OP_DENSE || kind == RL_OP_CONV2D; }
bool is_injective(int kind)
{
    switch (kind) {
    case RL_OP_BIAS_ADD: case RL_OP_ADD: case RL_OP_SUB: case RL_OP_MUL: case RL_OP_DIV: case RL_OP_NEG:
    case RL_OP_SQ: case RL_OP_RELU: case RL_OP_SIGMOID: case RL_OP_TANH: case RL_OP_CAST:
        return true;
    default:
        return false;
    }
}

bool same_type(const rl_type &a, const rl_type &b)
{
    if (a.dtype != b.dtype || a.rank != b.rank) return false;
    for (int i = 0; i < a.rank; ++i)
        if (a.dims[i] != b.dims[i]) return false;
    return true;
}

std::string type_str(const rl_type &t)
{
    std::ostringstream o;
    o << "Tensor(" << (t.dtype == RL_F32 ? "f32" : t.dtype == RL_BF16 ? "bf16" : "?") << ", Shape(";
    for (int i = 0; i < t.rank && i < RL_MAX_RANK; ++i) o << (i ? "," : "") << t.dims[i];
    o << "))";
    return o.str();
}

int64_t numel(const rl_type &t)
{
    int64_t n = 1;
    for (int i = 0; i < t.rank; ++i) n *= t.dims[i];
    return n;
}

size_t dtype_size(int dtype) { return dtype == RL_BF16 ? 2 : 4; }

rl_status check_tensor_type(const rl_type &t, std::string &msg)
{
    if (t.dtype != RL_F32 && t.dtype != RL_BF16) { msg = "unknown base type"; return RL_ERR_KIND; }
    if (t.rank < 0 || t.rank > RL_MAX_RANK) { msg = "rank out of range"; return RL_ERR_KIND; }
    for (int i = 0; i < t.rank; ++i)
        if (t.dims[i] < 1) { msg = "dimension is not a positive constant"; return RL_ERR_SHAPE; }
    if (numel(t) > (int64_t)1 << 40) { msg = "tensor too large"; return RL_ERR_SHAPE; }
    return RL_OK;
}

rl_status parse_attrs(int kind, const void *attrs, size_t size, Attrs &a, std::string &msg)
{
    auto want = [&](size_t s) -> bool {
        if (attrs && size != s) { msg = std::string("attribute struct size mismatch for ") + op_name(kind); return false; }
        return true;
    };
    switch (kind) {
    case RL_OP_DENSE: case RL_OP_DENSE_GRAD_X: case RL_OP_DENSE_GRAD_W:
        if (!want(sizeof(rl_attr_contract))) return RL_ERR_KIND;
        if (attrs) a.out_dtype = ((const rl_attr_contract *)attrs)->out_dtype;
        break;
    case RL_OP_CONV2D: case RL_OP_CONV2D_GRAD_X: case RL_OP_CONV2D_GRAD_W: {
        if (!attrs) { msg = std::string(op_name(kind)) + " needs rl_attr_conv2d"; return RL_ERR_KIND; }
        if (!want(sizeof(rl_attr_conv2d))) return RL_ERR_KIND;
        const rl_attr_conv2d *c = (const rl_attr_conv2d *)attrs;
        a.stride[0] = c->stride_h; a.stride[1] = c->stride_w; a.pad[0] = c->pad_h; a.pad[1] = c->pad_w;
        a.out_dtype = c->out_dtype;
        if (c->stride_h < 1 || c->stride_w < 1 || c->pad_h < 0 || c->pad_w < 0) { msg = "bad stride/pad"; return RL_ERR_KIND; }
        if (c->dilation_h != 1 || c->dilation_w != 1 || c->groups != 1) { msg = "dilation/groups other than 1"; return RL_ERR_UNSUPPORTED; }
        break;
    }
    case RL_OP_BIAS_ADD: case RL_OP_CONCAT:
        if (!want(sizeof(rl_attr_axis))) return RL_ERR_KIND;
        if (attrs) a.axis = ((const rl_attr_axis *)attrs)->axis;
        break;
    case RL_OP_MAXPOOL2D: {
        if (!attrs) { msg = "maxpool2d needs rl_attr_pool2d"; return RL_ERR_KIND; }
        if (!want(sizeof(rl_attr_pool2d))) return RL_ERR_KIND;
        const rl_attr_pool2d *c = (const rl_attr_pool2d *)attrs;
        a.kernel[0] = c->kernel_h; a.kernel[1] = c->kernel_w; a.stride[0] = c->stride_h; a.stride[1] = c->stride_w;
        a.pad[0] = c->pad_h; a.pad[1] = c->pad_w;
        if (c->kernel_h < 1 || c->kernel_w < 1 || c->stride_h < 1 || c->stride_w < 1 || c->pad_h < 0 || c->pad_w < 0 ||
            c->pad_h >= c->kernel_h || c->pad_w >= c->kernel_w) { msg = "bad pool attributes"; return RL_ERR_KIND; }
        break;
    }
    case RL_OP_CAST:
        if (!attrs) { msg = "cast needs rl_attr_cast"; return RL_ERR_KIND; }
        if (!want(sizeof(rl_attr_cast))) return RL_ERR_KIND;
        a.to = ((const rl_attr_cast *)attrs)->to;
        if (a.to != RL_F32 && a.to != RL_BF16) { msg = "cast to unknown base type"; return RL_ERR_KIND; }
        break;
    case RL_OP_LAYOUT_TRANSFORM: {
        if (!attrs) { msg = "layout_transform needs rl_attr_layout"; return RL_ERR_KIND; }
        if (!want(sizeof(rl_attr_layout))) return RL_ERR_KIND;
        for (int i = 0; i < RL_MAX_RANK; ++i) a.perm[i] = ((const rl_attr_layout *)attrs)->perm[i];
        break;                                  // checked against the operand's rank in infer_type
    }
    default:
        break;
    }
    return RL_OK;
}

static rl_type make_type(int dtype, std::initializer_list<int64_t> dims)
{
    rl_type t{};
    t.dtype = dtype;
    t.rank = (int32_t)dims.size();
    int i = 0;
    for (int64_t d : dims) t.dims[i++] = d;
    return t;
}

rl_status infer_type(int kind, const std::vector<rl_type> &in, const Attrs &a, const std::vector<rl_type> &declared,
                     std::vector<rl_type> &out, std::string &msg)
{
    auto arity = [&](size_t n) -> bool {
        if (in.size() != n) { msg = std::string(op_name(kind)) + ": wrong number of arguments"; return false; }
        return true;
    };
    auto out_dtype = [&](int in_dt, int &od) -> bool {
        od = a.out_dtype < 0 ? in_dt : a.out_dtype;
        if (od != in_dt && od != RL_F32) { msg = "out_dtype not allowed for these operands"; return false; }
        return true;
    };
    out.clear();
    switch (kind) {
    case RL_OP_NEG: case RL_OP_SQ: case RL_OP_RELU: case RL_OP_SIGMOID: case RL_OP_TANH:      // Type-UnaryOp
        if (!arity(1)) return RL_ERR_TYPE;
        out.push_back(in[0]);
        return RL_OK;
    case RL_OP_ADD: case RL_OP_SUB: case RL_OP_MUL: case RL_OP_DIV:                             // Type-Noncomp-BinaryOp
        if (!arity(2)) return RL_ERR_TYPE;
        if (!same_type(in[0], in[1])) {
            msg = std::string(op_name(kind)) + ": operands " + type_str(in[0]) + " and " + type_str(in[1]) +
                  " differ (no implicit broadcast or promotion)";
            return RL_ERR_TYPE;
        }
        out.push_back(in[0]);
        return RL_OK;
    case RL_OP_BIAS_ADD: {
        if (!arity(2)) return RL_ERR_TYPE;
        const rl_type &x = in[0], &b = in[1];
        if (a.axis < 0 || a.axis >= x.rank) { msg = "bias_add axis out of range"; return RL_ERR_TYPE; }
        if (b.rank != 1 || b.dims[0] != x.dims[a.axis]) { msg = "bias shape does not match the axis"; return RL_ERR_TYPE; }
        if (!(b.dtype == x.dtype || (x.dtype == RL_BF16 && b.dtype == RL_F32))) { msg = "bias dtype not allowed"; return RL_ERR_TYPE; }
        out.push_back(x);
        return RL_OK;
    }
    case RL_OP_DENSE: {
        if (!arity(2)) return RL_ERR_TYPE;
        const rl_type &x = in[0], &w = in[1];
        if (x.rank != 2 || w.rank != 2) { msg = "dense wants rank-2 operands"; return RL_ERR_TYPE; }
        if (x.dtype != w.dtype) { msg = "dense operands differ in base type"; return RL_ERR_TYPE; }
        if (x.dims[1] != w.dims[1]) { msg = "dense inner dimensions differ"; return RL_ERR_TYPE; }
        int od;
        if (!out_dtype(x.dtype, od)) return RL_ERR_TYPE;
        out.push_back(make_type(od, {x.dims[0], w.dims[0]}));
        return RL_OK;
    }
    case RL_OP_CONV2D: {
        if (!arity(2)) return RL_ERR_TYPE;
        const rl_type &x = in[0], &w = in[1];
        if (x.rank != 4 || w.rank != 4) { msg = "conv2d wants rank-4 operands"; return RL_ERR_TYPE; }
        if (x.dtype != w.dtype) { msg = "conv2d operands differ in base type"; return RL_ERR_TYPE; }
        if (x.dims[1] != w.dims[1]) { msg = "conv2d channel counts differ"; return RL_ERR_TYPE; }
        if (x.dims[2] + 2 * a.pad[0] < w.dims[2] || x.dims[3] + 2 * a.pad[1] < w.dims[3]) {
            msg = "kernel larger than padded input";
            return RL_ERR_SHAPE;
        }
        int od;
        if (!out_dtype(x.dtype, od)) return RL_ERR_TYPE;
        int64_t oh = (x.dims[2] + 2 * a.pad[0] - w.dims[2]) / a.stride[0] + 1;
        int64_t ow = (x.dims[3] + 2 * a.pad[1] - w.dims[3]) / a.stride[1] + 1;
        out.push_back(make_type(od, {x.dims[0], w.dims[0], oh, ow}));
        return RL_OK;
    }
    case RL_OP_DENSE_GRAD_X: case RL_OP_DENSE_GRAD_W: {
        if (!arity(2)) return RL_ERR_TYPE;
        const rl_type &dy = in[0], &b = in[1];
        if (dy.rank != 2 || b.rank != 2) { msg = std::string(op_name(kind)) + " wants rank-2 operands"; return RL_ERR_TYPE; }
        if (dy.dtype != b.dtype) { msg = std::string(op_name(kind)) + " operands differ in base type"; return RL_ERR_TYPE; }
        int od;
        if (!out_dtype(dy.dtype, od)) return RL_ERR_TYPE;
        if (kind == RL_OP_DENSE_GRAD_X) {
            if (dy.dims[1] != b.dims[0]) { msg = "dense_grad_x: dy's columns and W's rows differ"; return RL_ERR_TYPE; }
            out.push_back(make_type(od, {dy.dims[0], b.dims[1]}));
        } else {
            if (dy.dims[0] != b.dims[0]) { msg = "dense_grad_w: dy and x differ in their first dimension"; return RL_ERR_TYPE; }
            out.push_back(make_type(od, {dy.dims[1], b.dims[1]}));
        }
        return RL_OK;
    }
    case RL_OP_CONV2D_GRAD_X: case RL_OP_CONV2D_GRAD_W: {
        if (!arity(2)) return RL_ERR_TYPE;
        const rl_type &dy = in[0], &b = in[1];
        if (dy.rank != 4 || b.rank != 4) { msg = std::string(op_name(kind)) + " wants rank-4 operands"; return RL_ERR_TYPE; }
        if (dy.dtype != b.dtype) { msg = std::string(op_name(kind)) + " operands differ in base type"; return RL_ERR_TYPE; }
        if (declared.size() != 1 || declared[0].rank != 4) { msg = std::string(op_name(kind)) + ": the declared result must be rank 4"; return RL_ERR_TYPE; }
        const rl_type &d = declared[0];
        int64_t H, W, KH, KW;
        bool ok;
        if (kind == RL_OP_CONV2D_GRAD_X) {       // b = w[O,C,KH,KW], d = [N,C,H,W]
            H = d.dims[2]; W = d.dims[3]; KH = b.dims[2]; KW = b.dims[3];
            ok = d.dims[0] == dy.dims[0] && d.dims[1] == b.dims[1] && dy.dims[1] == b.dims[0];
        } else {                                 // b = x[N,C,H,W], d = [O,C,KH,KW]
            H = b.dims[2]; W = b.dims[3]; KH = d.dims[2]; KW = d.dims[3];
            ok = d.dims[0] == dy.dims[1] && d.dims[1] == b.dims[1] && dy.dims[0] == b.dims[0];
        }
        if (!ok) { msg = std::string(op_name(kind)) + ": batch / channel counts of operands and declared result disagree"; return RL_ERR_TYPE; }
        if (H + 2 * a.pad[0] < KH || W + 2 * a.pad[1] < KW) { msg = "kernel larger than padded input"; return RL_ERR_SHAPE; }
        if ((H + 2 * a.pad[0] - KH) / a.stride[0] + 1 != dy.dims[2] || (W + 2 * a.pad[1] - KW) / a.stride[1] + 1 != dy.dims[3]) {
            msg = std::string(op_name(kind)) + ": the forward convolution of the declared geometry does not give dy's size";
            return RL_ERR_TYPE;
        }
        int od;
        if (!out_dtype(dy.dtype, od)) return RL_ERR_TYPE;
        rl_type t = d;
        t.dtype = od;
        out.push_back(t);
        return RL_OK;
    }
    case RL_OP_MAXPOOL2D: {
        if (!arity(1)) return RL_ERR_TYPE;
        const rl_type &x = in[0];
        if (x.rank != 4) { msg = "maxpool2d wants rank 4"; return RL_ERR_TYPE; }
        if (x.dims[2] + 2 * a.pad[0] < a.kernel[0] || x.dims[3] + 2 * a.pad[1] < a.kernel[1]) {
            msg = "window larger than padded input";
            return RL_ERR_SHAPE;
        }
        out.push_back(make_type(x.dtype, {x.dims[0], x.dims[1], (x.dims[2] + 2 * a.pad[0] - a.kernel[0]) / a.stride[0] + 1,
                                          (x.dims[3] + 2 * a.pad[1] - a.kernel[1]) / a.stride[1] + 1}));
        return RL_OK;
    }
    case RL_OP_GLOBAL_AVGPOOL:
        if (!arity(1)) return RL_ERR_TYPE;
        if (in[0].rank != 4) { msg = "global_avgpool wants rank 4"; return RL_ERR_TYPE; }
        out.push_back(make_type(in[0].dtype, {in[0].dims[0], in[0].dims[1], 1, 1}));
        return RL_OK;
    case RL_OP_FLATTEN: {
        if (!arity(1)) return RL_ERR_TYPE;
        if (in[0].rank < 2) { msg = "flatten wants rank >= 2"; return RL_ERR_TYPE; }
        int64_t rest = 1;
        for (int i = 1; i < in[0].rank; ++i) rest *= in[0].dims[i];
        out.push_back(make_type(in[0].dtype, {in[0].dims[0], rest}));
        return RL_OK;
    }
    case RL_OP_CONCAT: {
        if (!arity(2)) return RL_ERR_TYPE;
        if (a.axis != 1 || in[0].rank != 2 || in[1].rank != 2) { msg = "concat: rank 2, axis 1 only"; return RL_ERR_UNSUPPORTED; }
        if (in[0].dtype != in[1].dtype || in[0].dims[0] != in[1].dims[0]) { msg = "concat operands disagree"; return RL_ERR_TYPE; }
        out.push_back(make_type(in[0].dtype, {in[0].dims[0], in[0].dims[1] + in[1].dims[1]}));
        return RL_OK;
    }
    case RL_OP_CAST:
        if (!arity(1)) return RL_ERR_TYPE;
        out.push_back(in[0]);
        out[0].dtype = a.to;
        return RL_OK;
    case RL_OP_LAYOUT_TRANSFORM: {
        if (!arity(1)) return RL_ERR_TYPE;
        const int r = in[0].rank;
        uint32_t seen = 0;
        for (int i = 0; i < r; ++i) {
            if (a.perm[i] < 0 || a.perm[i] >= r || (seen >> a.perm[i] & 1u)) { msg = "layout_transform: perm is not a permutation of the operand's axes"; return RL_ERR_KIND; }
            seen |= 1u << a.perm[i];
        }
        rl_type t = in[0];
        for (int i = 0; i < r; ++i) t.dims[i] = in[0].dims[a.perm[i]];
        out.push_back(t);
        return RL_OK;
    }
    case RL_OP_LSTM_GATES: {
        if (!arity(2)) return RL_ERR_TYPE;
        const rl_type &z = in[0], &c = in[1];
        if (z.dtype != RL_F32 || c.dtype != RL_F32) { msg = "lstm_gates wants f32 pre-activations and cell state"; return RL_ERR_TYPE; }
        if (z.rank != 2 || c.rank != 2 || z.dims[0] != c.dims[0] || z.dims[1] != 4 * c.dims[1]) {
            msg = "lstm_gates: z must be [B,4H] for c [B,H]";
            return RL_ERR_TYPE;
        }
        out.push_back(c);
        rl_type h = c;
        h.dtype = declared.size() == 2 ? declared[1].dtype : RL_F32;   // h' base type comes from the declaration
        out.push_back(h);
        return RL_OK;
    }
    default:
        msg = "unknown operator kind";
        return RL_ERR_KIND;
    }
}

rl_status check_group(const Graph &g, const std::vector<int> &ops_in, std::string &msg)
{
    if (ops_in.empty()) { msg = "empty group"; return RL_ERR_GROUP; }
    std::vector<int> ops = ops_in;
    std::sort(ops.begin(), ops.end());
    for (size_t i = 0; i < ops.size(); ++i) {
        if (ops[i] < 0 || ops[i] >= (int)g.ops.size()) { msg = "group names an unknown op"; return RL_ERR_GROUP; }
        if (i && ops[i] == ops[i - 1]) { msg = "op listed twice"; return RL_ERR_GROUP; }
    }
    std::set<int> gset(ops.begin(), ops.end());
    size_t lead = 0;
    if (ops.size() > 1 && g.ops[ops[0]].kind == RL_OP_CONCAT && g.ops[ops[1]].kind == RL_OP_DENSE) lead = 1;
    int n_anchor = 0;
    for (int o : ops) n_anchor += is_anchor(g.ops[o].kind);
    if (n_anchor > 1) { msg = "more than one contraction in a group"; return RL_ERR_GROUP; }
    if (n_anchor == 1 && !is_anchor(g.ops[ops[lead]].kind)) { msg = "the contraction is not the group's first operator"; return RL_ERR_GROUP; }
    size_t tail0 = n_anchor ? lead + 1 : 0;
    if (ops.size() > 1) {
        for (size_t i = tail0; i < ops.size(); ++i) {
            int k = g.ops[ops[i]].kind;
            // lstm_gates closes a group only behind a dense contraction (it is the contraction's epilogue there);
            // behind a bare injective chain it stays a group of its own
            bool last_gate = (k == RL_OP_LSTM_GATES && i + 1 == ops.size() && n_anchor == 1 && g.ops[ops[lead]].kind == RL_OP_DENSE);
            if (!is_injective(k) && !last_gate) { msg = std::string(op_name(k)) + " cannot be fused"; return RL_ERR_GROUP; }
            if (last_gate) {
                // its pre-activations are the value the rest of the group computes, its cell state comes from outside
                const OpNode &go = g.ops[ops[i]];
                const int zprod = g.values[go.in[0]].producer, cprod = g.values[go.in[1]].producer;
                if (zprod != ops[i - 1]) { msg = "lstm_gates must take the group's last result as its first operand"; return RL_ERR_GROUP; }
                if (cprod >= 0 && gset.count(cprod)) { msg = "lstm_gates' cell state must come from outside the group"; return RL_ERR_GROUP; }
            }
        }
    }
    // connected: every op after the first consumes something produced inside the group
    for (size_t i = 1; i < ops.size(); ++i) {
        bool linked = false;
        for (int v : g.ops[ops[i]].in)
            if (g.values[v].producer >= 0 && gset.count(g.values[v].producer)) linked = true;
        if (!linked) { msg = "group is not connected"; return RL_ERR_GROUP; }
    }
    // only the last op's results may be seen outside
    std::set<int> outs(g.outputs.begin(), g.outputs.end());
    for (size_t i = 0; i < ops.size(); ++i) {
        bool escapes = false;
        for (int v : g.ops[ops[i]].out) {
            if (outs.count(v)) escapes = true;
            for (size_t c = 0; c < g.ops.size(); ++c)
                if (!gset.count((int)c))
                    for (int u : g.ops[c].in)
                        if (u == v) escapes = true;
        }
        if (escapes && i + 1 != ops.size()) { msg = "an intermediate of the group is used outside it"; return RL_ERR_GROUP; }
    }
    if (ops.size() > 1) {
        const rl_type &ref = g.values[g.ops[ops[n_anchor ? lead : 0]].out[0]].type;
        for (size_t i = tail0; i < ops.size(); ++i) {
            const OpNode &o = g.ops[ops[i]];
            if (o.kind == RL_OP_LSTM_GATES) continue;
            const rl_type &t = g.values[o.out[0]].type;
            bool same_shape = t.rank == ref.rank;
            for (int d = 0; same_shape && d < t.rank; ++d) same_shape = t.dims[d] == ref.dims[d];
            if (!same_shape) { msg = "fused operators differ in output shape"; return RL_ERR_GROUP; }
        }
    }
    return RL_OK;
}

// Fusion groups for every call that has none yet, by the rule the hand-written groupings follow: a group is
// opened by the first ungrouped call in declaration order (a concat whose only use is an ungrouped dense
// opens it together with that dense) and then follows the chain of results: the group's last result is
// absorbed into its consumer while that result has exactly one use, is not a graph output, and the
// consumer is an ungrouped injective call (or lstm_gates, which then closes the group) that takes the result
// as its first operand, has every other operand defined before the group starts, keeps the group's output
// shape and leaves the epilogue within its length limits.  Pools, flatten and anything else that is neither a
// contraction nor injective stay alone.  Every group formed is checked by check_group like a declared one.
rl_status auto_group(Graph &g, int &n_new, std::string &msg)
{
    n_new = 0;
    std::vector<std::vector<int>> users(g.values.size());
    for (size_t c = 0; c < g.ops.size(); ++c)
        for (int v : g.ops[c].in) users[v].push_back((int)c);
    std::set<int> outs(g.outputs.begin(), g.outputs.end());
    auto sole_user = [&](int v) -> int {       // the one call that reads v (possibly through several operands), or -1
        if (outs.count(v) || users[v].empty()) return -1;
        for (int u : users[v]) if (u != users[v][0]) return -1;
        return users[v][0];
    };
    for (size_t o = 0; o < g.ops.size(); ++o) {
        if (g.ops[o].group >= 0) continue;
        std::vector<int> mem{(int)o};
        int kind = g.ops[o].kind;
        if (kind == RL_OP_CONCAT && g.ops[o].out.size() == 1) {
            const int d = sole_user(g.ops[o].out[0]);
            if (d >= 0 && g.ops[d].group < 0 && g.ops[d].kind == RL_OP_DENSE && g.ops[d].in[0] == g.ops[o].out[0]) { mem.push_back(d); kind = RL_OP_DENSE; }
        }
        const bool grows = is_anchor(kind) || is_injective(kind);
        int n_chain = 0, n_ptr = 0;            // epilogue steps and operand pointers used so far
        while (grows) {
            const OpNode &last = g.ops[mem.back()];
            if (last.out.size() != 1) break;
            const int v = last.out[0];
            const int c = sole_user(v);
            if (c < 0 || g.ops[c].group >= 0) break;
            const OpNode &cn = g.ops[c];
            if (!(is_injective(cn.kind) || cn.kind == RL_OP_LSTM_GATES) || cn.in.empty() || cn.in[0] != v) break;
            bool ok = true;
            int extra = 0;
            for (size_t i = 1; i < cn.in.size(); ++i) {
                const int u = cn.in[i];
                if (u == v || (g.values[u].producer >= 0 && g.values[u].producer >= mem[0])) ok = false;
                ++extra;
            }
            if (cn.kind == RL_OP_LSTM_GATES) extra = 0;      // its cell-state operand is not an epilogue pointer
            if (!ok || n_chain + 1 > RL_EPI_MAX_OPS || n_ptr + extra > RL_EPI_MAX_PTRS) break;
            std::vector<int> trial = mem;
            trial.push_back(c);
            std::string why;
            if (check_group(g, trial, why) != RL_OK) break;
            mem.swap(trial);
            ++n_chain; n_ptr += extra;
            if (cn.kind == RL_OP_LSTM_GATES) break;
        }
        rl_status st = check_group(g, mem, msg);
        if (st != RL_OK) return st;
        const int gi = (int)g.groups.size();
        for (int m : mem) g.ops[m].group = gi;
        g.groups.push_back(mem);
        ++n_new;
    }
    return RL_OK;
}

}  // namespace rl
