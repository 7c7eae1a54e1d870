// Host-side typed graph: values with Tensor(dtype, Shape) types, operator
// calls, caller-declared fusion groups.  Type inference per operator kind
// instantiates the operator's arrow type from its argument types (the paper's
// typing rules assume quantified variables are already instantiated) and the
// caller's declared result type is compared with it (rule Type-Call).
#pragma once
#include <memory>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/relayhip.h"

namespace rl {

struct ErrBox {
    std::mutex mu;
    std::string text;
    void set(const std::string &s) { std::lock_guard<std::mutex> g(mu); text = s; }
};

struct Attrs {
    int32_t out_dtype = -1;                       // dense / conv2d: -1 = operand dtype
    int32_t stride[2] = {1, 1}, pad[2] = {0, 0};  // conv2d / pool
    int32_t kernel[2] = {1, 1};                   // pool
    int32_t axis = 1;                             // bias_add / concat
    int32_t to = 0;                               // cast
    int32_t perm[RL_MAX_RANK] = {0, 1, 2, 3, 4, 5};   // layout_transform
};

enum Role { ROLE_INPUT = 0, ROLE_PARAM = 1, ROLE_OP = 2 };

struct Value {
    rl_type type;
    int role;
    int producer;     // op index or -1
};

struct OpNode {
    int kind;
    std::vector<int> in;
    std::vector<int> out;
    Attrs attrs;
    int group = -1;
};

struct Graph {
    std::shared_ptr<ErrBox> err;
    std::vector<Value> values;
    std::vector<OpNode> ops;
    std::vector<std::vector<int>> groups;
    std::vector<int> outputs;
};

bool same_type(const rl_type &a, const rl_type &b);
std::string type_str(const rl_type &t);
int64_t numel(const rl_type &t);
size_t dtype_size(int dtype);

// Tensor-T / Shape-T / BaseType-T.  Returns RL_OK or the error class, text in msg.
rl_status check_tensor_type(const rl_type &t, std::string &msg);

// Parse the kind's attribute struct.  RL_ERR_KIND on a size mismatch.
rl_status parse_attrs(int kind, const void *attrs, size_t size, Attrs &out, std::string &msg);

// Result types of `kind` on argument types `in`; declared is consulted only for
// what the operator leaves to its declaration (lstm_gates' h dtype).
rl_status infer_type(int kind, const std::vector<rl_type> &in, const Attrs &a, const std::vector<rl_type> &declared,
                     std::vector<rl_type> &out, std::string &msg);

// Fusion-group legality over the finished graph.
rl_status check_group(const Graph &g, const std::vector<int> &ops, std::string &msg);
// Puts every call that has no group yet into one (see graph.cpp); n_new = groups added.
rl_status auto_group(Graph &g, int &n_new, std::string &msg);

const char *op_name(int kind);
bool is_anchor(int kind);
bool is_injective(int kind);

}  // namespace rl
