// The opaque handles of the C ABI as the library's own sources see them.
#pragma once
#include <memory>

#include "plan.h"

struct rl_ctx { std::shared_ptr<rl::ErrBox> err; };
struct rl_graph { rl::Graph g; };
struct rl_plan { rl::Plan p; };
