// C ABI of the library (see include/relayhip.h for the contract).
#include <algorithm>
#include <cstring>
#include <new>

#include "handles.h"

using namespace rl;

namespace {

rl_status fail(const std::shared_ptr<ErrBox> &e, rl_status st, const std::string &m)
{
    if (e) e->set(m);
    return st;
}

template <typename F>
rl_status guarded(const std::shared_ptr<ErrBox> &e, F f)
{
    try {
        return f();
    } catch (const std::bad_alloc &) {
        return fail(e, RL_ERR_NULL, "out of host memory");
    } catch (const std::exception &ex) {
        return fail(e, RL_ERR_KIND, std::string("internal error: ") + ex.what());
    } catch (...) {
        return fail(e, RL_ERR_KIND, "internal error");
    }
}

rl_status add_value(rl_graph *g, const rl_type *t, int role, int32_t *value_id)
{
    if (!g) return RL_ERR_NULL;
    return guarded(g->g.err, [&]() -> rl_status {
        if (!t || !value_id) return fail(g->g.err, RL_ERR_NULL, "null argument");
        std::string msg;
        rl_status st = check_tensor_type(*t, msg);
        if (st != RL_OK) return fail(g->g.err, st, msg + ": " + type_str(*t));
        Value v;
        v.type = *t;
        for (int i = t->rank; i < RL_MAX_RANK; ++i) v.type.dims[i] = 0;
        v.role = role;
        v.producer = -1;
        g->g.values.push_back(v);
        *value_id = (int32_t)g->g.values.size() - 1;
        return RL_OK;
    });
}

// resolve the pointer of every buffer a plan touches
// A cell plan that is exactly one fused [x, h] contraction + gate step in bf16 can run with the input projection
// x_t . Wx^T of many steps hoisted into one large contraction (the recurrence only needs h_{t-1} . Wh^T per step).
// Returns that step, or null if the plan is anything else.
const Step *hoistable_cell(const Plan &p)
{
    if (p.steps.size() != 1 || p.opts.no_hoist) return nullptr;
    const Step &s = p.steps[0];
    const IgemmParams &g = s.ig;
    if (s.kind != S_IGEMM || !s.il.gates || !s.il.avec || !s.il.dma || s.slot[SL_X2] < 0 || g.in_dtype != DT_BF16 || g.h_dtype != DT_BF16) return nullptr;
    const int64_t I = g.K1, H = g.hidden;
    if (I < 128 || I % 64 != 0 || H < 64 || H % 64 != 0 || g.K != I + H || g.Kp != g.K || g.N != 4 * H || g.x2s_n != H || g.xs_n != I) return nullptr;
    if (g.epi.n_ops > 1 || (g.epi.n_ops == 1 && (epi_host_op(g.epi, 0) != E_BIAS || epi_host_dtype(g.epi, epi_host_arg(g.epi, 0)) != DT_F32)))
        return nullptr;
    if ((uint64_t)g.N * g.Kp * 2 >= 0x7fffffffull || (uint64_t)g.M * H * 16 >= 0x7fffffffull) return nullptr;
    return &s;
}
size_t hoist_bytes_per_step(const Step &s) { return (size_t)s.ig.M * s.ig.N * sizeof(float); }
size_t round256(size_t n) { return (n + 255) & ~(size_t)255; }

rl_status resolve(const Plan &p, const rl_binding *b, int32_t nb, void *ws, size_t ws_bytes, std::vector<void *> &ptrs, std::string &msg)
{
    const int nv = (int)p.values.size();
    std::vector<void *> by_value(nv, nullptr);
    std::vector<char> seen(nv, 0);
    for (int32_t i = 0; i < nb; ++i) {
        int v = b[i].value_id;
        if (v < 0 || v >= nv) { msg = "binding names an unknown value id"; return RL_ERR_BINDING; }
        if (seen[v]) { msg = "value id " + std::to_string(v) + " bound twice"; return RL_ERR_BINDING; }
        if (p.bound_buf[v] < 0) { msg = "value id " + std::to_string(v) + " is an intermediate, not bindable"; return RL_ERR_BINDING; }
        if (!b[i].dev_ptr) { msg = "null device pointer for value id " + std::to_string(v); return RL_ERR_BINDING; }
        if (((uintptr_t)b[i].dev_ptr & 15) != 0) { msg = "device pointer of value id " + std::to_string(v) + " is not 16-byte aligned"; return RL_ERR_ALIGN; }
        seen[v] = 1;
        by_value[v] = b[i].dev_ptr;
    }
    if (p.workspace_bytes > 0) {
        if (!ws || ws_bytes < p.workspace_bytes) { msg = "workspace missing or smaller than rl_plan_workspace_bytes"; return RL_ERR_WORKSPACE; }
        if (((uintptr_t)ws & 255) != 0) { msg = "workspace is not 256-byte aligned"; return RL_ERR_ALIGN; }
    }
    ptrs.assign(p.bufs.size(), nullptr);
    for (size_t i = 0; i < p.bufs.size(); ++i) {
        const BufDesc &d = p.bufs[i];
        if (d.bound_value >= 0) {
            if (d.first < 0) continue;                      // never touched by a step
            if (!seen[d.bound_value]) { msg = "value id " + std::to_string(d.bound_value) + " has no binding"; return RL_ERR_BINDING; }
            ptrs[i] = by_value[d.bound_value];
        } else {
            ptrs[i] = (char *)ws + d.offset;
        }
    }
    return RL_OK;
}

}  // namespace

extern "C" {

rl_status rl_ctx_create(rl_ctx **out)
{
    if (!out) return RL_ERR_NULL;
    rl_ctx *c = new (std::nothrow) rl_ctx;
    if (!c) return RL_ERR_NULL;
    try {
        c->err = std::make_shared<ErrBox>();
    } catch (...) {
        delete c;
        return RL_ERR_NULL;
    }
    *out = c;
    return RL_OK;
}

void rl_ctx_destroy(rl_ctx *ctx) { delete ctx; }

const char *rl_last_error(const rl_ctx *ctx)
{
    if (!ctx || !ctx->err) return "";
    return ctx->err->text.c_str();
}

rl_status rl_graph_create(rl_ctx *ctx, rl_graph **out)
{
    if (!ctx || !out) return RL_ERR_NULL;
    return guarded(ctx->err, [&]() -> rl_status {
        rl_graph *g = new rl_graph;
        g->g.err = ctx->err;
        *out = g;
        return RL_OK;
    });
}

void rl_graph_destroy(rl_graph *g) { delete g; }

rl_status rl_graph_input(rl_graph *g, const rl_type *t, int32_t *value_id) { return add_value(g, t, ROLE_INPUT, value_id); }
rl_status rl_graph_param(rl_graph *g, const rl_type *t, int32_t *value_id) { return add_value(g, t, ROLE_PARAM, value_id); }

rl_status rl_graph_op(rl_graph *g, int32_t op_kind, const int32_t *in_ids, int32_t n_in, const void *attrs, size_t attrs_size,
                      const rl_type *declared_outs, int32_t n_out, int32_t *op_id, int32_t *out_value_ids)
{
    if (!g) return RL_ERR_NULL;
    auto &err = g->g.err;
    return guarded(err, [&]() -> rl_status {
        if (!in_ids || !declared_outs || !out_value_ids) return fail(err, RL_ERR_NULL, "null argument");
        if (op_kind < 0 || op_kind >= RL_OP_KIND_COUNT) return fail(err, RL_ERR_KIND, "unknown operator kind");
        if (n_in < 0 || n_in > 8 || n_out < 1 || n_out > 2) return fail(err, RL_ERR_TYPE, "bad operand or result count");
        std::string msg;
        OpNode op;
        op.kind = op_kind;
        std::vector<rl_type> in_t, decl;
        for (int i = 0; i < n_in; ++i) {
            if (in_ids[i] < 0 || in_ids[i] >= (int)g->g.values.size())
                return fail(err, RL_ERR_TYPE, "operand value id is not defined at this call");
            op.in.push_back(in_ids[i]);
            in_t.push_back(g->g.values[in_ids[i]].type);
        }
        for (int i = 0; i < n_out; ++i) {
            rl_status st = check_tensor_type(declared_outs[i], msg);
            if (st != RL_OK) return fail(err, st, "declared result: " + msg);
            decl.push_back(declared_outs[i]);
        }
        rl_status st = parse_attrs(op_kind, attrs, attrs_size, op.attrs, msg);
        if (st != RL_OK) return fail(err, st, msg);
        std::vector<rl_type> inferred;
        st = infer_type(op_kind, in_t, op.attrs, decl, inferred, msg);
        if (st != RL_OK) return fail(err, st, msg);
        if ((int)inferred.size() != n_out) return fail(err, RL_ERR_TYPE, std::string(op_name(op_kind)) + ": wrong number of declared results");
        for (int i = 0; i < n_out; ++i)
            if (!same_type(inferred[i], decl[i]))
                return fail(err, RL_ERR_TYPE, std::string(op_name(op_kind)) + ": declared " + type_str(decl[i]) + " but the operator's type gives " + type_str(inferred[i]));
        const int oi = (int)g->g.ops.size();
        for (int i = 0; i < n_out; ++i) {
            Value v;
            v.type = inferred[i];
            v.role = ROLE_OP;
            v.producer = oi;
            g->g.values.push_back(v);
            op.out.push_back((int)g->g.values.size() - 1);
            out_value_ids[i] = op.out.back();
        }
        g->g.ops.push_back(op);
        if (op_id) *op_id = oi;
        return RL_OK;
    });
}

rl_status rl_graph_group(rl_graph *g, const int32_t *op_ids, int32_t n, int32_t *group_id)
{
    if (!g) return RL_ERR_NULL;
    auto &err = g->g.err;
    return guarded(err, [&]() -> rl_status {
        if (!op_ids) return fail(err, RL_ERR_NULL, "null argument");
        if (n < 1) return fail(err, RL_ERR_GROUP, "empty group");
        std::vector<int> ops(op_ids, op_ids + n);
        for (int o : ops) {
            if (o < 0 || o >= (int)g->g.ops.size()) return fail(err, RL_ERR_GROUP, "group names an unknown op");
            if (g->g.ops[o].group >= 0) return fail(err, RL_ERR_GROUP, "op already belongs to a group");
        }
        std::string msg;
        rl_status st = check_group(g->g, ops, msg);
        if (st != RL_OK) return fail(err, st, msg);
        const int gi = (int)g->g.groups.size();
        for (int o : ops) g->g.ops[o].group = gi;
        g->g.groups.push_back(ops);
        if (group_id) *group_id = gi;
        return RL_OK;
    });
}

rl_status rl_graph_autogroup(rl_graph *g, int32_t *n_groups)
{
    if (!g) return RL_ERR_NULL;
    auto &err = g->g.err;
    return guarded(err, [&]() -> rl_status {
        std::string msg;
        int n = 0;
        rl_status st = auto_group(g->g, n, msg);
        if (st != RL_OK) return fail(err, st, msg);
        if (n_groups) *n_groups = n;
        return RL_OK;
    });
}

rl_status rl_graph_group_of(const rl_graph *g, int32_t op_id, int32_t *group_id)
{
    if (!g || !group_id) return RL_ERR_NULL;
    if (op_id < 0 || op_id >= (int32_t)g->g.ops.size()) return fail(g->g.err, RL_ERR_GROUP, "unknown op id");
    *group_id = g->g.ops[op_id].group;
    return RL_OK;
}

rl_status rl_graph_output(rl_graph *g, int32_t value_id)
{
    if (!g) return RL_ERR_NULL;
    auto &err = g->g.err;
    return guarded(err, [&]() -> rl_status {
        if (value_id < 0 || value_id >= (int)g->g.values.size()) return fail(err, RL_ERR_TYPE, "output value id is not defined");
        for (int v : g->g.outputs)
            if (v == value_id) return RL_OK;
        g->g.outputs.push_back(value_id);
        return RL_OK;
    });
}

rl_status rl_plan_create(rl_graph *g, const rl_plan_opts *opts, rl_plan **out)
{
    if (!g || !out) return RL_ERR_NULL;
    auto err = g->g.err;
    return guarded(err, [&]() -> rl_status {
        if (opts && (opts->struct_size < sizeof(uint32_t) || opts->struct_size > sizeof(rl_plan_opts)))
            return fail(err, RL_ERR_KIND, "rl_plan_opts.struct_size is not one this library knows");
        rl_plan *p = new rl_plan;
        if (opts) memcpy(&p->p.opts, opts, opts->struct_size);
        p->p.opts.struct_size = (uint32_t)sizeof(rl_plan_opts);
        std::string msg;
        rl_status st = build_plan(g->g, p->p, msg);
        if (st != RL_OK) {
            delete p;
            return fail(err, st, msg);
        }
        *out = p;
        return RL_OK;
    });
}

void rl_plan_destroy(rl_plan *plan) { delete plan; }

rl_status rl_plan_describe(const rl_plan *plan, char *buf, size_t cap, size_t *needed)
{
    if (!plan) return RL_ERR_NULL;
    return guarded(plan->p.err, [&]() -> rl_status {
        std::string s = describe_plan(plan->p);
        if (needed) *needed = s.size() + 1;
        if (buf && cap > 0) {
            size_t n = s.size() < cap - 1 ? s.size() : cap - 1;
            memcpy(buf, s.data(), n);
            buf[n] = 0;
        }
        return RL_OK;
    });
}

rl_status rl_plan_workspace_bytes(const rl_plan *plan, size_t *bytes)
{
    if (!plan || !bytes) return RL_ERR_NULL;
    *bytes = plan->p.workspace_bytes;
    return RL_OK;
}

rl_status rl_plan_recurrent_workspace_bytes(const rl_plan *cell, int32_t steps, size_t *bytes)
{
    if (!cell || !bytes) return RL_ERR_NULL;
    if (steps < 0) return fail(cell->p.err, RL_ERR_BINDING, "negative step count");
    const Step *hs = hoistable_cell(cell->p);
    *bytes = hs ? round256(cell->p.workspace_bytes) + (size_t)steps * hoist_bytes_per_step(*hs) : cell->p.workspace_bytes;
    return RL_OK;
}

rl_status rl_plan_packed_bytes(const rl_plan *plan, int32_t v, size_t *bytes)
{
    if (!plan || !bytes) return RL_ERR_NULL;
    if (v < 0 || v >= (int)plan->p.values.size() || plan->p.values[v].role != ROLE_PARAM)
        return fail(plan->p.err, RL_ERR_BINDING, "not a param value id");
    auto it = plan->p.packs.find(v);
    *bytes = it == plan->p.packs.end() ? 0 : it->second.bytes;
    return RL_OK;
}

rl_status rl_plan_prepack(const rl_plan *plan, int32_t v, const void *src, void *dst, void *stream)
{
    if (!plan) return RL_ERR_NULL;
    auto &err = plan->p.err;
    return guarded(err, [&]() -> rl_status {
        if (!src || !dst) return fail(err, RL_ERR_NULL, "null device pointer");
        auto it = plan->p.packs.find(v);
        if (it == plan->p.packs.end()) return fail(err, RL_ERR_BINDING, "this value id needs no packing");
        if (((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return fail(err, RL_ERR_ALIGN, "device pointer is not 16-byte aligned");
        const PackSpec &k = it->second;
        hipError_t er = k.gather ? launch_pack_gather(src, dst, k.gp, (hipStream_t)stream)
                      : k.stem == 2 ? launch_pack_weight_stem_direct(src, dst, k.O, k.C, k.KH, k.KW, k.pw, (hipStream_t)stream)
                      : k.stem ? launch_pack_weight_stem(src, dst, k.O, k.C, k.KH, k.KW, k.Kp, (hipStream_t)stream)
                               : launch_pack_weight(src, dst, k.dtype, k.O, k.C, k.T, k.Kp, k.perm_block, (hipStream_t)stream);
        if (er != hipSuccess) return fail(err, RL_ERR_HIP, std::string("pack_weight: ") + hipGetErrorString(er));
        return RL_OK;
    });
}

rl_status rl_plan_run(const rl_plan *plan, const rl_binding *bindings, int32_t n_bindings, void *ws, size_t ws_bytes, void *stream)
{
    if (!plan) return RL_ERR_NULL;
    auto &err = plan->p.err;
    return guarded(err, [&]() -> rl_status {
        if (!bindings && n_bindings > 0) return fail(err, RL_ERR_NULL, "null bindings");
        std::vector<void *> ptrs;
        std::string msg;
        rl_status st = resolve(plan->p, bindings, n_bindings, ws, ws_bytes, ptrs, msg);
        if (st != RL_OK) return fail(err, st, msg);
        st = run_steps(plan->p, ptrs.data(), (hipStream_t)stream, msg);
        if (st != RL_OK) return fail(err, st, msg);
        return RL_OK;
    });
}

rl_status rl_plan_profile(const rl_plan *plan, const rl_binding *bindings, int32_t n_bindings, void *ws, size_t ws_bytes, void *stream,
                          int32_t reps, float *step_ms, int32_t cap, int32_t *n_steps)
{
    if (!plan) return RL_ERR_NULL;
    auto &err = plan->p.err;
    return guarded(err, [&]() -> rl_status {
        if (!step_ms || !n_steps) return fail(err, RL_ERR_NULL, "null argument");
        if (reps < 1 || reps > 10000) return fail(err, RL_ERR_BINDING, "reps out of range");
        const int ns = (int)plan->p.steps.size();
        *n_steps = ns;
        std::vector<void *> ptrs;
        std::string msg;
        rl_status st = resolve(plan->p, bindings, n_bindings, ws, ws_bytes, ptrs, msg);
        if (st != RL_OK) return fail(err, st, msg);
        std::vector<hipEvent_t> ev((size_t)reps * (ns + 1), nullptr);
        auto cleanup = [&]() { for (hipEvent_t e : ev) if (e) (void)hipEventDestroy(e); };
        for (auto &e : ev)
            if (hipEventCreate(&e) != hipSuccess) { cleanup(); return fail(err, RL_ERR_HIP, "hipEventCreate failed"); }
        for (int r = 0; r < reps && st == RL_OK; ++r) st = run_steps(plan->p, ptrs.data(), (hipStream_t)stream, msg, ev.data() + (size_t)r * (ns + 1));
        hipError_t er = hipStreamSynchronize((hipStream_t)stream);
        if (st == RL_OK && er != hipSuccess) { st = RL_ERR_HIP; msg = std::string("hipStreamSynchronize: ") + hipGetErrorString(er); }
        if (st == RL_OK) {
            std::vector<double> acc(ns, 0.0);
            for (int r = 0; r < reps; ++r)
                for (int i = 0; i < ns; ++i) {
                    float ms = 0.f;
                    if (hipEventElapsedTime(&ms, ev[(size_t)r * (ns + 1) + i], ev[(size_t)r * (ns + 1) + i + 1]) != hipSuccess) { st = RL_ERR_HIP; msg = "hipEventElapsedTime failed"; }
                    acc[i] += ms;
                }
            for (int i = 0; i < ns && i < cap; ++i) step_ms[i] = (float)(acc[i] / reps);
        }
        cleanup();
        if (st != RL_OK) return fail(err, st, msg);
        return RL_OK;
    });
}

rl_status rl_plan_run_recurrent(const rl_plan *cell, int32_t steps, const rl_recurrent *io, const rl_binding *pb, int32_t npb,
                                void *ws, size_t ws_bytes, void *stream)
{
    if (!cell) return RL_ERR_NULL;
    auto &err = cell->p.err;
    return guarded(err, [&]() -> rl_status {
        if (!io) return fail(err, RL_ERR_NULL, "null recurrent descriptor");
        if (steps < 0) return fail(err, RL_ERR_BINDING, "negative step count");
        if (!io->x_seq_dev || !io->h0_dev || !io->c_dev || !io->h_seq_dev) return fail(err, RL_ERR_NULL, "null device pointer");
        if ((io->x_step_bytes & 15) || (io->h_step_bytes & 15)) return fail(err, RL_ERR_ALIGN, "per-step strides must be multiples of 16 bytes");
        const Plan &p = cell->p;
        const int ids[5] = {io->x_id, io->h_in_id, io->c_in_id, io->h_out_id, io->c_out_id};
        for (int i = 0; i < 5; ++i) {
            if (ids[i] < 0 || ids[i] >= (int)p.values.size() || p.bound_buf[ids[i]] < 0)
                return fail(err, RL_ERR_BINDING, "recurrent role names a value that is not an input or output of the cell");
            for (int j = 0; j < i; ++j)
                if (ids[i] == ids[j]) return fail(err, RL_ERR_BINDING, "one value id given two recurrent roles");
        }
        // the step loop feeds h' back as h and c' back as c: each pair must be one tensor type, and a step's slice of
        // the sequences must hold a whole operand
        if (!same_type(p.values[io->h_in_id].type, p.values[io->h_out_id].type))
            return fail(err, RL_ERR_BINDING, "recurrent h input " + type_str(p.values[io->h_in_id].type) + " and h output " +
                                             type_str(p.values[io->h_out_id].type) + " differ in type");
        if (!same_type(p.values[io->c_in_id].type, p.values[io->c_out_id].type))
            return fail(err, RL_ERR_BINDING, "recurrent c input " + type_str(p.values[io->c_in_id].type) + " and c output " +
                                             type_str(p.values[io->c_out_id].type) + " differ in type");
        auto vbytes = [&](int v) { return (size_t)numel(p.values[v].type) * dtype_size(p.values[v].type.dtype); };
        if (io->x_step_bytes < vbytes(io->x_id)) return fail(err, RL_ERR_BINDING, "x_step_bytes is smaller than the cell's x operand");
        if (io->h_step_bytes < vbytes(io->h_out_id)) return fail(err, RL_ERR_BINDING, "h_step_bytes is smaller than the cell's h result");
        std::vector<rl_binding> b(pb, pb + (npb > 0 ? npb : 0));
        const size_t base = b.size();
        b.push_back({io->x_id, (void *)io->x_seq_dev});
        b.push_back({io->h_in_id, (void *)io->h0_dev});
        b.push_back({io->c_in_id, io->c_dev});
        b.push_back({io->h_out_id, io->h_seq_dev});
        b.push_back({io->c_out_id, io->c_dev});
        std::vector<void *> ptrs;
        std::string msg;
        rl_status st = resolve(p, b.data(), (int32_t)b.size(), ws, ws_bytes, ptrs, msg);
        if (st != RL_OK) return fail(err, st, msg);
        (void)base;
        const int bx = p.bound_buf[io->x_id], bh = p.bound_buf[io->h_in_id], bo = p.bound_buf[io->h_out_id];
        // Hoisted form: the input projection of a chunk of steps as one contraction into the workspace behind the
        // plan's own, then one small recurrent kernel per step.  Taken when the cell has that form, the x_t are
        // contiguous and the workspace holds at least 8 steps' projections (or all of them).
        if (const Step *hs = hoistable_cell(p)) {
            const IgemmParams &g0 = hs->ig;
            const int64_t B = g0.M, I = g0.K1, H = g0.hidden;
            const size_t base = round256(p.workspace_bytes), per = hoist_bytes_per_step(*hs);
            int64_t chunk = (ws && ws_bytes > base) ? (int64_t)((ws_bytes - base) / per) : 0;
            chunk = std::min<int64_t>(chunk, steps);
            chunk = std::min<int64_t>(chunk, (int64_t)(0x7fffffffull / (uint64_t)(B * std::max<int64_t>(I * 2, 4 * H * 4))));   // operands below 2 GiB
            const bool roles_ok = bx == hs->slot[SL_X] && bh == hs->slot[SL_X2] && bo == hs->slot[SL_HOUT] &&
                                  hs->slot[SL_CIN] >= 0 && hs->slot[SL_COUT] >= 0;
            if (roles_ok && steps > 0 && chunk >= std::min<int64_t>(steps, 8) && io->x_step_bytes == (size_t)(B * I * 2) &&
                (((uintptr_t)ws + base) & 255) == 0) {
                float *zx = (float *)((char *)ws + base);
                const void *bias = g0.epi.n_ops == 1 ? ptrs[hs->slot[SL_E0 + epi_host_arg(g0.epi, 0)]] : nullptr;
                const int bias_dt = g0.epi.n_ops == 1 ? epi_host_dtype(g0.epi, epi_host_arg(g0.epi, 0)) : DT_F32;
                for (int64_t t0 = 0; t0 < steps; t0 += chunk) {
                    const int64_t tc = std::min<int64_t>(chunk, steps - t0);
                    IgemmParams g = g0;
                    g.x = (const char *)io->x_seq_dev + (size_t)t0 * io->x_step_bytes; g.x2 = nullptr; g.x2_bytes = 0;
                    g.w = ptrs[hs->slot[SL_W]]; g.y = zx; g.y_dtype = DT_F32;
                    g.M = (int32_t)(tc * B); g.K = (int32_t)I; g.K1 = (int32_t)I; g.C = (int32_t)I;      // weight rows keep their stride Kp
                    g.x_bytes = (uint32_t)(tc * B * I * 2); g.y_bytes = (uint32_t)std::min<uint64_t>((uint64_t)tc * per, 0x7fffffffull);
                    g.ys_n = g.N; g.ys_p = g.N; g.ys_c = 1;
                    g.epi = Epilogue{}; finalize_epilogue(g.epi);
                    g.hidden = 0; g.c_in = nullptr; g.c_out = nullptr; g.h_out = nullptr;
                    IgemmLaunch l{};
                    l.avec = 1; l.dma = 1;
                    const int64_t b128 = ((g.M + 127) / 128) * (int64_t)((g.N + 127) / 128), b64 = ((g.M + 127) / 128) * (int64_t)((g.N + 63) / 64);
                    const int64_t b256 = ((g.M + 255) / 256) * (int64_t)((g.N + 127) / 128);
                    l.tile = b128 >= 192 ? TILE_128x128 : b64 >= 192 ? TILE_128x64 : TILE_64x64;
                    // the pixel-on-lane kernel with fp32 output where one of its two large tiles fills the chip
                    if (g.N % 8 == 0 && (b256 >= 190 || b128 >= 192) && !p.opts.no_lp) {
                        l.lp = 1;
                        l.tile = b256 >= 190 ? TILE_256x128 : TILE_128x128;
                        g.seg_stride = 64; g.ts_h = 0; g.ts_w = 0; g.tap_rep = 1;
                    }
                    hipError_t er = launch_igemm(g, l, (hipStream_t)stream);
                    if (er != hipSuccess) return fail(err, RL_ERR_HIP, std::string("launch of the hoisted input projection failed: ") + hipGetErrorString(er));
                    for (int64_t t = t0; t < t0 + tc; ++t) {
                        LstmStepParams q{};
                        q.h_prev = t == 0 ? io->h0_dev : (const void *)((const char *)io->h_seq_dev + (size_t)(t - 1) * io->h_step_bytes);
                        q.w = g.w; q.zx = zx + (size_t)(t - t0) * B * g.N;
                        q.bias = bias; q.bias_dtype = bias_dt;
                        q.c_in = (const float *)ptrs[hs->slot[SL_CIN]]; q.c_out = (float *)ptrs[hs->slot[SL_COUT]];
                        q.h_out = (char *)io->h_seq_dev + (size_t)t * io->h_step_bytes; q.h_dtype = g0.h_dtype;
                        q.B = (int32_t)B; q.H = (int32_t)H; q.Kp = g0.Kp; q.k_off = (int32_t)I;
                        q.h_bytes = (uint32_t)(B * H * 2); q.w_bytes = (uint32_t)((uint64_t)g0.N * g0.Kp * 2);
                        er = launch_lstm_step(q, (hipStream_t)stream);
                        if (er != hipSuccess) return fail(err, RL_ERR_HIP, std::string("launch of lstm_step failed: ") + hipGetErrorString(er));
                    }
                }
                return RL_OK;
            }
        }
        for (int32_t t = 0; t < steps; ++t) {
            ptrs[bx] = (char *)io->x_seq_dev + (size_t)t * io->x_step_bytes;
            ptrs[bh] = t == 0 ? (void *)io->h0_dev : (void *)((char *)io->h_seq_dev + (size_t)(t - 1) * io->h_step_bytes);
            ptrs[bo] = (char *)io->h_seq_dev + (size_t)t * io->h_step_bytes;
            st = run_steps(p, ptrs.data(), (hipStream_t)stream, msg);
            if (st != RL_OK) return fail(err, st, msg);
        }
        return RL_OK;
    });
}

rl_status rl_calibrate_mfma_bf16(rl_ctx *ctx, void *scratch, int32_t workgroups, int32_t iters, void *stream)
{
    if (!ctx) return RL_ERR_NULL;
    auto &err = ctx->err;
    return guarded(err, [&]() -> rl_status {
        if (!scratch) return fail(err, RL_ERR_NULL, "null device pointer");
        if (workgroups < 1 || iters < 1) return fail(err, RL_ERR_BINDING, "workgroups and iters must be positive");
        hipError_t er = launch_mfma_peak((float *)scratch, workgroups, iters, (hipStream_t)stream);
        if (er != hipSuccess) return fail(err, RL_ERR_HIP, std::string("mfma calibration kernel: ") + hipGetErrorString(er));
        return RL_OK;
    });
}

rl_status rl_prep_fold_batchnorm(rl_ctx *ctx, const void *w, const void *gamma, const void *beta, const void *mean, const void *var,
                                 double eps, void *w_out, int32_t out_dtype, void *b_out, int64_t O, int64_t per_o, void *stream)
{
    if (!ctx) return RL_ERR_NULL;
    auto &err = ctx->err;
    return guarded(err, [&]() -> rl_status {
        if (!w || !gamma || !beta || !mean || !var || !w_out || !b_out) return fail(err, RL_ERR_NULL, "null device pointer");
        if (O < 1 || per_o < 1) return fail(err, RL_ERR_SHAPE, "O and per_o must be positive");
        if (out_dtype != RL_F32 && out_dtype != RL_BF16) return fail(err, RL_ERR_KIND, "unknown base type");
        hipError_t er = launch_fold_bn((const float *)w, (const float *)gamma, (const float *)beta, (const float *)mean, (const float *)var,
                                       eps, w_out, out_dtype, (float *)b_out, O, per_o, (hipStream_t)stream);
        if (er != hipSuccess) return fail(err, RL_ERR_HIP, std::string("fold_batchnorm: ") + hipGetErrorString(er));
        return RL_OK;
    });
}

}  // extern "C"
