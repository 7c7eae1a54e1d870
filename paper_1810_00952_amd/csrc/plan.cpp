// Fusion-group planner and executor (host).
//
// For every caller-declared group the planner re-checks legality, picks the
// kernel (implicit-GEMM contraction with epilogue, single-pass elementwise
// chain, window reduction, gate kernel), the tile, and the private layout of
// each intermediate: rank-4 activations between contractions live
// channel-last so that a K slice of the implicit GEMM is a run of channels;
// tensors at the boundary keep the order of their Shape.  Layout changes are
// inserted only where a consumer cannot read what its producer wrote.
#include "plan.h"

#include <algorithm>
#include <set>
#include <sstream>

namespace rl {

namespace {

enum { L_NATIVE = 0, L_NHWC = 1 };

inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }
inline int kv_of(int dtype) { return dtype == RL_BF16 ? 8 : 4; }

struct Planner {
    const Graph &g;
    Plan &plan;
    std::string &msg;
    std::vector<int> phys[2];              // [layout][value] -> buffer index or -1
    std::set<int> out_set;
    std::vector<std::vector<int>> consumers;

    Planner(const Graph &g_, Plan &p_, std::string &m_) : g(g_), plan(p_), msg(m_) {}

    rl_status fail(rl_status st, const std::string &m) { msg = m; return st; }

    const rl_type &T(int v) const { return g.values[v].type; }
    bool hw1(int v) const { return T(v).rank == 4 && T(v).dims[2] * T(v).dims[3] == 1; }
    bool layout_free(int v) const { return T(v).rank != 4 || hw1(v) || T(v).dims[1] == 1; }
    size_t bytes_of(int v) const { return (size_t)numel(T(v)) * dtype_size(T(v).dtype); }

    int bound(int v)
    {
        if (plan.bound_buf[v] < 0) {
            BufDesc b;
            b.bound_value = v;
            b.bytes = bytes_of(v);
            plan.bufs.push_back(b);
            plan.bound_buf[v] = (int)plan.bufs.size() - 1;
        }
        return plan.bound_buf[v];
    }
    int new_ws(size_t bytes)
    {
        BufDesc b;
        b.bytes = round_up((int64_t)bytes, 256);
        plan.bufs.push_back(b);
        return (int)plan.bufs.size() - 1;
    }
    void set_phys(int v, int layout, int buf)
    {
        phys[layout][v] = buf;
        if (layout_free(v)) phys[1 - layout][v] = buf;
    }
    // A graph output that is the channel-last view (layout_transform with axes 0,2,3,1) of rank-4 value v, or -1:
    // v's channel-last storage then is that output's own buffer.
    int channel_last_output_of(int v) const
    {
        for (int c : consumers[v]) {
            const OpNode &o = g.ops[c];
            if (o.kind == RL_OP_LAYOUT_TRANSFORM && T(v).rank == 4 && o.attrs.perm[0] == 0 && o.attrs.perm[1] == 2 && o.attrs.perm[2] == 3 &&
                o.attrs.perm[3] == 1 && out_set.count(o.out[0]))
                return o.out[0];
        }
        return -1;
    }
    // buffer a step writes value v into, in `layout`
    int out_buf(int v, int layout)
    {
        int b, home;
        if (out_set.count(v) && (layout == L_NATIVE || layout_free(v))) b = bound(v);
        else if (layout == L_NHWC && !layout_free(v) && (home = channel_last_output_of(v)) >= 0) b = bound(home);
        else b = new_ws(bytes_of(v));
        set_phys(v, layout, b);
        return b;
    }
    Step &add_step(int kind, const std::string &name, const std::string &kernel)
    {
        plan.steps.emplace_back();
        Step &s = plan.steps.back();
        s.kind = kind;
        s.name = name;
        s.kernel = kernel;
        return s;
    }
    // make value v available in `layout`; returns the buffer
    rl_status need(int v, int layout, int &buf)
    {
        if (phys[layout][v] >= 0) { buf = phys[layout][v]; return RL_OK; }
        int other = phys[1 - layout][v];
        if (other < 0) return fail(RL_ERR_UNSUPPORTED, "internal: value has no storage yet");
        const rl_type &t = T(v);
        int dst = out_buf(v, layout);
        Step &s = add_step(layout == L_NHWC ? S_TO_NHWC : S_TO_NCHW, "layout", layout == L_NHWC ? "nchw_to_nhwc" : "nhwc_to_nchw");
        s.t_dtype = t.dtype; s.t_N = (int)t.dims[0]; s.t_C = (int)t.dims[1]; s.t_P = (int)(t.dims[2] * t.dims[3]);
        s.slot[SL_X] = other; s.slot[SL_Y] = dst;
        s.bytes = 2.0 * bytes_of(v);
        buf = dst;
        return RL_OK;
    }

    // ---- injective chain -------------------------------------------------
    struct Chain {
        Epilogue epi{};
        std::vector<int> operand;        // value id per pointer slot
        std::vector<bool> is_vec;        // bias vector (1-D) or full-shape tensor
        int bias_axis = -1;
        int last_value = -1;
    };
    rl_status push_op(Chain &c, uint8_t op, int operand, bool vec)
    {
        if (c.epi.n_ops >= RL_EPI_MAX_OPS) return fail(RL_ERR_UNSUPPORTED, "fused chain longer than the kernel's program");
        int a = 0;
        if (operand >= 0) {
            a = -1;
            for (size_t i = 0; i < c.operand.size(); ++i)
                if (c.operand[i] == operand) a = (int)i;
            if (a < 0) {
                if ((int)c.operand.size() >= RL_EPI_MAX_PTRS) return fail(RL_ERR_UNSUPPORTED, "fused chain has too many operands");
                c.operand.push_back(operand);
                c.is_vec.push_back(vec);
                a = (int)c.operand.size() - 1;
                epi_set_dtype(c.epi, a, T(operand).dtype);
            }
        }
        epi_set_op(c.epi, c.epi.n_ops, op, a);
        c.epi.n_ops++;
        return RL_OK;
    }
    // ops[from..to) applied to running value `cur`
    rl_status build_chain(const std::vector<int> &ops, size_t from, size_t to, int cur, const std::set<int> &gset, Chain &c)
    {
        for (size_t i = from; i < to; ++i) {
            const OpNode &o = g.ops[ops[i]];
            auto external = [&](int v) { return g.values[v].producer < 0 || !gset.count(g.values[v].producer); };
            rl_status st = RL_OK;
            switch (o.kind) {
            case RL_OP_NEG: case RL_OP_SQ: case RL_OP_RELU: case RL_OP_SIGMOID: case RL_OP_TANH: case RL_OP_CAST: {
                if (o.in[0] != cur) return fail(RL_ERR_UNSUPPORTED, "fused group is not a single chain");
                uint8_t code = o.kind == RL_OP_NEG ? E_NEG : o.kind == RL_OP_SQ ? E_SQ : o.kind == RL_OP_RELU ? E_RELU
                             : o.kind == RL_OP_SIGMOID ? E_SIGMOID : o.kind == RL_OP_TANH ? E_TANH
                             : (o.attrs.to == RL_BF16 ? E_ROUND_BF16 : E_NOP);
                st = push_op(c, code, -1, false);
                break;
            }
            case RL_OP_BIAS_ADD:
                if (o.in[0] != cur || !external(o.in[1])) return fail(RL_ERR_UNSUPPORTED, "fused group is not a single chain");
                if (c.bias_axis >= 0 && c.bias_axis != o.attrs.axis) return fail(RL_ERR_UNSUPPORTED, "bias_add along two axes in one group");
                c.bias_axis = o.attrs.axis;
                st = push_op(c, E_BIAS, o.in[1], true);
                break;
            case RL_OP_ADD: case RL_OP_SUB: case RL_OP_MUL: case RL_OP_DIV: {
                int a = o.in[0], b = o.in[1];
                if (a == cur && b == cur) {
                    uint8_t code = o.kind == RL_OP_ADD ? E_ADD_VV : o.kind == RL_OP_SUB ? E_SUB_VV : o.kind == RL_OP_MUL ? E_SQ : E_DIV_VV;
                    st = push_op(c, code, -1, false);
                } else if (a == cur && external(b)) {
                    uint8_t code = o.kind == RL_OP_ADD ? E_ADD : o.kind == RL_OP_SUB ? E_SUB : o.kind == RL_OP_MUL ? E_MUL : E_DIV;
                    st = push_op(c, code, b, false);
                } else if (b == cur && external(a)) {
                    uint8_t code = o.kind == RL_OP_ADD ? E_ADD : o.kind == RL_OP_SUB ? E_RSUB : o.kind == RL_OP_MUL ? E_MUL : E_RDIV;
                    st = push_op(c, code, a, false);
                } else {
                    return fail(RL_ERR_UNSUPPORTED, "fused group is not a single chain");
                }
                break;
            }
            default:
                return fail(RL_ERR_UNSUPPORTED, std::string(op_name(o.kind)) + " inside a chain");
            }
            if (st != RL_OK) return st;
            cur = o.out[0];
        }
        c.last_value = cur;
        return RL_OK;
    }
    // bind the chain's operands to step slots; full-shape operands in `layout`
    rl_status bind_chain(Chain &c, Step &s, int layout, double &bytes)
    {
        for (size_t i = 0; i < c.operand.size(); ++i) {
            int buf;
            rl_status st = need(c.operand[i], c.is_vec[i] ? L_NATIVE : layout, buf);
            if (st != RL_OK) return st;
            // `need` may have appended a layout step: s is re-fetched by the caller, so only indices are kept here
            s.slot[SL_E0 + i] = buf;
            bytes += (double)bytes_of(c.operand[i]);
        }
        return RL_OK;
    }

    // ---- contraction groups ------------------------------------------------
    // A contraction seen through other eyes than its op's: the gradient with respect to the first operand of a dense
    // or of a stride-1 conv2d is a dense / a stride-1 conv2d of dy with re-ordered weights, and runs on the same kernels.
    struct AnchorView {
        int kind;                         // RL_OP_DENSE or RL_OP_CONV2D
        int N, KH, KW, ph, pw;            // output channels (features), taps, padding; stride 1; contraction channels come from x
        GatherPack gp;                    // where the rows of the K-contiguous weight matrix come from
        int xbuf = -1;                    // >= 0: the activations are this channel-last buffer [xN][xH][xW][C] instead of x's own
        int xH = 0, xW = 0;
    };

    rl_status plan_anchor(int gi, const std::vector<int> &ops, const AnchorView *ov = nullptr)
    {
        std::set<int> gset(ops.begin(), ops.end());
        size_t ai = 0;
        int x = -1, x2 = -1;
        if (g.ops[ops[0]].kind == RL_OP_CONCAT) {
            ai = 1;
            const OpNode &cc = g.ops[ops[0]];
            if (g.ops[ops[1]].in[0] != cc.out[0]) return fail(RL_ERR_UNSUPPORTED, "concat must feed the dense's first operand");
            x = cc.in[0];
            x2 = cc.in[1];
        }
        const OpNode &an = g.ops[ops[ai]];
        const int akind = ov ? ov->kind : an.kind;
        if (x < 0) x = an.in[0];
        const int wv = an.in[1];
        if (g.values[wv].role != ROLE_PARAM) return fail(RL_ERR_UNSUPPORTED, "contraction weights must be a param");
        const int in_dt = T(x).dtype;
        const int KV = kv_of(in_dt);
        const bool gates = g.ops[ops.back()].kind == RL_OP_LSTM_GATES && ops.size() > ai + 1;
        Chain chain;
        rl_status st = build_chain(ops, ai + 1, gates ? ops.size() - 1 : ops.size(), an.out[0], gset, chain);
        if (st != RL_OK) return st;
        if (chain.bias_axis >= 0 && chain.bias_axis != 1) return fail(RL_ERR_UNSUPPORTED, "bias_add fused into a contraction must be along axis 1");
        if (gates) {
            const OpNode &go = g.ops[ops.back()];
            const int cprod = g.values[go.in[1]].producer;
            if (go.in[0] != chain.last_value || (cprod >= 0 && gset.count(cprod))) return fail(RL_ERR_UNSUPPORTED, "fused group is not a single chain");
        }
        if (gates)
            for (int i = 0; i < chain.epi.n_ops; ++i)
                if (epi_host_op(chain.epi, i) != E_BIAS) return fail(RL_ERR_UNSUPPORTED, "only bias_add may sit between the contraction and lstm_gates");

        IgemmParams p{};
        IgemmLaunch il{};
        PackSpec pack;
        bool need_pack = false;
        int xbuf = -1, x2buf = -1;
        double flops = 0.0;
        size_t x_extent = 0;                 // bytes of the tensor the kernel reads as x
        const rl_type &ot = T(an.out[0]);
        p.in_dtype = in_dt;
        int out_layout = L_NATIVE;
        const int vout = gates ? -1 : chain.last_value;

        // form of the injective chain, needed before the kernel variant is chosen
        Epilogue cls = chain.epi;
        finalize_epilogue(cls);
        const bool epi_any = cls.simple && (!cls.has_bias || cls.bias_dtype == DT_F32) && (cls.t_op < 0 || (cls.t_op == E_ADD && cls.t_dtype == DT_BF16));
        const bool relu_form = cls.rest_n == 0 || cls.relu_last;     // at most one ReLU behind them: every pixel-on-lane kernel; anything else: the general one
        const bool epi_lp = epi_any && relu_form;
        bool stem = false;
        const size_t lim = (size_t)1 << 31;

        if (akind == RL_OP_CONV2D) {
            const rl_type &xt = T(x), &wt = T(wv);
            p.C = (int)xt.dims[1]; p.H = (int)xt.dims[2]; p.W = (int)xt.dims[3];
            const bool xov = ov && ov->xbuf >= 0;
            if (xov) { p.H = ov->xH; p.W = ov->xW; }
            const size_t x_own = xov ? (size_t)xt.dims[0] * p.H * p.W * p.C * dtype_size(in_dt) : bytes_of(x);
            p.KH = (int)wt.dims[2]; p.KW = (int)wt.dims[3];
            p.OH = (int)ot.dims[2]; p.OW = (int)ot.dims[3]; p.OHW = p.OH * p.OW;
            p.sh = an.attrs.stride[0]; p.sw = an.attrs.stride[1]; p.ph = an.attrs.pad[0]; p.pw = an.attrs.pad[1];
            p.N = (int)wt.dims[0];
            if (ov) { p.N = ov->N; p.KH = ov->KH; p.KW = ov->KW; p.sh = p.sw = 1; p.ph = ov->ph; p.pw = ov->pw; }
            if (xt.dims[0] * (int64_t)p.OHW > 0x7fffffff) return fail(RL_ERR_UNSUPPORTED, "conv2d too large");
            p.M = (int)(xt.dims[0] * p.OHW); p.K = p.C * p.KH * p.KW; p.K1 = p.K;
            p.Kp = (int)round_up(p.K, KV);
            out_layout = (vout >= 0 && out_set.count(vout)) ? L_NATIVE : L_NHWC;
            flops = 2.0 * p.M * (double)p.N * p.K;
            // A bf16 result that is a graph output (Shape order): only the slower direct-load kernel stores in that order
            // itself.  From 0.4 GFLOP on, the pixel-on-lane kernels writing channel-last into the workspace plus a
            // transposition (one launch more, and one more for a channel-first residual) are faster: 64x128x28x28 through
            // 3x3 20 + 9 us against 56, with a residual 43 against 166; at 0.46 GFLOP 14.3 against 16.9; below, the
            // direct-load kernel with its K split is level or ahead (0.23 GFLOP: 16.4 against 14.6).
            if (out_layout == L_NATIVE && vout >= 0 && !plan.opts.no_out_transpose && !plan.opts.no_lp && in_dt == RL_BF16 && T(vout).dtype == RL_BF16 &&
                p.C % 64 == 0 && p.N % 8 == 0 && p.KH * p.KW <= 32 && x2 < 0 && !gates && epi_any && flops >= 4e8 &&
                channel_last_output_of(vout) < 0)
                out_layout = L_NHWC;
            if (out_layout == L_NHWC) { p.ys_n = (int64_t)p.OHW * p.N; p.ys_p = p.N; p.ys_c = 1; }
            else { p.ys_n = (int64_t)p.N * p.OHW; p.ys_p = 1; p.ys_c = p.OHW; }
            flops = 2.0 * p.M * (double)p.N * p.K;
            // Few-channel stem (e.g. 3 -> 64, 7x7, stride 2): gathering single elements starves the MFMAs.  Copy the
            // input into a zero-padded 4-channel channel-last frame instead; a K tile then holds two filter rows of
            // 8 pixels x 4 channels and travels by direct loads like any other (see launch_stem_pad).
            const int KH2 = (p.KH + 1) / 2;
            const int64_t Hp = (int64_t)(p.OH - 1) * p.sh + 2 * KH2, Wp = (int64_t)(p.OW - 1) * p.sw + 8;
            const size_t frame = (size_t)xt.dims[0] * Hp * Wp * 8;
            stem = in_dt == RL_BF16 && p.C <= 4 && p.KW <= 8 && p.sw % 2 == 0 && KH2 <= 32 && epi_lp && vout >= 0 && T(vout).dtype == RL_BF16 &&
                   out_layout == L_NHWC && p.N % 8 == 0 && bytes_of(vout) < lim && frame < lim && phys[L_NATIVE][x] >= 0 && !plan.opts.no_stem && !ov;
            if (stem) {
                int xnat;
                st = need(x, L_NATIVE, xnat);
                if (st != RL_OK) return st;
                xbuf = new_ws(frame);
                Step &ps = add_step(S_STEM_PAD, "stem_pad", "stem_pad_nhwc4");
                ps.t_N = (int)xt.dims[0]; ps.t_C = p.C; ps.st_H = p.H; ps.st_W = p.W; ps.st_Hp = (int)Hp; ps.st_Wp = (int)Wp;
                ps.st_ph = p.ph; ps.st_pw = p.pw;
                ps.slot[SL_X] = xnat; ps.slot[SL_Y] = xbuf;
                ps.bytes = (double)bytes_of(x) + (double)frame;
                pack.dtype = in_dt; pack.O = p.N; pack.C = p.C; pack.KH = p.KH; pack.KW = p.KW; pack.stem = 1; pack.T = p.KH * p.KW;
                // the contraction as the kernel sees it: 64 "channels" per tap, KH2 taps, taps two frame rows apart
                p.C = 64; p.KH = KH2; p.KW = 1; p.H = (int)Hp; p.W = (int)Wp; p.ph = 0; p.pw = 0;
                p.xs_n = Hp * Wp * 4; p.xs_h = Wp * 4; p.xs_w = 4; p.xs_c = 1;
                p.ts_h = 2 * Wp * 4; p.ts_w = 0; p.seg_stride = (uint32_t)(Wp * 8);
                p.K = KH2 * 64; p.K1 = p.K; p.Kp = p.K;
                pack.Kp = p.Kp; pack.perm_block = 0;
                il.avec = 1;
                need_pack = true;
                x_extent = frame;
            } else {
                il.avec = (p.C % KV == 0);
                int xl;
                if (il.avec || xov) xl = L_NHWC;
                else xl = phys[L_NATIVE][x] >= 0 ? L_NATIVE : L_NHWC;
                if (xov) xbuf = ov->xbuf;
                else st = need(x, xl, xbuf);
                if (st != RL_OK) return st;
                if (xl == L_NHWC) { p.xs_n = (int64_t)p.H * p.W * p.C; p.xs_h = (int64_t)p.W * p.C; p.xs_w = p.C; p.xs_c = 1; }
                else { p.xs_n = (int64_t)p.C * p.H * p.W; p.xs_c = (int64_t)p.H * p.W; p.xs_h = p.W; p.xs_w = 1; }
                p.ts_h = p.xs_h; p.ts_w = p.xs_w; p.seg_stride = 64;
                need_pack = !(p.KH * p.KW == 1 && p.C % KV == 0) || ov;
                pack.dtype = in_dt; pack.O = p.N; pack.C = p.C; pack.T = p.KH * p.KW; pack.Kp = p.Kp; pack.perm_block = 0;
                x_extent = x_own;
            }
        } else {
            const rl_type &wt = T(wv);
            const int64_t K = ov ? T(x).dims[1] : wt.dims[1], Nf = ov ? ov->N : wt.dims[0];
            if (ot.dims[0] > 0x7fffffff || K > 0x7ffffff0 || Nf > 0x7fffffff) return fail(RL_ERR_UNSUPPORTED, "dense too large");
            p.M = (int)ot.dims[0]; p.N = (int)Nf; p.K = (int)K; p.Kp = (int)round_up(K, KV);
            p.C = p.K; p.H = p.W = p.KH = p.KW = p.OH = p.OW = p.OHW = 1; p.sh = p.sw = 1;
            p.K1 = x2 >= 0 ? (int)T(x).dims[1] : p.K;
            const int K2 = p.K - p.K1;
            il.avec = (p.K1 % KV == 0) && (K2 % KV == 0);
            st = need(x, L_NATIVE, xbuf);
            if (st != RL_OK) return st;
            if (x2 >= 0) { st = need(x2, L_NATIVE, x2buf); if (st != RL_OK) return st; }
            p.xs_n = p.K1; p.xs_c = 1; p.xs_h = 0; p.xs_w = 0; p.x2s_n = K2;
            p.ts_h = 0; p.ts_w = 0; p.seg_stride = 64;
            flops = 2.0 * p.M * (double)p.N * p.K;
            x_extent = bytes_of(x);
            need_pack = (p.K % KV != 0) || gates || ov;
            pack.dtype = in_dt; pack.O = p.N; pack.C = p.K; pack.T = 1; pack.Kp = p.Kp; pack.perm_block = gates ? 64 : 0;
            p.ys_n = p.N; p.ys_p = p.N; p.ys_c = 1;
        }
        // 3x3 bf16 weights from 64 to 64 channels carry, behind the matrix, a second copy in the fragment order of the
        // kernel that keeps them in registers (whichever kernel a step ends up with, so that every user agrees)
        const bool dual = !ov && akind == RL_OP_CONV2D && !stem && in_dt == RL_BF16 && p.N == 64 && p.C == 64 && p.KH == 3 && p.KW == 3 && p.Kp == p.K;
        if (dual) pack.perm_block = -1;
        pack.bytes = (size_t)pack.O * pack.Kp * dtype_size(in_dt);
        // the vector-load kernel addresses its operands with 32-bit byte offsets and wants a K tile
        // (128 bytes per row) to lie inside one operand of a concatenation
        {
            if (x_extent >= lim || pack.bytes >= lim || (x2 >= 0 && bytes_of(x2) >= lim)) il.avec = 0;
            if (x2 >= 0 && p.K1 % (8 * KV) != 0) il.avec = 0;
            p.x_bytes = (uint32_t)std::min(x_extent, lim - 1);
            p.x2_bytes = x2 >= 0 ? (uint32_t)std::min(bytes_of(x2), lim - 1) : 0;
            p.w_bytes = (uint32_t)std::min(pack.bytes, lim - 1);
            if (dual) pack.bytes *= 2;
            // LDS-DMA variant: a K tile must lie inside one filter tap (and one concat operand)
            const int bke = 8 * KV;
            const size_t halo = (size_t)((int64_t)p.ph * p.xs_h + (int64_t)p.pw * p.xs_w) * dtype_size(in_dt);
            il.dma = !stem && il.avec && p.C % bke == 0 && p.K % bke == 0 && p.K / bke >= 2 && p.KH * p.KW <= 32 &&
                     (x2 < 0 || p.K1 % bke == 0) && x_extent + halo < lim && !plan.opts.no_dma;
            // a dense contraction whose K is a multiple of the vector but not of the K tile: the weights are packed
            // with zeros up to whole tiles and the kernel requests the activation chunks past K out of range
            if (!il.dma && akind == RL_OP_DENSE && !stem && !gates && x2 < 0 && il.avec && p.K % bke != 0 && p.K / bke >= 2 &&
                x_extent < lim && (size_t)p.N * round_up(p.K, bke) * dtype_size(in_dt) < lim && !plan.opts.no_dma) {
                il.dma = 1;
                p.Kp = (int)round_up(p.K, bke);
                need_pack = true;
                pack.Kp = p.Kp;
                pack.bytes = (size_t)pack.O * pack.Kp * dtype_size(in_dt);
                p.w_bytes = (uint32_t)pack.bytes;
            }
            // pixel-on-lane variant: bf16 throughout, output rows contiguous in n, epilogue [bias] [+residual] [relu]
            bool y_ok = vout >= 0 && T(vout).dtype == RL_BF16 && p.ys_c == 1 && p.ys_n == (int64_t)p.OHW * p.ys_p && p.N % 8 == 0 &&
                        bytes_of(vout) < lim;
            il.lp = stem || (il.avec && in_dt == RL_BF16 && p.C % bke == 0 && p.K % bke == 0 && p.KH * p.KW <= 32 && x2 < 0 && !gates &&
                             x_extent + halo < lim && epi_any && y_ok && !plan.opts.no_lp);
            il.anyact = il.lp && !stem && !relu_form;
            // weights-stationary persistent variant: pays off when the weights leave LDS for a deep ring (K <= 320);
            // the plan option ws_all also takes it up to K = 576, where its shallower ring is latency-bound
            il.ws = il.lp && !il.anyact && p.N <= 64 && (p.K / bke <= 5 || (p.K / bke <= 9 && plan.opts.ws_all)) && !plan.opts.no_ws;
            // 3x3 / stride 1 / pad 1 from 64 to 64 channels on rows of at most 63 pixels: weights in registers, every
            // input pixel fetched once per region
            il.c64 = il.lp && !il.anyact && !stem && akind == RL_OP_CONV2D && p.C == 64 && p.N == 64 && p.KH == 3 && p.KW == 3 && p.sh == 1 && p.sw == 1 &&
                     p.ph == 1 && p.pw == 1 && p.OH == p.H && p.OW == p.W && p.W <= 63 && p.Kp == p.K && p.ys_p == 64 && !plan.opts.no_c64;
            il.c64 = il.c64 && dual;
            if (il.c64) { il.ws = 0; p.w_bytes = (uint32_t)pack.bytes; }
            p.y_bytes = vout >= 0 ? (uint32_t)std::min(bytes_of(vout), lim - 1) : 0;
            make_fast_div((uint32_t)p.OHW, p.div_ohw_mul, p.div_ohw_sh);
            make_fast_div((uint32_t)p.OW, p.div_ow_mul, p.div_ow_sh);
            p.tap_rep = 0;
            if (p.KH * p.KW <= 32)
                for (int kh = 0; kh < p.KH; ++kh) p.tap_rep |= 1u << (kh * p.KW);
        }
        if (ov) { pack.gather = 1; pack.gp = ov->gp; pack.gp.Kp = pack.Kp; pack.perm_block = -3; }
        if (need_pack) {
            auto it = plan.packs.find(wv);
            if (it != plan.packs.end() && (ov || it->second.perm_block != pack.perm_block || it->second.Kp != pack.Kp))
                return fail(RL_ERR_UNSUPPORTED, "one param needs two different kernel-native layouts");
            plan.packs[wv] = pack;
        } else if (plan.packs.count(wv)) {
            return fail(RL_ERR_UNSUPPORTED, "one param needs two different kernel-native layouts");
        }

        // tile: the largest that still yields enough workgroups for 256 CUs
        auto nblk = [&](int bm, int bn) { return (int64_t)((p.M + bm - 1) / bm) * ((p.N + bn - 1) / bn); };
        if (gates) {
            il.tile = TILE_64x64;
            il.gates = 1;
            int64_t Hd = T(g.ops[ops.back()].in[1]).dims[1];
            if (Hd % 16 != 0) return fail(RL_ERR_UNSUPPORTED, "fused gate epilogue needs hidden size divisible by 16");
            p.hidden = (int)Hd;
            p.h_dtype = T(g.ops[ops.back()].out[1]).dtype;
        } else if (!il.avec) {
            il.tile = TILE_64x64;
        } else if (il.lp && p.N > 64 && nblk(256, 128) >= 190 && !plan.opts.no_lp_256) {
            il.tile = TILE_256x128;        // a quarter fewer operand bytes per MFMA than 128x128
        } else if (p.N > 64 && nblk(128, 128) >= 192) {
            il.tile = TILE_128x128;
        } else if (nblk(128, 64) >= 192) {
            il.tile = TILE_128x64;
        } else {
            il.tile = TILE_64x64;
        }

        // 3x3 / stride 1 / pad 1 on short image rows with whole 64-channel slices: the nine taps of a slice are read
        // from one copy of the input rows (needs one of the larger tiles)
        il.run = il.lp && !il.anyact && !il.c64 && !il.ws && !stem && akind == RL_OP_CONV2D && p.KH == 3 && p.KW == 3 && p.sh == 1 && p.sw == 1 && p.ph == 1 &&
                 p.pw == 1 && p.OH == p.H && p.OW == p.W && p.W <= 30 && p.C % 64 == 0 && p.Kp == p.K && il.tile != TILE_64x64 &&
                 !plan.opts.no_run;
        if (il.run && il.tile == TILE_128x64 && p.C % 128 == 0 && !plan.opts.no_run_ks) {
            il.run = 2;                                                 // K split over the waves
            // weights of all channel tiles larger than an XCD's share of L2 (4 MB): tiles are numbered channel-tile-major,
            // so that an XCD multiplies every pixel tile by one channel tile's weights
            p.nmajor = (int64_t)p.N * p.K * 2 > (3 << 20) ? 1 : 0;
        }

        double bytes = (double)bytes_of(x) + (x2 >= 0 ? (double)bytes_of(x2) : 0.0) + (double)bytes_of(wv);
        std::vector<int> eslots(RL_EPI_MAX_PTRS, -1);
        {
            Step tmp;
            st = bind_chain(chain, tmp, out_layout, bytes);
            if (st != RL_OK) return st;
            for (int i = 0; i < RL_EPI_MAX_PTRS; ++i) eslots[i] = tmp.slot[SL_E0 + i];
        }
        int cin_buf = -1, cout_buf = -1, hout_buf = -1, ybuf = -1;
        if (gates) {
            const OpNode &go = g.ops[ops.back()];
            st = need(go.in[1], L_NATIVE, cin_buf);
            if (st != RL_OK) return st;
            cout_buf = out_buf(go.out[0], L_NATIVE);
            hout_buf = out_buf(go.out[1], L_NATIVE);
            bytes += 2.0 * bytes_of(go.in[1]) + bytes_of(go.out[1]);
        } else {
            p.y_dtype = T(vout).dtype;
            ybuf = out_buf(vout, out_layout);
            bytes += (double)bytes_of(vout);
        }
        p.epi = chain.epi;
        // Few tiles and a long K (small batches, late stages): K is split over several workgroups per tile, whose fp32
        // sums meet in a scratch tensor [splits][M][N] that a second kernel adds up in order before the epilogue.
        int part_buf = -1;
        if (il.avec && !il.lp && !gates && x2 < 0 && !stem && !plan.opts.no_splitk) {
            static const int tbm[] = {128, 128, 64, 256}, tbn[] = {128, 64, 64, 128};
            const int64_t tiles = nblk(tbm[il.tile], tbn[il.tile]);
            const int nk = (p.K + 8 * KV - 1) / (8 * KV);
            // from 8 K tiles on (fewer: the adding launch costs more than the serial K loop); slices of at least two K tiles
            int want = (int)std::min<int64_t>(std::min<int64_t>(16, 256 / std::max<int64_t>(tiles, 1)), nk / 2);
            if (tiles <= 64 && nk >= 8 && want >= 2 && (int64_t)want * p.M * p.N * 4 < (int64_t)1 << 28) {
                const int per = (nk + want - 1) / want;
                il.splits = (nk + per - 1) / per;
                p.splits = il.splits; p.split_tiles = per;
                part_buf = new_ws((size_t)il.splits * p.M * p.N * 4);
                bytes += 2.0 * il.splits * p.M * (double)p.N * 4;
            }
        }
        static const char *tile_names[] = {"128x128", "128x64", "64x64", "256x128"};
        std::string kname = (ov ? std::string("igemm_") + op_name(an.kind) + "_" : std::string(akind == RL_OP_CONV2D ? "igemm_conv2d_" : "igemm_dense_")) + (in_dt == RL_BF16 ? "bf16_" : "f32_") +
                            (il.c64 ? "3x3_c64" : il.ws ? "128x64_ws" : tile_names[il.tile]) + (il.c64 || il.ws ? "" : il.run ? "_run" : il.lp ? "_lp" : il.avec ? (il.dma ? "_dma" : "") : "_gather") + (gates ? "_gates" : "") +
                            (il.splits > 1 ? "_splitk" : "");
        Step &s = add_step(S_IGEMM, std::string(op_name(an.kind)) + "#" + std::to_string(ops[ai]), kname);
        s.group = gi;
        s.ig = p; s.il = il;
        s.stem = stem ? 1 : 0;
        s.stem_kh = stem ? pack.KH : 0;
        s.slot[SL_X] = xbuf; s.slot[SL_X2] = x2buf; s.slot[SL_W] = bound(wv); s.slot[SL_Y] = ybuf;
        for (int i = 0; i < RL_EPI_MAX_PTRS; ++i) s.slot[SL_E0 + i] = eslots[i];
        s.slot[SL_CIN] = cin_buf; s.slot[SL_COUT] = cout_buf; s.slot[SL_HOUT] = hout_buf;
        s.slot[SL_PART] = part_buf;
        s.flops = flops;
        s.bytes = bytes;
        return RL_OK;
    }

    // ---- anchor-less injective groups ---------------------------------------
    rl_status plan_eltwise(int gi, const std::vector<int> &ops)
    {
        std::set<int> gset(ops.begin(), ops.end());
        const OpNode &first = g.ops[ops[0]];
        const int start = first.in[0];
        Chain chain;
        rl_status st = build_chain(ops, 0, ops.size(), start, gset, chain);
        if (st != RL_OK) return st;
        const int vout = chain.last_value;
        const rl_type &ot = T(vout);
        int layout = L_NATIVE;
        if (ot.rank == 4 && !layout_free(vout) && (chain.bias_axis < 0 || chain.bias_axis == 1) && phys[L_NATIVE][start] < 0 &&
            !out_set.count(vout))
            layout = L_NHWC;
        int xbuf;
        st = need(start, layout, xbuf);
        if (st != RL_OK) return st;
        EltwiseParams e{};
        e.x_dtype = T(start).dtype;
        e.y_dtype = ot.dtype;
        e.n = numel(ot);
        e.ch_inner = 1; e.ch_count = 1;
        if (chain.bias_axis >= 0) {
            if (layout == L_NHWC) { e.ch_inner = 1; e.ch_count = (int)ot.dims[1]; }
            else {
                int64_t inner = 1;
                for (int d = chain.bias_axis + 1; d < ot.rank; ++d) inner *= ot.dims[d];
                e.ch_inner = inner; e.ch_count = (int)ot.dims[chain.bias_axis];
            }
        }
        double bytes = (double)bytes_of(start) + (double)bytes_of(vout);
        Step tmp;
        st = bind_chain(chain, tmp, layout, bytes);
        if (st != RL_OK) return st;
        int ybuf = out_buf(vout, layout);
        e.epi = chain.epi;
        Step &s = add_step(S_ELTWISE, "eltwise#" + std::to_string(ops[0]), "eltwise_chain");
        s.group = gi;
        s.el = e;
        s.slot[SL_X] = xbuf; s.slot[SL_Y] = ybuf;
        for (int i = 0; i < RL_EPI_MAX_PTRS; ++i) s.slot[SL_E0 + i] = tmp.slot[SL_E0 + i];
        s.flops = (double)e.n * chain.epi.n_ops;
        s.bytes = bytes;
        return RL_OK;
    }

    rl_status plan_pool(int gi, int oi)
    {
        const OpNode &o = g.ops[oi];
        const rl_type &xt = T(o.in[0]), &ot = T(o.out[0]);
        int xbuf;
        rl_status st = need(o.in[0], L_NHWC, xbuf);
        if (st != RL_OK) return st;
        PoolParams p{};
        p.dtype = xt.dtype;
        p.N = (int)xt.dims[0]; p.C = (int)xt.dims[1]; p.H = (int)xt.dims[2]; p.W = (int)xt.dims[3];
        p.OH = (int)ot.dims[2]; p.OW = (int)ot.dims[3];
        bool mx = o.kind == RL_OP_MAXPOOL2D;
        if (mx) {
            p.KH = o.attrs.kernel[0]; p.KW = o.attrs.kernel[1]; p.sh = o.attrs.stride[0]; p.sw = o.attrs.stride[1];
            p.ph = o.attrs.pad[0]; p.pw = o.attrs.pad[1];
        }
        int ybuf = out_buf(o.out[0], L_NHWC);
        Step &s = add_step(mx ? S_MAXPOOL : S_GAVG, std::string(op_name(o.kind)) + "#" + std::to_string(oi), mx ? "maxpool_nhwc" : "gavgpool_nhwc");
        s.group = gi;
        s.po = p;
        s.slot[SL_X] = xbuf; s.slot[SL_Y] = ybuf;
        s.bytes = (double)bytes_of(o.in[0]) + (double)bytes_of(o.out[0]);
        s.flops = (double)numel(ot) * (mx ? p.KH * p.KW : p.H * p.W);
        return RL_OK;
    }

    rl_status plan_flatten(int oi)
    {
        const OpNode &o = g.ops[oi];
        int buf;
        rl_status st = need(o.in[0], L_NATIVE, buf);      // row-major order of the Shape is what flatten keeps
        if (st != RL_OK) return st;
        set_phys(o.out[0], L_NATIVE, buf);                // zero-copy alias
        return RL_OK;
    }

    // A change of layout (a permutation of the axes).  Rank-4 values live channel-last inside convolution, pool and
    // elementwise groups, so the two permutations between channel-first and channel-last Shapes are the other
    // view of storage that exists anyway: the result aliases it.  A permutation that keeps a prefix of the axes
    // and exchanges two blocks behind it is a batched transposition (LDS-tiled kernel); the rest gathers.
    rl_status plan_layout(int gi, int oi)
    {
        const OpNode &o = g.ops[oi];
        const int x = o.in[0], y = o.out[0];
        const rl_type &xt = T(x), &yt = T(y);
        const int r = xt.rank;
        const int32_t *pm = o.attrs.perm;
        bool ident = true;
        for (int i = 0; i < r; ++i) ident &= pm[i] == i;
        const bool to_last = r == 4 && pm[0] == 0 && pm[1] == 2 && pm[2] == 3 && pm[3] == 1;
        const bool to_first = r == 4 && pm[0] == 0 && pm[1] == 3 && pm[2] == 1 && pm[3] == 2;
        int buf;
        if (ident || (to_last && layout_free(x)) || (to_first && layout_free(y))) {     // same order in memory
            rl_status st = need(x, L_NATIVE, buf);
            if (st != RL_OK) return st;
            set_phys(y, L_NATIVE, buf);
            return RL_OK;
        }
        if (to_last && phys[L_NHWC][x] >= 0) { set_phys(y, L_NATIVE, phys[L_NHWC][x]); return RL_OK; }
        if (to_first) {
            rl_status st = need(x, L_NATIVE, buf);
            if (st != RL_OK) return st;
            set_phys(y, L_NHWC, buf);               // a consumer that wants y in Shape order gets the transposition then
            return RL_OK;
        }
        rl_status st = need(x, L_NATIVE, buf);
        if (st != RL_OK) return st;
        // identity prefix of length a, then blocks [a, a+R) and [a+R, r) exchanged?
        int a = 0;
        while (a < r && pm[a] == a) ++a;
        int split = -1;                             // first axis of the block that moves to the front
        if (a < r) {
            split = pm[a];
            bool ok = split > a;
            for (int i = a; i < r && ok; ++i) ok = pm[i] == (i - a + split < r ? i - a + split : i - a + split - r + a);
            if (!ok) split = -1;
        }
        const int ybuf = out_buf(y, L_NATIVE);
        if (split > 0) {
            int64_t outer = 1, R = 1, Q = 1;
            for (int i = 0; i < a; ++i) outer *= xt.dims[i];
            for (int i = a; i < split; ++i) R *= xt.dims[i];
            for (int i = split; i < r; ++i) Q *= xt.dims[i];
            if (outer <= 65535 && (R + 31) / 32 <= 65535 && Q <= 0x7fffffff && R <= 0x7fffffff) {
                Step &s = add_step(S_TO_NHWC, "layout_transform#" + std::to_string(oi), "transpose_tiled");
                s.group = gi;
                s.t_dtype = xt.dtype; s.t_N = (int)outer; s.t_C = (int)R; s.t_P = (int)Q;
                s.slot[SL_X] = buf; s.slot[SL_Y] = ybuf;
                s.bytes = 2.0 * bytes_of(x);
                if (to_last) phys[L_NHWC][x] = ybuf;     // the result doubles as the operand's channel-last form
                return RL_OK;
            }
        }
        PermuteParams pe{};
        pe.dtype = xt.dtype; pe.rank = r; pe.n = numel(xt);
        int64_t xs[RL_MAX_RANK];
        int64_t acc = 1;
        for (int i = r - 1; i >= 0; --i) { xs[i] = acc; acc *= xt.dims[i]; }
        for (int k = 0; k < r; ++k) { pe.ydims[k] = (int32_t)yt.dims[k]; pe.xstride[k] = xs[pm[k]]; }
        for (int k = 0; k < r; ++k) if (yt.dims[k] > 0x7fffffff) return fail(RL_ERR_UNSUPPORTED, "layout_transform: axis too long");
        Step &s = add_step(S_PERMUTE, "layout_transform#" + std::to_string(oi), "permute_gather");
        s.group = gi;
        s.pe = pe;
        s.slot[SL_X] = buf; s.slot[SL_Y] = ybuf;
        s.bytes = 2.0 * bytes_of(x);
        return RL_OK;
    }

    rl_status plan_gates(int gi, int oi)
    {
        const OpNode &o = g.ops[oi];
        int zbuf, cbuf;
        rl_status st = need(o.in[0], L_NATIVE, zbuf);
        if (st != RL_OK) return st;
        st = need(o.in[1], L_NATIVE, cbuf);
        if (st != RL_OK) return st;
        GatesParams p{};
        p.B = (int)T(o.in[1]).dims[0]; p.H = (int)T(o.in[1]).dims[1];
        p.h_dtype = T(o.out[1]).dtype;
        int cob = out_buf(o.out[0], L_NATIVE), hob = out_buf(o.out[1], L_NATIVE);
        Step &s = add_step(S_GATES, "lstm_gates#" + std::to_string(oi), "lstm_gates");
        s.group = gi;
        s.ga = p;
        s.slot[SL_X] = zbuf; s.slot[SL_CIN] = cbuf; s.slot[SL_COUT] = cob; s.slot[SL_HOUT] = hob;
        s.bytes = (double)bytes_of(o.in[0]) + 2.0 * bytes_of(o.in[1]) + bytes_of(o.out[1]);
        s.flops = 30.0 * p.B * p.H;
        return RL_OK;
    }

    // ---- partial derivatives of the contractions --------------------------------
    // Each is again a contraction C[m, n] = sum_k A[m, k] Wp[n, k] once its operands are looked at the right way round:
    //   dense_grad_x   m = batch row,       n = input feature k',  k = output feature:   A = dy,            Wp[k'][n] = W[n][k']
    //   dense_grad_w   m = output feature,  n = input feature,     k = batch row:        A[n][m] = dy[m][n], Wp[k'][m] = x[m][k']
    //   conv2d_grad_x  m = input pixel,     n = input channel,     k = (tap, out chan.): A = dy with stride-1 zeros between its
    //                  pixels and a border of K-1-pad, Wp = w with taps reversed and channel roles exchanged
    //   conv2d_grad_w  m = (in chan., tap), n = output channel,    k = (out pixel, image): A = x read with channel and image
    //                  exchanged and taps `stride` apart, Wp[o][(i, j), n] = dy[n][o][i][j]
    // A is read in place through the element-gather kernel's strides; Wp is gathered once into K-contiguous rows: at
    // prepack time when it comes from a param, by a step of the plan when it comes from an activation.
    rl_status plan_grad(int gi, int oi)
    {
        const OpNode &o = g.ops[oi];
        const int va = o.in[0], vb = o.in[1], vy = o.out[0];
        const rl_type &ta = T(va), &tb = T(vb), &ty = T(vy);
        const int dt = ta.dtype;
        const int KV = kv_of(dt);
        IgemmParams p{};
        GatherPack gp{};
        p.in_dtype = dt; p.y_dtype = ty.dtype;
        gp.dtype = dt;
        if (numel(ta) >= ((int64_t)1 << 31) || numel(tb) >= ((int64_t)1 << 31) || numel(ty) >= ((int64_t)1 << 31))
            return fail(RL_ERR_UNSUPPORTED, std::string(op_name(o.kind)) + ": tensor too large");
        // With respect to the first operand, through weights that are a param of their own: a dense, or a stride-1 conv2d
        // with reversed taps and exchanged channel roles, of dy; planned like the forward operator, onto its kernels.
        if (g.values[vb].role == ROLE_PARAM && consumers[vb].size() == 1 && !plan.packs.count(vb) && !plan.opts.no_grad_fwd) {
            AnchorView ov{};
            ov.gp.dtype = dt;
            if (o.kind == RL_OP_DENSE_GRAD_X) {
                const int N = (int)ta.dims[1], K = (int)tb.dims[1];
                ov.kind = RL_OP_DENSE; ov.N = K; ov.KH = ov.KW = 1;
                ov.gp.R = K; ov.gp.T = 1; ov.gp.TW = 1; ov.gp.Cq = N; ov.gp.s_row = 1; ov.gp.s_c = K;
                return plan_anchor(gi, std::vector<int>{oi}, &ov);
            }
            if (o.kind == RL_OP_CONV2D_GRAD_X && o.attrs.stride[0] == 1 && o.attrs.stride[1] == 1) {
                const int O = (int)ta.dims[1], C = (int)tb.dims[1], KH = (int)tb.dims[2], KW = (int)tb.dims[3];
                if (o.attrs.pad[0] > KH - 1 || o.attrs.pad[1] > KW - 1) return fail(RL_ERR_UNSUPPORTED, "conv2d_grad_x: padding larger than the kernel");
                ov.kind = RL_OP_CONV2D; ov.N = C; ov.KH = KH; ov.KW = KW; ov.ph = KH - 1 - o.attrs.pad[0]; ov.pw = KW - 1 - o.attrs.pad[1];
                ov.gp.R = C; ov.gp.T = KH * KW; ov.gp.TW = KW; ov.gp.Cq = O;
                ov.gp.s_row = (int64_t)KH * KW; ov.gp.s_c = (int64_t)C * KH * KW; ov.gp.s_ti = -KW; ov.gp.s_tj = -1; ov.gp.base = (int64_t)KH * KW - 1;
                return plan_anchor(gi, std::vector<int>{oi}, &ov);
            }
            // At a stride: the same stride-1 convolution of dy spread out with zeros (a step of its own writes that
            // tensor; three of four products are with zeros, on kernels that are many times faster than the gather).
            if (o.kind == RL_OP_CONV2D_GRAD_X && o.attrs.stride[0] == o.attrs.stride[1] && o.attrs.stride[0] > 1 &&
                (ta.dims[1] * (int64_t)dtype_size(dt)) % 16 == 0) {
                const int Nb = (int)ta.dims[0], O = (int)ta.dims[1], OH = (int)ta.dims[2], OW = (int)ta.dims[3];
                const int C = (int)tb.dims[1], KH = (int)tb.dims[2], KW = (int)tb.dims[3], H = (int)ty.dims[2], W = (int)ty.dims[3];
                const int sd = o.attrs.stride[0];
                if (o.attrs.pad[0] > KH - 1 || o.attrs.pad[1] > KW - 1) return fail(RL_ERR_UNSUPPORTED, "conv2d_grad_x: padding larger than the kernel");
                const int Hd = H + 2 * o.attrs.pad[0] - KH + 1, Wd = W + 2 * o.attrs.pad[1] - KW + 1;
                const size_t dbytes = (size_t)Nb * Hd * Wd * O * dtype_size(dt);
                if (Hd >= (OH - 1) * sd + 1 && Wd >= (OW - 1) * sd + 1 && dbytes < ((size_t)1 << 31)) {
                    int src;
                    rl_status st = need(va, L_NHWC, src);
                    if (st != RL_OK) return st;
                    const int dil = new_ws(dbytes);
                    Step &ds = add_step(S_DILATE, std::string(op_name(o.kind)) + "#" + std::to_string(oi) + ".spread", "dilate_nhwc");
                    ds.group = gi;
                    ds.t_N = Nb; ds.t_C = (int)(O * dtype_size(dt)); ds.st_H = OH; ds.st_W = OW; ds.st_Hp = Hd; ds.st_Wp = Wd; ds.st_ph = sd;
                    ds.slot[SL_X] = src; ds.slot[SL_Y] = dil;
                    ds.bytes = (double)bytes_of(va) + (double)dbytes;
                    ov.kind = RL_OP_CONV2D; ov.N = C; ov.KH = KH; ov.KW = KW; ov.ph = KH - 1 - o.attrs.pad[0]; ov.pw = KW - 1 - o.attrs.pad[1];
                    ov.gp.R = C; ov.gp.T = KH * KW; ov.gp.TW = KW; ov.gp.Cq = O;
                    ov.gp.s_row = (int64_t)KH * KW; ov.gp.s_c = (int64_t)C * KH * KW; ov.gp.s_ti = -KW; ov.gp.s_tj = -1; ov.gp.base = (int64_t)KH * KW - 1;
                    ov.xbuf = dil; ov.xH = Hd; ov.xW = Wd;
                    st = plan_anchor(gi, std::vector<int>{oi}, &ov);
                    if (st != RL_OK) return st;
                    for (size_t k = plan.steps.size(); k-- > 0;)
                        if (plan.steps[k].kind == S_IGEMM) { plan.steps[k].flops /= (double)(sd * sd); break; }     // the zeros are no work
                    return RL_OK;
                }
            }
        }
        p.C = 1; p.H = p.W = p.KH = p.KW = p.OH = p.OW = p.OHW = 1; p.sh = p.sw = 1;
        if (o.kind == RL_OP_DENSE_GRAD_X) {
            const int M = (int)ta.dims[0], N = (int)ta.dims[1], K = (int)tb.dims[1];
            p.M = M; p.N = K; p.K = N; p.C = N;
            p.xs_n = N; p.xs_c = 1;
            gp.R = K; gp.T = 1; gp.TW = 1; gp.Cq = N; gp.s_row = 1; gp.s_c = K;
        } else if (o.kind == RL_OP_DENSE_GRAD_W) {
            const int M = (int)ta.dims[0], N = (int)ta.dims[1], K = (int)tb.dims[1];
            p.M = N; p.N = K; p.K = M; p.C = M;
            p.xs_n = 1; p.xs_c = N;
            gp.R = K; gp.T = 1; gp.TW = 1; gp.Cq = M; gp.s_row = 1; gp.s_c = K;
        } else if (o.kind == RL_OP_CONV2D_GRAD_X) {
            // dy[N,O,OH,OW], w[O,C,KH,KW] -> dx[N,C,H,W]
            const int Nb = (int)ta.dims[0], O = (int)ta.dims[1], OH = (int)ta.dims[2], OW = (int)ta.dims[3];
            const int C = (int)tb.dims[1], KH = (int)tb.dims[2], KW = (int)tb.dims[3], H = (int)ty.dims[2], W = (int)ty.dims[3];
            if (o.attrs.stride[0] != o.attrs.stride[1]) return fail(RL_ERR_UNSUPPORTED, "conv2d_grad_x: strides must agree");
            if (o.attrs.pad[0] > KH - 1 || o.attrs.pad[1] > KW - 1) return fail(RL_ERR_UNSUPPORTED, "conv2d_grad_x: padding larger than the kernel");
            if ((int64_t)Nb * H * W > 0x7fffffff) return fail(RL_ERR_UNSUPPORTED, "conv2d_grad_x too large");
            p.M = Nb * H * W; p.N = C; p.K = O * KH * KW; p.C = O;
            p.H = OH; p.W = OW; p.KH = KH; p.KW = KW; p.OH = H; p.OW = W; p.OHW = H * W;
            p.sh = p.sw = 1; p.ph = KH - 1 - o.attrs.pad[0]; p.pw = KW - 1 - o.attrs.pad[1];
            p.in_dil_m1 = o.attrs.stride[0] - 1;
            p.xs_n = (int64_t)O * OH * OW; p.xs_c = (int64_t)OH * OW; p.xs_h = OW; p.xs_w = 1;
            p.ys_n = (int64_t)C * H * W; p.ys_p = 1; p.ys_c = (int64_t)H * W;
            // Wp[c][(a', b'), o] = w[o][c][KH-1-a'][KW-1-b']
            gp.R = C; gp.T = KH * KW; gp.TW = KW; gp.Cq = O;
            gp.s_row = (int64_t)KH * KW; gp.s_c = (int64_t)C * KH * KW; gp.s_ti = -KW; gp.s_tj = -1; gp.base = (int64_t)KH * KW - 1;
        } else {
            // dy[N,O,OH,OW], x[N,C,H,W] -> dw[O,C,KH,KW]
            const int Nb = (int)ta.dims[0], O = (int)ta.dims[1], OH = (int)ta.dims[2], OW = (int)ta.dims[3];
            const int C = (int)tb.dims[1], H = (int)tb.dims[2], W = (int)tb.dims[3], KH = (int)ty.dims[2], KW = (int)ty.dims[3];
            if (o.attrs.stride[0] != o.attrs.stride[1]) return fail(RL_ERR_UNSUPPORTED, "conv2d_grad_w: strides must agree");
            if (dt == RL_BF16 && conv_wgrad_ok(Nb, O, C, KH, KW, o.attrs.stride[0]) && o.attrs.pad[0] < KH && o.attrs.pad[1] < KW &&
                bytes_of(va) < ((size_t)1 << 31) && bytes_of(vb) < ((size_t)1 << 31) && !plan.opts.no_wgrad)
                return plan_wgrad(gi, oi);
            if ((int64_t)Nb * OH * OW > 0x7ffffff0) return fail(RL_ERR_UNSUPPORTED, "conv2d_grad_w too large");
            p.M = C * KH * KW; p.N = O; p.K = Nb * OH * OW; p.C = Nb;
            p.H = H; p.W = W; p.KH = OH; p.KW = OW; p.OH = KH; p.OW = KW; p.OHW = KH * KW;
            p.sh = p.sw = 1; p.ph = o.attrs.pad[0]; p.pw = o.attrs.pad[1];
            p.tap_dil_m1 = o.attrs.stride[0] - 1;
            p.xs_n = (int64_t)H * W; p.xs_c = (int64_t)C * H * W; p.xs_h = W; p.xs_w = 1;      // "image" = channel c, "channel" = image n
            p.ys_n = (int64_t)KH * KW; p.ys_p = 1; p.ys_c = (int64_t)C * KH * KW;               // dw[o][c][a][b] at n*ys_c + m
            // Wp[o][(i, j), n] = dy[n][o][i][j]
            gp.R = O; gp.T = OH * OW; gp.TW = OW; gp.Cq = Nb;
            gp.s_row = (int64_t)OH * OW; gp.s_c = (int64_t)O * OH * OW; gp.s_ti = OW; gp.s_tj = 1;
        }
        if (o.kind == RL_OP_DENSE_GRAD_X || o.kind == RL_OP_DENSE_GRAD_W) { p.ys_n = p.N; p.ys_p = p.N; p.ys_c = 1; }
        p.K1 = p.K;
        p.Kp = (int)round_up(p.K, KV);
        gp.Kp = p.Kp;
        p.ts_h = p.xs_h; p.ts_w = p.xs_w; p.seg_stride = 64;
        make_fast_div((uint32_t)p.OHW, p.div_ohw_mul, p.div_ohw_sh);
        make_fast_div((uint32_t)p.OW, p.div_ow_mul, p.div_ow_sh);
        const size_t lim = (size_t)1 << 31;
        const size_t wbytes = (size_t)gp.R * gp.Kp * dtype_size(dt);
        if (wbytes >= lim) return fail(RL_ERR_UNSUPPORTED, std::string(op_name(o.kind)) + ": operand too large");
        p.x_bytes = (uint32_t)std::min(bytes_of(va), lim - 1);
        p.w_bytes = (uint32_t)wbytes;
        p.y_bytes = (uint32_t)std::min(bytes_of(vy), lim - 1);

        int abuf, wbuf;
        rl_status st;
        // which of the two operands is A and which is gathered into Wp: dy is A except for conv2d_grad_w, where x is
        int a_val = va, w_val = vb;
        if (o.kind == RL_OP_CONV2D_GRAD_W) { a_val = vb; w_val = va; }
        st = need(a_val, L_NATIVE, abuf);
        if (st != RL_OK) return st;
        if (g.values[w_val].role == ROLE_PARAM && consumers[w_val].size() == 1) {     // a param with other uses keeps its own layout for them
            PackSpec pack;
            pack.dtype = dt; pack.gather = 1; pack.gp = gp; pack.bytes = wbytes; pack.Kp = gp.Kp; pack.perm_block = -3;
            auto it = plan.packs.find(w_val);
            if (it != plan.packs.end()) return fail(RL_ERR_UNSUPPORTED, "one param needs two different kernel-native layouts");
            plan.packs[w_val] = pack;
            wbuf = bound(w_val);
        } else {
            int src;
            st = need(w_val, L_NATIVE, src);
            if (st != RL_OK) return st;
            wbuf = new_ws(wbytes);
            Step &ps = add_step(S_PACK, std::string(op_name(o.kind)) + "#" + std::to_string(oi) + ".operand", "pack_gather");
            ps.group = gi;
            ps.gp = gp;
            ps.slot[SL_X] = src; ps.slot[SL_Y] = wbuf;
            ps.bytes = (double)bytes_of(w_val) + (double)wbytes;
        }
        const int ybuf = out_buf(vy, L_NATIVE);
        IgemmLaunch il{};
        il.tile = TILE_64x64;                         // element gather: any strides, any counts
        // few tiles and a long K (a weight gradient contracts over every pixel of the batch): K split over workgroups
        int part_buf = -1;
        if (!plan.opts.no_splitk) {
            const int64_t tiles = (int64_t)((p.M + 63) / 64) * ((p.N + 63) / 64);
            const int nk = (p.Kp + 8 * KV - 1) / (8 * KV);
            const int want = (int)std::min<int64_t>(std::min<int64_t>(64, 512 / std::max<int64_t>(tiles, 1)), nk / 4);
            if (tiles <= 128 && want >= 2 && (int64_t)want * p.M * p.N * 4 < (int64_t)1 << 28) {
                const int per = (nk + want - 1) / want;
                il.splits = (nk + per - 1) / per;
                p.splits = il.splits; p.split_tiles = per;
                part_buf = new_ws((size_t)il.splits * p.M * p.N * 4);
            }
        }
        Step &s = add_step(S_IGEMM, std::string(op_name(o.kind)) + "#" + std::to_string(oi),
                           std::string("igemm_") + op_name(o.kind) + (dt == RL_BF16 ? "_bf16" : "_f32") + "_64x64_gather");
        s.group = gi;
        s.ig = p; s.il = il;
        s.slot[SL_X] = abuf; s.slot[SL_W] = wbuf; s.slot[SL_Y] = ybuf; s.slot[SL_PART] = part_buf;
        if (il.splits > 1) s.kernel += "_splitk";
        s.flops = 2.0 * p.M * (double)p.N * p.K / (double)((p.in_dil_m1 + 1) * (p.in_dil_m1 + 1));     // the zeros between dy's pixels are no work
        s.bytes = (double)bytes_of(va) + (double)bytes_of(vb) + (double)bytes_of(vy);
        return RL_OK;
    }

    // conv2d_grad_w on bf16 batches of 64: both operands transposed so that the images are the fastest axis (two steps),
    // the contraction per output pixel and filter tap (conv_wgrad.hip), the row segments' sums added in order (a step).
    rl_status plan_wgrad(int gi, int oi)
    {
        const OpNode &o = g.ops[oi];
        const int vdy = o.in[0], vx = o.in[1], vy = o.out[0];
        const rl_type &ta = T(vdy), &tb = T(vx), &ty = T(vy);
        const int Nb = (int)ta.dims[0], O = (int)ta.dims[1], OH = (int)ta.dims[2], OW = (int)ta.dims[3];
        const int C = (int)tb.dims[1], H = (int)tb.dims[2], W = (int)tb.dims[3], KH = (int)ty.dims[2], KW = (int)ty.dims[3];
        WgradParams w{};
        w.O = O; w.C = C; w.H = H; w.W = W; w.OH = OH; w.OW = OW; w.KH = KH; w.KW = KW;
        w.s = o.attrs.stride[0]; w.ph = o.attrs.pad[0]; w.pw = o.attrs.pad[1];
        // an operand as the plan holds it (channel-last if some group already wrote or asked for that, else as declared),
        // viewed as a matrix [images][everything else] and transposed
        auto batch_last = [&](int v, int Cc, int P, int64_t &s_pix, int64_t &s_ch, int &tbuf) -> rl_status {
            int src;
            const bool cl = phys[L_NHWC][v] >= 0;
            rl_status st = need(v, cl ? L_NHWC : L_NATIVE, src);
            if (st != RL_OK) return st;
            if (cl) { s_pix = (int64_t)Cc * Nb; s_ch = Nb; }
            else { s_pix = Nb; s_ch = (int64_t)P * Nb; }
            tbuf = new_ws(bytes_of(v));
            Step &ts = add_step(S_TO_NHWC, std::string(op_name(o.kind)) + "#" + std::to_string(oi) + ".images_last", "transpose_images_last");
            ts.group = gi;
            ts.t_dtype = T(v).dtype; ts.t_N = 1; ts.t_C = Nb; ts.t_P = Cc * P;
            ts.slot[SL_X] = src; ts.slot[SL_Y] = tbuf;
            ts.bytes = 2.0 * bytes_of(v);
            return RL_OK;
        };
        int dyT, xT;
        rl_status st = batch_last(vdy, O, OH * OW, w.ys_pix, w.ys_o, dyT);
        if (st != RL_OK) return st;
        st = batch_last(vx, C, H * W, w.xs_pix, w.xs_c, xT);
        if (st != RL_OK) return st;
        w.nck = Nb / 64;
        w.n_ot = O % 128 == 0 ? O / 128 : O / 64;
        w.n_ct = C / 64;
        // one workgroup per CU (its LDS is full): as many row segments as keep the grid within one round
        const int tiles = OH * w.n_ot * w.n_ct;
        int nseg = std::max(1, std::min(OW, 256 / std::max(tiles, 1)));
        w.L = (OW + nseg - 1) / nseg;
        w.nseg = (OW + w.L - 1) / w.L;
        const int chunks = OH * w.nseg, Tt = KH * KW;
        const size_t part_bytes = (size_t)chunks * Tt * O * C * 4;
        if (part_bytes >= ((size_t)1 << 32)) return fail(RL_ERR_UNSUPPORTED, "conv2d_grad_w: partial sums too large");
        const int part = new_ws(part_bytes);
        Step &s = add_step(S_WGRAD, std::string(op_name(o.kind)) + "#" + std::to_string(oi), std::string("conv2d_grad_w_bf16_") + (O % 128 == 0 ? "128x64" : "64x64") + "_images_last");
        s.group = gi;
        s.wg = w;
        s.slot[SL_X] = xT; s.slot[SL_X2] = dyT; s.slot[SL_PART] = part;
        s.flops = 2.0 * Nb * OH * OW * (double)O * C * Tt;
        s.bytes = (double)bytes_of(vdy) + (double)bytes_of(vx) + (double)part_bytes;
        const int ybuf = out_buf(vy, L_NATIVE);
        Step &r = add_step(S_WGRAD_REDUCE, std::string(op_name(o.kind)) + "#" + std::to_string(oi) + ".segments", "wgrad_reduce");
        r.group = gi;
        r.wg = w;
        r.t_dtype = ty.dtype; r.t_N = chunks; r.t_C = Tt;
        r.slot[SL_X] = part; r.slot[SL_Y] = ybuf;
        r.bytes = (double)part_bytes + (double)bytes_of(vy);
        return RL_OK;
    }

    rl_status plan_group(int gi, std::vector<int> ops)
    {
        std::sort(ops.begin(), ops.end());
        rl_status st = check_group(g, ops, msg);
        if (st != RL_OK) return st;
        bool has_anchor = false;
        for (int o : ops) has_anchor |= is_anchor(g.ops[o].kind);
        if (has_anchor) return plan_anchor(gi, ops);
        int k0 = g.ops[ops[0]].kind;
        if (ops.size() == 1) {
            if (k0 == RL_OP_MAXPOOL2D || k0 == RL_OP_GLOBAL_AVGPOOL) return plan_pool(gi, ops[0]);
            if (k0 == RL_OP_FLATTEN) return plan_flatten(ops[0]);
            if (k0 == RL_OP_LSTM_GATES) return plan_gates(gi, ops[0]);
            if (k0 == RL_OP_LAYOUT_TRANSFORM) return plan_layout(gi, ops[0]);
            if (k0 >= RL_OP_DENSE_GRAD_X && k0 <= RL_OP_CONV2D_GRAD_W) return plan_grad(gi, ops[0]);
            if (k0 == RL_OP_CONCAT) return fail(RL_ERR_UNSUPPORTED, "concat is only implemented as the operand of a dense in its group");
        }
        return plan_eltwise(gi, ops);
    }

    rl_status run()
    {
        const int nv = (int)g.values.size();
        plan.values = g.values;
        plan.outputs = g.outputs;
        plan.err = g.err;
        plan.bound_buf.assign(nv, -1);
        phys[0].assign(nv, -1);
        phys[1].assign(nv, -1);
        out_set.insert(g.outputs.begin(), g.outputs.end());
        if (g.outputs.empty()) return fail(RL_ERR_TYPE, "graph has no output");
        consumers.assign(nv, {});
        for (size_t o = 0; o < g.ops.size(); ++o)
            for (int v : g.ops[o].in) consumers[v].push_back((int)o);
        for (int v = 0; v < nv; ++v)
            if (g.values[v].role != ROLE_OP) set_phys(v, L_NATIVE, bound(v));

        // groups: declared ones plus a singleton for every ungrouped call
        std::vector<std::vector<int>> groups = g.groups;
        std::vector<int> group_of(g.ops.size(), -1);
        for (size_t gi = 0; gi < groups.size(); ++gi)
            for (int o : groups[gi]) {
                if (o < 0 || o >= (int)g.ops.size() || group_of[o] >= 0) return fail(RL_ERR_GROUP, "an op is missing or in two groups");
                group_of[o] = (int)gi;
            }
        for (size_t o = 0; o < g.ops.size(); ++o)
            if (group_of[o] < 0) { group_of[o] = (int)groups.size(); groups.push_back({(int)o}); }

        // order groups so that producers run first; a cycle between groups is illegal
        const int ng = (int)groups.size();
        std::vector<std::set<int>> deps(ng);
        for (size_t o = 0; o < g.ops.size(); ++o)
            for (int v : g.ops[o].in) {
                int pr = g.values[v].producer;
                if (pr >= 0 && group_of[pr] != group_of[o]) deps[group_of[o]].insert(group_of[pr]);
            }
        std::vector<int> order, state(ng, 0);
        std::vector<int> key(ng);
        for (int i = 0; i < ng; ++i) key[i] = *std::min_element(groups[i].begin(), groups[i].end());
        std::vector<int> by_key(ng);
        for (int i = 0; i < ng; ++i) by_key[i] = i;
        std::sort(by_key.begin(), by_key.end(), [&](int a, int b) { return key[a] < key[b]; });
        bool cyc = false;
        std::vector<std::pair<int, std::set<int>::iterator>> stack;
        for (int root : by_key) {
            if (state[root]) continue;
            stack.push_back({root, deps[root].begin()});
            state[root] = 1;
            while (!stack.empty()) {
                auto &top = stack.back();
                if (top.second == deps[top.first].end()) {
                    state[top.first] = 2;
                    order.push_back(top.first);
                    stack.pop_back();
                } else {
                    int d = *top.second;
                    ++top.second;
                    if (state[d] == 1) { cyc = true; break; }
                    if (state[d] == 0) { state[d] = 1; stack.push_back({d, deps[d].begin()}); }
                }
            }
            if (cyc) return fail(RL_ERR_GROUP, "fusion groups depend on each other cyclically");
        }
        for (int gi : order) {
            rl_status st = plan_group(gi, groups[gi]);
            if (st != RL_OK) return st;
        }
        // every output must end up in its bound buffer in boundary order
        for (int v : g.outputs) {
            int b = bound(v);
            if (phys[L_NATIVE][v] == b) continue;
            if (phys[L_NATIVE][v] >= 0) {
                EltwiseParams e{};
                e.x_dtype = e.y_dtype = T(v).dtype;
                e.n = numel(T(v));
                e.ch_inner = 1; e.ch_count = 1;
                int src = phys[L_NATIVE][v];
                Step &s = add_step(S_ELTWISE, "copy_out", "eltwise_chain");
                s.el = e;
                s.slot[SL_X] = src; s.slot[SL_Y] = b;
                s.bytes = 2.0 * bytes_of(v);
            } else if (phys[L_NHWC][v] >= 0) {
                const rl_type &t = T(v);
                int src = phys[L_NHWC][v];
                Step &s = add_step(S_TO_NCHW, "layout_out", "nhwc_to_nchw");
                s.t_dtype = t.dtype; s.t_N = (int)t.dims[0]; s.t_C = (int)t.dims[1]; s.t_P = (int)(t.dims[2] * t.dims[3]);
                s.slot[SL_X] = src; s.slot[SL_Y] = b;
                s.bytes = 2.0 * bytes_of(v);
            } else {
                return fail(RL_ERR_TYPE, "an output is never computed");
            }
        }
        fuse_stem_pool();
        pair_contractions();
        chain_small_dense();
        assign_workspace();
        return RL_OK;
    }

    // A stem convolution group whose only consumer is the 3x3 / stride 2 / pad 1 max-pool group right behind it
    // runs as one kernel that pools the finished values in LDS: the full-size tensor between the two groups
    // (the largest of the whole graph) is then never written.  Same values as the two kernels, bit for bit
    // (max commutes with the bias, the ReLU and the rounding).
    void fuse_stem_pool()
    {
        if (plan.opts.no_stem_pool) return;
        for (size_t si = 0; si + 1 < plan.steps.size(); ++si) {
            Step &c = plan.steps[si];
            const Step &m = plan.steps[si + 1];
            const IgemmParams &g = c.ig;
            if (c.kind != S_IGEMM || !c.stem || !c.il.lp || m.kind != S_MAXPOOL) continue;
            const int mid = c.slot[SL_Y];
            if (mid < 0 || m.slot[SL_X] != mid || plan.bufs[mid].bound_value >= 0) continue;
            bool other_use = false;
            for (size_t sj = 0; sj < plan.steps.size(); ++sj)
                if (sj != si && sj != si + 1)
                    for (int b : plan.steps[sj].slot) other_use |= (b == mid);
            const PoolParams &po = m.po;
            Epilogue e = g.epi;                 // wanted: [f32 bias] [relu] and nothing else
            finalize_epilogue(e);
            if (other_use || g.sh != 2 || g.sw != 2 || g.N != 64 || g.y_dtype != DT_BF16 || po.dtype != DT_BF16 || po.C != 64 ||
                po.KH != 3 || po.KW != 3 || po.sh != 2 || po.sw != 2 || po.ph != 1 || po.pw != 1 || po.H != g.OH || po.W != g.OW ||
                po.OH != (g.OH - 1) / 2 + 1 || po.OW != (g.OW - 1) / 2 + 1 || !e.simple || e.t_op >= 0 ||
                (e.has_bias && e.bias_dtype != DT_F32) || (e.rest_n != 0 && !e.relu_last) ||
                (uint64_t)po.N * po.OH * po.OW * 64 * 2 >= ((uint64_t)1 << 31))
                continue;
            // Two forms of the fused kernel.  One fetches its patches from the channel-first planes themselves: the frame
            // copy in front of this step (the step before, whose result only this step reads) then goes, and the weights
            // are packed for that kernel's contraction order instead.  The other reads the frame (exactly four K tiles).
            bool direct = false;
            if (si > 0 && !plan.opts.no_stem_direct) {
                const Step &pd = plan.steps[si - 1];
                const int wbuf = c.slot[SL_W];
                const int wv = wbuf >= 0 ? plan.bufs[wbuf].bound_value : -1;
                auto pk = wv >= 0 ? plan.packs.find(wv) : plan.packs.end();
                bool frame_private = pd.kind == S_STEM_PAD && pd.slot[SL_Y] == c.slot[SL_X];
                for (size_t sj = 0; frame_private && sj < plan.steps.size(); ++sj)
                    if (sj != si && sj != si - 1)
                        for (int b : plan.steps[sj].slot) frame_private &= (b != pd.slot[SL_Y]);
                direct = frame_private && pk != plan.packs.end() && pk->second.stem == 1 && consumers[wv].size() == 1 &&
                         stem_direct_ok(pd.t_C, pd.st_H, pd.st_W, pk->second.KH, pk->second.KW, pd.st_ph, pd.st_pw) &&
                         (uint64_t)pd.t_N * pd.t_C * pd.st_H * pd.st_W * 2 < ((uint64_t)1 << 31);
                if (direct) {
                    c.stem_direct = 1;
                    c.t_N = pd.t_N; c.t_C = pd.t_C; c.st_H = pd.st_H; c.st_W = pd.st_W; c.st_ph = pd.st_ph; c.st_pw = pd.st_pw;
                    c.stem_kh = pk->second.KH; c.stem_kw = pk->second.KW;
                    c.bytes += (double)plan.bufs[pd.slot[SL_X]].bytes - (double)plan.bufs[pd.slot[SL_Y]].bytes;
                    c.slot[SL_X] = pd.slot[SL_X];
                    PackSpec &ps = pk->second;
                    ps.stem = 2; ps.pw = pd.st_pw; ps.Kp = STEM_DIRECT_KP; ps.bytes = (size_t)ps.O * STEM_DIRECT_KP * 2;
                }
            }
            if (!direct && (g.K != 256 || g.Kp != 256 || g.KH != 4)) continue;
            c.kind = S_STEM_POOL;
            c.sp_N = po.N; c.sp_PH = po.OH; c.sp_PW = po.OW;
            c.slot[SL_Y] = m.slot[SL_Y];
            c.name += "+" + m.name;
            c.kernel = direct ? "igemm_conv2d_bf16_stem_maxpool_direct" : "igemm_conv2d_bf16_stem_maxpool";
            c.bytes = c.bytes - (double)plan.bufs[mid].bytes + (double)plan.bufs[m.slot[SL_Y]].bytes;
            plan.steps.erase(plan.steps.begin() + (long)si + 1);
            if (direct) {
                plan.steps.erase(plan.steps.begin() + (long)si - 1);
                --si;
            }
        }
    }

    // Two consecutive contraction steps of which the second does not use the first one's result, and which run the
    // same variant of the pixel-on-lane kernel (a stage's stride-2 convolution and its 1x1 projection), share one
    // launch: each alone leaves a quarter of the CUs idle, and the projection's short tiles fit into that gap.
    void pair_contractions()
    {
        if (plan.opts.no_pair) return;
        for (size_t si = 0; si + 1 < plan.steps.size(); ++si) {
            Step &a = plan.steps[si];
            Step &b = plan.steps[si + 1];
            if (a.kind != S_IGEMM || b.kind != S_IGEMM || a.pair || b.pair || a.stem || b.stem) continue;
            // a 3x3 / stride 2 convolution and the 1x1 / stride 2 projection of the same tensor: one contraction, the
            // projection riding on the centre tap; any other two contractions of one kernel variant: one grid
            const bool fused = plan.opts.s2_pair && a.slot[SL_X] >= 0 && a.slot[SL_X] == b.slot[SL_X] && conv3x3s2_pair_ok(a.ig, a.il, b.ig, b.il);
            if (!fused && !igemm_lp_can_pair(a.ig, a.il, b.ig, b.il)) continue;
            const int ya = a.slot[SL_Y], yb = b.slot[SL_Y];
            if (ya < 0 || yb < 0 || ya == yb) continue;
            bool dep = false;
            for (int s : b.slot) dep |= (s == ya);          // b reads (or overwrites) a's result
            for (int s : a.slot) dep |= (s == yb);          // a reads what b writes
            if (dep) continue;
            a.pair = 1; b.pair = 2;
            if (fused) {
                a.il.s2pair = 1;
                a.kernel = "igemm_conv2d_bf16_3x3s2_pair";
                b.bytes -= (double)plan.bufs[b.slot[SL_X]].bytes;     // the shared input is read once
            }
            a.flops += b.flops; a.bytes += b.bytes;
            b.flops = 0; b.bytes = 0;
            a.name += " | " + b.name;
            b.kernel = "(launched with the step before)";
            ++si;
        }
    }

    // A dense contraction whose K is split over workgroups ends in a launch that adds the slices.  When its result feeds
    // nothing but a small dense layer right behind it (an MLP's output layer), that launch computes the small layer as
    // well, a row per workgroup, and the tensor between the two groups never leaves LDS: a launch fewer on graphs
    // whose time is the number of their launches.
    void chain_small_dense()
    {
        if (plan.opts.no_dense_chain) return;
        for (size_t si = 0; si + 1 < plan.steps.size(); ++si) {
            Step &a = plan.steps[si];
            Step &b = plan.steps[si + 1];
            if (a.kind != S_IGEMM || b.kind != S_IGEMM || a.pair || b.pair || a.chain || b.chain || a.stem || b.stem) continue;
            const IgemmParams &pa = a.ig, &pb = b.ig;
            if (a.il.splits < 2 || !a.il.avec || !a.il.dma || a.il.lp || a.il.gates || b.il.gates) continue;
            if (pa.OHW != 1 || pb.OHW != 1 || pa.KH * pa.KW != 1 || pb.KH * pb.KW != 1) continue;                       // two dense layers
            if (pa.ys_c != 1 || pa.ys_n != pa.N || pa.N > REDUCE_DENSE_MAX_N1 || pa.M > 65535) continue;
            if (pb.M != pa.M || pb.K != pa.N || pb.K1 != pb.K || pb.N > REDUCE_DENSE_MAX_N2 || pb.xs_c != 1 || pb.xs_n != pa.N) continue;
            if (b.slot[SL_X2] >= 0 || pb.in_dtype != pa.y_dtype) continue;
            const int h = a.slot[SL_Y];
            if (h < 0 || plan.bufs[h].bound_value >= 0 || b.slot[SL_X] != h) continue;                               // the result is the plan's own
            bool other = false;                                                                                        // ... and nobody else's
            for (size_t sj = 0; sj < plan.steps.size(); ++sj)
                for (int q = 0; q < SL_COUNT; ++q)
                    if (plan.steps[sj].slot[q] == h && !((sj == si && q == SL_Y) || (sj == si + 1 && q == SL_X))) other = true;
            if (other) continue;
            a.chain = 1; b.chain = 2;
            b.slot[SL_PART] = -1;                       // the small layer's own K split, if it had one, is not used
            b.il.splits = 1; b.ig.splits = 0; b.ig.split_tiles = 0;
            a.kernel += "+dense";
            a.name += " > " + b.name;
            a.flops += b.flops; a.bytes += b.bytes - 2.0 * plan.bufs[h].bytes;      // the tensor between them is neither written nor read
            b.flops = 0; b.bytes = 0;
            b.kernel = "(launched with the step before)";
            ++si;
        }
    }

    // liveness-based first-fit packing of workspace buffers
    void assign_workspace()
    {
        for (size_t si = 0; si < plan.steps.size(); ++si)
            for (int b : plan.steps[si].slot)
                if (b >= 0) {
                    BufDesc &d = plan.bufs[b];
                    // the second step of a pair runs when the first is launched
                    const int at = plan.steps[si].pair == 2 ? (int)si - 1 : (int)si;
                    if (d.first < 0) d.first = at;
                    d.last = (int)si;
                }
        std::vector<int> ws;
        for (size_t b = 0; b < plan.bufs.size(); ++b)
            if (plan.bufs[b].bound_value < 0 && plan.bufs[b].first >= 0) ws.push_back((int)b);
        std::sort(ws.begin(), ws.end(), [&](int a, int b) { return plan.bufs[a].first < plan.bufs[b].first; });
        std::vector<int> placed;
        size_t total = 0;
        for (int b : ws) {
            BufDesc &d = plan.bufs[b];
            std::vector<std::pair<size_t, size_t>> busy;
            for (int q : placed) {
                const BufDesc &o = plan.bufs[q];
                if (o.last >= d.first && o.first <= d.last) busy.push_back({o.offset, o.offset + o.bytes});
            }
            std::sort(busy.begin(), busy.end());
            size_t off = 0;
            for (auto &iv : busy) {
                if (off + d.bytes <= iv.first) break;
                if (iv.second > off) off = iv.second;
            }
            d.offset = off;
            total = std::max(total, off + d.bytes);
            placed.push_back(b);
        }
        plan.workspace_bytes = total;
    }
};

}  // namespace

rl_status build_plan(const Graph &g, Plan &plan, std::string &msg)
{
    Planner pl(g, plan, msg);
    return pl.run();
}

std::string describe_plan(const Plan &p)
{
    std::ostringstream o;
    o << "{\"workspace_bytes\": " << p.workspace_bytes << ", \"steps\": [";
    for (size_t i = 0; i < p.steps.size(); ++i) {
        const Step &s = p.steps[i];
        o << (i ? ", " : "") << "{\"name\": \"" << s.name << "\", \"kernel\": \"" << s.kernel << "\", \"group\": " << s.group
          << ", \"flops\": " << (long long)s.flops << ", \"bytes\": " << (long long)s.bytes;
        if (s.kind == S_IGEMM)
            o << ", \"M\": " << s.ig.M << ", \"N\": " << s.ig.N << ", \"K\": " << s.ig.K << ", \"epilogue_ops\": " << s.ig.epi.n_ops
              << ", \"k_split_waves\": " << (s.il.run == 2 ? 1 : 0) << ", \"channel_tile_major\": " << s.ig.nmajor << ", \"k_split_workgroups\": " << (s.il.splits > 1 ? s.il.splits : 1);
        if (s.kind == S_ELTWISE) o << ", \"n\": " << (long long)s.el.n << ", \"chain_ops\": " << s.el.epi.n_ops;
        o << "}";
    }
    // workspace buffers with the steps between which each one holds live data (first writer .. last reader)
    o << "], \"buffers\": [";
    bool firstb = true;
    for (size_t i = 0; i < p.bufs.size(); ++i) {
        const BufDesc &d = p.bufs[i];
        if (d.bound_value >= 0 || d.first < 0) continue;
        o << (firstb ? "" : ", ") << "{\"offset\": " << d.offset << ", \"bytes\": " << d.bytes << ", \"first\": " << d.first << ", \"last\": " << d.last
          << "}";
        firstb = false;
    }
    o << "], \"packed_params\": [";
    bool firstp = true;
    for (auto &kv : p.packs) {
        o << (firstp ? "" : ", ") << "{\"value\": " << kv.first << ", \"bytes\": " << kv.second.bytes << "}";
        firstp = false;
    }
    o << "]}";
    return o.str();
}

void finalize_epilogue(Epilogue &e)
{
    int s = 0;
    e.has_bias = 0; e.t_op = -1; e.bias_ptr = nullptr; e.t_ptr = nullptr; e.bias_dtype = 0; e.t_dtype = 0;
    if (s < e.n_ops && epi_host_op(e, s) == E_BIAS) {
        const int a = epi_host_arg(e, s);
        e.has_bias = 1; e.bias_ptr = e.ptr[a]; e.bias_dtype = epi_host_dtype(e, a); ++s;
    }
    if (s < e.n_ops && epi_host_op(e, s) >= E_ADD && epi_host_op(e, s) <= E_RDIV) {
        const int a = epi_host_arg(e, s);
        e.t_op = epi_host_op(e, s); e.t_ptr = e.ptr[a]; e.t_dtype = epi_host_dtype(e, a); ++s;
    }
    e.simple = 1;
    e.rest_n = 0;
    e.rest_ops = 0;
    for (; s < e.n_ops; ++s) {
        const int op = epi_host_op(e, s);
        if (op <= E_RDIV || e.rest_n >= 8) { e.simple = 0; break; }      // E_BIAS .. E_RDIV take operands
        e.rest_ops |= (uint64_t)op << (8 * e.rest_n);
        e.rest_n++;
    }
    e.relu_last = (e.simple && e.rest_n == 1 && e.rest_ops == (uint64_t)E_RELU) ? 1 : 0;
}

void make_fast_div(uint32_t d, uint32_t &mul, uint32_t &sh)
{
    mul = 0; sh = 0;
    if (d < 2) return;
    uint32_t l = 0;
    while (((uint64_t)1 << l) < d) ++l;                  // ceil(log2 d) >= 1
    const uint64_t pw = (uint64_t)1 << (31 + l);         // 2^31 <= pw / d < 2^32; exact quotients for n < 2^31
    mul = (uint32_t)((pw + d - 1) / d);
    sh = l - 1;
}

rl_status run_steps(const Plan &plan, void *const *ptrs, hipStream_t stream, std::string &msg, hipEvent_t *events)
{
    size_t si = 0;
    auto P = [&](const Step &s, int slot) -> void * { return s.slot[slot] >= 0 ? ptrs[s.slot[slot]] : nullptr; };
    for (const Step &s : plan.steps) {
        hipError_t er = hipSuccess;
        if (events) er = hipEventRecord(events[si], stream);
        ++si;
        if (er == hipSuccess) switch (s.kind) {
        case S_IGEMM: {
            if (s.pair == 2 || s.chain == 2) break; // went out with the step before
            auto params = [&](const Step &t) {
                IgemmParams p = t.ig;
                p.x = P(t, SL_X); p.x2 = P(t, SL_X2); p.w = P(t, SL_W); p.y = P(t, SL_Y);
                for (int i = 0; i < RL_EPI_MAX_PTRS; ++i) p.epi.ptr[i] = P(t, SL_E0 + i);
                finalize_epilogue(p.epi);
                p.c_in = (const float *)P(t, SL_CIN); p.c_out = (float *)P(t, SL_COUT); p.h_out = P(t, SL_HOUT);
                p.partial = (float *)P(t, SL_PART);
                return p;
            };
            if (s.chain == 1) {
                const Step &t = plan.steps[si];     // si already counts this step: the next one
                IgemmParams pa = params(s), pb = params(t);
                pa.skip_reduce = 1;
                er = launch_igemm(pa, s.il, stream);
                if (er == hipSuccess) {
                    ReduceDenseParams r{};
                    r.partial = pa.partial; r.splits = pa.splits; r.M = pa.M; r.N1 = pa.N;
                    r.epi1 = pa.epi; r.hs_n = pa.ys_n; r.hs_c = pa.ys_c; r.h_dtype = pa.y_dtype;
                    r.w2 = pb.w; r.w_dtype = pb.in_dtype; r.N2 = pb.N; r.Kp2 = pb.Kp;
                    r.epi2 = pb.epi; r.y = pb.y; r.y_dtype = pb.y_dtype; r.ys_n = pb.ys_n; r.ys_c = pb.ys_c;
                    er = launch_reduce_dense(r, stream);
                }
            } else if (s.pair == 1) {
                const Step &t = plan.steps[si];     // si already counts this step: the next one
                er = s.il.s2pair ? launch_conv3x3s2_pair(params(s), s.il, params(t), t.il, stream)
                                 : launch_igemm_lp_pair(params(s), s.il, params(t), t.il, stream);
            } else {
                er = launch_igemm(params(s), s.il, stream);
            }
            break;
        }
        case S_ELTWISE: {
            EltwiseParams p = s.el;
            p.x = P(s, SL_X); p.y = P(s, SL_Y);
            for (int i = 0; i < RL_EPI_MAX_PTRS; ++i) p.epi.ptr[i] = P(s, SL_E0 + i);
            finalize_epilogue(p.epi);
            er = launch_eltwise(p, stream);
            break;
        }
        case S_GATES: {
            GatesParams p = s.ga;
            p.z = (const float *)P(s, SL_X); p.c_in = (const float *)P(s, SL_CIN); p.c_out = (float *)P(s, SL_COUT); p.h_out = P(s, SL_HOUT);
            er = launch_lstm_gates(p, stream);
            break;
        }
        case S_MAXPOOL: case S_GAVG: {
            PoolParams p = s.po;
            p.x = P(s, SL_X); p.y = P(s, SL_Y);
            er = s.kind == S_MAXPOOL ? launch_maxpool_nhwc(p, stream) : launch_gavgpool_nhwc(p, stream);
            break;
        }
        case S_TO_NHWC:
            er = launch_nchw_to_nhwc(P(s, SL_X), P(s, SL_Y), s.t_dtype, s.t_N, s.t_C, s.t_P, stream);
            break;
        case S_TO_NCHW:
            er = launch_nhwc_to_nchw(P(s, SL_X), P(s, SL_Y), s.t_dtype, s.t_N, s.t_C, s.t_P, stream);
            break;
        case S_STEM_POOL: {
            if (s.stem_direct) {
                StemDirectParams q{};
                q.x = P(s, SL_X); q.w = P(s, SL_W);
                q.x_bytes = (uint32_t)((uint64_t)s.t_N * s.t_C * s.st_H * s.st_W * 2);
                q.w_bytes = (uint32_t)(64 * STEM_DIRECT_KP * 2);
                q.epi = s.ig.epi;
                for (int i = 0; i < RL_EPI_MAX_PTRS; ++i) q.epi.ptr[i] = P(s, SL_E0 + i);
                finalize_epilogue(q.epi);
                q.yp = P(s, SL_Y);
                q.yp_bytes = (uint32_t)((uint64_t)s.sp_N * s.sp_PH * s.sp_PW * 64 * 2);
                q.n_img = s.sp_N; q.C = s.t_C; q.H = s.st_H; q.W = s.st_W; q.KH = s.stem_kh; q.KW = s.stem_kw; q.ph = s.st_ph; q.pw = s.st_pw;
                q.OH = s.ig.OH; q.OW = s.ig.OW; q.PH = s.sp_PH; q.PW = s.sp_PW;
                er = launch_stem_pool_direct(q, stream);
                break;
            }
            StemPoolParams q{};
            q.g = s.ig;
            q.g.x = P(s, SL_X); q.g.w = P(s, SL_W); q.g.y = nullptr;
            for (int i = 0; i < RL_EPI_MAX_PTRS; ++i) q.g.epi.ptr[i] = P(s, SL_E0 + i);
            finalize_epilogue(q.g.epi);
            q.yp = P(s, SL_Y);
            q.n_img = s.sp_N; q.PH = s.sp_PH; q.PW = s.sp_PW;
            q.kh = s.stem_kh;
            q.yp_bytes = (uint32_t)((uint64_t)s.sp_N * s.sp_PH * s.sp_PW * 64 * 2);
            er = launch_stem_pool(q, stream);
            break;
        }
        case S_PERMUTE: {
            PermuteParams p = s.pe;
            p.x = P(s, SL_X); p.y = P(s, SL_Y);
            er = launch_permute(p, stream);
            break;
        }
        case S_PACK:
            er = launch_pack_gather(P(s, SL_X), P(s, SL_Y), s.gp, stream);
            break;
        case S_WGRAD: {
            WgradParams q = s.wg;
            q.xT = P(s, SL_X); q.dyT = P(s, SL_X2); q.part = (float *)P(s, SL_PART);
            q.dy_bytes = (uint32_t)((uint64_t)q.OH * q.OW * q.O * 64 * q.nck * 2);
            q.x_bytes = (uint32_t)((uint64_t)q.H * q.W * q.C * 64 * q.nck * 2);
            er = launch_conv_wgrad(q, stream);
            break;
        }
        case S_DILATE:
            er = launch_dilate_nhwc(P(s, SL_X), P(s, SL_Y), s.t_N, s.st_H, s.st_W, s.st_Hp, s.st_Wp, s.t_C, s.st_ph, stream);
            break;
        case S_WGRAD_REDUCE:
            er = launch_wgrad_reduce((const float *)P(s, SL_X), P(s, SL_Y), s.t_dtype, s.t_N, s.t_C, s.wg.O, s.wg.C, stream);
            break;
        case S_STEM_PAD:
            er = launch_stem_pad(P(s, SL_X), P(s, SL_Y), s.t_N, s.t_C, s.st_H, s.st_W, s.st_Hp, s.st_Wp, s.st_ph, s.st_pw, stream);
            break;
        }
        if (er != hipSuccess) {
            msg = "launch of " + s.kernel + " (" + s.name + ") failed: " + hipGetErrorString(er);
            return RL_ERR_HIP;
        }
    }
    if (events && hipEventRecord(events[si], stream) != hipSuccess) { msg = "hipEventRecord failed"; return RL_ERR_HIP; }
    return RL_OK;
}

}  // namespace rl
