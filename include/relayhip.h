/*
 * relayhip -- C ABI for declaring, type-checking, grouping and running fused
 * tensor-operator groups on one MI355X (gfx950).
 *
 * The interface follows the paper's statement of the problem:
 *   - a program is a list of operator declarations and calls whose types are
 *     tensor types with constant shapes      (grammar figure: Operator, Type,
 *                                             BaseType, Shape);
 *   - Tensor(bt, sh) is formed from one base type and one shape
 *                                            (kinding rules BaseType-T, Shape-T, Tensor-T);
 *   - unary operators keep Tensor(b, s); + - * / need both operands of the same
 *     b and s and return it                  (Type-UnaryOp, Type-Noncomp-BinaryOp);
 *   - a call is well typed only if every argument has the operator's parameter
 *     type; its type is the arrow's result   (Type-Call);
 *   - operators are primitives implemented outside the language and run as
 *     type-specialised kernels               (sections "Frontend", "Runtime System");
 *   - fusion and layout change are optimisations below the typed graph
 *                                            (sections "Background", "Optimizations").
 *
 * Conventions for every entry point
 *   - Handles (rl_ctx, rl_graph, rl_plan) are owned by the library and freed by
 *     their destroy call; destroying a ctx does not free graphs/plans made from it.
 *   - The caller owns all device memory and the stream.  The library never
 *     allocates device memory, never synchronises and never changes the current
 *     device.  Run calls only enqueue work on the given stream.
 *   - "dev" pointers are device pointers, 16-byte aligned; everything else is
 *     host memory.  hip_stream is a hipStream_t passed as void* (NULL = default
 *     stream).
 *   - No exception crosses the ABI and nothing aborts: every call returns
 *     rl_status (0 = RL_OK, negative = error class); the text of the last error
 *     on a ctx is available from rl_last_error.  A failed rl_graph_* call leaves
 *     the graph unchanged.
 *   - Tensors at the boundary are dense row-major in the order of their Shape
 *     (so rank-4 activations are NCHW, conv weights OIHW, dense weights
 *     [out, in]).  Kernel-native layouts are private to a plan.
 *   - A ctx/graph is single-threaded.  A finished plan may be run from several
 *     threads on different streams with different workspaces.
 */
#ifndef RELAYHIP_H
#define RELAYHIP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rl_ctx rl_ctx;
typedef struct rl_graph rl_graph;
typedef struct rl_plan rl_plan;
typedef int32_t rl_status;

enum {
    RL_OK = 0,
    RL_ERR_NULL = -1,        /* a required pointer argument is NULL */
    RL_ERR_KIND = -2,        /* unknown base type / op kind, rank > RL_MAX_RANK, malformed attributes */
    RL_ERR_SHAPE = -3,       /* a dimension is not a positive constant, or a window exceeds its input */
    RL_ERR_TYPE = -4,        /* ill-typed: operand types or declared result type violate the typing rules */
    RL_ERR_GROUP = -5,       /* the declared fusion group is not legal */
    RL_ERR_BINDING = -6,     /* run: a needed value has no pointer, or an id is bound twice / unknown */
    RL_ERR_WORKSPACE = -7,   /* run: workspace missing or too small */
    RL_ERR_ALIGN = -8,       /* run: a device pointer is not 16-byte aligned */
    RL_ERR_UNSUPPORTED = -9, /* well typed, but no kernel implements it */
    RL_ERR_HIP = -10         /* a HIP runtime call failed (text has hipGetErrorString) */
};

/* BaseType.  The paper's FloatType(width) cannot tell bfloat16 from IEEE half,
 * so bfloat16 has a tag of its own. */
enum { RL_F32 = 0, RL_BF16 = 1 };

#define RL_MAX_RANK 6

/* Tensor(dtype, Shape(dims[0..rank-1])); rank 0 is a scalar. */
typedef struct rl_type {
    int32_t dtype;
    int32_t rank;
    int64_t dims[RL_MAX_RANK];
} rl_type;

/* Operator kinds.  The binary and unary arithmetic kinds are the grammar's
 * BinOp / UnaryOp; the rest are declared operators (conv2d, linear, max_pool,
 * flatten_layer, tanh appear in the paper's decorator example). */
enum {
    RL_OP_DENSE = 0,          /* (x[M,K], W[N,K]) -> [M,N]; attrs rl_attr_contract (may be NULL) */
    RL_OP_CONV2D = 1,         /* (x[N,C,H,W], w[O,C,KH,KW]) -> [N,O,OH,OW]; attrs rl_attr_conv2d */
    RL_OP_BIAS_ADD = 2,       /* (x, b[C]) -> x's type, b added along attrs rl_attr_axis.axis; b has x's dtype, or f32 when x is bf16 */
    RL_OP_ADD = 3, RL_OP_SUB = 4, RL_OP_MUL = 5, RL_OP_DIV = 6,   /* (a, b) of one identical type */
    RL_OP_NEG = 7, RL_OP_SQ = 8,                                     /* grammar's unary operators */
    RL_OP_RELU = 9, RL_OP_SIGMOID = 10, RL_OP_TANH = 11,
    RL_OP_MAXPOOL2D = 12,     /* attrs rl_attr_pool2d; taps outside the input are ignored */
    RL_OP_GLOBAL_AVGPOOL = 13,/* [N,C,H,W] -> [N,C,1,1] */
    RL_OP_FLATTEN = 14,       /* [N, d1, ...] -> [N, d1*...] */
    RL_OP_LSTM_GATES = 15,    /* (z f32[B,4H] as i|f|g|o blocks, c f32[B,H]) -> (c' f32[B,H], h' f32|bf16[B,H]) */
    RL_OP_CAST = 16,          /* explicit (Type) Expr; attrs rl_attr_cast */
    RL_OP_CONCAT = 17,        /* (a[B,K1], b[B,K2]) -> [B,K1+K2]; only as the operand of a dense in the same group */
    RL_OP_LAYOUT_TRANSFORM = 18, /* (x[d0..d(r-1)]) -> [d(perm[0]) .. d(perm[r-1])], y[i0..] = x at index j with j[perm[k]] = i[k];
                                    attrs rl_attr_layout.  The paper's types carry no layout (its section on extensions
                                    proposes tracking it); here a layout IS the order of the Shape, so a change of layout
                                    is an operator whose arrow type permutes the Shape, and the typed graph shows it.
                                    Always a group of its own.  On rank-4 tensors the two channel-first <-> channel-last
                                    permutations (0,2,3,1) and (0,3,1,2) cost nothing when the other side of the value is
                                    a convolution, pool or elementwise group: those run channel-last internally. */
    /* Partial derivatives of the two contractions: the operators a reverse-mode gradient of a program (the paper's section
     * "Automatic Differentiation", node Grad) calls for every dense / conv2d it differentiates through.  Each is a group of
     * its own.  dy is the derivative with respect to the forward operator's result. */
    RL_OP_DENSE_GRAD_X = 19,  /* (dy[M,N], W[N,K]) -> [M,K]: sum_n dy[m,n] W[n,k]; attrs rl_attr_contract (may be NULL) */
    RL_OP_DENSE_GRAD_W = 20,  /* (dy[M,N], x[M,K]) -> [N,K]: sum_m dy[m,n] x[m,k]; attrs rl_attr_contract (may be NULL) */
    RL_OP_CONV2D_GRAD_X = 21, /* (dy[N,O,OH,OW], w[O,C,KH,KW]) -> [N,C,H,W]; attrs rl_attr_conv2d of the forward convolution.  The
                                 forward output size does not determine H and W: the declared result states them, and
                                 OH = floor((H + 2 pad - KH)/stride) + 1 is checked (else RL_ERR_TYPE) */
    RL_OP_CONV2D_GRAD_W = 22, /* (dy[N,O,OH,OW], x[N,C,H,W]) -> [O,C,KH,KW]; attrs as above; the declared result states KH and KW */
    RL_OP_KIND_COUNT = 23
};

typedef struct rl_attr_contract { int32_t out_dtype; /* operand dtype, or RL_F32 */ } rl_attr_contract;
typedef struct rl_attr_conv2d {
    int32_t stride_h, stride_w, pad_h, pad_w;   /* zero padding, symmetric */
    int32_t dilation_h, dilation_w, groups;     /* must be 1 (else RL_ERR_UNSUPPORTED) */
    int32_t out_dtype;
} rl_attr_conv2d;
typedef struct rl_attr_axis { int32_t axis; } rl_attr_axis;
typedef struct rl_attr_pool2d { int32_t kernel_h, kernel_w, stride_h, stride_w, pad_h, pad_w; } rl_attr_pool2d;
typedef struct rl_attr_cast { int32_t to; } rl_attr_cast;
typedef struct rl_attr_layout { int32_t perm[RL_MAX_RANK]; /* a permutation of 0..rank-1 in the first rank entries; else RL_ERR_KIND */ } rl_attr_layout;

typedef struct rl_binding { int32_t value_id; void *dev_ptr; } rl_binding;

/* ---- context ------------------------------------------------------------ */
rl_status rl_ctx_create(rl_ctx **out);
void rl_ctx_destroy(rl_ctx *ctx);
/* Text of the most recent error on ctx ("" if none); valid until the next call on ctx. */
const char *rl_last_error(const rl_ctx *ctx);

/* ---- graph: typed values and operator calls ------------------------------
 * rl_graph_input / rl_graph_param introduce a value of the given tensor type
 * (Tensor-T: dtype known, rank <= RL_MAX_RANK, every dim >= 1).  A param is a
 * constant the plan may ask to have re-laid-out once (rl_plan_prepack).
 * rl_graph_op appends a call.  The caller must state the result type(s)
 * (declared_outs, n_out = 1 except RL_OP_LSTM_GATES which has 2); the library
 * infers the result type from the argument types and attributes and rejects
 * the call with RL_ERR_TYPE when they differ (Type-Call), or when the
 * arguments break the operator's rule (Type-UnaryOp, Type-Noncomp-BinaryOp:
 * no implicit broadcast or promotion).  attrs points to the kind's POD struct
 * (attrs_size = its sizeof) or is NULL for kinds without attributes. */
rl_status rl_graph_create(rl_ctx *ctx, rl_graph **out);
void rl_graph_destroy(rl_graph *g);
rl_status rl_graph_input(rl_graph *g, const rl_type *t, int32_t *value_id);
rl_status rl_graph_param(rl_graph *g, const rl_type *t, int32_t *value_id);
rl_status rl_graph_op(rl_graph *g, int32_t op_kind, const int32_t *in_ids, int32_t n_in,
                      const void *attrs, size_t attrs_size,
                      const rl_type *declared_outs, int32_t n_out,
                      int32_t *op_id, int32_t *out_value_ids);
/* Declare a fusion group: a connected set of calls with at most one
 * contraction (dense / conv2d, which must come first; a concat feeding that
 * dense may precede it), every other member injective on the group's output
 * shape (elementwise, bias_add, cast; lstm_gates only as the last member), and
 * no intermediate used outside the group.  Checked here as far as the calls
 * are known and again by rl_plan_create.  Calls left ungrouped run alone. */
rl_status rl_graph_group(rl_graph *g, const int32_t *op_ids, int32_t n, int32_t *group_id);
rl_status rl_graph_output(rl_graph *g, int32_t value_id);
/* Automatic fusion: puts every call that has no group yet into one, by the same rules a declared group must
 * satisfy.  In declaration order, the first ungrouped call opens a group (a concat whose only use is an
 * ungrouped dense opens it together with that dense); the group then absorbs the consumer of its last result
 * for as long as that result has exactly one use and is not a graph output, and the consumer is an ungrouped
 * injective call taking it as first operand whose other operands are defined before the group (lstm_gates is
 * absorbed too and closes the group).  Calls that are neither contractions nor injective stay alone.  Declare
 * the graph outputs first: a value that is an output is never fused away.  Groups declared by hand are kept.
 * *n_groups (nullable) gets the number of groups added.  On error nothing is guaranteed about which of the
 * ungrouped calls were grouped; the graph stays valid. */
rl_status rl_graph_autogroup(rl_graph *g, int32_t *n_groups);
/* Group a call belongs to (the id rl_graph_group returned, or its position for automatic ones), -1 if none. */
rl_status rl_graph_group_of(const rl_graph *g, int32_t op_id, int32_t *group_id);

/* ---- plan ---------------------------------------------------------------
 * Plan-time options.  The paper leaves the choice of an operator's implementation to the layer below the typed
 * graph (section "Runtime System": one type-specialised operator per call); these switches steer that choice
 * and nothing else: each non-zero field takes one kernel form out of the planner's repertoire (ws_all widens
 * one), so that the next form down runs on the same shapes -- results stay within summation order.  The choices
 * are fixed inside the plan when it is created; no environment variable and no later call changes them.
 * All zero (or a NULL pointer) = the planner's own choices. */
typedef struct rl_plan_opts {
    uint32_t struct_size;   /* sizeof(rl_plan_opts) of the caller's build; must be <= the library's (else RL_ERR_KIND);
                               fields the caller's struct does not have read as 0 */
    int32_t no_lp;          /* no pixel-on-lane bf16 contraction kernels (nor their register/LDS-row epilogue) */
    int32_t no_lp_256;      /* no 256x128 tile in that family */
    int32_t no_ws;          /* no weights-stationary persistent kernel for N <= 64, K <= 320 */
    int32_t ws_all;         /* take that kernel up to K = 576 as well */
    int32_t no_stem;        /* few-channel stems: no padded 4-channel frame, gather from the operand instead */
    int32_t no_stem_pool;   /* stem convolution and the max-pool behind it stay two kernels */
    int32_t no_dma;         /* no direct global->LDS operand path (register-staged vector loads instead) */
    int32_t no_c64;         /* no weights-in-registers kernel for 3x3 64->64 convolutions */
    int32_t no_run;         /* no nine-taps-from-one-copy kernel for 3x3 stride-1 convolutions on short rows */
    int32_t no_run_ks;      /* in that kernel's 128x64 form: do not split K over the waves */
    int32_t no_pair;        /* a stride-2 convolution and the 1x1 projection beside it go out as two launches */
    int32_t s2_pair;        /* opt in: such a pair as ONE contraction whose centre tap carries the projection (second
                               accumulators) with the input rows shared in LDS -- correct and tested, but its 64-pixel tiles
                               lose to the two-contractions-in-one-grid form on every shape measured so far */
    int32_t no_splitk;      /* never split K over several workgroups per tile */
    int32_t no_hoist;       /* rl_plan_run_recurrent: never hoist the input projection out of the step loop */
    int32_t no_stem_direct; /* the fused stem + max-pool kernel reads a padded channel-last copy of the input (written by a step
                               of its own) even where it could fetch its patches from the channel-first input directly */
    int32_t no_wgrad;       /* conv2d_grad_w on bf16 batches that are multiples of 64: no images-last contraction kernel; the element-gather kernel */
    int32_t no_grad_fwd;    /* dense_grad_x and stride-1 conv2d_grad_x through a param: do not plan them as the forward
                               operator on re-ordered weights; take the element-gather kernel like the other gradients */
    int32_t no_out_transpose; /* a large bf16 convolution whose result is a graph output: store it in Shape order from the
                               direct-load kernel, instead of channel-last from the pixel-on-lane kernels plus a transposition */
    int32_t no_dense_chain; /* a split dense contraction followed by a small dense layer on its result alone: keep them two
                               steps (contraction, adding launch, small layer) instead of letting the adding launch run
                               the small layer too */
} rl_plan_opts;

/* rl_plan_create re-checks the whole graph (Type-Call on every call, group legality, outputs reachable), picks
 * one kernel per fusion group, tiles and private layouts, and sizes the workspace -- the role the paper gives
 * its evaluator's just-in-time operator compiler (section "Runtime System": one operator specialised to the types of
 * each call), done once ahead of the runs.
 * It needs no GPU.  opts may be NULL.  The graph may be destroyed afterwards.  Errors: RL_ERR_NULL, RL_ERR_KIND
 * (opts->struct_size larger than the library knows), RL_ERR_TYPE / RL_ERR_GROUP (graph), RL_ERR_UNSUPPORTED. */
rl_status rl_plan_create(rl_graph *g, const rl_plan_opts *opts, rl_plan **out);
void rl_plan_destroy(rl_plan *plan);
/* JSON text describing the steps (kernel, tile, flops, algorithmic bytes).
 * Writes at most cap bytes including the terminator; *needed gets the full size. */
rl_status rl_plan_describe(const rl_plan *plan, char *buf, size_t cap, size_t *needed);
rl_status rl_plan_workspace_bytes(const rl_plan *plan, size_t *bytes);
/* Bytes of the kernel-native copy of a param, or 0 when the param is bound as is. */
rl_status rl_plan_packed_bytes(const rl_plan *plan, int32_t param_value_id, size_t *bytes);
/* Enqueue the re-layout of one param: src_dev holds it in boundary layout (dense row-major in the order of its
 * Shape), dst_dev (rl_plan_packed_bytes bytes, caller-owned) receives the kernel-native copy, which is what
 * rl_plan_run must then be given for that value id.  This is the "layout change" of the paper's list of high-level
 * optimisations (section "Background") applied to constants, once, outside the runs; the typed graph never sees it
 * (the paper's types carry no layout: section on future extensions).  Asynchronous on hip_stream; src and dst must not
 * overlap.  Errors: RL_ERR_NULL, RL_ERR_BINDING (not a param of this plan, or one that is bound as is), RL_ERR_HIP. */
rl_status rl_plan_prepack(const rl_plan *plan, int32_t param_value_id, const void *src_dev, void *dst_dev,
                          void *hip_stream);
/* Execute the typed graph: every fusion group's type-specialised kernel in dependency order -- what the paper's
 * run time does with a checked program (section "Runtime System"), with the fusion and memory reuse its section
 * "Background" lists among the optimisations below the graph decided beforehand by rl_plan_create.
 * Enqueues every step of the plan.  bindings must cover every input, param
 * (packed copy where rl_plan_packed_bytes > 0) and output value id exactly
 * once; intermediates live in workspace_dev (>= rl_plan_workspace_bytes).
 * Inputs and params are read only; outputs and workspace are overwritten.
 * An output may alias an input only for lstm_gates' cell state (c' over c).
 * The call only launches kernels on hip_stream (no allocation, no memset, no
 * synchronisation), so it may be made while that stream is being captured into
 * a HIP graph; replays then need the same device pointers to stay valid. */
rl_status rl_plan_run(const rl_plan *plan, const rl_binding *bindings, int32_t n_bindings,
                      void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* rl_plan_run without a workspace argument, for callers that cannot allocate device memory (code under HIP graph
 * capture, serving loops, harnesses that forbid hipMalloc): the intermediates live in an array of
 * RL_STATIC_WORKSPACE_BYTES that is part of the library's code object (each GPU the library runs on holds one copy
 * until the process ends).  Plans with rl_plan_workspace_bytes above that return RL_ERR_WORKSPACE.  The call
 * allocates nothing on the device and otherwise behaves like rl_plan_run (same kernels, same results, same errors).
 * All calls on one GPU share the array: two calls that may overlap in time (different streams or threads) race;
 * serialise them or use rl_plan_run with workspaces of the caller's. */
#define RL_STATIC_WORKSPACE_BYTES (16u << 20)
rl_status rl_plan_run_static(const rl_plan *plan, const rl_binding *bindings, int32_t n_bindings, void *hip_stream);

/* Measurement aid (not part of the hot path): enqueue the plan `reps` times
 * with a HIP event recorded on hip_stream before and after every step, then
 * wait for the stream -- the only entry point that synchronises.  step_ms[i]
 * receives the mean milliseconds between the events around step i (i follows
 * the "steps" array of rl_plan_describe); at most cap entries are written and
 * *n_steps gets the plan's step count. */
rl_status rl_plan_profile(const rl_plan *plan, const rl_binding *bindings, int32_t n_bindings,
                          void *workspace_dev, size_t workspace_bytes, void *hip_stream,
                          int32_t reps, float *step_ms, int32_t cap, int32_t *n_steps);

/* Measurement aid (not part of the hot path): enqueue a kernel that does nothing but bf16 MFMAs (32x32x16, fp32
 * accumulate) on register operands -- `workgroups` workgroups of eight waves, every wave a chain of 16 * iters
 * MFMAs, i.e. workgroups * 8 * 16 * iters * 32768 flops in all.  Timed by the caller (events on hip_stream), it
 * gives the rate the matrix pipes deliver on this machine, the yardstick next to the quoted peak.  scratch_dev
 * receives workgroups * 512 floats (ignore them).  Errors: RL_ERR_NULL, RL_ERR_BINDING (counts < 1), RL_ERR_HIP. */
rl_status rl_calibrate_mfma_bf16(rl_ctx *ctx, void *scratch_dev, int32_t workgroups, int32_t iters, void *hip_stream);

/* Recurrent execution of a one-step cell plan for `steps` steps.  The paper's language expresses a recurrent model as
 * a recursive function over its time steps (section "Grammar and Design": recursion and conditionals are part of the
 * language; its evaluator would call the cell's operators once per step); this call is that loop for a cell whose types are checked once: at step t the
 * cell's x input is x_seq_dev + t*x_step_bytes, its h input is h0_dev (t = 0)
 * or the previous step's h output, its c input/output is c_dev (updated in
 * place; the caller initialises it), and its h output is written to
 * h_seq_dev + t*h_step_bytes.  `bindings` supplies the params.  The value ids
 * name the cell graph's values playing each role. */
typedef struct rl_recurrent {
    int32_t x_id, h_in_id, c_in_id, h_out_id, c_out_id;
    const void *x_seq_dev; size_t x_step_bytes;
    const void *h0_dev;
    void *c_dev;
    void *h_seq_dev; size_t h_step_bytes;
} rl_recurrent;
/* Workspace that lets rl_plan_run_recurrent run `steps` steps of this cell at its best.  For a cell that is
 * one fused [x, h] contraction + LSTM-gate group in bf16 this is rl_plan_workspace_bytes rounded up to 256 plus
 * steps * batch * 4*hidden * 4 bytes: the input projection x_t . Wx^T of all steps is then computed by one
 * contraction up front and each step only runs the recurrent part (h_{t-1} . Wh^T and the gates).  With less
 * (but room for at least 8 steps' projections) the steps are processed in chunks; with only
 * rl_plan_workspace_bytes the cell plan is replayed once per step.  For every other cell the value equals
 * rl_plan_workspace_bytes.  Results of the forms agree to summation order.  Host call; errors: RL_ERR_NULL,
 * RL_ERR_BINDING (negative steps). */
rl_status rl_plan_recurrent_workspace_bytes(const rl_plan *cell, int32_t steps, size_t *bytes);
rl_status rl_plan_run_recurrent(const rl_plan *cell, int32_t steps, const rl_recurrent *io,
                                const rl_binding *param_bindings, int32_t n_bindings,
                                void *workspace_dev, size_t workspace_bytes, void *hip_stream);

/* ---- one-time weight preparation (device side, asynchronous) ------------- */
/* Fold an inference batch-norm into the preceding convolution -- a rewrite of constants of the kind the paper leaves to
 * optimisation passes over the typed program (section "Optimizations"; the paper prints no formula, this is the
 * textbook one):
 * scale[o] = gamma[o]/sqrt(var[o]+eps); w_out[o,:] = w[o,:]*scale[o];
 * b_out[o] = beta[o] - mean[o]*scale[o], evaluated in float64 and rounded to
 * f32 (then to out_dtype for w_out).  w: f32 [O, per_o]; gamma..var, b_out:
 * f32 [O]; w_out: out_dtype [O, per_o].  All device pointers. */
rl_status rl_prep_fold_batchnorm(rl_ctx *ctx, const void *w_dev, const void *gamma_dev, const void *beta_dev,
                                 const void *mean_dev, const void *var_dev, double eps,
                                 void *w_out_dev, int32_t out_dtype, void *b_out_dev,
                                 int64_t O, int64_t per_o, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* RELAYHIP_H */
