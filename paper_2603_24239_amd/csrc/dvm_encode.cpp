// The host side of libdvm: program builder, bytecode encoder, stacker, validator, disassembler.
//
// Everything in this file runs on the CPU and makes no HIP call.  dvm_encode does, in order
// (Section 4.2 of the paper unless noted):
//   1. shape inference with broadcasting, dominant shape S_d ("Shape tiling", first step);
//   2. pattern fusion check: all ops must share one iteration space so that they become one
//      meta-kernel whose intermediates stay in registers (Section 5.1);
//   3. collapsing of the iteration space to rows x columns and per-tensor strides (the worked
//      example tiles the flattened 32768 elements of a [32,1024] tensor);
//   4. linearisation of the op DAG into accumulator-machine code with liveness-driven tile
//      register allocation (Algorithm 1's n_max: the peak number of live tiles);
//   5. the tile plan: interpreter variant K (T_max = register budget / n_max), lanes per row,
//      rows or columns per tile chosen by the cost model ceil(#tiles/N) * (tile + c);
//   6. emission of header + body, every unused bit zero.
// No heap allocation happens in dvm_encode: all scratch lives on the stack.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "../../include/dvm.h"
#include "dvm_bytecode.h"
#include "dvm_internal.h"

using namespace dvmbc;

// ------------------------------------------------------------------------------------------------
// errors
// ------------------------------------------------------------------------------------------------
namespace {
thread_local char t_detail[256] = "";
}

extern "C" int dvm_set_error(int status, const char *detail) {
    if (detail) {
        strncpy(t_detail, detail, sizeof(t_detail) - 1);
        t_detail[sizeof(t_detail) - 1] = 0;
    } else {
        t_detail[0] = 0;
    }
    return status;
}
extern "C" const char *dvm_last_error_detail(void) { return t_detail; }

extern "C" const char *dvm_strerror(int status) {
    switch (status) {
        case DVM_OK: return "ok";
        case DVM_E_ARGS: return "bad argument";
        case DVM_E_SHAPE: return "shapes do not broadcast";
        case DVM_E_RANK: return "rank not supported";
        case DVM_E_DTYPE: return "unknown dtype";
        case DVM_E_UNSUPPORTED: return "program not supported by the VM";
        case DVM_E_BUFSZ: return "buffer too small";
        case DVM_E_BADCODE: return "malformed bytecode";
        case DVM_E_HIP: return "HIP error";
        case DVM_E_ALIGN: return "tensor pointer misaligned";
        case DVM_E_LIMIT: return "program exceeds a size limit";
        case DVM_E_STATE: return "wrong program state";
        default: return "unknown status";
    }
}

extern "C" int dvm_shape_contiguous(dvm_shape *s, int rank, const int64_t *dims) {
    if (!s || rank < 0 || rank > DVM_MAX_RANK || (rank > 0 && !dims)) return dvm_set_error(DVM_E_ARGS, "dvm_shape_contiguous");
    memset(s, 0, sizeof(*s));
    s->rank = rank;
    int64_t st = 1;
    for (int i = rank - 1; i >= 0; --i) {
        if (dims[i] < 0) return dvm_set_error(DVM_E_SHAPE, "negative dimension");
        s->dim[i] = dims[i];
        s->stride[i] = st;
        st *= dims[i] > 0 ? dims[i] : 1;
    }
    return DVM_OK;
}

// ------------------------------------------------------------------------------------------------
// context
// ------------------------------------------------------------------------------------------------
constexpr int NR_LIMIT = 6;      // tile registers of the largest interpreter variant

struct dvm_ctx {
    int device;
    int n_cu;
    int overhead;   // per-tile overhead of the cost model, in elements
    int max_k;      // largest elements-per-lane the planner may choose
    int max_nr;     // most tile registers a program may use
    // plan overrides (dvm_ctx_set_plan_override): tests and tuning walk plans the cost model would not pick
    int dbg_k;      // preferred elements per lane (0 = planner's choice)
    int dbg_grid_x; // workgroups launched per resident slot (default 1)
    int dbg_rp;     // rows per tile, or waves per unit of a reduction along the penultimate axis (0 = cost model)
    int assignment; // DVM_ASSIGN_*: how the tiles of a meta-kernel are dealt out to the workgroups
    int lds_operands;   // row-invariant operands may live in LDS instead of pinned tile registers
    int lds_budget;     // bytes of LDS images per workgroup
    int64_t workspace_limit;    // bytes of workspace dvm_encode may plan for (0: programs never need one)
    int copies;                 // copies of every program that share a launch (tensor sets of a batched run): tiles count that many times in the cost model
    int64_t sync_limit;     // polls a workgroup spends at a grid-wide synchronisation point before it gives up
};

extern "C" int dvm_ctx_create(int hip_device, dvm_ctx **out) {
    if (!out) return dvm_set_error(DVM_E_ARGS, "dvm_ctx_create: null out");
    dvm_ctx *c = new (std::nothrow) dvm_ctx;
    if (!c) return dvm_set_error(DVM_E_LIMIT, "out of memory");
    c->device = hip_device;
    c->n_cu = 256;          // MI355X
    c->overhead = 512;
    c->max_k = 32;
    c->max_nr = NR_LIMIT;
    c->dbg_k = 0;
    c->dbg_grid_x = 1;
    c->dbg_rp = 0;
    c->assignment = DVM_ASSIGN_AUTO;
    c->lds_operands = 1;
    c->workspace_limit = 0;
    c->copies = 1;
    c->lds_budget = 40 * 1024 - 640;    // four workgroups per compute unit keep their images in its 160 KiB
    c->sync_limit = 1 << 20;
    if (hip_device >= 0) {
        int n = 0;
        int st = dvm_ctx_query_device(hip_device, &n);
        if (st != DVM_OK) {
            delete c;
            return dvm_set_error(st, "dvm_ctx_create: device query failed");
        }
        if (n > 0) c->n_cu = n;
    } else if (hip_device != -1) {
        delete c;
        return dvm_set_error(DVM_E_ARGS, "dvm_ctx_create: device must be >= 0 or -1");
    }
    *out = c;
    return DVM_OK;
}
extern "C" void dvm_ctx_destroy(dvm_ctx *c) { delete c; }
extern "C" int dvm_ctx_device(const dvm_ctx *c) { return c ? c->device : -1; }
extern "C" void dvm_ctx_planner_get(const dvm_ctx *c, int *n_cu, int *overhead) {
    if (!c) return;
    if (n_cu) *n_cu = c->n_cu;
    if (overhead) *overhead = c->overhead;
}
extern "C" int dvm_ctx_set_limits(dvm_ctx *c, int max_k, int max_nr) {
    if (!c) return dvm_set_error(DVM_E_ARGS, "null context");
    if (max_k > 0) {
        if (max_k != 4 && max_k != 8 && max_k != 16 && max_k != 32 && max_k != 64) return dvm_set_error(DVM_E_ARGS, "elements per lane must be 4, 8, 16, 32 or 64");
        c->max_k = max_k;
    }
    if (max_nr > 0) {
        if (max_nr != 1 && max_nr != 2 && max_nr != 4 && max_nr != 6) return dvm_set_error(DVM_E_ARGS, "tile registers must be 1, 2, 4 or 6");
        c->max_nr = max_nr;
    }
    return DVM_OK;
}

extern "C" int dvm_ctx_set_plan_override(dvm_ctx *c, int elems_per_lane, int rows_per_tile, int grid_multiplier) {
    if (!c) return dvm_set_error(DVM_E_ARGS, "null context");
    if (elems_per_lane != 0 && elems_per_lane != 4 && elems_per_lane != 8 && elems_per_lane != 16 && elems_per_lane != 32 && elems_per_lane != 64)
        return dvm_set_error(DVM_E_ARGS, "elements per lane must be 0, 4, 8, 16, 32 or 64");
    if (rows_per_tile < 0 || rows_per_tile > 1024) return dvm_set_error(DVM_E_ARGS, "rows per tile must be 0 .. 1024");
    if (grid_multiplier < 0 || grid_multiplier > 64) return dvm_set_error(DVM_E_ARGS, "grid multiplier must be 0 .. 64");
    c->dbg_k = elems_per_lane;
    c->dbg_rp = rows_per_tile;
    c->dbg_grid_x = grid_multiplier > 0 ? grid_multiplier : 1;
    return DVM_OK;
}

extern "C" int dvm_ctx_set_sync_limit(dvm_ctx *c, int64_t polls) {
    if (!c || polls < 1) return dvm_set_error(DVM_E_ARGS, "dvm_ctx_set_sync_limit: null context or limit below 1");
    c->sync_limit = polls > 0x7FFFFFFF ? 0x7FFFFFFF : polls;
    return DVM_OK;
}
extern "C" int64_t dvm_ctx_sync_limit(const dvm_ctx *c) { return c ? c->sync_limit : 0; }

extern "C" int dvm_ctx_set_copies_in_flight(dvm_ctx *c, int copies) {
    if (!c || copies < 1 || copies > 4096) return dvm_set_error(DVM_E_ARGS, "dvm_ctx_set_copies_in_flight: null context, or copies not in 1 .. 4096");
    c->copies = copies;
    return DVM_OK;
}
extern "C" int dvm_ctx_set_workspace_limit(dvm_ctx *c, int64_t bytes) {
    if (!c || bytes < 0) return dvm_set_error(DVM_E_ARGS, "dvm_ctx_set_workspace_limit: null context or negative size");
    c->workspace_limit = bytes;
    return DVM_OK;
}

extern "C" int dvm_ctx_set_lds_operands(dvm_ctx *c, int enabled) {
    if (!c) return dvm_set_error(DVM_E_ARGS, "dvm_ctx_set_lds_operands: null context");
    c->lds_operands = enabled != 0;
    if (enabled > 1) c->lds_budget = enabled < (int)LDS_IMAGE_MAX_BYTES ? enabled : (int)LDS_IMAGE_MAX_BYTES;
    return DVM_OK;
}

extern "C" int dvm_ctx_set_assignment(dvm_ctx *c, int assignment) {
    if (!c) return dvm_set_error(DVM_E_ARGS, "null context");
    if (assignment != DVM_ASSIGN_BLOCKED && assignment != DVM_ASSIGN_INTERLEAVED && assignment != DVM_ASSIGN_AUTO) return dvm_set_error(DVM_E_ARGS, "unknown tile assignment");
    c->assignment = assignment;
    return DVM_OK;
}

extern "C" int dvm_ctx_set_planner(dvm_ctx *c, int n_cu, int overhead) {
    if (!c) return dvm_set_error(DVM_E_ARGS, "null context");
    if (n_cu > 0) c->n_cu = n_cu;
    if (overhead > 0) c->overhead = overhead;
    return DVM_OK;
}

// ------------------------------------------------------------------------------------------------
// program builder and front end (decomposition into basic ops)
// ------------------------------------------------------------------------------------------------
namespace {

enum NodeKind : uint8_t { N_IN = 0, N_UN, N_BIN, N_BINI, N_SEL, N_RED, N_DEAD, N_CRED };
enum ImmKind : uint8_t { IMM_LIT = 0, IMM_INV_H = 1 };   // literal, or 1 / (row length of operand a)

constexpr int MAX_NODES = 160;
constexpr int MAX_VALUES = DVM_MAX_OPS + DVM_MAX_TENSORS;

struct Node {
    uint8_t kind, op, immkind, pad;
    int16_t a, b, c;
    int16_t input;       // for N_IN: input index
    float imm;
};

struct UserOp { int opcode; int args[3]; int n_args; double imm[2]; int n_imm; };

}  // namespace

struct dvm_prog {
    bool finished;
    int n_in, n_out, n_values, n_nodes;
    int in_dtype[DVM_MAX_TENSORS];
    int out_value[DVM_MAX_TENSORS], out_dtype[DVM_MAX_TENSORS];
    int out_node[DVM_MAX_TENSORS];
    // values in declaration order: inputs and user ops
    bool value_is_input[MAX_VALUES];
    int value_input_index[MAX_VALUES];
    UserOp value_op[MAX_VALUES];
    int value_node[MAX_VALUES];
    Node nodes[MAX_NODES];
};

extern "C" int dvm_prog_create(dvm_prog **out) {
    if (!out) return dvm_set_error(DVM_E_ARGS, "dvm_prog_create: null out");
    dvm_prog *p = new (std::nothrow) dvm_prog;
    if (!p) return dvm_set_error(DVM_E_LIMIT, "out of memory");
    memset(p, 0, sizeof(*p));
    *out = p;
    return DVM_OK;
}
extern "C" void dvm_prog_destroy(dvm_prog *p) { delete p; }
extern "C" int dvm_prog_num_inputs(const dvm_prog *p) { return p ? p->n_in : 0; }
extern "C" int dvm_prog_num_outputs(const dvm_prog *p) { return p ? p->n_out : 0; }

extern "C" int dvm_prog_input(dvm_prog *p, int dtype, int *value_id) {
    if (!p || !value_id) return dvm_set_error(DVM_E_ARGS, "dvm_prog_input: null argument");
    if (p->finished) return dvm_set_error(DVM_E_STATE, "program already finished");
    if (dtype != DVM_F32 && dtype != DVM_BF16) return dvm_set_error(DVM_E_DTYPE, "dvm_prog_input: dtype");
    if (p->n_in >= DVM_MAX_TENSORS - 1 || p->n_values >= MAX_VALUES) return dvm_set_error(DVM_E_LIMIT, "too many inputs");
    const int v = p->n_values++;
    p->value_is_input[v] = true;
    p->value_input_index[v] = p->n_in;
    p->in_dtype[p->n_in++] = dtype;
    *value_id = v;
    return DVM_OK;
}

static int op_arity(int opcode, int *n_imm) {
    *n_imm = 0;
    if (opcode >= DVM_OP_COPY && opcode <= DVM_OP_SILU) return 1;
    if (opcode == DVM_OP_CAST) { *n_imm = 1; return 1; }
    if (opcode == DVM_OP_ADDS || opcode == DVM_OP_MULS) { *n_imm = 1; return 1; }
    if (opcode >= DVM_OP_ADD && opcode <= DVM_OP_CMP_GE) return 2;
    if (opcode == DVM_OP_SELECT) return 3;
    if (opcode >= DVM_OP_SUM && opcode <= DVM_OP_MEANSQ) return 1;
    if (opcode >= DVM_OP_CSUM && opcode <= DVM_OP_CMIN) return 1;
    if (opcode == DVM_OP_SOFTMAX) return 1;
    if (opcode == DVM_OP_RMSNORM) { *n_imm = 1; return 2; }
    if (opcode == DVM_OP_LAYERNORM) { *n_imm = 1; return 3; }
    return -1;
}

extern "C" int dvm_prog_op(dvm_prog *p, int opcode, const int *arg_ids, int n_args, const double *imm, int n_imm,
                           int *value_id) {
    if (!p || !value_id || (n_args > 0 && !arg_ids)) return dvm_set_error(DVM_E_ARGS, "dvm_prog_op: null argument");
    if (p->finished) return dvm_set_error(DVM_E_STATE, "program already finished");
    int want_imm = 0;
    const int ar = op_arity(opcode, &want_imm);
    if (ar < 0) return dvm_set_error(DVM_E_ARGS, "dvm_prog_op: unknown opcode");
    if (n_args != ar) return dvm_set_error(DVM_E_ARGS, "dvm_prog_op: wrong number of arguments");
    if (n_imm < want_imm || (want_imm > 0 && !imm)) return dvm_set_error(DVM_E_ARGS, "dvm_prog_op: missing immediate");
    if (p->n_values >= MAX_VALUES) return dvm_set_error(DVM_E_LIMIT, "too many ops");
    const int v = p->n_values;
    UserOp &u = p->value_op[v];
    memset(&u, 0, sizeof(u));
    u.opcode = opcode;
    u.n_args = n_args;
    for (int i = 0; i < n_args; ++i) {
        if (arg_ids[i] < 0 || arg_ids[i] >= v) return dvm_set_error(DVM_E_ARGS, "dvm_prog_op: argument is not an earlier value");
        u.args[i] = arg_ids[i];
    }
    u.n_imm = want_imm;
    for (int i = 0; i < want_imm; ++i) u.imm[i] = imm[i];
    p->value_is_input[v] = false;
    p->n_values++;
    *value_id = v;
    return DVM_OK;
}

extern "C" int dvm_prog_output(dvm_prog *p, int value_id, int dtype) {
    if (!p) return dvm_set_error(DVM_E_ARGS, "dvm_prog_output: null program");
    if (p->finished) return dvm_set_error(DVM_E_STATE, "program already finished");
    if (dtype != DVM_F32 && dtype != DVM_BF16) return dvm_set_error(DVM_E_DTYPE, "dvm_prog_output: dtype");
    if (value_id < 0 || value_id >= p->n_values) return dvm_set_error(DVM_E_ARGS, "dvm_prog_output: bad value id");
    if (p->n_in + p->n_out >= DVM_MAX_TENSORS) return dvm_set_error(DVM_E_LIMIT, "too many tensors");
    p->out_value[p->n_out] = value_id;
    p->out_dtype[p->n_out] = dtype;
    p->n_out++;
    return DVM_OK;
}

namespace {

struct Lower {
    dvm_prog *p;
    bool overflow;
    int add(uint8_t kind, uint8_t op, int a, int b = -1, int c = -1, float imm = 0.0f, uint8_t immkind = IMM_LIT) {
        if (p->n_nodes >= MAX_NODES) { overflow = true; return 0; }
        Node &n = p->nodes[p->n_nodes];
        memset(&n, 0, sizeof(n));
        n.kind = kind; n.op = op; n.immkind = immkind;
        n.a = (int16_t)a; n.b = (int16_t)b; n.c = (int16_t)c; n.input = -1; n.imm = imm;
        return p->n_nodes++;
    }
    int un(uint32_t u, int a) { return add(N_UN, (uint8_t)u, a); }
    int bin(uint32_t b, int x, int y) { return add(N_BIN, (uint8_t)b, x, y); }
    int bini(uint32_t b, int x, float imm) { return add(N_BINI, (uint8_t)b, x, -1, -1, imm); }
    int inv_h(int x) { return add(N_BINI, (uint8_t)B_MUL, x, -1, -1, 0.0f, IMM_INV_H); }   // x * (1/H)
    int red(uint32_t r, int a) { return add(N_RED, (uint8_t)r, a); }
};

}  // namespace

extern "C" int dvm_prog_finish(dvm_prog *p) {
    if (!p) return dvm_set_error(DVM_E_ARGS, "dvm_prog_finish: null program");
    if (p->finished) return dvm_set_error(DVM_E_STATE, "program already finished");
    if (p->n_out == 0) return dvm_set_error(DVM_E_ARGS, "program has no output");
    Lower L{p, false};
    p->n_nodes = 0;
    for (int v = 0; v < p->n_values; ++v) {
        if (p->value_is_input[v]) {
            int n = L.add(N_IN, 0, -1);
            p->nodes[n].input = (int16_t)p->value_input_index[v];
            p->value_node[v] = n;
            continue;
        }
        const UserOp &u = p->value_op[v];
        const int a = p->value_node[u.args[0]];
        const int b = u.n_args > 1 ? p->value_node[u.args[1]] : -1;
        const int c = u.n_args > 2 ? p->value_node[u.args[2]] : -1;
        int r = -1;
        switch (u.opcode) {
            case DVM_OP_COPY: r = a; break;
            case DVM_OP_SQRT: r = L.un(U_SQRT, a); break;
            case DVM_OP_ABS: r = L.un(U_ABS, a); break;
            case DVM_OP_LOG: r = L.un(U_LOG, a); break;
            case DVM_OP_EXP: r = L.un(U_EXP, a); break;
            case DVM_OP_ROUND: r = L.un(U_ROUND, a); break;
            case DVM_OP_FLOOR: r = L.un(U_FLOOR, a); break;
            case DVM_OP_ISFINITE: r = L.un(U_ISFINITE, a); break;
            case DVM_OP_NEG: r = L.un(U_NEG, a); break;
            case DVM_OP_RSQRT: r = L.un(U_RSQRT, a); break;
            case DVM_OP_RCP: r = L.un(U_RCP, a); break;
            case DVM_OP_TANH: r = L.un(U_TANH, a); break;
            case DVM_OP_ERF: r = L.un(U_ERF, a); break;
            case DVM_OP_SIGMOID: r = L.un(U_SIGMOID, a); break;
            case DVM_OP_SQUARE: r = L.un(U_SQUARE, a); break;
            case DVM_OP_GELU_TANH: r = L.un(U_GELU_TANH, a); break;
            case DVM_OP_GELU_ERF: r = L.un(U_GELU_ERF, a); break;
            case DVM_OP_SILU: r = L.un(U_SILU, a); break;
            case DVM_OP_CAST:
                if ((int)u.imm[0] == DVM_BF16) r = L.un(U_CAST_BF16, a);
                else if ((int)u.imm[0] == DVM_F32) r = a;
                else return dvm_set_error(DVM_E_DTYPE, "cast: unknown target dtype");
                break;
            case DVM_OP_ADDS: r = L.bini(B_ADD, a, (float)u.imm[0]); break;
            case DVM_OP_MULS: r = L.bini(B_MUL, a, (float)u.imm[0]); break;
            case DVM_OP_ADD: r = L.bin(B_ADD, a, b); break;
            case DVM_OP_SUB: r = L.bin(B_SUB, a, b); break;
            case DVM_OP_MUL: r = L.bin(B_MUL, a, b); break;
            case DVM_OP_DIV: r = L.bin(B_DIV, a, b); break;
            case DVM_OP_MIN: r = L.bin(B_MIN, a, b); break;
            case DVM_OP_MAX: r = L.bin(B_MAX, a, b); break;
            case DVM_OP_POW: r = L.bin(B_POW, a, b); break;
            case DVM_OP_CMP_EQ: r = L.bin(B_EQ, a, b); break;
            case DVM_OP_CMP_NE: r = L.bin(B_NE, a, b); break;
            case DVM_OP_CMP_LT: r = L.bin(B_LT, a, b); break;
            case DVM_OP_CMP_LE: r = L.bin(B_LE, a, b); break;
            case DVM_OP_CMP_GT: r = L.bin(B_GT, a, b); break;
            case DVM_OP_CMP_GE: r = L.bin(B_GE, a, b); break;
            case DVM_OP_SELECT: r = L.add(N_SEL, 0, a, b, c); break;
            case DVM_OP_SUM: r = L.red(R_SUM, a); break;
            case DVM_OP_RMAX: r = L.red(R_MAX, a); break;
            case DVM_OP_RMIN: r = L.red(R_MIN, a); break;
            case DVM_OP_CSUM: r = L.add(N_CRED, (uint8_t)R_SUM, a); break;
            case DVM_OP_CMAX: r = L.add(N_CRED, (uint8_t)R_MAX, a); break;
            case DVM_OP_CMIN: r = L.add(N_CRED, (uint8_t)R_MIN, a); break;
            case DVM_OP_MEAN: r = L.inv_h(L.red(R_SUM, a)); p->nodes[r].b = (int16_t)a; break;
            case DVM_OP_MEANSQ: r = L.inv_h(L.red(R_SUMSQ, a)); p->nodes[r].b = (int16_t)a; break;
            case DVM_OP_SOFTMAX: {       // exp(z - max z) / sum exp(z - max z)
                int m = L.red(R_MAX, a);
                int d = L.bin(B_SUB, a, m);
                int e = L.un(U_EXP, d);
                int s = L.red(R_SUM, e);
                r = L.bin(B_DIV, e, s);
                break;
            }
            case DVM_OP_RMSNORM: {       // x * rsqrt(mean(x^2) + eps) * w
                int ms = L.inv_h(L.red(R_SUMSQ, a));
                p->nodes[ms].b = (int16_t)a;
                int rs = L.un(U_RSQRT, L.bini(B_ADD, ms, (float)u.imm[0]));
                r = L.bin(B_MUL, L.bin(B_MUL, a, rs), b);
                break;
            }
            case DVM_OP_LAYERNORM: {     // (h - mu) * rsqrt(mean((h - mu)^2) + eps) * gamma + beta
                int mu = L.inv_h(L.red(R_SUM, a));
                p->nodes[mu].b = (int16_t)a;
                int d = L.bin(B_SUB, a, mu);
                int var = L.inv_h(L.red(R_SUMSQ, d));
                p->nodes[var].b = (int16_t)d;
                int rs = L.un(U_RSQRT, L.bini(B_ADD, var, (float)u.imm[0]));
                r = L.bin(B_ADD, L.bin(B_MUL, L.bin(B_MUL, d, rs), b), c);
                break;
            }
            default: return dvm_set_error(DVM_E_ARGS, "dvm_prog_finish: unknown opcode");
        }
        if (L.overflow) return dvm_set_error(DVM_E_LIMIT, "program too long after decomposition");
        p->value_node[v] = r;
    }
    for (int i = 0; i < p->n_out; ++i) p->out_node[i] = p->value_node[p->out_value[i]];

    // peephole: sum(square(x)) or sum(x * x), the square used nowhere else -> one sum-of-squares
    int uses[MAX_NODES];
    memset(uses, 0, sizeof(uses));
    for (int n = 0; n < p->n_nodes; ++n) {
        const Node &nd = p->nodes[n];
        if (nd.kind == N_IN) continue;
        if (nd.a >= 0) uses[nd.a]++;
        if ((nd.kind == N_BIN || nd.kind == N_SEL) && nd.b >= 0) uses[nd.b]++;
        if (nd.kind == N_SEL && nd.c >= 0) uses[nd.c]++;
    }
    for (int i = 0; i < p->n_out; ++i) uses[p->out_node[i]]++;
    for (int n = 0; n < p->n_nodes; ++n) {
        Node &nd = p->nodes[n];
        if (nd.kind != N_RED || nd.op != R_SUM) continue;
        Node &sq = p->nodes[nd.a];
        const bool is_sq = (sq.kind == N_UN && sq.op == U_SQUARE) || (sq.kind == N_BIN && sq.op == B_MUL && sq.a == sq.b);
        if (is_sq && uses[nd.a] == 1) {
            nd.op = R_SUMSQ;
            nd.a = sq.a;
            sq.kind = N_DEAD;
        }
    }
    // peephole: exp(a - b), the difference used nowhere else -> one fused op (the softmax core)
    for (int n = 0; n < p->n_nodes; ++n) {
        Node &nd = p->nodes[n];
        if (nd.kind != N_UN || nd.op != U_EXP) continue;
        Node &d = p->nodes[nd.a];
        if (d.kind == N_BIN && d.op == B_SUB && uses[nd.a] == 1) {
            const int16_t da = d.a, db = d.b;
            d.kind = N_DEAD;
            nd.kind = N_BIN;
            nd.op = B_EXPSUB;
            nd.a = da;
            nd.b = db;
        }
    }
    p->finished = true;
    return DVM_OK;
}

// ------------------------------------------------------------------------------------------------
// small integer helpers
// ------------------------------------------------------------------------------------------------
namespace {

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline uint32_t pow2ceil(uint32_t x) {
    uint32_t p = 1;
    while (p < x) p <<= 1;
    return p;
}

// multiplier and shifts that divide any 32-bit unsigned number by d (1 <= d < 2^31):
// l = ceil(log2 d), m = floor(2^32 (2^l - d) / d) + 1, q = (t + ((n - t) >> sh1)) >> sh2 with
// t = mulhi(m, n), sh1 = min(l, 1), sh2 = max(l - 1, 0).
void magic_u32(uint32_t d, uint32_t *m, uint32_t *sh) {
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;
    const uint64_t mm = ((((uint64_t)1 << l) - d) << 32) / d + 1;
    *m = (uint32_t)mm;
    const uint32_t sh1 = l < 1 ? l : 1, sh2 = l > 0 ? l - 1 : 0;
    *sh = sh1 | (sh2 << 8);
}

// The tile-size rule on a one-dimensional space of `total` elements (Section 4.2): minimise
// ceil(ceil(total/t)/n) * (t + c) over t in 1..min(t_max,total); ties go to the larger tile.
// For a given number of rounds w the cheapest tile is the smallest one that needs no more than
// w rounds, t_w = ceil(total / (w n)); rounds are tried upwards until total/n + w c, a lower bound
// of any cost with w rounds, reaches the best cost found.
int64_t min_cost_tile(int64_t total, int64_t n, int64_t t_max, int64_t c) {
    const int64_t t0 = t_max < total ? t_max : total;
    int64_t w = cdiv(cdiv(total, t0), n);
    int64_t best_t = t0, best_c = w * (t0 + c);
    for (;; ++w) {
        const int64_t t = cdiv(total, w * n);
        const int64_t wa = cdiv(cdiv(total, t), n);
        const int64_t cost = wa * (t + c);
        if (cost < best_c || (cost == best_c && t > best_t)) { best_c = cost; best_t = t; }
        if (t == 1) break;
        if (total / n + (w + 1) * c >= best_c && c > 0) break;
    }
    return best_t;
}

int64_t align_up_capped(int64_t t, int64_t align, int64_t t_max) {
    const int64_t up = cdiv(t, align) * align;
    if (up <= t_max) return up;
    const int64_t down = (t_max / align) * align;
    return down >= align ? down : t;
}

}  // namespace

extern "C" int dvm_plan(int64_t total, int n_cores, int64_t t_max, int align, int overhead, int64_t *t_min_cost,
                        int64_t *t_aligned, int64_t *n_tiles) {
    if (total < 1 || n_cores < 1 || t_max < 1 || align < 1 || overhead < 0) return dvm_set_error(DVM_E_ARGS, "dvm_plan");
    const int64_t t = min_cost_tile(total, n_cores, t_max, overhead);
    const int64_t ta = align_up_capped(t, align, t_max);
    if (t_min_cost) *t_min_cost = t;
    if (t_aligned) *t_aligned = ta;
    if (n_tiles) *n_tiles = cdiv(total, ta);
    return DVM_OK;
}

// ------------------------------------------------------------------------------------------------
// the encoder
// ------------------------------------------------------------------------------------------------
namespace {

constexpr int NR_MAX = 6;
constexpr int MAX_AI = 4 * MAX_NODES;

struct Access {             // one tensor of the launch as the kernel addresses it
    int dtype;
    bool is_output;
    bool rows;              // one value per row (last-axis extent 1)
    int align_log2;
    int64_t min_bytes;
    int64_t ostride[DVM_MAX_RANK];   // per original axis, right aligned, 0 where broadcast
    int64_t s[4];           // collapsed: s[0] inner (0 or 1), s[1..3] outer groups
};

struct AI {                 // abstract instruction before emission
    uint8_t op, a, b, c;
    uint8_t kind, srck;
    int16_t tensor;
    float imm, imm2;
};

struct Enc {
    const dvm_prog *p;
    int R;                              // rank of the dominant shape
    int64_t shape[MAX_NODES][DVM_MAX_RANK];
    int64_t dom[DVM_MAX_RANK];
    bool rows_class[MAX_NODES];
    bool row_axis;                      // the dominant shape's last axis has extent > 1
    Access acc[DVM_MAX_TENSORS];
    int n_acc;
    // collapsed space
    int64_t D0, nrows, Dg[4];
    int n_groups;
    bool has_red;
    bool has_cred;                      // some value is reduced along the penultimate axis
    bool cred_real[MAX_NODES];          // N_CRED over an axis of extent > 1 (otherwise the identity)
    bool post[MAX_NODES];               // computed from such a reduction: once per unit, in the epilogue
    int n_epilog;                       // first abstract instruction of the epilogue
    bool cstream;                       // the per-row part only reduces input tensors: one streaming record each
    int n_fence;                        // peepholes do not reach back across this instruction index
    // linearisation
    AI ai[MAX_AI];
    int n_ai, n_prolog, n_prolog_a;
    int uses[MAX_NODES];
    int reg_of[MAX_NODES], sreg_of[MAX_NODES];
    int regs[NR_MAX], sregs[NS];
    int nr_limit;           // tile registers the program may use
    bool reload_inputs;     // never keep an input tile in a register: load it again at every use
    bool keep_sregs;        // never give a row-scalar register a second value (rows longer than a tile: the body runs once per pass)
    int lds_of[MAX_NODES];  // LDS image (slot) of a row-invariant input that only multiplies or is added, or -1
    int n_lds;
    int lds_node[LDS_SLOTS];
    int in_acc;
    int nr_used, ns_used;
    const char *err;
    int err_code;

    bool fail(int code, const char *msg) { if (!err) { err = msg; err_code = code; } return false; }

    void emit(uint8_t op, uint8_t a = 0, uint8_t b = 0, int tensor = -1, float imm = 0.0f, uint8_t kind = 0,
              uint8_t srck = 0, uint8_t c = 0) {
        if (n_ai >= MAX_AI) { fail(DVM_E_LIMIT, "too many instructions"); return; }
        // adjacent multiplies by a row scalar and by a tile register, and an add of a tile register after
        // them, become one fused record: acc = acc * S * R + R (kind: S index + 1, 0 = no scalar)
        if (op == I_BIN && n_ai > n_fence) {
            AI &p = ai[n_ai - 1];
            const bool is_r = a < SRC_S0, is_s = a >= SRC_S0 && a < SRC_S0 + NS;
            if (b == B_ADD && is_r) {
                if (p.op == I_BIN && p.b == B_MUL && p.a < SRC_S0) { p.op = I_FMA; p.b = a; p.kind = 0; return; }
                if (p.op == I_FMA && p.b == FMA_NO_ADDEND) { p.b = a; return; }
            }
            if (b == B_MUL && p.op == I_BIN && p.b == B_MUL) {
                const bool p_r = p.a < SRC_S0, p_s = p.a >= SRC_S0 && p.a < SRC_S0 + NS;
                if (p_s && is_r) { const uint8_t s = (uint8_t)(p.a - SRC_S0 + 1); p.op = I_FMA; p.a = a; p.b = FMA_NO_ADDEND; p.kind = s; return; }
                if (p_r && is_s) { p.op = I_FMA; p.b = FMA_NO_ADDEND; p.kind = (uint8_t)(a - SRC_S0 + 1); return; }
            }
        }
        AI &x = ai[n_ai++];
        x.op = op; x.a = a; x.b = b; x.c = c; x.kind = kind; x.srck = srck; x.tensor = (int16_t)tensor; x.imm = imm;
        x.imm2 = 0.0f;
    }
    // acc = acc * L or acc + L with L the LDS image in `slot`: joins the record before it where that keeps the
    // order of the operations (acc * S, then * L, then + L), else a record of its own.
    // I_LFMA: a = multiplier slot or LFMA_NONE, b = addend slot or LFMA_NONE, kind = S index + 1 or 0.
    void emit_lds(bool mul, int slot) {
        if (n_ai > n_fence && n_ai > 0) {
            AI &p = ai[n_ai - 1];
            if (mul && p.op == I_BIN && p.b == B_MUL && p.a >= SRC_S0 && p.a < SRC_S0 + NS) {      // acc * S, then * L
                p.op = I_LFMA; p.kind = (uint8_t)(p.a - SRC_S0 + 1); p.a = (uint8_t)slot; p.b = LFMA_NONE;
                return;
            }
            if (!mul && p.op == I_LFMA && p.b == LFMA_NONE) { p.b = (uint8_t)slot; return; }        // ... * L, then + L
        }
        emit(I_LFMA, mul ? (uint8_t)slot : (uint8_t)LFMA_NONE, mul ? (uint8_t)LFMA_NONE : (uint8_t)slot);
    }
    // Row-scalar op on the value a reduction has just produced, that value being used nowhere
    // else: fold it into the reduction's record as post(x) = U(x * scale + shift).
    // what: 0 = multiply by imm, 1 = add imm, 2 = unary uop.  srck of the RED record tracks the
    // stage reached (0 nothing, 1 scaled, 2 shifted, 3 unary applied).
    bool fold_into_red(int src_sreg, int what, float v, uint8_t uop) {
        if (n_ai == 0) return false;
        AI &r = ai[n_ai - 1];
        if (r.op != I_RED || r.a != src_sreg) return false;
        if (what == 0 && r.srck <= 1) { r.imm *= v; r.srck = 1; return true; }
        if (what == 0 && r.srck == 2) { r.imm *= v; r.imm2 *= v; return true; }
        if (what == 1 && r.srck <= 2) { r.imm2 += v; r.srck = 2; return true; }
        if (what == 2 && r.srck <= 2) { r.kind = uop; r.srck = 3; return true; }
        return false;
    }
    // the folded result takes over the source's S register
    void take_over_sreg(int src_node, int dst_node) {
        const int sr = sreg_of[src_node];
        sreg_of[src_node] = -1;
        sregs[sr] = dst_node;
        sreg_of[dst_node] = sr;
    }
    int alloc_reg(int node) {
        for (int i = 0; i < nr_limit; ++i)
            if (regs[i] < 0) {
                regs[i] = node;
                reg_of[node] = i;
                if (i + 1 > nr_used) nr_used = i + 1;
                return i;
            }
        fail(DVM_E_UNSUPPORTED, "program needs more live tile registers than available");
        return 0;
    }
    int alloc_sreg(int node) {
        for (int i = 0; i < NS; ++i)
            if (sregs[i] < 0) {
                sregs[i] = node;
                if (node >= 0) sreg_of[node] = i;
                if (i + 1 > ns_used) ns_used = i + 1;
                return i;
            }
        fail(DVM_E_UNSUPPORTED, "program needs more than 4 live row-scalar registers");
        return 0;
    }
    void release(int node) {            // called when the last use of `node` is gone
        if (reg_of[node] >= 0) { regs[reg_of[node]] = -1; reg_of[node] = -1; }
        if (sreg_of[node] >= 0 && !keep_sregs) { sregs[sreg_of[node]] = -1; sreg_of[node] = -1; }
        if (in_acc == node) in_acc = -1;
    }
    void use(int node) {
        if (--uses[node] <= 0) release(node);
    }
    bool is_input(int n) const { return p->nodes[n].kind == N_IN; }
    int tensor_of_input(int n) const { return p->nodes[n].input; }

    // keep the accumulator's value alive if something still needs it
    void save_acc_if_live() {
        const int v = in_acc;
        if (v < 0 || uses[v] <= 0 || reg_of[v] >= 0) return;
        if (is_input(v)) return;        // an input tile can be loaded again
        const int r = alloc_reg(v);
        emit(I_MOVRA, (uint8_t)r);
    }
    void load_rows_input(int n) {       // a [.., 1] input: one value per row into an S register
        if (sreg_of[n] >= 0) return;
        const int s = alloc_sreg(n);
        emit(I_LOADS, (uint8_t)s, 0, tensor_of_input(n));
    }
    bool to_acc(int n) {
        if (in_acc == n) return true;
        save_acc_if_live();
        if (reg_of[n] >= 0) emit(I_MOVAR, (uint8_t)reg_of[n]);
        else if (rows_class[n]) emit(I_BIN, (uint8_t)(SRC_S0 + sreg(n)), (uint8_t)B_NONE);   // Table 1 Broadcast: row value -> tile
        else if (is_input(n)) emit(I_LOAD, (uint8_t)SRC_ACC, (uint8_t)B_NONE, tensor_of_input(n));
        else return fail(DVM_E_UNSUPPORTED, "internal: value lost during linearisation");
        in_acc = n;
        return true;
    }
    // the accumulator holds `n` and is about to be overwritten: keep a copy if n is needed later
    void preserve(int n, int pending_uses) {
        if (uses[n] - pending_uses <= 0 || reg_of[n] >= 0) return;
        if (rows_class[n]) return;          // a row value lives on in its row-scalar register
        if (is_input(n)) {
            int free_regs = 0;
            for (int i = 0; i < nr_limit; ++i) free_regs += regs[i] < 0;
            if (free_regs == 0 || reload_inputs) return;   // reload it later instead
        }
        const int r = alloc_reg(n);
        emit(I_MOVRA, (uint8_t)r);
    }
    int to_reg(int n) {                 // make sure a tile value sits in some R register
        if (reg_of[n] >= 0) return reg_of[n];
        if (rows_class[n] && in_acc != n) {     // a row value needed as a tile: broadcast it through the accumulator
            to_acc(n);
        }
        if (in_acc == n) {
            const int r = alloc_reg(n);
            emit(I_MOVRA, (uint8_t)r);
            return r;
        }
        if (is_input(n)) {
            const int r = alloc_reg(n);
            emit(I_LOAD, (uint8_t)r, (uint8_t)B_NONE, tensor_of_input(n));
            return r;
        }
        fail(DVM_E_UNSUPPORTED, "internal: value lost during linearisation");
        return 0;
    }
    int sreg(int n) {
        if (sreg_of[n] < 0 && is_input(n)) load_rows_input(n);
        if (sreg_of[n] < 0) { fail(DVM_E_UNSUPPORTED, "internal: row value lost"); return 0; }
        return sreg_of[n];
    }
};

uint32_t reversed(uint32_t b) {
    switch (b) {
        case B_SUB: return B_RSUB;
        case B_DIV: return B_RDIV;
        case B_POW: return B_RPOW;
        case B_EXPSUB: return B_REXPSUB;
        case B_LT: return B_GT;
        case B_LE: return B_GE;
        case B_GT: return B_LT;
        case B_GE: return B_LE;
        default: return b;      // commutative
    }
}

float f32_bits(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
uint32_t bits_f32(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

}  // namespace

static int stack_impl(const void *const *codes, const size_t *lens, int n, const int *same_as, int n_same_as, void *out, size_t cap,
                      size_t *len, bool spatial, bool by_launch = false);

// dvm_encode of a program whose single reduction along the penultimate axis (node c, over `size` rows) is split S ways.
// Part 1: the ops before the reduction and the reduction itself over tensors seen as [.., S, size/S, N]: its output,
// [.., S, 1, N] fp32, is the data area of the launch's workspace.  Part 2: the same reduction over that area seen as
// [.., S, N], then the ops after it.  The two are encoded on their own and joined into one temporally stacked program
// whose tensor table is the program's inputs, its outputs and the workspace; part 2 is a kernel launch of its own.
static int encode_split_reduction(const dvm_ctx *ctx, const dvm_prog *prog, const dvm_shape *in_shapes, const dvm_shape *out_layout,
                                  void *bytecode, size_t cap, size_t *len, dvm_shape *out_shapes, const bool *post, int c, int R, int S,
                                  int64_t size, const int64_t *dom) {
    const int NN = prog->n_nodes, n_in = prog->n_in, n_out = prog->n_out;
    dvm_ctx sub = *ctx;
    sub.workspace_limit = 0;
    if (sub.max_k > 8) sub.max_k = 8;       // (the streaming form of the reduction runs in the variants up to 8 elements per lane)
    if (sub.dbg_rp == 0) sub.dbg_rp = 4;    // four waves per unit: workgroups of 256 threads, four of them per compute unit
    // ---- part 1
    dvm_prog p1;
    memset(&p1, 0, sizeof(p1));
    p1.finished = true;
    p1.n_in = n_in;
    for (int i = 0; i < n_in; ++i) p1.in_dtype[i] = prog->in_dtype[i];
    p1.n_nodes = NN;
    for (int n = 0; n < NN; ++n) {
        p1.nodes[n] = prog->nodes[n];
        if (post[n] && n != c) p1.nodes[n].kind = N_DEAD;
    }
    p1.n_out = 1;
    p1.out_node[0] = c;
    p1.out_dtype[0] = DVM_F32;
    dvm_shape sh1[DVM_MAX_TENSORS];
    for (int i = 0; i < n_in; ++i) {
        const dvm_shape &a = in_shapes[i];
        dvm_shape &b = sh1[i];
        b = a;
        if (a.rank >= 2) {              // [.., d, last] -> [.., S, d / S, last] (a broadcast extent of 1 -> 1, 1)
            const int ax = a.rank - 2;
            b.rank = a.rank + 1;
            for (int k = 0; k < ax; ++k) { b.dim[k] = a.dim[k]; b.stride[k] = a.stride[k]; }
            if (a.dim[ax] == 1) {
                b.dim[ax] = 1; b.stride[ax] = 0;
                b.dim[ax + 1] = 1; b.stride[ax + 1] = 0;
            } else {
                if (a.dim[ax] != size) return dvm_set_error(DVM_E_SHAPE, "internal: extent of the reduced axis");
                b.dim[ax] = S; b.stride[ax] = a.stride[ax] * (size / S);
                b.dim[ax + 1] = size / S; b.stride[ax + 1] = a.stride[ax];
            }
            b.dim[ax + 2] = a.dim[ax + 1];
            b.stride[ax + 2] = a.stride[ax + 1];
        }
    }
    unsigned char code1[DVM_CODE_MAX_BYTES + 512], code2[DVM_CODE_MAX_BYTES + 512];
    size_t len1 = 0, len2 = 0;
    dvm_shape part_shape;
    int st = dvm_encode(&sub, &p1, sh1, n_in, nullptr, code1, sizeof(code1), &len1, &part_shape);
    if (st != DVM_OK) return st;
    int64_t part_elems = 1;
    for (int k = 0; k < part_shape.rank; ++k) part_elems *= part_shape.dim[k];
    // ---- part 2: [partial results, the inputs the later ops take] -> the program's outputs
    dvm_prog p2;
    memset(&p2, 0, sizeof(p2));
    p2.finished = true;
    int map[MAX_NODES], in_of[DVM_MAX_TENSORS];
    for (int n = 0; n < NN; ++n) map[n] = -1;
    int nn = 0;
    p2.in_dtype[0] = DVM_F32;
    p2.nodes[nn] = Node{N_IN, 0, 0, 0, -1, -1, -1, 0, 0.0f};
    const int part_node = nn++;
    p2.n_in = 1;
    dvm_shape sh2[DVM_MAX_TENSORS];
    {
        int64_t dims[DVM_MAX_RANK];
        for (int k = 0; k < R; ++k) dims[k] = dom[k];
        dims[R - 2] = S;
        dvm_shape_contiguous(&sh2[0], R, dims);
        sh2[0].align_bytes = 16;
    }
    for (int n = 0; n < NN; ++n) {          // inputs of the ops after the reduction
        if (!post[n] || n == c) continue;
        const Node &nd = prog->nodes[n];
        const int args[3] = {nd.a, (nd.kind == N_BIN || nd.kind == N_SEL) ? nd.b : -1, nd.kind == N_SEL ? nd.c : -1};
        for (int j = 0; j < 3; ++j) {
            const int a = args[j];
            if (a < 0 || map[a] >= 0 || prog->nodes[a].kind != N_IN) continue;
            const int t = prog->nodes[a].input;
            in_of[p2.n_in] = t;
            p2.in_dtype[p2.n_in] = prog->in_dtype[t];
            sh2[p2.n_in] = in_shapes[t];
            p2.nodes[nn] = Node{N_IN, 0, 0, 0, -1, -1, -1, (int16_t)p2.n_in, 0.0f};
            map[a] = nn++;
            ++p2.n_in;
        }
    }
    p2.nodes[nn] = Node{N_CRED, prog->nodes[c].op, 0, 0, (int16_t)part_node, -1, -1, 0, 0.0f};
    map[c] = nn++;
    for (int n = 0; n < NN; ++n) {
        if (!post[n] || n == c) continue;
        Node nd = prog->nodes[n];
        if (nd.kind == N_DEAD) continue;
        if (nd.a >= 0) nd.a = (int16_t)map[nd.a];
        if ((nd.kind == N_BIN || nd.kind == N_SEL) && nd.b >= 0) nd.b = (int16_t)map[nd.b];
        if (nd.kind == N_SEL && nd.c >= 0) nd.c = (int16_t)map[nd.c];
        p2.nodes[nn] = nd;
        map[n] = nn++;
    }
    p2.n_nodes = nn;
    p2.n_out = n_out;
    for (int o = 0; o < n_out; ++o) {
        if (map[prog->out_node[o]] < 0) return dvm_set_error(DVM_E_UNSUPPORTED, "internal: output of a split reduction not computed after it");
        p2.out_node[o] = map[prog->out_node[o]];
        p2.out_dtype[o] = prog->out_dtype[o];
    }
    st = dvm_encode(&sub, &p2, sh2, p2.n_in, out_layout, code2, sizeof(code2), &len2, out_shapes);
    if (st != DVM_OK) return st;
    // ---- join: stack the two, then fold their tensor tables into [inputs, outputs, workspace]
    unsigned char both[2 * DVM_CODE_MAX_BYTES + 1024];
    const void *codes[2] = {code1, code2};
    const size_t lens[2] = {len1, len2};
    size_t lenb = 0;
    st = stack_impl(codes, lens, 2, nullptr, 0, both, sizeof(both), &lenb, false);
    if (st != DVM_OK) return st;
    const uint32_t *sw = (const uint32_t *)both;
    const uint32_t nt1 = (uint32_t)n_in + 1, nt2 = (uint32_t)p2.n_in + (uint32_t)n_out, ntf = (uint32_t)(n_in + n_out + 1);
    const uint32_t ws_index = (uint32_t)(n_in + n_out);
    uint32_t final_of[2 * DVM_MAX_TENSORS];     // index in the stacked table -> index in the final table
    for (uint32_t t = 0; t < nt1; ++t) final_of[t] = t < (uint32_t)n_in ? t : ws_index;
    for (uint32_t t = 0; t < nt2; ++t)
        final_of[nt1 + t] = t == 0 ? ws_index : (t < (uint32_t)p2.n_in ? (uint32_t)in_of[t] : (uint32_t)n_in + (t - (uint32_t)p2.n_in));
    const uint32_t segs_off_s = PH_WORDS_N + (nt1 + nt2) * TT_WORDS;
    const uint32_t seg_words = sw[PH_WORDS] - segs_off_s;
    const size_t words = PH_WORDS_N + (size_t)ntf * TT_WORDS + seg_words;
    *len = words * 4;
    if (seg_words * 4 > DVM_CODE_MAX_BYTES) return dvm_set_error(DVM_E_LIMIT, "bytecode exceeds the per-launch limit");
    if (!bytecode || cap < words * 4) return dvm_set_error(DVM_E_BUFSZ, "bytecode buffer too small");
    uint32_t *w = (uint32_t *)bytecode;
    memset(w, 0, words * 4);
    memcpy(w, sw, PH_WORDS_N * 4);
    w[PH_WORDS] = (uint32_t)words;
    w[PH_NTENS] = ntf;
    uint32_t *tt = w + PH_WORDS_N;
    for (uint32_t t = 0; t < (uint32_t)n_in; ++t) memcpy(tt + t * TT_WORDS, sw + PH_WORDS_N + t * TT_WORDS, TT_WORDS * 4);
    for (uint32_t o = 0; o < (uint32_t)n_out; ++o)
        memcpy(tt + ((uint32_t)n_in + o) * TT_WORDS, sw + PH_WORDS_N + (nt1 + (uint32_t)p2.n_in + o) * TT_WORDS, TT_WORDS * 4);
    {
        uint32_t *te = tt + ws_index * TT_WORDS;
        const uint64_t bytes = (uint64_t)DVM_WORKSPACE_BYTES + (uint64_t)part_elems * 4;
        te[TT_INFO] = (uint32_t)DVM_F32 | TI_OUTPUT | TI_WORKSPACE | (8u << 16);
        te[TT_BYTES_LO] = (uint32_t)(bytes & 0xFFFFFFFFu);
        te[TT_BYTES_HI] = (uint32_t)(bytes >> 32);
    }
    uint32_t *sg = w + PH_WORDS_N + ntf * TT_WORDS;
    memcpy(sg, sw + segs_off_s, (size_t)seg_words * 4);
    uint32_t at = 0;
    for (uint32_t k = 0; k < sw[PH_NSEG]; ++k) {
        uint32_t *sh = sg + at;
        const uint32_t tb = sh[S_TBASE];
        for (uint32_t pc = SH_WORDS; pc < sh[S_WORDS]; pc += (sh[pc] >> 8) & 0xFF) {
            const uint32_t op = sh[pc] & 0xFF;
            if (op == I_LOAD || op == I_VLOAD || op == I_STORE || op == I_VSTORE || op == I_LOADS || op == I_STORES || op == I_CSTREAM ||
                op == I_LDSCOPY)
                sh[pc + 1] = (sh[pc + 1] & ~0xFFu) | final_of[tb + (sh[pc + 1] & 0xFF)];
        }
        sh[S_TBASE] = 0;
        sh[S_NTENS] = ntf;
        if (k > 0) sh[S_FLAGS] |= SF_NEW_LAUNCH;
        at += sh[S_WORDS];
    }
    return dvm_validate(bytecode, words * 4);
}

extern "C" int dvm_encode(const dvm_ctx *ctx, const dvm_prog *prog, const dvm_shape *in_shapes, int n_in,
                          const dvm_shape *out_layout, void *bytecode, size_t cap, size_t *len, dvm_shape *out_shapes) {
    if (!ctx || !prog || !len || (n_in > 0 && !in_shapes)) return dvm_set_error(DVM_E_ARGS, "dvm_encode: null argument");
    if (!prog->finished) return dvm_set_error(DVM_E_STATE, "dvm_encode: program not finished");
    if (n_in != prog->n_in) return dvm_set_error(DVM_E_ARGS, "dvm_encode: number of input shapes");
    Enc E;
    E.p = prog;
    E.err = nullptr;
    E.err_code = 0;
    const int NN = prog->n_nodes;

    // ---- 1. shapes ---------------------------------------------------------------------------
    int R = 1;
    for (int i = 0; i < n_in; ++i) {
        if (in_shapes[i].rank < 0 || in_shapes[i].rank > DVM_MAX_RANK) return dvm_set_error(DVM_E_RANK, "input rank");
        if (in_shapes[i].rank > R) R = in_shapes[i].rank;
    }
    E.R = R;
    for (int n = 0; n < NN; ++n) {
        const Node &nd = prog->nodes[n];
        int64_t *sh = E.shape[n];
        if (nd.kind == N_DEAD) continue;
        if (nd.kind == N_IN) {
            const dvm_shape &s = in_shapes[nd.input];
            for (int k = 0; k < R; ++k) sh[k] = 1;
            for (int k = 0; k < s.rank; ++k) {
                if (s.dim[k] < 0) return dvm_set_error(DVM_E_SHAPE, "negative dimension");
                sh[R - s.rank + k] = s.dim[k];
            }
            continue;
        }
        const int args[3] = {nd.a, (nd.kind == N_BIN || nd.kind == N_SEL) ? nd.b : -1, nd.kind == N_SEL ? nd.c : -1};
        for (int k = 0; k < R; ++k) sh[k] = 1;
        for (int j = 0; j < 3; ++j) {
            if (args[j] < 0) continue;
            const int64_t *as = E.shape[args[j]];
            for (int k = 0; k < R; ++k) {
                if (as[k] == sh[k] || as[k] == 1) continue;
                if (sh[k] == 1) sh[k] = as[k];
                else return dvm_set_error(DVM_E_SHAPE, "operands do not broadcast together");
            }
        }
        if (nd.kind == N_RED) sh[R - 1] = 1;
        if (nd.kind == N_CRED) {
            if (R < 2) return dvm_set_error(DVM_E_RANK, "a reduction along the penultimate axis needs rank >= 2");
            sh[R - 2] = 1;
        }
    }
    for (int k = 0; k < R; ++k) E.dom[k] = 1;
    for (int n = 0; n < NN; ++n) {
        if (prog->nodes[n].kind == N_DEAD) continue;
        for (int k = 0; k < R; ++k) {
            const int64_t d = E.shape[n][k];
            if (d == E.dom[k] || d == 1) continue;
            if (E.dom[k] == 1) E.dom[k] = d;
            else return dvm_set_error(DVM_E_UNSUPPORTED, "ops have different iteration spaces: cannot fuse into one meta-kernel");
        }
    }
    if (out_shapes) {
        for (int i = 0; i < prog->n_out; ++i) {
            dvm_shape_contiguous(&out_shapes[i], R, E.shape[prog->out_node[i]]);
        }
    }
    int64_t total = 1;
    for (int k = 0; k < R; ++k) total *= E.dom[k];

    // ---- 2. classes ---------------------------------------------------------------------------
    E.row_axis = E.dom[R - 1] > 1;
    E.has_red = false;
    for (int n = 0; n < NN; ++n) {
        const Node &nd = prog->nodes[n];
        if (nd.kind == N_DEAD) continue;
        E.rows_class[n] = E.row_axis && E.shape[n][R - 1] == 1;
        if (nd.kind == N_RED && !E.rows_class[nd.a] && E.row_axis) E.has_red = true;
    }
    // Reductions along the penultimate axis.  The values computed from one (`post`) exist once per unit
    // (outer index, column tile) and are evaluated by an epilogue after the unit's last row; everything
    // else is evaluated row by row as usual.
    E.has_cred = false;
    for (int n = 0; n < NN; ++n) {
        const Node &nd = prog->nodes[n];
        E.cred_real[n] = nd.kind == N_CRED && E.shape[nd.a][R - 2] > 1;
        if (nd.kind == N_CRED && E.shape[nd.a][R - 2] == 0) return dvm_set_error(DVM_E_UNSUPPORTED, "reduction along an empty axis");
        E.post[n] = false;
        E.has_cred |= E.cred_real[n];
    }
    if (E.has_cred) {
        if (!E.row_axis) return dvm_set_error(DVM_E_UNSUPPORTED, "reduction along the penultimate axis of a tensor whose last axis has extent 1: reduce the last axis of [M, size] instead");
        for (int n = 0; n < NN; ++n) {
            const Node &nd = prog->nodes[n];
            if (nd.kind == N_DEAD || nd.kind == N_IN) continue;
            if (nd.kind == N_RED) return dvm_set_error(DVM_E_UNSUPPORTED, "a program reduces along one axis only");
            const int args[3] = {nd.a, (nd.kind == N_BIN || nd.kind == N_SEL) ? nd.b : -1, nd.kind == N_SEL ? nd.c : -1};
            bool any_post = false;
            for (int j = 0; j < 3; ++j) any_post |= args[j] >= 0 && E.post[args[j]];
            if (E.cred_real[n]) {
                if (E.rows_class[nd.a]) return dvm_set_error(DVM_E_UNSUPPORTED, "reduction along the penultimate axis of a row value");
                if (any_post) return dvm_set_error(DVM_E_UNSUPPORTED, "internal: reduced value reduced again");
                E.post[n] = true;
                continue;
            }
            if (!any_post) continue;
            if (E.shape[n][R - 2] != 1)
                return dvm_set_error(DVM_E_UNSUPPORTED, "a value reduced along the penultimate axis feeds a full-size op: that needs a second pass over the data");
            for (int j = 0; j < 3; ++j)
                if (args[j] >= 0 && !E.post[args[j]] && prog->nodes[args[j]].kind != N_IN)
                    return dvm_set_error(DVM_E_UNSUPPORTED, "an op after the reduction takes a value computed before it");
            E.post[n] = true;
        }
    }

    // A program whose per-row part does nothing but reduce input tensors gets one streaming record per
    // reduction (several rows in flight per wave) instead of a load and an accumulate per row.
    E.cstream = E.has_cred;
    for (int n = 0; n < NN && E.cstream; ++n) {
        const Node &nd = prog->nodes[n];
        if (nd.kind == N_DEAD || nd.kind == N_IN || E.post[n]) {
            if (E.cred_real[n] && (prog->nodes[nd.a].kind != N_IN || E.rows_class[nd.a])) E.cstream = false;
            continue;
        }
        E.cstream = false;              // some other per-row computation
    }
    for (int o = 0; o < prog->n_out && E.cstream; ++o)
        if (prog->nodes[prog->out_node[o]].kind == N_IN) E.cstream = false;     // an input copied to an output, row by row
    // (several reductions of one input share its load when they go row by row; streaming records would each read it)
    for (int n = 0; n < NN && E.cstream; ++n)
        for (int m = n + 1; m < NN && E.cstream; ++m)
            if (E.cred_real[n] && E.cred_real[m] && prog->nodes[n].a == prog->nodes[m].a) E.cstream = false;

    // A reduction along the penultimate axis with few units of work (outer index, column tile) and a long reduced
    // axis is split when the context allows a workspace: the rows of every unit are dealt out to S units that each
    // leave a partial result in the workspace, and a second meta-kernel, behind a grid-wide synchronisation
    // point, combines the S partial results in their fixed order and runs the ops that follow the reduction.
    if (E.has_cred && ctx->workspace_limit > 0 && total > 0) {
        int c = -1, n_cred = 0;
        for (int n = 0; n < NN; ++n)
            if (E.cred_real[n]) { c = n; ++n_cred; }
        bool all_post = true;
        for (int o = 0; o < prog->n_out; ++o) all_post &= E.post[prog->out_node[o]];
        const int64_t size = E.dom[R - 2], N = E.dom[R - 1];
        int64_t outer = 1;
        for (int k = 0; k < R - 2; ++k) outer *= E.dom[k];
        const int64_t units = outer * cdiv(N, 512);     // (at tiles of 64 lanes by 8 elements)
        const int64_t want_units = (int64_t)ctx->n_cu * 4;
        int64_t S = 0;
        if (n_cred == 1 && all_post && R < DVM_MAX_RANK && units * 4 <= want_units && size >= 64) {
            // the smallest divisor of the reduced extent that fills the machine and leaves every unit 16 rows or more
            for (int64_t d = 2; d <= size / 16 && S == 0; ++d)
                if (size % d == 0 && units * d >= want_units) S = d;
            if (S == 0)
                for (int64_t d = size / 16; d >= 2 && S == 0; --d)
                    if (size % d == 0) S = d;
        }
        if (S >= 2 && (int64_t)DVM_WORKSPACE_BYTES + outer * S * N * 4 <= ctx->workspace_limit) {
            const int st_split = encode_split_reduction(ctx, prog, in_shapes, out_layout, bytecode, cap, len, out_shapes, E.post, c, R, (int)S,
                                                        size, E.dom);
            // (the two parts may fit no common interpreter variant: the program then runs unsplit)
            if (st_split != DVM_E_UNSUPPORTED && st_split != DVM_E_LIMIT) return st_split;
            t_detail[0] = 0;
        }
    }

    // ---- 3. tensor accesses, collapse -------------------------------------------------------------
    E.n_acc = prog->n_in + prog->n_out;
    for (int t = 0; t < E.n_acc; ++t) {
        Access &A = E.acc[t];
        memset(&A, 0, sizeof(A));
        const bool is_out = t >= prog->n_in;
        const dvm_shape *s = nullptr;
        dvm_shape tmp;
        int node;
        if (!is_out) {
            s = &in_shapes[t];
            A.dtype = prog->in_dtype[t];
            node = -1;
            for (int n = 0; n < NN; ++n)
                if (prog->nodes[n].kind == N_IN && prog->nodes[n].input == t) node = n;
        } else {
            const int o = t - prog->n_in;
            node = prog->out_node[o];
            A.dtype = prog->out_dtype[o];
            dvm_shape_contiguous(&tmp, R, E.shape[node]);
            if (out_layout) {
                if (out_layout[o].rank != R) return dvm_set_error(DVM_E_SHAPE, "output layout rank differs from the inferred rank");
                for (int k = 0; k < R; ++k) {
                    if (out_layout[o].dim[k] != tmp.dim[k]) return dvm_set_error(DVM_E_SHAPE, "output layout dims differ from the inferred shape");
                    tmp.stride[k] = out_layout[o].stride[k];
                }
                tmp.align_bytes = out_layout[o].align_bytes;
            }
            s = &tmp;
            // an output must cover the whole iteration space (except the row axis for row values)
            for (int k = 0; k < R; ++k) {
                const bool row_value = (k == R - 1) && E.rows_class[node];
                const bool reduced = (k == R - 2) && E.post[node];
                if (E.shape[node][k] != E.dom[k] && !row_value && !reduced)
                    return dvm_set_error(DVM_E_UNSUPPORTED, "an output is smaller than the fused iteration space");
            }
        }
        A.is_output = is_out;
        const int es = A.dtype == DVM_F32 ? 4 : 2;
        int al = s->align_bytes > 0 ? s->align_bytes : 16;
        int lg = 0;
        while ((2 << lg) <= al && lg < 8) ++lg;
        if (lg > 4) lg = 4;
        if ((1 << lg) < es) return dvm_set_error(DVM_E_ALIGN, "tensor alignment below its element size");
        A.align_log2 = lg;
        int64_t maxoff = 0;
        bool empty = false;
        for (int k = 0; k < R; ++k) A.ostride[k] = 0;
        for (int k = 0; k < s->rank; ++k) {
            const int ax = R - s->rank + k;
            const int64_t d = s->dim[k], st = s->stride[k];
            if (d == 0) empty = true;
            if (d > 1) {
                if (st < 0) return dvm_set_error(DVM_E_UNSUPPORTED, "negative strides are not supported");
                A.ostride[ax] = st;
                maxoff += (d - 1) * st;
            }
        }
        A.min_bytes = empty ? 0 : (maxoff + 1) * es;
        if (is_out && !empty) {
            // an output element must have a memory location of its own: no broadcast stride, no two index
            // tuples at one address (sufficient test: strides sorted ascending, each at least the span below it)
            int64_t ds[DVM_MAX_RANK], ss[DVM_MAX_RANK];
            int m = 0;
            for (int k = 0; k < s->rank; ++k)
                if (s->dim[k] > 1) {
                    if (s->stride[k] == 0) return dvm_set_error(DVM_E_SHAPE, "an output layout repeats elements (stride 0 on an axis of extent > 1)");
                    int at = m++;
                    while (at > 0 && ss[at - 1] > s->stride[k]) { ss[at] = ss[at - 1]; ds[at] = ds[at - 1]; --at; }
                    ss[at] = s->stride[k];
                    ds[at] = s->dim[k];
                }
            int64_t span = 1;       // elements covered by the axes below
            for (int k = 0; k < m; ++k) {
                if (ss[k] < span) return dvm_set_error(DVM_E_SHAPE, "an output layout maps two elements to one address");
                span = ss[k] * (ds[k] - 1) + span;
            }
        }
        A.rows = E.row_axis && (node >= 0 ? E.rows_class[node] : false);
        if (E.row_axis && !A.rows && A.ostride[R - 1] == 0 && E.dom[R - 1] > 1) {
            // the tensor has the full row extent in its shape; a zero stride there is an expanded view
            if (E.shape[node][R - 1] > 1) return dvm_set_error(DVM_E_UNSUPPORTED, "zero stride on the last axis of a full tensor");
        }
    }

    // group the axes of the dominant shape from the innermost outwards
    int ax_list[DVM_MAX_RANK], n_ax = 0;
    for (int k = R - 1; k >= 0; --k)
        if (E.dom[k] > 1) ax_list[n_ax++] = k;
    int grp_first[4], grp_last[4];      // innermost and outermost axis of each group
    int64_t grp_ext[4];
    int ng = 0;
    for (int i = 0; i < n_ax; ++i) {
        const int ax = ax_list[i];
        bool merge = ng > 0;
        if (merge && ng == 1 && E.row_axis && E.has_red) merge = false;     // rows stay whole under a reduction
        if (merge && E.has_cred && ng <= 2) merge = false;      // the reduced axis is outer group 1, by itself
        if (merge) {
            const int inner = grp_last[ng - 1];
            for (int t = 0; t < E.n_acc && merge; ++t) {
                const Access &A = E.acc[t];
                if (A.ostride[ax] != A.ostride[inner] * E.dom[inner]) merge = false;
            }
        }
        if (merge) {
            grp_last[ng - 1] = ax;
            grp_ext[ng - 1] *= E.dom[ax];
        } else {
            if (ng == 4) return dvm_set_error(DVM_E_RANK, "iteration space does not reduce to four dimensions");
            grp_first[ng] = ax;
            grp_last[ng] = ax;
            grp_ext[ng] = E.dom[ax];
            ++ng;
        }
    }
    // Order of the outer groups = order in which rows are visited (group 1 varies fastest).  A group
    // along which some input is broadcast goes first: consecutive rows, and so the tiles one workgroup
    // runs back to back, then read the same part of that input again and find it in cache, instead of
    // every workgroup streaming the whole broadcast tensor once per repetition (a causal mask [S,S]
    // under scores [B,H,S,S] would otherwise be fetched from memory B*H times).
    if (ng > 2 && !E.has_cred) {
        auto carries_broadcast = [&](int g) {
            for (int t = 0; t < prog->n_in; ++t) {
                const Access &A = E.acc[t];
                bool varies_elsewhere = false;
                for (int h = 1; h < ng; ++h) varies_elsewhere |= (h != g && A.ostride[grp_first[h]] != 0 && grp_ext[h] > 1);
                if (A.ostride[grp_first[g]] == 0 && grp_ext[g] > 1 && varies_elsewhere) return true;
            }
            return false;
        };
        int order[4] = {0, 1, 2, 3};
        int n_first = 1;
        for (int g = 1; g < ng; ++g)
            if (carries_broadcast(g)) {     // move group g to position n_first, keeping the others in order
                const int moved = order[g];
                for (int h = g; h > n_first; --h) order[h] = order[h - 1];
                order[n_first++] = moved;
            }
        int gf[4], gl[4];
        int64_t ge[4];
        for (int g = 0; g < ng; ++g) { gf[g] = grp_first[order[g]]; gl[g] = grp_last[order[g]]; ge[g] = grp_ext[order[g]]; }
        for (int g = 0; g < ng; ++g) { grp_first[g] = gf[g]; grp_last[g] = gl[g]; grp_ext[g] = ge[g]; }
    }
    // if the row axis exists it must be group 0; otherwise group 0 is whatever is innermost
    E.n_groups = ng;
    const bool g0_is_row = ng > 0 && E.row_axis && grp_first[0] == R - 1;
    E.D0 = ng > 0 ? grp_ext[0] : 1;
    E.nrows = 1;
    for (int g = 1; g < ng; ++g) E.nrows *= grp_ext[g];
    for (int g = 0; g < 4; ++g) E.Dg[g] = g < ng ? grp_ext[g] : 1;
    if (total == 0) { E.D0 = 0; E.nrows = 0; }
    if (E.nrows >= (1ll << 31)) return dvm_set_error(DVM_E_LIMIT, "more than 2^31 rows");
    bool any_bf16_full = false;
    for (int t = 0; t < E.n_acc; ++t) {
        Access &A = E.acc[t];
        for (int g = 0; g < 4; ++g) A.s[g] = g < ng ? A.ostride[grp_first[g]] : 0;
        if (ng > 0 && !A.rows && A.s[0] != 1 && A.s[0] != 0)
            return dvm_set_error(DVM_E_UNSUPPORTED, "innermost stride of a tensor must be 1 (or 0 for a broadcast)");
        if (ng > 0 && A.s[0] == 0 && !(A.rows && g0_is_row)) {
            // broadcast along the innermost group without being a row value: only legal when the
            // tensor is constant along that group, which the row-value path handles
            A.rows = true;
        }
        if (!A.rows && A.dtype == DVM_BF16) any_bf16_full = true;
    }
    (void)g0_is_row;

    // ---- 4. linearise ---------------------------------------------------------------------------
    const uint32_t V = any_bf16_full ? 8 : 4;      // elements per 16-byte chunk of a tile
    auto linearize = [&](int hoist_budget, bool use_lds = false) {
    memset(E.uses, 0, sizeof(E.uses));
    for (int n = 0; n < NN; ++n) {
        const Node &nd = prog->nodes[n];
        if (nd.kind == N_IN || nd.kind == N_DEAD) continue;
        if (nd.a >= 0) E.uses[nd.a]++;
        if ((nd.kind == N_BIN || nd.kind == N_SEL) && nd.b >= 0) E.uses[nd.b]++;
        if (nd.kind == N_SEL && nd.c >= 0) E.uses[nd.c]++;
    }
    for (int i = 0; i < prog->n_out; ++i) E.uses[prog->out_node[i]]++;
    for (int n = 0; n < NN; ++n) { E.reg_of[n] = -1; E.sreg_of[n] = -1; }
    for (int i = 0; i < NR_MAX; ++i) E.regs[i] = -1;
    for (int i = 0; i < NS; ++i) E.sregs[i] = -1;
    E.in_acc = -1;
    E.n_ai = 0;
    E.nr_used = 0;
    E.ns_used = 0;
    E.n_epilog = -1;
    E.n_fence = 0;
    // input tensors that are row values by layout (see above) make their nodes row values too
    for (int n = 0; n < NN; ++n)
        if (prog->nodes[n].kind == N_IN && E.acc[prog->nodes[n].input].rows) E.rows_class[n] = true;

    // Tile-invariant operands (every outer stride zero: a weight vector broadcast over the rows) that the
    // program only multiplies by or adds can stay in LDS instead of a tile register: the prologue copies
    // them there once per workgroup, and the multiply / add reads them from there.
    E.n_lds = 0;
    for (int n = 0; n < NN; ++n) E.lds_of[n] = -1;
    if (use_lds) {
        int64_t lds_bytes = 0;
        auto invariant_input = [&](int n) {
            if (prog->nodes[n].kind != N_IN || E.rows_class[n]) return false;
            const Access &A = E.acc[prog->nodes[n].input];
            return A.s[1] == 0 && A.s[2] == 0 && A.s[3] == 0;
        };
        for (int n = 0; n < NN && E.n_lds < LDS_SLOTS; ++n) {
            if (!invariant_input(n) || E.uses[n] == 0) continue;
            bool ok = true;
            for (int o = 0; o < prog->n_out; ++o) ok &= prog->out_node[o] != n;
            for (int m = 0; m < NN && ok; ++m) {
                const Node &u = prog->nodes[m];
                if (u.kind == N_IN || u.kind == N_DEAD) continue;
                const bool is_a = u.a == n, is_b = (u.kind == N_BIN || u.kind == N_SEL) && u.b == n, is_c = u.kind == N_SEL && u.c == n;
                if (!is_a && !is_b && !is_c) continue;
                const int other = is_a ? u.b : u.a;
                ok = u.kind == N_BIN && (u.op == B_ADD || u.op == B_MUL) && !(is_a && is_b) && other >= 0 &&
                     !E.rows_class[other] && !invariant_input(other) && !E.cred_real[m] && !E.post[m];
            }
            const int64_t bytes = cdiv(E.D0 > 0 ? E.D0 : 1, V) * V * (E.acc[prog->nodes[n].input].dtype == DVM_F32 ? 4 : 2);
            if (!ok || lds_bytes + bytes > (int64_t)ctx->lds_budget) continue;
            lds_bytes += bytes;
            E.lds_of[n] = E.n_lds;
            E.lds_node[E.n_lds++] = n;
            E.uses[n] += 1 << 20;       // never released
        }
    }
    // The other tile-invariant operands are loaded once per workgroup into a pinned tile register by a
    // prologue that runs before the first tile, instead of once per tile.
    E.n_prolog = 0;
    for (int k = 0; k < E.n_lds; ++k)
        E.emit(I_LDSCOPY, (uint8_t)k, (uint8_t)(k + 1 == E.n_lds), prog->nodes[E.lds_node[k]].input);
    int hoisted = 0;
    for (int n = 0, left = hoist_budget; n < NN && left > 0; ++n) {
        const Node &nd = prog->nodes[n];
        if (nd.kind != N_IN || E.rows_class[n] || E.uses[n] == 0 || E.lds_of[n] >= 0) continue;
        const Access &A = E.acc[nd.input];
        if (A.s[1] != 0 || A.s[2] != 0 || A.s[3] != 0) continue;
        bool is_out = false;
        for (int o = 0; o < prog->n_out; ++o) is_out |= prog->out_node[o] == n;
        if (is_out) continue;
        const int r = E.alloc_reg(n);
        E.emit(I_LOAD, (uint8_t)r, (uint8_t)B_NONE, nd.input);
        E.uses[n] += 1 << 20;           // pinned: never released
        --left;
        ++hoisted;
    }
    E.n_prolog_a = E.n_ai;
    // Operands that are invariant along the fastest outer dim only (a mask [S,S] under [B*H,S,S] once that
    // dim is the fastest) are pinned too; their loads run again when the slower index changes.
    for (int n = 0, left = hoist_budget - hoisted; n < NN && left > 0 && ng >= 3 && E.Dg[1] >= 16 && !E.has_cred; ++n) {
        const Node &nd = prog->nodes[n];
        if (nd.kind != N_IN || E.rows_class[n] || E.uses[n] == 0) continue;
        const Access &A = E.acc[nd.input];
        if (A.s[1] != 0 || (A.s[2] == 0 && A.s[3] == 0)) continue;
        bool is_out = false;
        for (int o = 0; o < prog->n_out; ++o) is_out |= prog->out_node[o] == n;
        if (is_out) continue;
        const int r = E.alloc_reg(n);
        E.emit(I_LOAD, (uint8_t)r, (uint8_t)B_NONE, nd.input);
        E.uses[n] += 1 << 20;
        --left;
    }
    E.n_prolog = E.n_ai;

    auto store_outputs = [&](int n) {
        for (int o = 0; o < prog->n_out; ++o) {
            if (prog->out_node[o] != n) continue;
            const int t = prog->n_in + o;
            if (E.rows_class[n]) {
                E.emit(I_STORES, (uint8_t)E.sreg(n), 0, t);
            } else if (E.in_acc == n) {
                // a multiply by a row scalar whose only use is this store rides along with the store record
                uint8_t scale = 0;
                if (E.uses[n] == 1 && E.n_ai > E.n_prolog && E.n_ai > E.n_fence) {
                    const AI &p = E.ai[E.n_ai - 1];
                    if (p.op == I_BIN && p.b == B_MUL && p.a >= SRC_S0 && p.a < SRC_S0 + NS) {
                        scale = (uint8_t)(p.a - SRC_S0 + 1);
                        --E.n_ai;
                    }
                }
                E.emit(I_STORE, (uint8_t)SRC_ACC, scale, t);
            } else if (E.reg_of[n] >= 0) {
                E.emit(I_STORE, (uint8_t)E.reg_of[n], 0, t);
            } else {
                E.to_acc(n);
                E.emit(I_STORE, (uint8_t)SRC_ACC, 0, t);
            }
            E.use(n);
        }
    };

    // The accumulators of reductions along the penultimate axis live across the rows of a unit: each
    // gets a tile register of its own before anything else, so that no temporary of the per-row code
    // is ever placed in it.
    for (int n = 0; n < NN && !E.err; ++n)
        if (E.cred_real[n] && E.uses[n] > 0) E.alloc_reg(n);
    for (int pass = 0; pass < (E.has_cred ? 2 : 1) && !E.err; ++pass) {
    if (pass == 1) {            // the epilogue: values computed from the reductions, once per unit
        E.n_epilog = E.n_ai;
        E.in_acc = -1;
        // each wave of the workgroup accumulated its own share of the rows: combine them first
        for (int n = 0; n < NN; ++n)
            if (E.cred_real[n] && E.uses[n] > 0) E.emit(I_CCOMB, (uint8_t)E.reg_of[n], prog->nodes[n].op);
        E.n_fence = E.n_ai;
    }
    for (int n = 0; n < NN && !E.err; ++n) {
        Node nd = prog->nodes[n];
        if (nd.kind == N_DEAD) continue;
        if (E.cred_real[n]) {
            if (pass == 0) {
                if (E.uses[n] > 0) {
                    if (E.cstream) {
                        E.emit(I_CSTREAM, (uint8_t)E.reg_of[n], nd.op, E.tensor_of_input(nd.a));
                    } else {
                        E.to_acc(nd.a);
                        E.emit(I_CACC, (uint8_t)E.reg_of[n], nd.op);
                    }
                }
                E.use(nd.a);
            } else {
                store_outputs(n);
            }
            continue;
        }
        if (E.post[n] != (pass == 1)) continue;
        if (nd.kind == N_CRED) {        // over an axis of extent 1: the identity (x * 1 keeps every value, NaNs and signed zeros included)
            nd.kind = N_BINI; nd.op = (uint8_t)B_MUL; nd.imm = 1.0f; nd.immkind = IMM_LIT;
        }
        if (nd.kind == N_IN) {
            store_outputs(n);       // an input that is also an output: a plain copy
            continue;
        }
        if (E.uses[n] == 0) {       // dead code: still consume the operands
            if (nd.a >= 0) E.use(nd.a);
            if ((nd.kind == N_BIN || nd.kind == N_SEL) && nd.b >= 0) E.use(nd.b);
            if (nd.kind == N_SEL && nd.c >= 0) E.use(nd.c);
            continue;
        }
        const bool rows = E.rows_class[n];
        float imm = nd.imm;
        if (nd.kind == N_BINI && nd.immkind == IMM_INV_H) {
            const int64_t H = E.shape[nd.b][R - 1];
            imm = (float)(1.0 / (double)(H > 0 ? H : 1));
        }
        switch (nd.kind) {
            case N_UN:
                if (rows) {
                    const int sa = E.sreg(nd.a);
                    if (E.uses[nd.a] == 1 && E.fold_into_red(sa, 2, 0.0f, nd.op)) {
                        E.take_over_sreg(nd.a, n);
                        E.use(nd.a);
                        break;
                    }
                    E.use(nd.a);
                    const int sd = E.alloc_sreg(n);
                    E.emit(I_SOP, (uint8_t)sd, (uint8_t)sa, -1, 0.0f, (uint8_t)(SOP_UNARY + nd.op), 0, 0);
                } else {
                    E.to_acc(nd.a);
                    E.preserve(nd.a, 1);
                    E.use(nd.a);
                    E.emit(I_UN, 0, nd.op);
                    E.in_acc = n;
                }
                break;
            case N_BINI:
                if (rows) {
                    const int sa = E.sreg(nd.a);
                    if (E.uses[nd.a] == 1 && (nd.op == B_MUL || nd.op == B_ADD) &&
                        E.fold_into_red(sa, nd.op == B_MUL ? 0 : 1, imm, 0)) {
                        E.take_over_sreg(nd.a, n);
                        E.use(nd.a);
                        break;
                    }
                    E.use(nd.a);
                    const int sd = E.alloc_sreg(n);
                    E.emit(I_SOP, (uint8_t)sd, (uint8_t)sa, -1, imm, nd.op, 1, 0);
                } else {
                    E.to_acc(nd.a);
                    E.preserve(nd.a, 1);
                    E.use(nd.a);
                    E.emit(I_BIN, (uint8_t)SRC_IMM, nd.op, -1, imm);
                    E.in_acc = n;
                }
                break;
            case N_BIN: {
                int a = nd.a, b = nd.b;
                uint32_t op = nd.op;
                const bool ra = E.rows_class[a], rb = E.rows_class[b];
                if (rows) {                         // both operands are row values
                    const int sa = E.sreg(a), sb = E.sreg(b);
                    E.use(a);
                    E.use(b);
                    const int sd = E.alloc_sreg(n);
                    E.emit(I_SOP, (uint8_t)sd, (uint8_t)sa, -1, 0.0f, (uint8_t)op, 0, (uint8_t)sb);
                    break;
                }
                if (ra && !rb) {                    // row value on the left: swap and reverse
                    int t = a; a = b; b = t;
                    op = reversed(op);
                } else if (!ra && !rb && E.in_acc == b && a != b) {
                    int t = a; a = b; b = t;
                    op = reversed(op);
                }
                // now `a` is a tile and goes through the accumulator
                if (E.lds_of[a] >= 0 || E.lds_of[b] >= 0) {     // (add or multiply: commutative)
                    if (E.lds_of[a] >= 0) { int t = a; a = b; b = t; }
                    E.to_acc(a);
                    E.preserve(a, 1);
                    E.use(a);
                    E.emit_lds(op == B_MUL, E.lds_of[b]);
                    E.use(b);
                    E.in_acc = n;
                    break;
                }
                if (E.rows_class[b]) {
                    int sb = E.sreg(b);
                    E.to_acc(a);
                    E.preserve(a, 1);
                    E.use(a);
                    if (op == B_DIV) {              // tile / row value = tile * (1 / row value)
                        if (E.uses[b] == 1 && E.fold_into_red(sb, 2, 0.0f, U_RCP)) {
                            E.emit(I_BIN, (uint8_t)(SRC_S0 + sb), (uint8_t)B_MUL);
                        } else {
                            const int st = E.alloc_sreg(-1);
                            E.emit(I_SOP, (uint8_t)st, (uint8_t)sb, -1, 0.0f, (uint8_t)(SOP_UNARY + U_RCP), 0, 0);
                            E.emit(I_BIN, (uint8_t)(SRC_S0 + st), (uint8_t)B_MUL);
                            if (!E.keep_sregs) E.sregs[st] = -1;
                        }
                    } else {
                        E.emit(I_BIN, (uint8_t)(SRC_S0 + sb), (uint8_t)op);
                    }
                    E.use(b);
                } else if (a == b) {
                    E.to_acc(a);
                    E.preserve(a, 2);
                    E.use(a);
                    E.use(a);
                    E.emit(I_BIN, (uint8_t)SRC_ACC, (uint8_t)op);
                } else {
                    E.to_acc(a);
                    E.preserve(a, 1);
                    E.use(a);
                    if (E.reg_of[b] >= 0) {
                        E.emit(I_BIN, (uint8_t)E.reg_of[b], (uint8_t)op);
                    } else if (E.is_input(b)) {
                        // the operand is loaded into a tile register of its own (its load then shares a group with
                        // the loads before it); when inputs are not kept, the register is free again after the op
                        const int r = E.to_reg(b);
                        E.emit(I_BIN, (uint8_t)r, (uint8_t)op);
                        if (E.reload_inputs && E.uses[b] > 1) { E.regs[r] = -1; E.reg_of[b] = -1; }
                    } else {
                        E.fail(DVM_E_UNSUPPORTED, "internal: operand lost during linearisation");
                    }
                    E.use(b);
                }
                E.in_acc = n;
                break;
            }
            case N_SEL: {
                if (rows) {
                    E.fail(DVM_E_UNSUPPORTED, "select among row values only");
                    break;
                }
                const int rb = E.to_reg(nd.b);
                const int rc = E.to_reg(nd.c);
                E.to_acc(nd.a);
                E.preserve(nd.a, 1);
                E.use(nd.a);
                E.emit(I_SEL, (uint8_t)rb, (uint8_t)rc);
                E.use(nd.b);
                E.use(nd.c);
                E.in_acc = n;
                break;
            }
            case N_RED: {
                if (E.rows_class[nd.a] || !E.row_axis) {
                    // a row of one element: sum, max and min are the element, sum of squares its square
                    if (E.row_axis) {
                        const int sa = E.sreg(nd.a);
                        E.use(nd.a);
                        const int sd = E.alloc_sreg(n);
                        if (nd.op == R_SUMSQ) E.emit(I_SOP, (uint8_t)sd, (uint8_t)sa, -1, 0.0f, (uint8_t)(SOP_UNARY + U_SQUARE), 0, 0);
                        else E.emit(I_SOP, (uint8_t)sd, (uint8_t)sa, -1, 0.0f, (uint8_t)B_ADD, 1, 0);
                    } else {
                        E.to_acc(nd.a);
                        E.preserve(nd.a, 1);
                        E.use(nd.a);
                        if (nd.op == R_SUMSQ) E.emit(I_UN, 0, (uint8_t)U_SQUARE);
                        E.in_acc = n;
                    }
                    break;
                }
                E.to_acc(nd.a);
                const int sd = E.alloc_sreg(n);
                E.emit(I_RED, (uint8_t)sd, nd.op, -1, 1.0f, (uint8_t)U_NONE, 0, 0);
                E.use(nd.a);
                break;
            }
            default: E.fail(DVM_E_BADCODE, "internal: bad node"); break;
        }
        if (!E.err) store_outputs(n);
    }
    }
    if (E.n_epilog < 0) E.n_epilog = E.n_ai;
    };
    // first without hoisting, to learn how many tile registers the body needs; then, in row mode,
    // again with as many pinned operands as keep the program within four tile registers
    E.nr_limit = ctx->max_nr < NR_MAX ? ctx->max_nr : NR_MAX;
    E.reload_inputs = false;
    E.keep_sregs = false;
    linearize(0);
    if (E.err) {                // too many live tiles: trade registers for repeated (cached) loads
        E.err = nullptr;
        E.reload_inputs = true;
        linearize(0);
    }
    {
        int reg_cap = 4;
        if (reg_cap > ctx->max_nr) reg_cap = ctx->max_nr;
        if (!E.err && E.nrows > 1 && !(!E.has_red && E.D0 > 4096) && E.nr_used < reg_cap && !E.has_cred) {
            const int body_regs = E.nr_used;
            linearize(reg_cap - body_regs);
            if (E.err || E.nr_used > reg_cap) { E.err = nullptr; linearize(0); }
        }
    }
    // LDS images instead of pinned registers when that lets the program run in an interpreter variant with fewer
    // tile registers (more resident waves), or when it did not fit the registers at all
    {
        auto cls = [](int n) { return n <= 2 ? 2 : (n <= 4 ? 4 : (n <= 6 ? 6 : 8)); };
        const bool row_mode_ok = E.nrows > 1 && !(!E.has_red && E.D0 > 4096) && !E.has_cred && E.D0 > 0;
        const int before = E.err ? 99 : E.nr_used;
        bool any_invariant = false;     // (without a row-invariant input tensor there is nothing to keep in LDS: skip the attempt)
        for (int n = 0; n < NN && !any_invariant; ++n) {
            if (prog->nodes[n].kind != N_IN || E.acc[prog->nodes[n].input].rows) continue;
            const Access &A = E.acc[prog->nodes[n].input];
            any_invariant = A.s[1] == 0 && A.s[2] == 0 && A.s[3] == 0;
        }
        if (row_mode_ok && ctx->lds_operands && any_invariant && (before > 2 || E.reload_inputs)) {
            const bool was_reload = E.reload_inputs;
            E.err = nullptr;
            E.reload_inputs = false;
            linearize(0, true);
            if (!E.err && E.n_lds > 0 && (cls(E.nr_used) < cls(before) || was_reload)) {
                const int body_regs = E.nr_used;
                const int cap = cls(body_regs) < ctx->max_nr ? cls(body_regs) : ctx->max_nr;
                if (body_regs < cap) {          // pin what is left over in the registers of the same variant class
                    linearize(cap - body_regs, true);
                    if (E.err || E.nr_used > cap) { E.err = nullptr; linearize(0, true); }
                }
            } else {                            // no gain: back to the plan without LDS images
                E.err = nullptr;
                E.reload_inputs = false;
                linearize(0);
                if (E.err) { E.err = nullptr; E.reload_inputs = true; linearize(0); }
                int reg_cap = 4;
                if (reg_cap > ctx->max_nr) reg_cap = ctx->max_nr;
                if (!E.err && E.nrows > 1 && !(!E.has_red && E.D0 > 4096) && E.nr_used < reg_cap && !E.has_cred) {
                    const int body_regs = E.nr_used;
                    linearize(reg_cap - body_regs);
                    if (E.err || E.nr_used > reg_cap) { E.err = nullptr; linearize(0); }
                }
            }
        }
    }
    if (E.err) return dvm_set_error(E.err_code, E.err);
    if (E.nr_used > ctx->max_nr) return dvm_set_error(DVM_E_UNSUPPORTED, "program needs more tile registers than the context allows");

    // Loads are issued as early as the registers allow: a load record further down the body whose destination
    // register nothing touches before it moves up into the group of loads the body starts with, so that all of
    // them are in flight together and the tile waits for memory once.
    if (!E.has_cred) {
        auto touches = [&](const AI &x, int r) {
            switch (x.op) {
                case I_LOAD: case I_STORE: case I_MOVRA: case I_MOVAR: return x.a == r;
                case I_BIN: return x.a == r;
                case I_SEL: return x.a == r || x.b == r;
                case I_FMA: return x.a == r || x.b == r;
                default: return false;
            }
        };
        int top = E.n_prolog;
        while (top < E.n_ai && (E.ai[top].op == I_LOAD || E.ai[top].op == I_LOADS)) ++top;
        if (top > E.n_prolog) {
            for (int i = top + 1; i < E.n_ai; ++i) {
                if (E.ai[i].op != I_LOAD || E.ai[i].a >= SRC_S0) continue;
                bool free_reg = true;
                for (int j = top; j < i && free_reg; ++j) free_reg = !touches(E.ai[j], E.ai[i].a);
                // (the registers of the prologue's pinned operands are never a body load's destination)
                if (!free_reg) continue;
                const AI moved = E.ai[i];
                for (int j = i; j > top; --j) E.ai[j] = E.ai[j - 1];
                E.ai[top++] = moved;
            }
        }
    }

    // ---- 5. tile plan ---------------------------------------------------------------------------
    const int need_nr = E.nr_used;
    const int64_t Cr = cdiv(E.D0 > 0 ? E.D0 : 1, V);
    int vi = -1;                    // chosen variant
    bool long_row = false;          // rows longer than a tile, with reductions along them
    uint32_t G = 1, RP = 1, nvec = 1, nct = 1, TC = 0;
    auto find_variant = [&](int K) {
        int best = -1;
        for (int i = 0; i < N_VARIANTS; ++i)
            if ((VARIANTS[i].cred || !E.has_cred) && VARIANTS[i].K == K && K <= ctx->max_k && VARIANTS[i].NR >= need_nr && VARIANTS[i].NR <= ctx->max_nr && (best < 0 || VARIANTS[i].NR < VARIANTS[best].NR)) best = i;
        return best;
    };
    // LDS images of this program: offsets and sizes (each a whole number of chunks, zero-filled behind the row's end)
    uint32_t lds_off[LDS_SLOTS] = {0, 0, 0, 0}, lds_size[LDS_SLOTS] = {0, 0, 0, 0}, lds_total = 0;
    for (int k = 0; k < E.n_lds; ++k) {
        lds_off[k] = lds_total;
        lds_size[k] = (uint32_t)(cdiv(E.D0 > 0 ? E.D0 : 1, V) * V * (E.acc[prog->nodes[E.lds_node[k]].input].dtype == DVM_F32 ? 4 : 2));
        lds_total += lds_size[k];
    }
    auto slots_per_cu = [&](const Variant &v, uint32_t threads) {
        const int waves_wg = (int)((threads + 63) / 64);
        int s = v.waves_per_simd * 4 / waves_wg;
        if (lds_total > 0) {            // 160 KiB of LDS per compute unit, allocated in steps of 512 bytes
            const int by_lds = (int)(163840u / ((lds_total + 128u + 511u) / 512u * 512u));
            if (by_lds < s) s = by_lds;
        }
        return s < 1 ? 1 : s;
    };
    const int64_t ovh = ctx->overhead;
    const int64_t copies = ctx->copies;
    bool column_mode = !E.has_red && E.D0 > 4096;
    bool has_rows_output = false;
    for (int t = prog->n_in; t < E.n_acc; ++t) has_rows_output |= E.acc[t].rows;
    if (has_rows_output) column_mode = false;
    const int64_t cred_outer = E.has_cred && E.Dg[1] > 0 ? E.nrows / E.Dg[1] : 0;
    if (E.has_cred) {
        // Reduction along the penultimate axis: a unit of work is (outer index, column tile); one wave
        // walks the `size` rows of a unit and accumulates in a tile register.  The tile is as wide as
        // still leaves enough units to fill the machine.
        if (has_rows_output) return dvm_set_error(DVM_E_UNSUPPORTED, "a row-value output beside a reduction along the penultimate axis");
        column_mode = false;
        const int ks[5] = {4, 8, 16, 32, 64};
        int pick = -1;
        for (int i = 0; i < 5; ++i) {
            const int K = ks[i];
            if ((uint32_t)K < V) continue;
            const int v = find_variant(K);
            if (v < 0) continue;
            // (a workgroup holds up to 16 waves, each taking every RP-th row of the unit)
            int64_t rp_max = VARIANTS[v].max_threads / 64 < 16 ? VARIANTS[v].max_threads / 64 : 16;
            if (rp_max > E.Dg[1]) rp_max = E.Dg[1];
            const int64_t waves = cred_outer * cdiv(E.D0 > 0 ? E.D0 : 1, 64 * K) * rp_max;
            if (pick < 0 || waves * copies >= (int64_t)ctx->n_cu * slots_per_cu(VARIANTS[v], 64)) pick = v;
        }
        if (pick < 0) return dvm_set_error(DVM_E_UNSUPPORTED, "no interpreter variant with enough tile registers");
        vi = pick;
        G = 64;
        {
            const Variant &vr = VARIANTS[vi];
            int64_t rp_max = vr.max_threads / 64 < 16 ? vr.max_threads / 64 : 16;
            if (rp_max > E.Dg[1]) rp_max = E.Dg[1];
            const int64_t units = cred_outer * cdiv(E.D0 > 0 ? E.D0 : 1, 64 * vr.K);
            const int64_t want = cdiv((int64_t)ctx->n_cu * slots_per_cu(vr, 64), (units > 0 ? units : 1) * copies);
            RP = (uint32_t)(want < 1 ? 1 : (want > rp_max ? rp_max : want));
            if (ctx->dbg_rp > 0 && ctx->dbg_rp <= rp_max) RP = (uint32_t)ctx->dbg_rp;
        }
        nvec = (uint32_t)(VARIANTS[vi].K / V);
        TC = G * nvec * V;
        nct = (uint32_t)cdiv(E.D0 > 0 ? E.D0 : 1, TC);
        if (nct == 1) {                 // a short row: only as many chunks per lane as it needs
            nvec = (uint32_t)cdiv(Cr, G);
            TC = G * nvec * V;
        }
        // The streaming record keeps several rows' loads in registers at once: only the variants with few
        // elements per lane have room for that (they are the ones picked when units are scarce, which is
        // where it matters); wider tiles go row by row.
        if (E.cstream && VARIANTS[vi].K > 8) {
            E.cstream = false;
            linearize(0);
            if (E.err) return dvm_set_error(E.err_code, E.err);
            if (E.nr_used > VARIANTS[vi].NR) return dvm_set_error(DVM_E_UNSUPPORTED, "internal: register count changed between linearisations");
        }
    } else if (!column_mode) {
        const int ks[5] = {4, 8, 16, 32, 64};
        int pick = -1;
        uint32_t nv_cap = 0;        // chunks per lane the geometry may use (0: as many as the variant holds)
        // the largest K that still spreads a row over >= 16 lanes (K = 32: over >= 32 lanes, since that
        // variant keeps only two waves per SIMD resident); fewer lanes per row mean fewer interpreted
        // records per element, which measured faster than the higher occupancy of the smaller variants
        for (int i = 0; i < 5; ++i) {
            const int K = ks[i];
            if ((uint32_t)K < V) continue;
            const int v = find_variant(K);
            if (v < 0) continue;
            const int64_t gneed = cdiv(Cr, K / V);
            if (gneed > VARIANTS[v].max_threads) continue;
            if (pick < 0 || gneed >= (K >= 32 ? 32 : 16)) pick = v;
        }
        // Short rows (a variant exists that holds a row in less than a wave).  What a wave spends on a tile is
        // mostly fixed -- record decode, addresses, the steps of a reduction across lanes: measured at about four
        // chunk slots' worth of instructions -- so fewer lanes per row and more chunks per lane mean less work per
        // row, as long as the waves still fill the machine.  Every (variant, chunks per lane) pair is priced in the
        // form of the cost model of Section 4.2, ceil(wave tiles / SIMDs) * (4 + chunks per lane), a wave tile
        // being the part of a tile that one wave holds; the cheapest wins, the smaller variant on a tie.
        if (pick >= 0 && ctx->dbg_k < (int)V) {
            int kmax = 0;
            for (int i = 0; i < 5; ++i)
                if ((uint32_t)ks[i] >= V && find_variant(ks[i]) >= 0) kmax = ks[i];
            if (kmax > 0 && cdiv(Cr, kmax / V) < 64) {
                int64_t best = -1;
                int prev_k = 0;
                const int64_t n_simd = 4 * (int64_t)ctx->n_cu;
                const int64_t nr = E.nrows > 0 ? E.nrows : 1;
                for (int i = 0; i < 5; ++i) {
                    const int K = ks[i];
                    if ((uint32_t)K < V) continue;
                    const int v = find_variant(K);
                    if (v < 0) continue;
                    for (int nv = prev_k / (int)V + 1; nv <= K / (int)V; ++nv) {     // (chunk counts a smaller variant holds were priced with it)
                        const int64_t gneed = cdiv(Cr, nv);
                        if (gneed > VARIANTS[v].max_threads) continue;
                        const int64_t g = gneed <= 64 ? pow2ceil((uint32_t)gneed) : cdiv(gneed, 64) * 64;
                        if (nv > 1 && g < 2) continue;                               // (keep a few lanes side by side on a row)
                        const int64_t nvec_g = cdiv(Cr, g);
                        const int64_t wt = g < 64 ? cdiv(nr, 64 / g) : nr * (g / 64);
                        const int64_t cost = cdiv(wt * copies, n_simd) * (4 + nvec_g + (g > 64 ? 3 : 0));   // (rows over several waves: a barrier per reduction)
                        if (best < 0 || cost < best) { best = cost; pick = v; nv_cap = (uint32_t)nv; }
                    }
                    prev_k = K;
                }
            }
        }
        if (ctx->dbg_k >= (int)V) {
            const int v = find_variant(ctx->dbg_k);
            if (v >= 0 && cdiv(Cr, ctx->dbg_k / V) <= VARIANTS[v].max_threads) pick = v;
        }
        if (pick < 0) {                         // long rows: more elements per lane
            for (int i = 0; i < 5 && pick < 0; ++i) {
                const int K = ks[i];
                if ((uint32_t)K < V) continue;
                const int v = find_variant(K);
                if (v >= 0 && cdiv(Cr, K / V) <= VARIANTS[v].max_threads) pick = v;
            }
        }
        if (pick < 0 && (E.has_red || has_rows_output)) {
            // Rows longer than the widest tile: the row is cut into column tiles and the workgroup passes over it
            // once per reduction, then once more for the rest (SF_LONGROW).  The body must be a pure function of the
            // loads and of the reductions before: no pinned operands, no row-scalar register used twice.
            if (has_rows_output && !E.has_red) return dvm_set_error(DVM_E_UNSUPPORTED, "row too long for a row-value output without a reduction");
            E.err = nullptr;
            E.reload_inputs = false;
            E.keep_sregs = true;
            linearize(0);
            if (E.err) { E.err = nullptr; E.reload_inputs = true; linearize(0); }
            if (E.err) return dvm_set_error(E.err_code, E.err);
            int v = -1;
            for (int i = 4; i >= 0 && v < 0; --i) {             // the widest tile register first
                if ((uint32_t)ks[i] < V || ks[i] > ctx->max_k) continue;
                for (int j = 0; j < N_VARIANTS; ++j)
                    if (VARIANTS[j].K == ks[i] && VARIANTS[j].NR >= E.nr_used && VARIANTS[j].NR <= ctx->max_nr && (v < 0 || VARIANTS[j].NR < VARIANTS[v].NR)) v = j;
            }
            if (v < 0) return dvm_set_error(DVM_E_UNSUPPORTED, "no interpreter variant with enough tile registers");
            vi = v;
            long_row = true;
            const Variant &vr = VARIANTS[vi];
            G = (uint32_t)(vr.max_threads < 512 ? vr.max_threads : 512);
            nvec = (uint32_t)(vr.K / V);
            TC = G * nvec * V;
            nct = (uint32_t)cdiv(E.D0, TC);
            RP = 1;
        } else if (pick < 0) {
            column_mode = true;
        } else {
            vi = pick;
            const Variant &vr = VARIANTS[vi];
            const int64_t gneed = cdiv(Cr, nv_cap != 0 ? nv_cap : vr.K / V);
            G = gneed <= 64 ? pow2ceil((uint32_t)gneed) : (uint32_t)(cdiv(gneed, 64) * 64);
            nvec = (uint32_t)cdiv(Cr, G);
            TC = G * nvec * V;
            nct = 1;
            // rows per tile by the cost model (Section 4.2): candidates keep the workgroup a
            // whole number of waves and at most 256 threads (or one row if a row needs more)
            const uint32_t step = G < 64 ? 64 / G : 1;
            const uint32_t rp_max = G >= 256 ? 1 : 256 / G;
            // (with plenty of rows a workgroup of four waves is the smallest candidate: tiles of 8 KiB and more per
            // tensor measured 3-4 % faster than the same rows dealt out two waves at a time)
            uint32_t rp_first = step;
            if (rp_max > step && E.nrows * copies >= (int64_t)8 * ctx->n_cu * rp_max) rp_first = rp_max;
            int64_t best_cost = -1;
            RP = rp_first;
            for (uint32_t rp = rp_first; rp <= (rp_max > step ? rp_max : step); rp += step) {
                const uint32_t threads = rp * G;
                if (threads > (uint32_t)vr.max_threads) break;
                const int64_t N = (int64_t)ctx->n_cu * slots_per_cu(vr, threads);
                const int64_t tiles = cdiv(E.nrows > 0 ? E.nrows : 1, rp);
                const int64_t cost = cdiv(tiles * copies, N) * ((int64_t)rp * (E.D0 > 0 ? E.D0 : 1) + ovh);
                if (best_cost < 0 || cost <= best_cost) { best_cost = cost; RP = rp; }
            }
            if (ctx->dbg_rp > 0 && (uint32_t)ctx->dbg_rp % step == 0 && (uint32_t)ctx->dbg_rp * G <= (uint32_t)vr.max_threads)
                RP = (uint32_t)ctx->dbg_rp;
        }
    }
    if (column_mode) {
        // (the widest tile register first: 128 bytes per lane and tensor in flight measured 2-9 % above 64)
        int v = ctx->dbg_k >= (int)V ? find_variant(ctx->dbg_k) : -1;
        if (v < 0) v = find_variant(32);        // (64 elements at three waves per SIMD measured 18 % slower than 32 at four on a flat bf16 add)
        if (v < 0) v = find_variant(64);
        if (v < 0) v = find_variant(16);
        if (v < 0) v = find_variant(8);
        if (v < 0) v = find_variant(4);
        if (v < 0) return dvm_set_error(DVM_E_UNSUPPORTED, "no interpreter variant with enough tile registers");
        vi = v;
        const Variant &vr = VARIANTS[vi];
        G = 256;
        RP = 1;
        const int64_t t_max = (int64_t)G * vr.K;
        const int64_t N = (int64_t)ctx->n_cu * slots_per_cu(vr, G);
        // columns per tile by the cost model: try numbers of column tiles around whole rounds of N
        const int64_t nct_min = cdiv(E.D0, t_max);
        int64_t best_cost = -1, best_nct = nct_min;
        auto consider = [&](int64_t k) {
            if (k < nct_min) k = nct_min;
            int64_t tc = cdiv(cdiv(E.D0, k), V) * V;
            const int64_t tc_min = (int64_t)G * V;      // at least one chunk for every lane
            if (tc < tc_min) tc = tc_min;
            if (tc > t_max) return;
            const int64_t kk = cdiv(E.D0, tc);
            const int64_t cost = cdiv(E.nrows * kk * copies, N) * (tc + ovh);
            if (best_cost < 0 || cost < best_cost || (cost == best_cost && kk < best_nct)) { best_cost = cost; best_nct = kk; }
        };
        consider(nct_min);
        const int64_t w0 = cdiv(E.nrows * nct_min * copies, N);
        for (int64_t w = w0; w < w0 + 8; ++w) consider((w * N) / (E.nrows * copies));
        int64_t tc = cdiv(cdiv(E.D0, best_nct), V) * V;
        if (tc < (int64_t)G * V) tc = (int64_t)G * V;
        TC = (uint32_t)tc;
        nct = (uint32_t)cdiv(E.D0, tc);
        nvec = (uint32_t)cdiv(cdiv(tc, V), G);
    }
    const Variant &vr = VARIANTS[vi];
    const uint32_t threads = G * RP;
    const int64_t M64 = total == 0 ? 0 : (E.has_cred ? cred_outer * nct : (long_row ? E.nrows : cdiv(E.nrows, RP) * nct));
    if (M64 >= (1ll << 31)) return dvm_set_error(DVM_E_LIMIT, "more than 2^31 tiles");
    const int64_t Nslots = (int64_t)ctx->n_cu * slots_per_cu(vr, threads);
    const int64_t Ngrid = Nslots * ctx->dbg_grid_x;
    const uint32_t grid = (uint32_t)(M64 < Ngrid ? M64 : Ngrid);
    const bool wgsync = G > 64;

    // ---- 6. emit ---------------------------------------------------------------------------
    // size first
    size_t body_words = 0, prolog_words = 0, prolog_a_words = 0, epilog_words = 0;
    const bool view = ng > 2;       // more than one outer group: rows need the multi-stride form
    for (int i = 0; i < E.n_ai; ++i) {
        const AI &x = E.ai[i];
        if (i == E.n_prolog) prolog_words = body_words;
        if (i == E.n_prolog_a) prolog_a_words = body_words;
        if (i == E.n_epilog) epilog_words = body_words;
        switch (x.op) {
            case I_LOAD: case I_STORE: body_words += view ? LEN_VLOAD : LEN_LOAD; break;
            case I_LOADS: case I_STORES: case I_CSTREAM: body_words += LEN_VLOAD; break;
            default: body_words += LEN_REC; break;
        }
    }
    const size_t words = PH_WORDS_N + (size_t)E.n_acc * TT_WORDS + SH_WORDS + body_words;
    *len = words * 4;
    if ((SH_WORDS + body_words) * 4 > DVM_CODE_MAX_BYTES) return dvm_set_error(DVM_E_LIMIT, "bytecode exceeds the per-launch limit");
    if (!bytecode || cap < words * 4) return dvm_set_error(DVM_E_BUFSZ, "bytecode buffer too small");
    uint32_t *w = (uint32_t *)bytecode;
    memset(w, 0, words * 4);
    w[PH_MAGIC] = MAGIC;
    w[PH_TYPE] = KT_META | (VERSION << 16);
    w[PH_WORDS] = (uint32_t)words;
    w[PH_NSEG] = 1;
    w[PH_BLOCK] = threads;
    w[PH_GRID] = grid;
    w[PH_VARIANT] = (uint32_t)vr.K | ((uint32_t)vr.NR << 8) | ((uint32_t)(E.nr_used + 1) << 16);
    w[PH_NTENS] = (uint32_t)E.n_acc;
    for (int t = 0; t < E.n_acc; ++t) {
        uint32_t *tt = w + PH_WORDS_N + t * TT_WORDS;
        const Access &A = E.acc[t];
        // a full tensor is read in chunks of V elements at element alignment; only the element
        // alignment is required of the pointer
        const int es_log2 = A.dtype == DVM_F32 ? 2 : 1;
        tt[TT_INFO] = (uint32_t)A.dtype | ((uint32_t)A.is_output << 8) | ((uint32_t)es_log2 << 16);
        tt[TT_BYTES_LO] = (uint32_t)((uint64_t)A.min_bytes & 0xFFFFFFFFu);
        tt[TT_BYTES_HI] = (uint32_t)((uint64_t)A.min_bytes >> 32);
    }
    uint32_t *sh = w + PH_WORDS_N + E.n_acc * TT_WORDS;
    sh[S_WORDS] = (uint32_t)(SH_WORDS + body_words);
    sh[S_CODESIZE] = (uint32_t)body_words;
    sh[S_NTILES] = (uint32_t)M64;
    sh[S_GEOM] = G | (V << 16) | (nvec << 24);
    sh[S_RP] = RP | (threads << 16);
    sh[S_NCT] = nct;
    sh[S_TC] = TC;
    sh[S_D0LO] = (uint32_t)((uint64_t)E.D0 & 0xFFFFFFFFu);
    sh[S_D0HI] = (uint32_t)((uint64_t)E.D0 >> 32);
    sh[S_NROWS] = (uint32_t)E.nrows;
    if (ng > 2) {
        sh[S_D1] = (uint32_t)E.Dg[1];
        magic_u32((uint32_t)E.Dg[1], &sh[S_M1], &sh[S_SH1]);
        if (ng > 3) {
            sh[S_D2] = (uint32_t)E.Dg[2];
            magic_u32((uint32_t)E.Dg[2], &sh[S_M2], &sh[S_SH2]);
        }
    }
    if (long_row) {
        uint32_t n_red = 0;
        for (int i = 0; i < E.n_ai; ++i) n_red += E.ai[i].op == I_RED;
        sh[S_NCTSH] = n_red;
    } else if (nct > 1) {
        magic_u32(nct, &sh[S_NCTM], &sh[S_NCTSH]);
    }
    sh[S_TBASE] = 0;
    sh[S_NTENS] = (uint32_t)E.n_acc;
    // DVM_ASSIGN_AUTO: round-robin, except for a program that keeps an operand pinned while consecutive rows share it
    // (the reloading part of the prologue) and whose rows are not whole 128-byte lines: there a workgroup that walks
    // consecutive rows keeps the operand and meets the lines its rows share with their neighbours again at once
    // (measured 2-8 % faster; with rows of whole lines the round-robin order is 4 % faster).
    bool interleaved = ctx->assignment == DVM_ASSIGN_INTERLEAVED;
    if (ctx->assignment == DVM_ASSIGN_AUTO)
        interleaved = !(E.n_prolog > E.n_prolog_a && (E.D0 * (int64_t)(any_bf16_full ? 2 : 4)) % 128 != 0);
    sh[S_FLAGS] = (wgsync ? SF_WGSYNC : 0) | (E.has_cred && E.cstream ? SF_CSTREAM : 0) |
                  (interleaved ? SF_INTERLEAVED : 0) | (E.n_lds > 0 ? SF_LDS : 0) | (long_row ? SF_LONGROW : 0);
    sh[S_PROLOG] = (uint32_t)(E.n_prolog == E.n_ai ? body_words : prolog_words);
    sh[S_PROLOGA] = (uint32_t)(E.n_prolog_a == E.n_ai ? body_words : prolog_a_words);
    if (E.has_cred) {
        sh[S_INNER] = (uint32_t)E.Dg[1];
        sh[S_EPILOG] = (uint32_t)(E.n_epilog >= E.n_ai ? body_words : epilog_words);
    }
    uint32_t imask = 0;
    uint32_t *b = sh + SH_WORDS;
    auto put_i64 = [&](int64_t v) { *b++ = (uint32_t)((uint64_t)v & 0xFFFFFFFFu); *b++ = (uint32_t)((uint64_t)v >> 32); };
    for (int i = 0; i < E.n_ai; ++i) {
        const AI &x = E.ai[i];
        switch (x.op) {
            case I_LOAD: case I_STORE: {
                const Access &A = E.acc[x.tensor];
                const uint32_t op = view ? (x.op == I_LOAD ? I_VLOAD : I_VSTORE) : x.op;
                imask |= 1u << op;
                *b++ = w0(op, view ? LEN_VLOAD : LEN_LOAD, x.a, x.b);
                uint32_t mflags = 0;
                if (x.op == I_LOAD) {
                    bool once = !A.rows;        // read exactly once: no outer dim is broadcast
                    for (int g = 1; g < ng; ++g) once &= !(E.Dg[g] > 1 && A.s[g] == 0);
                    if (once && !long_row) mflags |= MF_STREAM;     // (a long row is read once per pass: keep it cached)
                }
                *b++ = (uint32_t)x.tensor | ((uint32_t)A.dtype << 8) | (mflags << 16);
                put_i64(A.s[1]);
                if (view) { put_i64(A.s[2]); put_i64(A.s[3]); }
                break;
            }
            case I_CSTREAM: {
                const Access &A = E.acc[x.tensor];
                imask |= 1u << I_CSTREAM;
                *b++ = w0(I_CSTREAM, LEN_VLOAD, x.a, x.b);
                bool once = true;       // read exactly once: no outer dim is broadcast
                for (int g = 1; g < ng; ++g) once &= !(E.Dg[g] > 1 && A.s[g] == 0);
                *b++ = (uint32_t)x.tensor | ((uint32_t)A.dtype << 8) | ((once ? MF_STREAM : 0u) << 16);
                put_i64(A.s[1]); put_i64(A.s[2]); put_i64(A.s[3]);
                break;
            }
            case I_LOADS: case I_STORES: {
                const Access &A = E.acc[x.tensor];
                imask |= 1u << x.op;
                *b++ = w0(x.op, LEN_VLOAD, x.a, 0);
                *b++ = (uint32_t)x.tensor | ((uint32_t)A.dtype << 8);
                put_i64(A.s[1]); put_i64(A.s[2]); put_i64(A.s[3]);
                break;
            }
            case I_LDSCOPY:
                imask |= 1u << I_LDSCOPY;
                b[0] = w0(I_LDSCOPY, LEN_REC, x.a, x.b);
                b[1] = (uint32_t)x.tensor | ((uint32_t)E.acc[x.tensor].dtype << 8);
                b[2] = lds_off[x.a];
                b[3] = lds_size[x.a];
                b += LEN_REC;
                break;
            case I_LFMA: {
                imask |= 1u << I_LFMA;
                uint32_t dts = 0;
                if (x.a != LFMA_NONE && E.acc[prog->nodes[E.lds_node[x.a]].input].dtype == DVM_BF16) dts |= 1u;
                if (x.b != LFMA_NONE && E.acc[prog->nodes[E.lds_node[x.b]].input].dtype == DVM_BF16) dts |= 2u;
                b[0] = w0(I_LFMA, LEN_REC, (uint32_t)x.a | ((uint32_t)x.b << 4), dts);
                b[1] = x.kind;
                b[2] = x.a != LFMA_NONE ? lds_off[x.a] : 0u;
                b[3] = x.b != LFMA_NONE ? lds_off[x.b] : 0u;
                b += LEN_REC;
                break;
            }
            case I_BIN:
                imask |= 1u << I_BIN;
                b[0] = w0(I_BIN, LEN_REC, x.a, x.b);
                b[1] = x.a == SRC_IMM ? bits_f32(x.imm) : 0u;
                b += LEN_REC;
                break;
            case I_SOP:
                imask |= 1u << I_SOP;
                b[0] = w0(I_SOP, LEN_SOP, x.a, x.b);
                b[1] = (uint32_t)x.kind | ((uint32_t)x.srck << 8) | ((uint32_t)x.c << 16);
                b[2] = x.srck == 1 ? bits_f32(x.imm) : 0u;
                b += LEN_SOP;
                break;
            case I_FMA:
                imask |= 1u << I_FMA;
                b[0] = w0(I_FMA, LEN_REC, x.a, x.b);
                b[1] = x.kind;
                b += LEN_REC;
                break;
            case I_RED:
                imask |= 1u << I_RED;
                b[0] = w0(I_RED, LEN_REC, x.a, x.b);
                b[1] = x.kind;                  // post unary op (U_NONE: none)
                b[2] = bits_f32(x.imm);         // scale
                b[3] = bits_f32(x.imm2);        // shift
                b += LEN_REC;
                break;
            default:
                imask |= 1u << x.op;
                b[0] = w0(x.op, LEN_REC, x.a, x.b);
                b += LEN_REC;
                break;
        }
    }
    sh[S_IMASK] = imask;
    t_detail[0] = 0;
    return DVM_OK;
}

// ------------------------------------------------------------------------------------------------
// validation, introspection, disassembly
// ------------------------------------------------------------------------------------------------
namespace {

int bad(const char *msg) { return dvm_set_error(DVM_E_BADCODE, msg); }

const Variant *variant_of(uint32_t word) {
    for (int i = 0; i < N_VARIANTS; ++i)
        if ((uint32_t)VARIANTS[i].K == (word & 0xFF) && (uint32_t)VARIANTS[i].NR == ((word >> 8) & 0xFF)) return &VARIANTS[i];
    return nullptr;
}

bool reg_ok(uint32_t r, const Variant *v) { return r < (uint32_t)v->NR; }
bool sreg_ok(uint32_t s) { return s < (uint32_t)NS; }

}  // namespace

extern "C" int dvm_validate(const void *bytecode, size_t len) {
    if (!bytecode) return dvm_set_error(DVM_E_ARGS, "dvm_validate: null bytecode");
    if (len < PH_WORDS_N * 4 || (len & 3)) return bad("bytecode shorter than its header");
    const uint32_t *w = (const uint32_t *)bytecode;
    if (w[PH_MAGIC] != MAGIC) return bad("bad magic");
    if ((w[PH_TYPE] >> 16) != VERSION) return bad("unknown version");
    const uint32_t kt = w[PH_TYPE] & 0xFFFF;
    if (kt != KT_META && kt != KT_STACK && kt != KT_STACK_SPATIAL) return bad("unknown kernel type");
    const uint32_t words = w[PH_WORDS];
    if ((size_t)words * 4 != len) return bad("length field does not match the buffer");
    const uint32_t nseg = w[PH_NSEG], ntens = w[PH_NTENS];
    if (nseg == 0 || nseg > 64) return bad("bad segment count");
    if (kt == KT_META && nseg != 1) return bad("a meta-kernel has one segment");
    if (ntens > DVM_MAX_TENSORS) return bad("too many tensors");
    const Variant *vr = variant_of(w[PH_VARIANT]);
    if (!vr) return bad("unknown interpreter variant");
    const uint32_t block = w[PH_BLOCK];
    if (block == 0 || (block & 63) || block > (uint32_t)vr->max_threads) return bad("bad workgroup size");
    size_t at = PH_WORDS_N + (size_t)ntens * TT_WORDS;
    if (at > words) return bad("tensor table runs past the end");
    for (uint32_t t = 0; t < ntens; ++t) {
        const uint32_t info = w[PH_WORDS_N + t * TT_WORDS + TT_INFO];
        if ((info & 0xFF) > 1) return bad("tensor dtype");
        if (((info >> 16) & 0xFF) > 8) return bad("tensor alignment");
        if ((info >> 24) > t) return bad("a tensor names a later one as the same buffer");
        if (info & TI_WORKSPACE) {
            if (t + 1 != ntens || kt != KT_STACK) return bad("the workspace is the last tensor of a temporally stacked program");
            const uint64_t bytes = (uint64_t)w[PH_WORDS_N + t * TT_WORDS + TT_BYTES_LO] | ((uint64_t)w[PH_WORDS_N + t * TT_WORDS + TT_BYTES_HI] << 32);
            if (bytes < WS_SYNC_WORDS * 4 || (info >> 24) != 0 || ((info >> 16) & 0xFF) < 6) return bad("workspace entry");
        }
    }
    const bool has_ws = ntens > 0 && (w[PH_WORDS_N + (ntens - 1) * TT_WORDS + TT_INFO] & TI_WORKSPACE);
    if ((words - at) * 4 > DVM_CODE_MAX_BYTES) return bad("segments exceed the per-launch limit");
    uint64_t tiles_total = 0;
    uint32_t wg_next = 0;       // spatial stacking: first workgroup of the next segment's share
    for (uint32_t s = 0; s < nseg; ++s) {
        if (at + SH_WORDS > words) return bad("segment header runs past the end");
        const uint32_t *sh = w + at;
        const uint32_t sw = sh[S_WORDS], cs = sh[S_CODESIZE];
        if (sw != SH_WORDS + cs || at + sw > words) return bad("segment length");
        const uint32_t G = sh[S_GEOM] & 0xFFFF, V = (sh[S_GEOM] >> 16) & 0xFF, nvec = sh[S_GEOM] >> 24;
        const uint32_t RP = sh[S_RP] & 0xFFFF, thr = sh[S_RP] >> 16;
        if (V != 4 && V != 8) return bad("chunk width");
        if (G == 0 || RP == 0 || nvec == 0) return bad("zero geometry field");
        if (G > 64 ? (G & 63) != 0 : (G & (G - 1)) != 0) return bad("lanes per row");
        if (nvec * V > (uint32_t)vr->K) return bad("chunks per lane exceed the variant");
        if (thr != G * RP || thr > block || (thr & 63)) return bad("segment threads");
        if (G > 1024) return bad("row group larger than a workgroup");
        const uint32_t nct = sh[S_NCT], TC = sh[S_TC];
        if (nct == 0) return bad("column tiles");
        if (TC > G * nvec * V) return bad("tile wider than the lanes can hold");
        const uint64_t D0 = (uint64_t)sh[S_D0LO] | ((uint64_t)sh[S_D0HI] << 32);
        const uint64_t nrows = sh[S_NROWS];
        const uint64_t M = sh[S_NTILES];
        if (M != 0) {
            if ((uint64_t)nct * TC < D0) return bad("column tiles do not cover the row");
            if (nct > 1 && (uint64_t)(nct - 1) * TC >= D0) return bad("an empty column tile");
            if (sh[S_INNER] == 0 && !(sh[S_FLAGS] & SF_LONGROW) && M != ((nrows + RP - 1) / RP) * nct) return bad("tile count");
            if ((sh[S_FLAGS] & SF_LONGROW) && (M != nrows || RP != 1 || sh[S_INNER] != 0 || sh[S_PROLOG] != 0 || nct < 2 || G < 64))
                return bad("geometry of a segment over rows longer than a tile");
        }
        if (sh[S_INNER] != 0) {        // units of (outer index, column tile), `size` rows each
            if (!vr->cred) return bad("interpreter variant does not run reductions along the penultimate axis");
            if (RP > 16 || G != 64) return bad("geometry of a reduction along the penultimate axis");
            if (nrows % sh[S_INNER] != 0 || M != (nrows / sh[S_INNER]) * nct) return bad("unit count");
            if (M != 0 && (sh[S_D1] != 0 ? sh[S_D1] != sh[S_INNER] : nrows != sh[S_INNER])) return bad("reduced axis is not the fastest outer dim");
            if (sh[S_PROLOG] != 0) return bad("prologue in a segment that reduces along the penultimate axis");
            if (sh[S_EPILOG] > cs || (sh[S_EPILOG] & 3)) return bad("epilogue offset");
        } else if (sh[S_EPILOG] != 0) {
            return bad("epilogue without a reduced axis");
        }
        if (sh[S_D1] == 0 && sh[S_D2] != 0) return bad("outer dims");
        if (sh[S_D1] != 0) {
            uint32_t m, sft;
            magic_u32(sh[S_D1], &m, &sft);
            if (m != sh[S_M1] || sft != sh[S_SH1]) return bad("division constants of outer dim 1");
        }
        if (sh[S_D2] != 0) {
            uint32_t m, sft;
            magic_u32(sh[S_D2], &m, &sft);
            if (m != sh[S_M2] || sft != sh[S_SH2]) return bad("division constants of outer dim 2");
        }
        if (nct > 1 && !(sh[S_FLAGS] & SF_LONGROW)) {
            uint32_t m, sft;
            magic_u32(nct, &m, &sft);
            if (m != sh[S_NCTM] || sft != sh[S_NCTSH]) return bad("division constants of the column tiles");
        }
        uint32_t n_red_seen = 0;
        if (sh[S_PROLOG] > cs || (sh[S_PROLOG] & 3) || (sh[S_PROLOG] != 0 && nct != 1)) return bad("prologue length");
        if (kt == KT_STACK_SPATIAL) {
            if (sh[S_NWG] == 0 || sh[S_WG0] != wg_next) return bad("workgroup share of a spatially stacked segment");
            if (sh[S_NTILES] != 0) {
                if ((uint64_t)wg_next + sh[S_NWG] > w[PH_GRID]) return bad("workgroup shares exceed the grid");
                wg_next += sh[S_NWG];
            } else if (sh[S_NWG] != 1) {
                return bad("workgroup share of an empty segment");
            }
        } else if (sh[S_NWG] != 0 || sh[S_WG0] != 0) {
            return bad("workgroup share outside a spatially stacked program");
        }
        if (sh[S_PROLOGA] > sh[S_PROLOG] || (sh[S_PROLOGA] & 3)) return bad("prologue split");
        if (sh[S_PROLOGA] != sh[S_PROLOG] && sh[S_D1] == 0) return bad("reloading prologue without a second outer dim");
        bool prolog_ends_on_record = sh[S_PROLOG] == 0;
        bool prolog_a_ends_on_record = sh[S_PROLOGA] == 0;
        bool epilog_on_record = sh[S_INNER] == 0 || sh[S_EPILOG] == 0;
        const uint32_t tbase = sh[S_TBASE], nt = sh[S_NTENS];
        if ((uint64_t)tbase + nt > ntens) return bad("segment tensor range");
        if (sh[S_FLAGS] & (SF_SYNC_WG | SF_SYNC_GRID | SF_NEW_LAUNCH)) {
            if (kt != KT_STACK || s == 0) return bad("synchronisation point outside a temporally stacked program, or on its first segment");
            if ((sh[S_FLAGS] & SF_SYNC_GRID) && !has_ws) return bad("grid-wide synchronisation without a workspace");
        }
        tiles_total += M;
        // body
        uint32_t lds_seen = 0, lds_at[LDS_SLOTS] = {0, 0, 0, 0};
        bool lds_bf16[LDS_SLOTS] = {false, false, false, false}, lds_last_sync = false;
        size_t pc = at + SH_WORDS;
        const size_t end = pc + cs;
        while (pc < end) {
            const uint32_t x = w[pc];
            const uint32_t op = x & 0xFF, l = (x >> 8) & 0xFF, a = (x >> 16) & 0xFF, bb = x >> 24;
            if ((l != LEN_REC && l != LEN_VLOAD) || pc + l > end) return bad("instruction length");
            if (pc + l == at + SH_WORDS + sh[S_PROLOG]) prolog_ends_on_record = true;
            if (pc + l == at + SH_WORDS + sh[S_PROLOGA]) prolog_a_ends_on_record = true;
            if (pc + l == at + SH_WORDS + sh[S_EPILOG]) epilog_on_record = true;
            if (pc < at + SH_WORDS + sh[S_PROLOG] && op != I_LOAD && op != I_VLOAD && op != I_LDSCOPY) return bad("prologue holds loads only");
            uint32_t want = LEN_REC;
            switch (op) {
                case I_LOAD: case I_VLOAD: case I_STORE: case I_VSTORE: {
                    want = (op == I_LOAD || op == I_STORE) ? LEN_LOAD : LEN_VLOAD;
                    if (l != want) return bad("memory instruction length");
                    if (a != SRC_ACC && !reg_ok(a, vr)) return bad("tile register index");
                    if ((op == I_LOAD || op == I_VLOAD) ? bb != B_NONE : (bb > (uint32_t)NS || (bb != 0 && a != SRC_ACC)))
                        return bad("combine op");
                    const uint32_t w1 = w[pc + 1];
                    if ((w1 & 0xFF) >= nt) return bad("tensor index");
                    const uint32_t info = w[PH_WORDS_N + (tbase + (w1 & 0xFF)) * TT_WORDS + TT_INFO];
                    if (((w1 >> 8) & 0xFF) != (info & 0xFF)) return bad("dtype differs from the tensor table");
                    if ((op == I_STORE || op == I_VSTORE) && !((info >> 8) & 1)) return bad("store to an input tensor");
                    if (((w1 >> 8) & 0xFF) == DVM_BF16 && V != 8) return bad("bf16 tile with 4-element chunks");
                    if ((w1 >> 16) & ~MF_STREAM) return bad("memory flags");
                    if (((w1 >> 16) & MF_STREAM) && op != I_LOAD && op != I_VLOAD) return bad("stream hint on a store");
                    break;
                }
                case I_LOADS: case I_STORES: {
                    want = LEN_VLOAD;
                    if (l != want) return bad("memory instruction length");
                    if (!sreg_ok(a)) return bad("row register index");
                    const uint32_t w1 = w[pc + 1];
                    if ((w1 & 0xFF) >= nt) return bad("tensor index");
                    const uint32_t info = w[PH_WORDS_N + (tbase + (w1 & 0xFF)) * TT_WORDS + TT_INFO];
                    if (((w1 >> 8) & 0xFF) != (info & 0xFF)) return bad("dtype differs from the tensor table");
                    if (op == I_STORES && !((info >> 8) & 1)) return bad("store to an input tensor");
                    break;
                }
                case I_MOVRA: case I_MOVAR:
                    if (l != LEN_REC || !reg_ok(a, vr)) return bad("move");
                    break;
                case I_UN:
                    if (l != LEN_REC || bb == 0 || bb >= U_COUNT) return bad("unary op");
                    break;
                case I_BIN:
                    if (bb >= B_COUNT || (bb == B_NONE && a < SRC_S0)) return bad("binary op");
                    if (l != LEN_REC) return bad("binary op length");
                    if (!(a == SRC_IMM || a == SRC_ACC || reg_ok(a, vr) || (a >= SRC_S0 && sreg_ok(a - SRC_S0)))) return bad("binary source");
                    break;
                case I_SEL:
                    if (l != LEN_REC || !reg_ok(a, vr) || !reg_ok(bb, vr)) return bad("select");
                    break;
                case I_FMA:
                    if (l != LEN_REC || !reg_ok(a, vr) || !(reg_ok(bb, vr) || bb == FMA_NO_ADDEND)) return bad("fused multiply-add");
                    if (w[pc + 1] > (uint32_t)NS || (w[pc + 1] == 0 && bb == FMA_NO_ADDEND)) return bad("fused multiply-add scalar");
                    break;
                case I_RED:
                    ++n_red_seen;
                    if (l != LEN_REC || !sreg_ok(a) || bb >= R_COUNT) return bad("reduction");
                    if (w[pc + 1] >= U_COUNT) return bad("reduction post op");
                    break;
                case I_SOP: {
                    if (l != LEN_SOP || !sreg_ok(a) || !sreg_ok(bb)) return bad("row-scalar op");
                    const uint32_t w1 = w[pc + 1];
                    const uint32_t kind = w1 & 0xFF, srck = (w1 >> 8) & 0xFF, c = (w1 >> 16) & 0xFF;
                    if (kind >= SOP_UNARY ? (kind - SOP_UNARY == 0 || kind - SOP_UNARY >= U_COUNT) : (kind == 0 || kind >= B_COUNT)) return bad("row-scalar op kind");
                    if (srck > 1 || (srck == 0 && !sreg_ok(c))) return bad("row-scalar source");
                    break;
                }
                case I_CACC:
                    if (l != LEN_REC || !reg_ok(a, vr) || bb > R_MIN) return bad("accumulate");
                    if (sh[S_INNER] == 0 || pc >= at + SH_WORDS + sh[S_EPILOG]) return bad("accumulate outside the per-row part of a reducing segment");
                    if (sh[S_FLAGS] & SF_CSTREAM) return bad("per-row accumulate in a segment marked as streaming reductions only");
                    break;
                case I_CSTREAM: {
                    if (l != LEN_VLOAD || !reg_ok(a, vr) || bb > R_MIN) return bad("streaming reduction");
                    if (vr->K > 8) return bad("streaming reduction in a variant that does not run it");
                    if (sh[S_INNER] == 0 || !(sh[S_FLAGS] & SF_CSTREAM) || pc >= at + SH_WORDS + sh[S_EPILOG])
                        return bad("streaming reduction outside the per-row part of a segment marked for it");
                    const uint32_t w1 = w[pc + 1];
                    if ((w1 & 0xFF) >= nt) return bad("tensor index");
                    const uint32_t info = w[PH_WORDS_N + (tbase + (w1 & 0xFF)) * TT_WORDS + TT_INFO];
                    if (((w1 >> 8) & 0xFF) != (info & 0xFF)) return bad("dtype differs from the tensor table");
                    if (((w1 >> 8) & 0xFF) == DVM_BF16 && V != 8) return bad("bf16 tile with 4-element chunks");
                    if ((w1 >> 16) & ~MF_STREAM) return bad("memory flags");
                    break;
                }
                case I_CCOMB:
                    if (l != LEN_REC || !reg_ok(a, vr) || bb > R_MIN) return bad("combine");
                    if (sh[S_INNER] == 0 || pc < at + SH_WORDS + sh[S_EPILOG]) return bad("combine outside the epilogue of a reducing segment");
                    break;
                case I_LDSCOPY: {
                    if (l != LEN_REC || a >= (uint32_t)LDS_SLOTS || bb > 1) return bad("LDS copy");
                    if (pc >= at + SH_WORDS + sh[S_PROLOGA] || !(sh[S_FLAGS] & SF_LDS) || sh[S_INNER] != 0) return bad("LDS copy outside the once-per-workgroup prologue");
                    const uint32_t w1 = w[pc + 1];
                    if ((w1 & 0xFF) >= nt || (w1 >> 16) != 0) return bad("tensor index");
                    const uint32_t info = w[PH_WORDS_N + (tbase + (w1 & 0xFF)) * TT_WORDS + TT_INFO];
                    if (((w1 >> 8) & 0xFF) != (info & 0xFF)) return bad("dtype differs from the tensor table");
                    const uint32_t es = (info & 0xFF) == DVM_F32 ? 4 : 2;
                    const uint64_t need = (D0 + V - 1) / V * V * es;
                    if ((w[pc + 3] & 15) || w[pc + 3] < need || (w[pc + 2] & 15) || (uint64_t)w[pc + 2] + w[pc + 3] > LDS_IMAGE_MAX_BYTES)
                        return bad("LDS image extent");
                    if (lds_seen & (1u << a)) return bad("LDS image copied twice");
                    lds_seen |= 1u << a;
                    lds_at[a] = w[pc + 2];
                    lds_bf16[a] = (info & 0xFF) == DVM_BF16;
                    lds_last_sync = bb != 0;
                    break;
                }
                case I_LFMA: {
                    const uint32_t la = a & 0xF, lb = a >> 4;
                    if (l != LEN_REC || (la == LFMA_NONE && lb == LFMA_NONE) || bb > 3) return bad("LDS multiply-add");
                    if (pc < at + SH_WORDS + sh[S_PROLOG]) return bad("LDS multiply-add in the prologue");
                    if (la != LFMA_NONE && (la >= (uint32_t)LDS_SLOTS || !(lds_seen & (1u << la)) || w[pc + 2] != lds_at[la] || ((bb & 1u) != 0) != lds_bf16[la])) return bad("LDS multiplier");
                    if (lb != LFMA_NONE && (lb >= (uint32_t)LDS_SLOTS || !(lds_seen & (1u << lb)) || w[pc + 3] != lds_at[lb] || ((bb & 2u) != 0) != lds_bf16[lb])) return bad("LDS addend");
                    if (w[pc + 1] > (uint32_t)NS) return bad("LDS multiply-add scalar");
                    if (!lds_last_sync) return bad("LDS images used without a synchronisation after the last copy");
                    break;
                }
                case I_NOP:
                    if (l != LEN_REC) return bad("nop");
                    break;
                default: return bad("unknown instruction id");
            }
            pc += l;
        }
        if (((sh[S_FLAGS] & SF_LDS) != 0) != (lds_seen != 0)) return bad("LDS flag does not match the prologue");
        if ((sh[S_FLAGS] & SF_LONGROW) && (sh[S_NCTSH] != n_red_seen || n_red_seen == 0)) return bad("reduction count of a segment over rows longer than a tile");
        if (!prolog_ends_on_record || !prolog_a_ends_on_record) return bad("prologue does not end on a record boundary");
        if (!epilog_on_record) return bad("epilogue does not start on a record boundary");
        at += sw;
    }
    if (at != words) return bad("trailing words after the last segment");
    if (tiles_total != 0 && w[PH_GRID] == 0) return bad("zero grid for a non-empty program");
    if (w[PH_GRID] > 65535u * 16) return bad("grid too large");
    return DVM_OK;
}

extern "C" int dvm_code_info_get(const void *bytecode, size_t len, dvm_code_info *info) {
    if (!info) return dvm_set_error(DVM_E_ARGS, "dvm_code_info_get: null info");
    int st = dvm_validate(bytecode, len);
    if (st != DVM_OK) return st;
    const uint32_t *w = (const uint32_t *)bytecode;
    memset(info, 0, sizeof(*info));
    info->kernel_type = (int32_t)(w[PH_TYPE] & 0xFFFF);
    info->n_segments = (int32_t)w[PH_NSEG];
    info->n_tensors = (int32_t)w[PH_NTENS];
    info->grid = (int32_t)w[PH_GRID];
    info->block = (int32_t)w[PH_BLOCK];
    info->variant_k = (int32_t)(w[PH_VARIANT] & 0xFF);
    info->variant_nr = (int32_t)((w[PH_VARIANT] >> 8) & 0xFF);
    size_t at = PH_WORDS_N + (size_t)w[PH_NTENS] * TT_WORDS;
    info->n_launches = 1;
    for (uint32_t s = 0; s < w[PH_NSEG]; ++s) {
        const uint32_t *sh = w + at;
        if (sh[S_FLAGS] & SF_NEW_LAUNCH) info->n_launches++;
        info->n_tiles += sh[S_NTILES];
        info->code_bytes += (int64_t)sh[S_CODESIZE] * 4;
        size_t pc = at + SH_WORDS;
        const size_t end = pc + sh[S_CODESIZE];
        while (pc < end) { info->n_instructions++; pc += (w[pc] >> 8) & 0xFF; }
        at += sh[S_WORDS];
    }
    return DVM_OK;
}

extern "C" int dvm_code_tensor(const void *bytecode, size_t len, int index, int64_t *min_bytes, int *is_output,
                               int *dtype, int *align_bytes) {
    int st = dvm_validate(bytecode, len);
    if (st != DVM_OK) return st;
    const uint32_t *w = (const uint32_t *)bytecode;
    if (index < 0 || (uint32_t)index >= w[PH_NTENS]) return dvm_set_error(DVM_E_ARGS, "dvm_code_tensor: index");
    const uint32_t *tt = w + PH_WORDS_N + index * TT_WORDS;
    if (min_bytes) *min_bytes = (int64_t)((uint64_t)tt[TT_BYTES_LO] | ((uint64_t)tt[TT_BYTES_HI] << 32));
    if (is_output) *is_output = (tt[TT_INFO] & TI_WORKSPACE) ? 2 : (int)((tt[TT_INFO] >> 8) & 1);
    if (dtype) *dtype = (int)(tt[TT_INFO] & 0xFF);
    if (align_bytes) *align_bytes = 1 << ((tt[TT_INFO] >> 16) & 0xFF);
    return DVM_OK;
}

namespace {

// Does every record of segment `sh` that names its tensor `t` address it row by row with the flat row index
// (the short memory record, or a row-scalar record with one stride) and row stride `*s1`?  (*s1 < 0: take it
// from the first such record.)  False if a record uses another form.
bool rows_addressed_flat(const uint32_t *sh, uint32_t t, int64_t *s1) {
    for (uint32_t pc = SH_WORDS; pc < sh[S_WORDS]; pc += (sh[pc] >> 8) & 0xFF) {
        const uint32_t op = sh[pc] & 0xFF;
        const bool mem = op == I_LOAD || op == I_STORE, view = op == I_VLOAD || op == I_VSTORE || op == I_CSTREAM;
        const bool rowv = op == I_LOADS || op == I_STORES;
        if (!(mem || view || rowv) || (sh[pc + 1] & 0xFF) != t) continue;
        if (view) return false;
        const int64_t st = (int64_t)((uint64_t)sh[pc + 2] | ((uint64_t)sh[pc + 3] << 32));
        if (rowv && (sh[pc + 4] | sh[pc + 5] | sh[pc + 6] | sh[pc + 7]) != 0) return false;
        if (*s1 < 0) *s1 = st;
        if (st != *s1) return false;
    }
    return true;
}

// Producer segment A (its tensor ta) and consumer segment B (its tensor tb, the same buffer): does every
// workgroup of the launch touch in B only rows of the buffer that it touched itself in A?  True when both
// segments deal the same rows and columns to the same tiles (equal row count, rows per tile, column tiles and
// tile width, the same assignment of tiles to workgroups, no outer dims) and both address the buffer by the
// flat row index.
bool same_rows_per_workgroup(const uint32_t *A, uint32_t ta, const uint32_t *B, uint32_t tb) {
    if (A[S_INNER] != 0 || B[S_INNER] != 0 || A[S_NCT] != B[S_NCT] || (A[S_NCT] != 1 && A[S_TC] != B[S_TC])) return false;
    if (A[S_NROWS] != B[S_NROWS] || (A[S_RP] & 0xFFFF) != (B[S_RP] & 0xFFFF) || A[S_NTILES] != B[S_NTILES]) return false;
    if (A[S_D1] != 0 || B[S_D1] != 0) return false;
    if ((A[S_FLAGS] & SF_INTERLEAVED) != (B[S_FLAGS] & SF_INTERLEAVED)) return false;
    int64_t s1 = -1;
    return rows_addressed_flat(A, ta, &s1) && rows_addressed_flat(B, tb, &s1);
}

}  // namespace

static int stack_impl(const void *const *codes, const size_t *lens, int n, const int *same_as, int n_same_as, void *out, size_t cap,
                      size_t *len, bool spatial, bool by_launch) {
    if (!codes || !lens || !len || n < 1) return dvm_set_error(DVM_E_ARGS, "dvm_stack: bad argument");
    size_t seg_words = 0;
    uint32_t ntens = 0, nseg = 0, block = 0, K = 0, NR = 0;
    bool need_cred = false, need_cstream = false;   // (streaming reductions run in the variants with at most 8 elements per lane)
    uint64_t grid = 0;
    for (int i = 0; i < n; ++i) {
        int st = dvm_validate(codes[i], lens[i]);
        if (st != DVM_OK) return st;
        const uint32_t *w = (const uint32_t *)codes[i];
        const uint32_t off = PH_WORDS_N + w[PH_NTENS] * TT_WORDS;
        seg_words += w[PH_WORDS] - off;
        ntens += w[PH_NTENS];
        nseg += w[PH_NSEG];
        if (w[PH_BLOCK] > block) block = w[PH_BLOCK];
        if ((w[PH_VARIANT] & 0xFF) > K) K = w[PH_VARIANT] & 0xFF;
        {   // tile registers the part uses (recorded beside its variant; bytecode without the note: its variant's)
            const uint32_t noted = (w[PH_VARIANT] >> 16) & 0xFF;
            const uint32_t need = noted != 0 ? noted - 1 : (w[PH_VARIANT] >> 8) & 0xFF;
            if (need > NR) NR = need;
        }
        for (uint32_t s = 0, at = off; s < w[PH_NSEG]; ++s) {      // (a part that reduces along the penultimate axis)
            need_cred |= w[at + S_INNER] != 0;
            need_cstream |= (w[at + S_FLAGS] & SF_CSTREAM) != 0;
            at += w[at + S_WORDS];
        }
        // every part was planned to fill the machine with workgroups of its own size: what carries
        // over to the common workgroup size is the number of resident waves, not of workgroups
        const uint64_t part_waves = (uint64_t)w[PH_GRID] * ((w[PH_BLOCK] + 63) / 64);
        if (part_waves > grid) grid = part_waves;
    }
    grid = grid / ((block + 63) / 64);
    if (grid == 0 && nseg > 0) grid = 1;
    if (same_as && (uint32_t)n_same_as != ntens) return dvm_set_error(DVM_E_ARGS, "dvm_stack_dependent: one same_as entry per tensor of the launch");
    for (uint32_t t = 0; same_as && t < ntens; ++t)
        if (same_as[t] < -1 || same_as[t] >= (int)t) return dvm_set_error(DVM_E_ARGS, "dvm_stack_dependent: same_as names an earlier entry, or -1");
    if (ntens > DVM_MAX_TENSORS) return dvm_set_error(DVM_E_LIMIT, "dvm_stack: too many tensors for one launch");
    if (nseg > 64) return dvm_set_error(DVM_E_LIMIT, "dvm_stack: too many segments");
    if (seg_words * 4 > DVM_CODE_MAX_BYTES) return dvm_set_error(DVM_E_LIMIT, "dvm_stack: bytecode exceeds the per-launch limit");
    // the stacked launch runs one interpreter variant: the smallest one that holds every part
    const Variant *vr = nullptr;
    for (int i = 0; i < N_VARIANTS; ++i) {
        const Variant &v = VARIANTS[i];
        if ((uint32_t)v.K >= K && (uint32_t)v.NR >= NR && (uint32_t)v.max_threads >= block && (v.cred || !need_cred) && (v.K <= 8 || !need_cstream)) {
            if (!vr || v.K < vr->K || (v.K == vr->K && v.NR < vr->NR)) vr = &v;
        }
    }
    if (!vr) return dvm_set_error(DVM_E_UNSUPPORTED, "dvm_stack: no interpreter variant fits all parts");
    // (a dependent stack may need the workspace entry: reserve its place, drop it again if no segment waits grid-wide)
    const uint32_t ntens_parts = ntens;
    if (same_as) {
        if (ntens + 1 > DVM_MAX_TENSORS) return dvm_set_error(DVM_E_LIMIT, "dvm_stack_dependent: too many tensors for one launch");
        for (int i = 0; i < n; ++i)
            if (((const uint32_t *)codes[i])[PH_NTENS] > 0 &&
                (((const uint32_t *)codes[i])[PH_WORDS_N + (((const uint32_t *)codes[i])[PH_NTENS] - 1) * TT_WORDS + TT_INFO] & TI_WORKSPACE))
                return dvm_set_error(DVM_E_UNSUPPORTED, "dvm_stack_dependent: a part is itself a dependent stack");
        ++ntens;
    }
    size_t words = PH_WORDS_N + (size_t)ntens * TT_WORDS + seg_words;
    *len = words * 4;
    if (!out || cap < words * 4) return dvm_set_error(DVM_E_BUFSZ, "dvm_stack: buffer too small");
    uint32_t *w = (uint32_t *)out;
    memset(w, 0, words * 4);
    w[PH_MAGIC] = MAGIC;
    w[PH_TYPE] = (spatial ? KT_STACK_SPATIAL : KT_STACK) | (VERSION << 16);
    w[PH_WORDS] = (uint32_t)words;
    w[PH_NSEG] = nseg;
    w[PH_BLOCK] = block;
    w[PH_GRID] = (uint32_t)grid;
    w[PH_VARIANT] = (uint32_t)vr->K | ((uint32_t)vr->NR << 8) | ((NR + 1) << 16);
    w[PH_NTENS] = ntens;
    uint32_t *tt = w + PH_WORDS_N;
    uint32_t *sg = w + PH_WORDS_N + ntens * TT_WORDS;
    uint32_t tbase = 0;
    for (int i = 0; i < n; ++i) {
        const uint32_t *c = (const uint32_t *)codes[i];
        const uint32_t nt = c[PH_NTENS];
        memcpy(tt, c + PH_WORDS_N, (size_t)nt * TT_WORDS * 4);
        tt += nt * TT_WORDS;
        const uint32_t off = PH_WORDS_N + nt * TT_WORDS;
        const uint32_t sw = c[PH_WORDS] - off;
        memcpy(sg, c + off, (size_t)sw * 4);
        // rebase the tensor indices of the copied segments, and re-tile row-mode segments to the
        // launch's workgroup size: a part planned for fewer threads takes more rows per tile
        // instead of leaving the other threads of the common workgroup idle
        uint32_t at = 0;
        for (uint32_t s = 0; s < c[PH_NSEG]; ++s) {
            uint32_t *sh = sg + at;
            sh[S_TBASE] += tbase;
            const uint32_t G = sh[S_GEOM] & 0xFFFF, RP = sh[S_RP] & 0xFFFF;
            if (sh[S_NCT] == 1 && G <= block && sh[S_NROWS] > 0 && sh[S_INNER] == 0) {
                const uint32_t rp_new = block / G;
                if (rp_new > RP && rp_new <= 0xFFFF) {
                    sh[S_RP] = rp_new | ((rp_new * G) << 16);
                    sh[S_NTILES] = (sh[S_NROWS] + rp_new - 1) / rp_new;
                }
            }
            at += sh[S_WORDS];
        }
        sg += sw;
        tbase += nt;
    }
    if (same_as) {
        // Dependences between the parts follow from the buffers they share: a part that touches a buffer an
        // earlier part wrote (or writes one an earlier part read) starts behind a synchronisation point.
        uint32_t *tt0 = w + PH_WORDS_N;
        uint32_t *seg_of_part[64];          // first segment of every part
        uint32_t part_of[DVM_MAX_TENSORS], local_of[DVM_MAX_TENSORS], root[DVM_MAX_TENSORS];
        uint32_t nsegs_of_part[64];
        {
            uint32_t t = 0, at = PH_WORDS_N + ntens * TT_WORDS;
            for (int i = 0; i < n; ++i) {
                const uint32_t *c = (const uint32_t *)codes[i];
                seg_of_part[i] = w + at;
                nsegs_of_part[i] = c[PH_NSEG];
                for (uint32_t k = 0; k < c[PH_NTENS]; ++k, ++t) { part_of[t] = (uint32_t)i; local_of[t] = k; }
                for (uint32_t sgi = 0; sgi < c[PH_NSEG]; ++sgi) at += w[at + S_WORDS];
            }
        }
        for (uint32_t t = 0; t < ntens_parts; ++t) {
            root[t] = same_as[t] < 0 ? t : root[same_as[t]];
            if (same_as[t] >= 0) {
                if ((tt0[t * TT_WORDS + TT_INFO] & 0xFF) != (tt0[root[t] * TT_WORDS + TT_INFO] & 0xFF))
                    return dvm_set_error(DVM_E_DTYPE, "dvm_stack_dependent: entries named as the same buffer differ in dtype");
                tt0[t * TT_WORDS + TT_INFO] |= (uint32_t)(same_as[t] + 1) << 24;
            }
        }
        bool any_grid = false;
        for (uint32_t t = 0; t < ntens_parts; ++t) {
            if (same_as[t] < 0) continue;
            const uint32_t pi = part_of[t];
            for (uint32_t u = 0; u < t; ++u) {
                if (root[u] != root[t] || part_of[u] >= pi) continue;
                const bool wu = (tt0[u * TT_WORDS + TT_INFO] & TI_OUTPUT) != 0, wt = (tt0[t * TT_WORDS + TT_INFO] & TI_OUTPUT) != 0;
                if (!wu && !wt) continue;           // both parts only read it
                uint32_t *cons = seg_of_part[pi];
                const uint32_t *prod = seg_of_part[part_of[u]];
                const bool aligned = nsegs_of_part[pi] == 1 && nsegs_of_part[part_of[u]] == 1 &&
                                     same_rows_per_workgroup(prod, local_of[u], cons, local_of[t]);
                cons[S_FLAGS] |= aligned ? SF_SYNC_WG : (by_launch ? SF_NEW_LAUNCH : SF_SYNC_GRID);
            }
        }
        for (int i = 0; i < n; ++i) {
            uint32_t *sh = seg_of_part[i];
            if (sh[S_FLAGS] & SF_SYNC_GRID) { sh[S_FLAGS] &= ~SF_SYNC_WG; any_grid = true; }
            if (sh[S_FLAGS] & SF_NEW_LAUNCH) sh[S_FLAGS] &= ~SF_SYNC_WG;
            // (a segment that only waits for its own workgroup relies on the producer having run in the same launch
            // with the same tiles per workgroup: true across a launch boundary too -- the tiles are dealt out alike --
            // and everything before a boundary is complete anyway)
        }
        if (any_grid) {
            uint32_t *te = tt0 + ntens_parts * TT_WORDS;
            te[TT_INFO] = (uint32_t)DVM_F32 | TI_WORKSPACE | (8u << 16);
            te[TT_BYTES_LO] = DVM_WORKSPACE_BYTES;
            te[TT_BYTES_HI] = 0;
        } else {
            // no workspace after all: close the gap its table entry left
            memmove(tt0 + ntens_parts * TT_WORDS, tt0 + ntens * TT_WORDS, seg_words * 4);
            --ntens;
            words -= TT_WORDS;
            w[PH_WORDS] = (uint32_t)words;
            w[PH_NTENS] = ntens;
            *len = words * 4;
        }
    }
    if (spatial) {
        // Spatial stacking (Section 5.1): the segments run side by side, each on a share of the workgroups
        // in proportion to its estimated run time, at least one and at most one per tile.
        uint32_t *seg[64];
        double cost[64];
        uint32_t share[64];
        uint32_t ns = 0, at = PH_WORDS_N + ntens * TT_WORDS;
        double total = 0;
        for (uint32_t k = 0; k < nseg; ++k) {
            uint32_t *sh = w + at;
            seg[ns] = sh;
            double c = 0;
            for (uint32_t t = 0; t < sh[S_NTENS]; ++t) {
                const uint32_t *te = w + PH_WORDS_N + (sh[S_TBASE] + t) * TT_WORDS;
                c += (double)((uint64_t)te[TT_BYTES_LO] | ((uint64_t)te[TT_BYTES_HI] << 32));
            }
            // time of a part ~ tiles * (interpreted records + bytes per tile / 2 KiB): short tiles are bound by
            // the per-record work of the interpreter, long ones by memory
            uint32_t n_rec = 0;
            for (uint32_t pc = SH_WORDS + sh[S_PROLOG]; pc < sh[S_WORDS]; pc += (sh[pc] >> 8) & 0xFF) ++n_rec;
            // (a unit of a segment that reduces along the penultimate axis runs its per-row records once per step)
            const double steps = sh[S_INNER] != 0 ? (double)((sh[S_INNER] + (sh[S_RP] & 0xFFFF) - 1) / (sh[S_RP] & 0xFFFF)) : 1.0;
            c = (double)sh[S_NTILES] * steps * n_rec + c / 2048.0;
            if (sh[S_NTILES] == 0) c = 0;
            cost[ns] = c;
            total += c;
            ++ns;
            at += sh[S_WORDS];
        }
        uint32_t live = 0;
        for (uint32_t k = 0; k < ns; ++k) live += seg[k][S_NTILES] != 0;
        if (live > grid) return dvm_set_error(DVM_E_UNSUPPORTED, "dvm_stack_spatial: more non-empty parts than resident workgroups");
        uint32_t used = 0;
        for (uint32_t k = 0; k < ns; ++k) {
            uint32_t sh_k = 0;
            if (seg[k][S_NTILES] != 0) {
                sh_k = total > 0 ? (uint32_t)((double)grid * cost[k] / total) : 1;
                if (sh_k < 1) sh_k = 1;
                if (sh_k > seg[k][S_NTILES]) sh_k = seg[k][S_NTILES];
            }
            share[k] = sh_k;
            used += sh_k;
        }
        // rounding may overshoot (minimum of one each) or leave workgroups over: trim from / add to the largest shares
        while (used > grid) {
            uint32_t best = 0;
            for (uint32_t k = 1; k < ns; ++k) if (share[k] > share[best]) best = k;
            --share[best];
            --used;
        }
        for (bool grew = true; used < grid && grew;) {
            grew = false;
            for (uint32_t k = 0; k < ns && used < grid; ++k)
                if (share[k] != 0 && share[k] < seg[k][S_NTILES] && cost[k] * grid >= total * share[k]) { ++share[k]; ++used; grew = true; }
        }
        uint32_t wg0 = 0;
        for (uint32_t k = 0; k < ns; ++k) {
            seg[k][S_WG0] = wg0;
            seg[k][S_NWG] = share[k] ? share[k] : 1;       // an empty segment is skipped by its (zero) tile count anyway
            wg0 += share[k];
        }
        w[PH_GRID] = wg0 ? wg0 : 1;
    }
    return dvm_validate(out, words * 4);
}

extern "C" int dvm_stack(const void *const *codes, const size_t *lens, int n, void *out, size_t cap, size_t *len) {
    return stack_impl(codes, lens, n, nullptr, 0, out, cap, len, false);
}

extern "C" int dvm_stack_dependent(const void *const *codes, const size_t *lens, int n, const int *same_as, int n_same_as, int order_by,
                                   void *out, size_t cap, size_t *len) {
    if (!same_as) return dvm_set_error(DVM_E_ARGS, "dvm_stack_dependent: null same_as");
    if (order_by != DVM_ORDER_IN_KERNEL && order_by != DVM_ORDER_BY_LAUNCH) return dvm_set_error(DVM_E_ARGS, "dvm_stack_dependent: order_by");
    return stack_impl(codes, lens, n, same_as, n_same_as, out, cap, len, false, order_by == DVM_ORDER_BY_LAUNCH);
}

extern "C" int dvm_stack_spatial(const void *const *codes, const size_t *lens, int n, void *out, size_t cap, size_t *len) {
    for (int i = 0; codes && lens && i < n; ++i) {
        if (dvm_validate(codes[i], lens[i]) == DVM_OK && (((const uint32_t *)codes[i])[PH_TYPE] & 0xFFFF) != KT_META)
            return dvm_set_error(DVM_E_UNSUPPORTED, "dvm_stack_spatial: parts must be single meta-kernels");
    }
    return stack_impl(codes, lens, n, nullptr, 0, out, cap, len, true);
}

namespace {

const char *const UN_NAMES[] = {"none", "sqrt", "abs", "log", "exp", "round", "floor", "isfinite", "neg", "rsqrt", "rcp",
                                "tanh", "erf", "sigmoid", "square", "gelu_tanh", "gelu_erf", "silu", "cast_bf16"};
const char *const BIN_NAMES[] = {"mov", "add", "sub", "rsub", "mul", "div", "rdiv", "min", "max", "pow", "rpow",
                                 "cmp_eq", "cmp_ne", "cmp_lt", "cmp_le", "cmp_gt", "cmp_ge", "expsub", "rexpsub"};
const char *const RED_NAMES[] = {"sum", "max", "min", "sumsq"};

struct Out {
    char *p;
    size_t cap, n;
    void put(const char *fmt, ...) __attribute__((format(printf, 2, 3))) {
        va_list ap;
        va_start(ap, fmt);
        if (n < cap) {
            int k = vsnprintf(p + n, cap - n, fmt, ap);
            if (k > 0) n += (size_t)k;
            if (n >= cap) n = cap - 1;
        }
        va_end(ap);
    }
};

void reg_name(char *buf, uint32_t r) {
    if (r == SRC_ACC) snprintf(buf, 8, "acc");
    else if (r == SRC_IMM) snprintf(buf, 8, "imm");
    else if (r >= SRC_S0) snprintf(buf, 8, "s%u", r - SRC_S0);
    else snprintf(buf, 8, "r%u", r);
}

}  // namespace

extern "C" int dvm_disasm(const void *bytecode, size_t len, char *txt, size_t cap) {
    if (!txt || cap == 0) return dvm_set_error(DVM_E_ARGS, "dvm_disasm: null text buffer");
    txt[0] = 0;
    int st = dvm_validate(bytecode, len);
    if (st != DVM_OK) return st;
    const uint32_t *w = (const uint32_t *)bytecode;
    Out o{txt, cap, 0};
    const uint32_t kt = w[PH_TYPE] & 0xFFFF;
    o.put("dvm program: kernel_type=%s block_dim=%u threads=%u variant=K%u/R%u segments=%u tensors=%u words=%u\n",
          kt == KT_META ? "vmain.v" : (kt == KT_STACK ? "vstack.t" : "vstack.s"), w[PH_GRID], w[PH_BLOCK], w[PH_VARIANT] & 0xFF, (w[PH_VARIANT] >> 8) & 0xFF,
          w[PH_NSEG], w[PH_NTENS], w[PH_WORDS]);
    for (uint32_t t = 0; t < w[PH_NTENS]; ++t) {
        const uint32_t *tt = w + PH_WORDS_N + t * TT_WORDS;
        o.put("  tensor %u: %s %s min_bytes=%llu", t, (tt[TT_INFO] & 0xFF) ? "bf16" : "f32",
              (tt[TT_INFO] & TI_WORKSPACE) ? "workspace" : ((tt[TT_INFO] & TI_OUTPUT) ? "out" : "in"),
              (unsigned long long)((uint64_t)tt[TT_BYTES_LO] | ((uint64_t)tt[TT_BYTES_HI] << 32)));
        if (tt[TT_INFO] >> 24) o.put(" same_buffer_as=%u", (tt[TT_INFO] >> 24) - 1);
        o.put("\n");
    }
    size_t at = PH_WORDS_N + (size_t)w[PH_NTENS] * TT_WORDS;
    for (uint32_t s = 0; s < w[PH_NSEG]; ++s) {
        const uint32_t *sh = w + at;
        const uint32_t M = sh[S_NTILES], N = w[PH_GRID];
        const uint32_t body_tile = N ? (M + N - 1) / N : 0;
        o.put("segment %u: tiles=%u body_tile=%u code_size=%u rows=%u row_len=%llu lanes_per_row=%u chunk=%u chunks_per_lane=%u "
              "rows_per_tile=%u col_tiles=%u tile_cols=%u outer=[%u,%u] tensor_base=%u tiles_to_workgroups=%s\n",
              s, M, body_tile, sh[S_CODESIZE] * 4, sh[S_NROWS],
              (unsigned long long)((uint64_t)sh[S_D0LO] | ((uint64_t)sh[S_D0HI] << 32)), sh[S_GEOM] & 0xFFFF,
              (sh[S_GEOM] >> 16) & 0xFF, sh[S_GEOM] >> 24, sh[S_RP] & 0xFFFF, sh[S_NCT], sh[S_TC], sh[S_D1], sh[S_D2], sh[S_TBASE],
              (sh[S_FLAGS] & SF_INTERLEAVED) ? "interleaved" : "blocked");
        if (sh[S_FLAGS] & SF_LONGROW) o.put("  ; rows longer than a tile: %u passes over a row, %u column tiles each\n", sh[S_NCTSH] + 1, sh[S_NCT]);
        if (sh[S_FLAGS] & SF_NEW_LAUNCH) o.put("  ; a kernel launch of its own: starts when the segments before are complete\n");
        if (sh[S_FLAGS] & SF_SYNC_GRID) o.put("  ; waits until every workgroup has finished the segments before\n");
        else if (sh[S_FLAGS] & SF_SYNC_WG) o.put("  ; waits for this workgroup's own stores of the segments before\n");
        size_t pc = at + SH_WORDS;
        const size_t end = pc + sh[S_CODESIZE];
        if (sh[S_PROLOGA]) o.put("  ; prologue (once per workgroup)\n");
        while (pc < end) {
            if (sh[S_PROLOG] && pc == at + SH_WORDS + sh[S_PROLOG]) o.put("  ; body (once per tile)\n");
            else if (sh[S_PROLOGA] != sh[S_PROLOG] && pc == at + SH_WORDS + sh[S_PROLOGA])
                o.put("  ; prologue (again whenever the second outer index changes)\n");
            if (sh[S_INNER] && pc == at + SH_WORDS + sh[S_EPILOG]) o.put("  ; epilogue (after the last of the %u rows of a unit)\n", sh[S_INNER]);
            const uint32_t x = w[pc];
            const uint32_t op = x & 0xFF, l = (x >> 8) & 0xFF, a = (x >> 16) & 0xFF, b = x >> 24;
            char ra[8], rb[8];
            reg_name(ra, a);
            reg_name(rb, b);
            auto i64 = [&](size_t i) { return (long long)((uint64_t)w[i] | ((uint64_t)w[i + 1] << 32)); };
            switch (op) {
                case I_LOAD:
                    o.put("  %04zu load    %s %s= t%u stride=%lld%s\n", pc - at - SH_WORDS, ra, b ? BIN_NAMES[b] : "", w[pc + 1] & 0xFF, i64(pc + 2),
                          ((w[pc + 1] >> 16) & MF_STREAM) ? "  [read once]" : "");
                    break;
                case I_VLOAD:
                    o.put("  %04zu viewload %s %s= t%u strides=[%lld,%lld,%lld]%s\n", pc - at - SH_WORDS, ra, b ? BIN_NAMES[b] : "",
                          w[pc + 1] & 0xFF, i64(pc + 2), i64(pc + 4), i64(pc + 6), ((w[pc + 1] >> 16) & MF_STREAM) ? "  [read once]" : "");
                    break;
                case I_STORE:
                    if (b) o.put("  %04zu store   t%u = %s * s%u stride=%lld\n", pc - at - SH_WORDS, w[pc + 1] & 0xFF, ra, b - 1, i64(pc + 2));
                    else o.put("  %04zu store   t%u = %s stride=%lld\n", pc - at - SH_WORDS, w[pc + 1] & 0xFF, ra, i64(pc + 2));
                    break;
                case I_VSTORE:
                    o.put("  %04zu viewstore t%u = %s%s strides=[%lld,%lld,%lld]\n", pc - at - SH_WORDS, w[pc + 1] & 0xFF, ra,
                          b ? " * s" : "", i64(pc + 2), i64(pc + 4), i64(pc + 6));
                    break;
                case I_LOADS:
                    o.put("  %04zu loads   s%u = t%u strides=[%lld,%lld,%lld]\n", pc - at - SH_WORDS, a, w[pc + 1] & 0xFF, i64(pc + 2),
                          i64(pc + 4), i64(pc + 6));
                    break;
                case I_STORES:
                    o.put("  %04zu stores  t%u = s%u strides=[%lld,%lld,%lld]\n", pc - at - SH_WORDS, w[pc + 1] & 0xFF, a, i64(pc + 2),
                          i64(pc + 4), i64(pc + 6));
                    break;
                case I_MOVRA: o.put("  %04zu copy    r%u = acc\n", pc - at - SH_WORDS, a); break;
                case I_MOVAR: o.put("  %04zu copy    acc = r%u\n", pc - at - SH_WORDS, a); break;
                case I_UN: o.put("  %04zu %-7s acc\n", pc - at - SH_WORDS, UN_NAMES[b]); break;
                case I_BIN:
                    if (a == SRC_IMM) o.put("  %04zu %-7s acc, %.9g\n", pc - at - SH_WORDS, BIN_NAMES[b], (double)f32_bits(w[pc + 1]));
                    else o.put("  %04zu %-7s acc, %s\n", pc - at - SH_WORDS, BIN_NAMES[b], ra);
                    break;
                case I_SEL: o.put("  %04zu select  acc = acc ? r%u : r%u\n", pc - at - SH_WORDS, a, b); break;
                case I_CSTREAM:
                    o.put("  %04zu stream.%-3s r%u = %s over this wave's rows of t%u strides=[%lld,%lld,%lld]%s\n", pc - at - SH_WORDS, RED_NAMES[b], a,
                          RED_NAMES[b], w[pc + 1] & 0xFF, i64(pc + 2), i64(pc + 4), i64(pc + 6), ((w[pc + 1] >> 16) & MF_STREAM) ? "  [read once]" : "");
                    break;
                case I_CCOMB: o.put("  %04zu comb.%-3s r%u = %s of r%u over the workgroup's waves\n", pc - at - SH_WORDS, RED_NAMES[b], a, RED_NAMES[b], a); break;
                case I_CACC: o.put("  %04zu acc.%-4s r%u = first row ? acc : %s(r%u, acc)\n", pc - at - SH_WORDS, RED_NAMES[b], a, RED_NAMES[b], a); break;
                case I_FMA: {
                    char sc[8] = "", ad[8] = "";
                    if (w[pc + 1]) snprintf(sc, sizeof sc, " * s%u", w[pc + 1] - 1);
                    if (b != FMA_NO_ADDEND) snprintf(ad, sizeof ad, " + r%u", b);
                    o.put("  %04zu fma     acc = acc%s * r%u%s\n", pc - at - SH_WORDS, sc, a, ad);
                    break;
                }
                case I_LDSCOPY:
                    o.put("  %04zu ldscopy L%u = t%u  [%u bytes of LDS at %u%s]\n", pc - at - SH_WORDS, a, w[pc + 1] & 0xFF, w[pc + 3], w[pc + 2],
                          b ? ", then workgroup sync" : "");
                    break;
                case I_LFMA: {
                    char sc[8] = "", mu[8] = "", ad[8] = "";
                    if (w[pc + 1]) snprintf(sc, sizeof sc, " * s%u", w[pc + 1] - 1);
                    if ((a & 0xF) != LFMA_NONE) snprintf(mu, sizeof mu, " * L%u", a & 0xF);
                    if ((a >> 4) != LFMA_NONE) snprintf(ad, sizeof ad, " + L%u", a >> 4);
                    o.put("  %04zu lfma    acc = acc%s%s%s\n", pc - at - SH_WORDS, sc, mu, ad);
                    break;
                }
                case I_RED:
                    o.put("  %04zu red.%-5s s%u = %s(acc * %.9g + %.9g)%s\n", pc - at - SH_WORDS, RED_NAMES[b], a,
                          w[pc + 1] ? UN_NAMES[w[pc + 1]] : "", (double)f32_bits(w[pc + 2]), (double)f32_bits(w[pc + 3]),
                          (sh[S_GEOM] & 0xFFFF) > 64 ? "  [workgroup sync]" : "");
                    break;
                case I_SOP: {
                    const uint32_t w1 = w[pc + 1];
                    const uint32_t kind = w1 & 0xFF, srck = (w1 >> 8) & 0xFF, c = (w1 >> 16) & 0xFF;
                    if (kind >= SOP_UNARY) o.put("  %04zu s.%-6s s%u = s%u\n", pc - at - SH_WORDS, UN_NAMES[kind - SOP_UNARY], a, b);
                    else if (srck == 1) o.put("  %04zu s.%-6s s%u = s%u, %.9g\n", pc - at - SH_WORDS, BIN_NAMES[kind], a, b, (double)f32_bits(w[pc + 2]));
                    else o.put("  %04zu s.%-6s s%u = s%u, s%u\n", pc - at - SH_WORDS, BIN_NAMES[kind], a, b, c);
                    break;
                }
                default: o.put("  %04zu nop\n", pc - at - SH_WORDS); break;
            }
            pc += l;
        }
        at += sh[S_WORDS];
    }
    return DVM_OK;
}
