// Streaming fuser for dynamic graphs (Section 5.2 of the paper, "dynamic graph fuser"): operators
// arrive one at a time, as an eager framework issues them; they are buffered lazily and fused as they
// arrive while their iteration spaces merge.  An operator that does not merge with the buffered ones
// cuts the buffer: it opens the next piece, and at the flush the pieces are encoded one by one and
// stacked into ONE launch, later pieces waiting for the earlier ones they read (cut-and-stack: a
// sequence that is no single meta-kernel still runs as one kernel).  The buffer runs when it is
// full or when the caller asks for a result (flush).  Values that the caller released before the flush
// and that no later piece reads are pure intermediates and never reach memory.
//
// Built on the public C ABI only (program builder, dvm_encode, dvm_stack_dependent, dvm_run): host
// code, no HIP call of its own.
#include <stdint.h>
#include <string.h>

#include <new>

#include "../../include/dvm.h"
#include "dvm_internal.h"

namespace {

constexpr int MAX_VALUES = 4096;        // values alive in one fuser (tensors + pending results)
constexpr int MAX_PENDING = 48;         // operators buffered before a forced flush
constexpr int MAX_GROUP_TENSORS = 24;   // distinct tensors (inputs + results) of one launch
constexpr int MAX_PIECES = 8;           // pieces of one launch
constexpr size_t PIECE_CODE_CAP = 4096;

struct Val {
    uint8_t used, pending, released, dtype;
    void *ptr;
    dvm_shape shape;
};

struct PendingOp {
    int opcode, n_args, n_imm;
    int args[3];
    double imm[2];
    int value;
};

}  // namespace

struct dvm_fuser {
    dvm_ctx *ctx;
    void *stream;
    Val vals[MAX_VALUES];
    int n_vals_hint;                    // search start for a free slot
    PendingOp ops[MAX_PENDING];
    int n_ops;
    int piece_lo[MAX_PIECES + 1];       // piece k holds ops [piece_lo[k], piece_lo[k + 1]); the last one is open
    int n_pieces;
    dvm_shape dom;                      // broadcast of the shapes of the results of the open piece
    void *workspace;                    // device memory lent for grid-wide waits (dvm_fuser_set_workspace), or null
    int64_t stat_ops, stat_launches, stat_flushes, stat_elided;
    unsigned char code[8192];
    size_t code_len;
    unsigned char piece_code[MAX_PIECES][PIECE_CODE_CAP];
};

namespace {

bool is_reduction(int opcode) { return opcode >= DVM_OP_SUM && opcode <= DVM_OP_MEANSQ; }

// NumPy broadcasting of b into a (right aligned); false if the shapes do not broadcast together
bool broadcast_into(dvm_shape &a, const dvm_shape &b) {
    const int r = a.rank > b.rank ? a.rank : b.rank;
    int64_t out[DVM_MAX_RANK];
    for (int k = 0; k < r; ++k) {
        const int ia = a.rank - r + k, ib = b.rank - r + k;
        const int64_t da = ia >= 0 ? a.dim[ia] : 1, db = ib >= 0 ? b.dim[ib] : 1;
        if (da == db || db == 1) out[k] = da;
        else if (da == 1) out[k] = db;
        else return false;
    }
    a.rank = r;
    for (int k = 0; k < r; ++k) a.dim[k] = out[k];
    return true;
}

int alloc_value(dvm_fuser *f) {
    for (int i = 0; i < MAX_VALUES; ++i) {
        const int k = (f->n_vals_hint + i) % MAX_VALUES;
        if (!f->vals[k].used) {
            f->n_vals_hint = k + 1;
            memset(&f->vals[k], 0, sizeof(Val));
            f->vals[k].used = 1;
            return k;
        }
    }
    return -1;
}

bool valid_value(const dvm_fuser *f, int v) { return v >= 0 && v < MAX_VALUES && f->vals[v].used; }

// Is the result of a buffered operator read by an operator at or after index `from`?
bool read_later(const dvm_fuser *f, int value, int from) {
    for (int i = from; i < f->n_ops; ++i)
        for (int a = 0; a < f->ops[i].n_args; ++a)
            if (f->ops[i].args[a] == value) return true;
    return false;
}

struct Piece {          // ops [lo, hi) as one encoded program and its tensors (inputs, then outputs)
    size_t code_len;
    int n_in, n_out;
    void *tensors[DVM_MAX_TENSORS];
    int values[DVM_MAX_TENSORS];        // the fuser value behind every tensor
};

// Encode ops [lo, hi) of the buffer as one program into `code`.  Its outputs are the results that the caller still
// references or that a later buffered operator reads; the others stay in tile registers.
int encode_range(dvm_fuser *f, int lo, int hi, unsigned char *code, size_t cap, Piece *pc) {
    dvm_prog *p = nullptr;
    int st = dvm_prog_create(&p);
    if (st != DVM_OK) return st;
    // value -> SSA id, kept sparse: the range touches at most MAX_GROUP_TENSORS + MAX_PENDING values
    int map_val[MAX_PENDING * 4 + MAX_GROUP_TENSORS], map_ssa[MAX_PENDING * 4 + MAX_GROUP_TENSORS], n_map = 0;
    auto find = [&](int v) { for (int i = 0; i < n_map; ++i) if (map_val[i] == v) return map_ssa[i]; return -1; };
    dvm_shape in_shapes[DVM_MAX_TENSORS];
    pc->n_in = pc->n_out = 0;
    pc->code_len = 0;
    // inputs: every argument that is not produced inside the range, in first-use order (a tensor, or the result
    // of an earlier piece, which is in its buffer by the time this piece runs)
    for (int i = lo; i < hi && st == DVM_OK; ++i) {
        const PendingOp &o = f->ops[i];
        for (int a = 0; a < o.n_args && st == DVM_OK; ++a) {
            const int v = o.args[a];
            bool inside = false, earlier = false;
            for (int j = lo; j < i; ++j) inside |= f->ops[j].value == v;
            for (int j = 0; j < lo; ++j) earlier |= f->ops[j].value == v;
            if (inside || find(v) >= 0) continue;
            if (f->vals[v].pending && !earlier) { st = dvm_set_error(DVM_E_STATE, "dvm_fuser: argument is neither a tensor nor buffered"); break; }
            if (pc->n_in >= DVM_MAX_TENSORS) { st = dvm_set_error(DVM_E_LIMIT, "dvm_fuser: too many tensors in one launch"); break; }
            int id = -1;
            st = dvm_prog_input(p, f->vals[v].dtype, &id);
            map_val[n_map] = v; map_ssa[n_map++] = id;
            in_shapes[pc->n_in] = f->vals[v].shape;
            pc->values[pc->n_in] = v;
            pc->tensors[pc->n_in++] = f->vals[v].ptr;
        }
    }
    for (int i = lo; i < hi && st == DVM_OK; ++i) {
        const PendingOp &o = f->ops[i];
        int ids[3] = {0, 0, 0};
        for (int a = 0; a < o.n_args; ++a) ids[a] = find(o.args[a]);
        int id = -1;
        st = dvm_prog_op(p, o.opcode, ids, o.n_args, o.imm, o.n_imm, &id);
        map_val[n_map] = o.value; map_ssa[n_map++] = id;
    }
    for (int i = lo; i < hi && st == DVM_OK; ++i) {
        const int v = f->ops[i].value;
        if (f->vals[v].released && !read_later(f, v, hi)) continue;
        if (pc->n_in + pc->n_out >= DVM_MAX_TENSORS) { st = dvm_set_error(DVM_E_LIMIT, "dvm_fuser: too many tensors in one launch"); break; }
        st = dvm_prog_output(p, find(v), f->vals[v].dtype);
        pc->values[pc->n_in + pc->n_out] = v;
        pc->tensors[pc->n_in + pc->n_out++] = f->vals[v].ptr;
    }
    if (st == DVM_OK && pc->n_out > 0) {
        st = dvm_prog_finish(p);
        dvm_shape out_shapes[DVM_MAX_TENSORS];
        if (st == DVM_OK) st = dvm_encode(f->ctx, p, in_shapes, pc->n_in, nullptr, code, cap, &pc->code_len, out_shapes);
        for (int k = 0; k < pc->n_out && st == DVM_OK; ++k) {
            const Val &v = f->vals[pc->values[pc->n_in + k]];
            if (v.shape.rank != out_shapes[k].rank || memcmp(v.shape.dim, out_shapes[k].dim, sizeof(int64_t) * v.shape.rank) != 0)
                st = dvm_set_error(DVM_E_SHAPE, "dvm_fuser: inferred shape differs from the encoder's");
        }
    }
    dvm_prog_destroy(p);
    return st;
}

// The results of ops [lo, hi) have run as one program: they are plain tensors now.  (Released ones are freed at the
// end of the flush: a later piece may still read them.)
void settle(dvm_fuser *f, int lo, int hi) {
    for (int i = lo; i < hi; ++i) {
        Val &v = f->vals[f->ops[i].value];
        v.pending = 0;
        if (v.released && !read_later(f, f->ops[i].value, hi)) ++f->stat_elided;    // it never reached memory
    }
}

// Execute ops [lo, hi) of the buffer as one launch.
int run_range(dvm_fuser *f, int lo, int hi) {
    Piece pc;
    int st = encode_range(f, lo, hi, f->code, sizeof(f->code), &pc);
    if (st != DVM_OK) return st;
    if (pc.n_out > 0) {
        f->code_len = pc.code_len;
        if (dvm_ctx_device(f->ctx) >= 0) st = dvm_run(f->ctx, f->code, f->code_len, pc.tensors, pc.n_in + pc.n_out, f->stream);
        if (st != DVM_OK) return st;
        ++f->stat_launches;
    }
    settle(f, lo, hi);
    return DVM_OK;
}

// One piece as a launch of its own; if it is no single meta-kernel after all (registers, tensor table, iteration
// space), operator by operator: every result then reaches its buffer, released or not.
int run_piece_alone(dvm_fuser *f, int lo, int hi) {
    int st = run_range(f, lo, hi);
    if (st == DVM_E_UNSUPPORTED || st == DVM_E_LIMIT || st == DVM_E_RANK) {
        for (int i = lo; i < hi; ++i) {
            Val &v = f->vals[f->ops[i].value];
            const uint8_t was_released = v.released;
            v.released = 0;
            st = run_range(f, i, i + 1);
            v.released = was_released;
            if (st != DVM_OK) break;
        }
    }
    return st;
}

// All pieces as one launch: encode each, stack them with the dependences that follow from the values they share.
// DVM_E_UNSUPPORTED / DVM_E_LIMIT / DVM_E_RANK: the caller falls back to one launch per piece.
int run_stacked(dvm_fuser *f) {
    Piece pcs[MAX_PIECES];
    const void *codes[MAX_PIECES];
    size_t lens[MAX_PIECES];
    void *tensors[DVM_MAX_TENSORS];
    int values[DVM_MAX_TENSORS], same_as[DVM_MAX_TENSORS];
    int n_parts = 0, n_t = 0, n_launches = 1;
    for (int k = 0; k < f->n_pieces; ++k) {
        Piece &pc = pcs[n_parts];
        int st = encode_range(f, f->piece_lo[k], f->piece_lo[k + 1], f->piece_code[n_parts], PIECE_CODE_CAP, &pc);
        if (st == DVM_E_BUFSZ) st = dvm_set_error(DVM_E_LIMIT, "dvm_fuser: a piece's bytecode exceeds the fuser's buffer");
        if (st != DVM_OK) return st;
        if (pc.n_out == 0) continue;        // every result released and unread: nothing to run
        if (n_t + pc.n_in + pc.n_out + 1 > DVM_MAX_TENSORS) return dvm_set_error(DVM_E_LIMIT, "dvm_fuser: too many tensors in one launch");
        for (int t = 0; t < pc.n_in + pc.n_out; ++t) {
            same_as[n_t] = -1;
            for (int u = 0; u < n_t; ++u)
                if (values[u] == pc.values[t]) { same_as[n_t] = u; break; }
            values[n_t] = pc.values[t];
            tensors[n_t++] = pc.tensors[t];
        }
        codes[n_parts] = f->piece_code[n_parts];
        lens[n_parts] = pc.code_len;
        ++n_parts;
    }
    if (n_parts > 0) {
        int st;
        if (n_parts == 1) {
            memcpy(f->code, codes[0], lens[0]);
            f->code_len = lens[0];
        } else {
            st = dvm_stack_dependent(codes, lens, n_parts, same_as, n_t, f->workspace ? DVM_ORDER_IN_KERNEL : DVM_ORDER_BY_LAUNCH, f->code,
                                     sizeof(f->code), &f->code_len);
            if (st == DVM_E_BUFSZ) st = dvm_set_error(DVM_E_LIMIT, "dvm_fuser: the stacked bytecode exceeds the fuser's buffer");
            if (st != DVM_OK) return st;
            int is_ws = 0;
            dvm_code_info info;
            st = dvm_code_info_get(f->code, f->code_len, &info);
            if (st == DVM_OK) st = dvm_code_tensor(f->code, f->code_len, info.n_tensors - 1, nullptr, &is_ws, nullptr, nullptr);
            if (st != DVM_OK) return st;
            if (is_ws == 2) tensors[n_t++] = f->workspace;
            n_launches = info.n_launches;
        }
        if (dvm_ctx_device(f->ctx) >= 0) {
            st = dvm_run(f->ctx, f->code, f->code_len, tensors, n_t, f->stream);
            if (st != DVM_OK) return st;
        }
        f->stat_launches += n_launches;
    }
    for (int k = 0; k < f->n_pieces; ++k) settle(f, f->piece_lo[k], f->piece_lo[k + 1]);
    return DVM_OK;
}

int flush_all(dvm_fuser *f) {
    if (f->n_ops == 0) return DVM_OK;
    ++f->stat_flushes;
    f->piece_lo[f->n_pieces] = f->n_ops;
    int st = f->n_pieces > 1 ? run_stacked(f) : DVM_E_UNSUPPORTED;
    if (st == DVM_E_UNSUPPORTED || st == DVM_E_LIMIT || st == DVM_E_RANK) {
        for (int k = 0; k < f->n_pieces; ++k) {
            st = run_piece_alone(f, f->piece_lo[k], f->piece_lo[k + 1]);
            if (st != DVM_OK) break;
        }
    }
    if (st == DVM_OK) {
        for (int i = 0; i < f->n_ops; ++i) {
            Val &v = f->vals[f->ops[i].value];
            if (v.released) v.used = 0;
        }
    }
    f->n_ops = 0;
    f->n_pieces = 1;
    f->piece_lo[0] = 0;
    f->dom.rank = 0;
    return st;
}

}  // namespace

extern "C" int dvm_fuser_create(dvm_ctx *ctx, void *hip_stream, dvm_fuser **out) {
    if (!ctx || !out) return dvm_set_error(DVM_E_ARGS, "dvm_fuser_create: null argument");
    dvm_fuser *f = new (std::nothrow) dvm_fuser;
    if (!f) return dvm_set_error(DVM_E_LIMIT, "out of memory");
    memset(f, 0, sizeof(*f));
    f->ctx = ctx;
    f->stream = hip_stream;
    f->n_pieces = 1;
    *out = f;
    return DVM_OK;
}

extern "C" void dvm_fuser_destroy(dvm_fuser *f) { delete f; }

extern "C" int dvm_fuser_tensor(dvm_fuser *f, void *device_ptr, int dtype, const dvm_shape *shape, int *value) {
    if (!f || !shape || !value) return dvm_set_error(DVM_E_ARGS, "dvm_fuser_tensor: null argument");
    if (dtype != DVM_F32 && dtype != DVM_BF16) return dvm_set_error(DVM_E_DTYPE, "dvm_fuser_tensor: dtype");
    if (shape->rank < 0 || shape->rank > DVM_MAX_RANK) return dvm_set_error(DVM_E_RANK, "dvm_fuser_tensor: rank");
    const int v = alloc_value(f);
    if (v < 0) return dvm_set_error(DVM_E_LIMIT, "dvm_fuser: too many live values");
    f->vals[v].ptr = device_ptr;
    f->vals[v].dtype = (uint8_t)dtype;
    f->vals[v].shape = *shape;
    *value = v;
    return DVM_OK;
}

extern "C" int dvm_fuser_op(dvm_fuser *f, int opcode, const int *args, int n_args, const double *imm, int n_imm,
                            int out_dtype, void *out_ptr, int *value) {
    if (!f || !args || !value || n_args < 1 || n_args > 3 || n_imm < 0 || n_imm > 2 || (n_imm > 0 && !imm))
        return dvm_set_error(DVM_E_ARGS, "dvm_fuser_op: bad argument");
    if (out_dtype != DVM_F32 && out_dtype != DVM_BF16) return dvm_set_error(DVM_E_DTYPE, "dvm_fuser_op: dtype");
    for (int a = 0; a < n_args; ++a)
        if (!valid_value(f, args[a])) return dvm_set_error(DVM_E_ARGS, "dvm_fuser_op: unknown value");
    // shape of the result: broadcast of the arguments; a reduction keeps its axis with extent 1
    dvm_shape s = f->vals[args[0]].shape;
    for (int a = 1; a < n_args; ++a)
        if (!broadcast_into(s, f->vals[args[a]].shape)) return dvm_set_error(DVM_E_SHAPE, "dvm_fuser_op: operands do not broadcast together");
    if (is_reduction(opcode) && s.rank > 0) s.dim[s.rank - 1] = 1;
    if (opcode >= DVM_OP_CSUM && opcode <= DVM_OP_CMIN) {       // along the penultimate axis
        if (s.rank < 2) return dvm_set_error(DVM_E_RANK, "dvm_fuser_op: a reduction along the penultimate axis needs rank >= 2");
        s.dim[s.rank - 2] = 1;
    }
    {
        int64_t dims[DVM_MAX_RANK];
        for (int k = 0; k < s.rank; ++k) dims[k] = s.dim[k];
        dvm_shape_contiguous(&s, s.rank, dims);
    }
    // fuse on arrival: the operator joins the open piece if its iteration space merges with that piece's
    // (its result broadcasts with the piece's dominant shape, or is that shape reduced along the row) and the
    // piece stays within a launch's limits; otherwise it cuts the buffer and opens the next piece; a full
    // buffer runs first
    if (f->n_ops >= MAX_PENDING) {
        int st = flush_all(f);
        if (st != DVM_OK) return st;
    }
    const int lo = f->piece_lo[f->n_pieces - 1];
    bool fits = true;
    if (f->n_ops > lo) {
        dvm_shape d = f->dom;
        fits = broadcast_into(d, s);
        if (fits) {
            // the merged space must be the old dominant shape or the new result's shape: two results
            // that only agree after broadcasting both would need a third, larger iteration space
            const bool same_as_old = d.rank == f->dom.rank && memcmp(d.dim, f->dom.dim, sizeof(int64_t) * d.rank) == 0;
            const bool same_as_new = d.rank == s.rank && memcmp(d.dim, s.dim, sizeof(int64_t) * d.rank) == 0;
            fits = same_as_old || same_as_new;
        }
        int distinct = 0;
        for (int i = lo; i < f->n_ops; ++i) distinct += 1 + f->ops[i].n_args;
        if (distinct + 1 + n_args > MAX_GROUP_TENSORS * 2) fits = false;
    }
    if (!fits) {
        if (f->n_pieces < MAX_PIECES) {
            f->piece_lo[f->n_pieces++] = f->n_ops;      // cut
        } else {
            int st = flush_all(f);
            if (st != DVM_OK) return st;
        }
    }
    const bool piece_empty = f->n_ops == f->piece_lo[f->n_pieces - 1];
    const int v = alloc_value(f);
    if (v < 0) return dvm_set_error(DVM_E_LIMIT, "dvm_fuser: too many live values");
    Val &val = f->vals[v];
    val.pending = 1;
    val.ptr = out_ptr;
    val.dtype = (uint8_t)out_dtype;
    val.shape = s;
    PendingOp &o = f->ops[f->n_ops++];
    o.opcode = opcode;
    o.n_args = n_args;
    o.n_imm = n_imm;
    for (int a = 0; a < n_args; ++a) o.args[a] = args[a];
    for (int k = 0; k < n_imm; ++k) o.imm[k] = imm[k];
    o.value = v;
    if (piece_empty) f->dom = s;
    else broadcast_into(f->dom, s);
    ++f->stat_ops;
    *value = v;
    return DVM_OK;
}

extern "C" int dvm_fuser_release(dvm_fuser *f, int value) {
    if (!f || !valid_value(f, value)) return dvm_set_error(DVM_E_ARGS, "dvm_fuser_release: unknown value");
    Val &v = f->vals[value];
    if (v.pending) v.released = 1;      // still an argument of buffered operators: dropped at the flush
    else v.used = 0;
    return DVM_OK;
}

extern "C" int dvm_fuser_flush(dvm_fuser *f) {
    if (!f) return dvm_set_error(DVM_E_ARGS, "dvm_fuser_flush: null fuser");
    return flush_all(f);
}

extern "C" int dvm_fuser_set_workspace(dvm_fuser *f, void *workspace, size_t bytes) {
    if (!f) return dvm_set_error(DVM_E_ARGS, "dvm_fuser_set_workspace: null fuser");
    if (workspace && (bytes < DVM_WORKSPACE_BYTES || ((uintptr_t)workspace & 255)))
        return dvm_set_error(DVM_E_ARGS, "dvm_fuser_set_workspace: DVM_WORKSPACE_BYTES of 256-byte aligned device memory, or null");
    f->workspace = workspace;
    return DVM_OK;
}

extern "C" int dvm_fuser_stats(const dvm_fuser *f, int64_t *n_ops, int64_t *n_launches, int64_t *n_flushes, int64_t *n_elided) {
    if (!f) return dvm_set_error(DVM_E_ARGS, "dvm_fuser_stats: null fuser");
    if (n_ops) *n_ops = f->stat_ops;
    if (n_launches) *n_launches = f->stat_launches;
    if (n_flushes) *n_flushes = f->stat_flushes;
    if (n_elided) *n_elided = f->stat_elided;
    return DVM_OK;
}

extern "C" int dvm_fuser_last_code(const dvm_fuser *f, void *bytecode, size_t cap, size_t *len) {
    if (!f || !len) return dvm_set_error(DVM_E_ARGS, "dvm_fuser_last_code: null argument");
    *len = f->code_len;
    if (!bytecode || cap < f->code_len) return dvm_set_error(DVM_E_BUFSZ, "dvm_fuser_last_code: buffer too small");
    memcpy(bytecode, f->code, f->code_len);
    return DVM_OK;
}
