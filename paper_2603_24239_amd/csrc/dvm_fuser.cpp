// Streaming fuser for dynamic graphs (Section 5.2 of the paper, "dynamic graph fuser"): operators
// arrive one at a time, as an eager framework issues them; they are buffered lazily, fused as they
// arrive while their iteration spaces merge, and executed as one VM launch when an operator arrives
// that does not fuse, when the buffer is full, or when the caller asks for a result (flush).
// Values that the caller released before the flush are pure intermediates and never reach memory.
//
// Built on the public C ABI only (program builder, dvm_encode, dvm_run): host code, no HIP call of
// its own.
#include <stdint.h>
#include <string.h>

#include <new>

#include "../../include/dvm.h"
#include "dvm_internal.h"

namespace {

constexpr int MAX_VALUES = 4096;        // values alive in one fuser (tensors + pending results)
constexpr int MAX_PENDING = 48;         // operators buffered before a forced flush
constexpr int MAX_GROUP_TENSORS = 24;   // distinct tensors (inputs + results) of one launch

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
    dvm_shape dom;                      // broadcast of the shapes of the buffered results
    int64_t stat_ops, stat_launches, stat_flushes, stat_elided;
    unsigned char code[8192];
    size_t code_len;
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

// Execute ops [lo, hi) of the buffer as one program.  Results that are still referenced are written
// to their buffers and become plain tensors; released ones are dropped.
int run_range(dvm_fuser *f, int lo, int hi) {
    dvm_prog *p = nullptr;
    int st = dvm_prog_create(&p);
    if (st != DVM_OK) return st;
    // value -> SSA id, kept sparse: the range touches at most MAX_GROUP_TENSORS + MAX_PENDING values
    int map_val[MAX_PENDING * 4 + MAX_GROUP_TENSORS], map_ssa[MAX_PENDING * 4 + MAX_GROUP_TENSORS], n_map = 0;
    auto find = [&](int v) { for (int i = 0; i < n_map; ++i) if (map_val[i] == v) return map_ssa[i]; return -1; };
    dvm_shape in_shapes[DVM_MAX_TENSORS];
    void *tensors[DVM_MAX_TENSORS];
    int n_in = 0;
    // inputs: every argument that is not produced inside the range, in first-use order
    for (int i = lo; i < hi && st == DVM_OK; ++i) {
        const PendingOp &o = f->ops[i];
        for (int a = 0; a < o.n_args && st == DVM_OK; ++a) {
            const int v = o.args[a];
            bool inside = false;
            for (int j = lo; j < i; ++j) inside |= f->ops[j].value == v;
            if (inside || find(v) >= 0) continue;
            if (f->vals[v].pending) { st = dvm_set_error(DVM_E_STATE, "dvm_fuser: argument is neither a tensor nor buffered"); break; }
            if (n_in >= DVM_MAX_TENSORS) { st = dvm_set_error(DVM_E_LIMIT, "dvm_fuser: too many tensors in one launch"); break; }
            int id = -1;
            st = dvm_prog_input(p, f->vals[v].dtype, &id);
            map_val[n_map] = v; map_ssa[n_map++] = id;
            in_shapes[n_in] = f->vals[v].shape;
            tensors[n_in++] = f->vals[v].ptr;
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
    int n_out = 0;
    int out_vals[MAX_PENDING];
    for (int i = lo; i < hi && st == DVM_OK; ++i) {
        const int v = f->ops[i].value;
        if (f->vals[v].released) continue;
        if (n_in + n_out >= DVM_MAX_TENSORS) { st = dvm_set_error(DVM_E_LIMIT, "dvm_fuser: too many tensors in one launch"); break; }
        st = dvm_prog_output(p, find(v), f->vals[v].dtype);
        tensors[n_in + n_out] = f->vals[v].ptr;
        out_vals[n_out++] = v;
    }
    if (st == DVM_OK && n_out > 0) {
        st = dvm_prog_finish(p);
        dvm_shape out_shapes[DVM_MAX_TENSORS];
        if (st == DVM_OK) st = dvm_encode(f->ctx, p, in_shapes, n_in, nullptr, f->code, sizeof(f->code), &f->code_len, out_shapes);
        if (st == DVM_OK && dvm_ctx_device(f->ctx) >= 0)
            st = dvm_run(f->ctx, f->code, f->code_len, tensors, n_in + n_out, f->stream);
        if (st == DVM_OK) {
            ++f->stat_launches;
            for (int k = 0; k < n_out; ++k) {
                Val &v = f->vals[out_vals[k]];
                if (v.shape.rank != out_shapes[k].rank || memcmp(v.shape.dim, out_shapes[k].dim, sizeof(int64_t) * v.shape.rank) != 0)
                    st = dvm_set_error(DVM_E_SHAPE, "dvm_fuser: inferred shape differs from the encoder's");
            }
        }
    }
    dvm_prog_destroy(p);
    if (st != DVM_OK) return st;
    for (int i = lo; i < hi; ++i) {
        Val &v = f->vals[f->ops[i].value];
        if (v.released) { v.used = 0; ++f->stat_elided; }
        else v.pending = 0;
    }
    return DVM_OK;
}

int flush_all(dvm_fuser *f) {
    if (f->n_ops == 0) return DVM_OK;
    ++f->stat_flushes;
    int st = run_range(f, 0, f->n_ops);
    if (st == DVM_E_UNSUPPORTED || st == DVM_E_LIMIT || st == DVM_E_RANK) {
        // the chain does not fit one meta-kernel after all (registers, tensor table, iteration space):
        // run it operator by operator; every result then reaches its buffer, released or not
        for (int i = 0; i < f->n_ops; ++i) {
            Val &v = f->vals[f->ops[i].value];
            const uint8_t was_released = v.released;
            v.released = 0;
            st = run_range(f, i, i + 1);
            v.released = was_released;
            if (st != DVM_OK) break;
        }
        if (st == DVM_OK)
            for (int i = 0; i < f->n_ops; ++i) {
                Val &v = f->vals[f->ops[i].value];
                if (v.released) v.used = 0;
            }
    }
    f->n_ops = 0;
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
    // fuse on arrival: the operator joins the buffer if its iteration space merges with the buffered
    // ones (its result broadcasts with their dominant shape, or is that shape reduced along the row)
    // and the launch stays within its limits; otherwise the buffer runs first
    bool fits = f->n_ops < MAX_PENDING;
    if (fits && f->n_ops > 0) {
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
        for (int i = 0; i < f->n_ops; ++i) distinct += 1 + f->ops[i].n_args;
        if (distinct + 1 + n_args > MAX_GROUP_TENSORS * 2) fits = false;
    }
    if (!fits) {
        int st = flush_all(f);
        if (st != DVM_OK) return st;
    }
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
    if (f->n_ops == 1) f->dom = s;
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
