// The device side of libdvm: the bytecode interpreter kernel for gfx950 and dvm_run.
//
// One workgroup plays the role of one "AI Core" of Algorithm 2 (Section 4.3): it takes a
// contiguous range of tiles, and for every tile walks the code body from its first record to
// CodeSize, dispatching each record on its instruction id.  Decoding is wave-uniform: the
// bytecode sits in the kernel-argument segment and is read with scalar loads into SGPRs, the
// dispatch is a scalar branch tree, so no vector lane ever spends an issue slot on decoding
// (the GPU analogue of decoding on the NPU's Scalar unit, Section 4.3).
//
// Local memory of the paper's AI Core = the vector register file here.  A tile register is K
// fp32 values per lane; the accumulator ACC and the registers R0..R(NR-1) hold fused
// intermediates, which therefore never touch HBM (Section 5.1, vector-vector fusion).  Every
// register reference in a handler is a compile-time constant: handlers are selected by scalar
// switches on the register ids, because a GPU cannot index vector registers dynamically.
//
// Layout of a tile: RP rows x up to G*nvec*V columns.  Row r of the tile is held by the G
// lanes [r*G, (r+1)*G); lane l of the group owns the chunks of V consecutive elements number
// l, l+G, l+2G, ... so that each load instruction of a wave covers whole contiguous runs of
// 16 bytes per lane.  Loads/stores do all address arithmetic (strides, broadcast, views), so
// compute instructions see one canonical layout (Section 4.1, last paragraph).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>
#include <atomic>
#include <mutex>
#include <utility>

#include "../../include/dvm.h"
#include "dvm_bytecode.h"
#include "dvm_internal.h"

using namespace dvmbc;

namespace {

constexpr int CODE_WORDS = DVM_CODE_MAX_BYTES / 4;

struct KArgs {
    uint32_t code[CODE_WORDS];          // the segments of the program (headers + bodies)
    uint64_t tensors[DVM_MAX_TENSORS];  // device addresses
    uint64_t ws;                        // the launch's workspace (0: none)
    uint32_t nseg;
    uint32_t spin_limit;                // polls a workgroup spends at a grid-wide synchronisation point before it gives up
    uint64_t sets;                      // batched launch: device array of n_sets * n_tensors addresses (0: `tensors` above)
    uint32_t n_sets;                    // times the program runs, each time on the next set of tensors (at least 1)
    uint32_t n_tensors;
    uint32_t rotate;                    // 1: every segment deals its tiles out starting at the workgroup after the one the
                                        // segment before stopped at (short segments then do not all land on the first workgroups)
    uint32_t seg_first;                 // this launch runs segments seg_first .. nseg - 1
};

#define DI __device__ __forceinline__
#define LI __attribute__((always_inline))

// Compile-time loop: f.operator()<I>() for I = 0..N-1.  Every register-array index in this file
// is a template constant, so that the arrays are split into scalar registers before any other
// optimisation can merge the handlers of different registers into one body with a run-time index.
template <class F, int... I> DI void sfor_impl(F &f, std::integer_sequence<int, I...>) {
    (f.template operator()<I>(), ...);
}
template <int N, class F> DI void sfor(F &&f) { sfor_impl(f, std::make_integer_sequence<int, N>{}); }

// ------------------------------------------------------------------------------------------
// scalar math on fp32 lanes
// ------------------------------------------------------------------------------------------
DI float f_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
DI float f_log2(float x) { return __builtin_amdgcn_logf(x); }
DI float f_rcp(float x) { return __builtin_amdgcn_rcpf(x); }
DI float f_rsq(float x) { return __builtin_amdgcn_rsqf(x); }
DI float f_sqrt(float x) { return __builtin_amdgcn_sqrtf(x); }
DI float f_fma(float a, float b, float c) { return __builtin_fmaf(a, b, c); }
// Table 1's Max / Min are read as propagating a NaN operand (what NumPy's maximum / minimum and the frameworks
// this VM serves do).  gfx950 has that operation as one instruction (v_maximum3_f32 / v_minimum3_f32), which the
// compiler selects for the IEEE-754-2019 maximum / minimum builtins: element-wise ops and every stage of a
// reduction use it, so a NaN anywhere in a row or column reaches the result.
DI float f_maxp(float a, float b) { return __builtin_elementwise_maximum(a, b); }
DI float f_minp(float a, float b) { return __builtin_elementwise_minimum(a, b); }

constexpr float LOG2E    = 1.44269504088896340736f;
constexpr float LOG2E_LO = 1.92596303e-8f;      // log2(e) - (float)log2(e)
constexpr float LN2      = 0.69314718055994530942f;

// exp(x) = 2^(x*log2e); the rounding error of the product is carried as a first-order correction
// so that the relative error stays near 1 ulp for |x| up to the overflow threshold.
DI float f_exp(float x) {
    float t = x * LOG2E;
    float e = f_fma(x, LOG2E, -t);
    e = f_fma(x, LOG2E_LO, e);
    e = (__builtin_fabsf(x) < __builtin_inff()) ? e : 0.0f;
    float r = f_exp2(t);
    return f_fma(r, e * LN2, r);
}
DI float f_sigmoid(float x) { return f_rcp(1.0f + f_exp2(-LOG2E * x)); }
DI float f_silu(float x) { return x * f_sigmoid(x); }
// 0.5 u (1 + tanh(c (u + 0.044715 u^3)))  ==  u * sigmoid(2 c (u + 0.044715 u^3))
DI float f_gelu_tanh(float u) {
    constexpr float C0 = -2.0f * LOG2E * 0.7978845608028654f;
    constexpr float C1 = -2.0f * LOG2E * 0.7978845608028654f * 0.044715f;
    float p = u * f_fma(u * u, C1, C0);
    return u * f_rcp(1.0f + f_exp2(p));
}
DI float f_tanh(float x) {
    float a = __builtin_fabsf(x);
    float t = f_exp2(-2.0f * LOG2E * a);
    float big = (1.0f - t) * f_rcp(1.0f + t);
    float s = a * a;                               // odd Taylor series below 0.04
    float small = a * f_fma(s, f_fma(s, 0.13333333f, -0.33333333f), 1.0f);
    float r = a < 0.04f ? small : big;
    return __builtin_copysignf(r, x);
}
// erf: odd polynomial in x on |x| <= 1, 1 - exp(q(|x| - 2.5)) on 1 < |x| <= 4, 1 beyond.
// Coefficients: least-squares Chebyshev fits of erf(x)/x in x^2 on [0,1] (degree 6) and of
// log(erfc(a)) in a-2.5 on [1,4] (degree 8), converted to the monomial basis.
DI float f_erf(float x) {
    float a = __builtin_fabsf(x);
    float s = a * a;
    float p = 7.882497448008507e-05f;
    p = f_fma(p, s, -0.0008018855005502701f);
    p = f_fma(p, s, 0.005189312156289816f);
    p = f_fma(p, s, -0.02685432881116867f);
    p = f_fma(p, s, 0.11283597350120544f);
    p = f_fma(p, s, -0.3761262595653534f);
    p = f_fma(p, s, 1.1283791065216064f);
    float lo = a * p;
    float u = __builtin_fminf(a, 4.0f) - 2.5f;
    float q = 1.6140616025950294e-06f;
    q = f_fma(q, u, -1.3309389942151029e-05f);
    q = f_fma(q, u, 7.739442662568763e-05f);
    q = f_fma(q, u, -0.0004201445553917438f);
    q = f_fma(q, u, 0.0021651603747159243f);
    q = f_fma(q, u, -0.01085851714015007f);
    q = f_fma(q, u, -0.9438936114311218f);
    q = f_fma(q, u, -5.352680683135986f);
    q = f_fma(q, u, -7.806815147399902f);
    float hi = 1.0f - f_exp2(q * LOG2E);
    float r = a <= 1.0f ? lo : hi;
    r = (a != a) ? a : r;
    return __builtin_copysignf(r, x);
}
DI float f_gelu_erf(float u) { return 0.5f * u * (1.0f + f_erf(u * 0.70710678118654752f)); }
// pow(a, b) = 2^(b log2 |a|) with the sign and the special cases of the C library's pow: a finite negative base
// is defined for integer exponents only (odd ones keep the sign), pow(x, 0) = pow(1, y) = 1 for every x and y,
// pow(-1, +-inf) = 1; zeros and infinities fall out of log2 and exp2.
DI float f_pow(float a, float b) {
    // (conditions are combined with integer and / or: a logical && would become a branch that differs between lanes)
    const float aa = __builtin_fabsf(a), ab = __builtin_fabsf(b);
    float r = f_exp2(b * f_log2(aa));
    const int b_int = __builtin_truncf(b) == b;
    const float half = 0.5f * b;
    const int b_odd = b_int & (int)(__builtin_truncf(half) != half) & (int)(ab < 16777216.0f);
    const int neg_base = (__builtin_bit_cast(uint32_t, a) >> 31) != 0;
    const int no_real_power = (int)(a < 0.0f) & (int)(aa < __builtin_inff()) & (b_int ^ 1);
    r = no_real_power ? __builtin_nanf("") : r;
    r = (neg_base & b_odd) ? -r : r;
    r = ((int)(aa == 1.0f) & (int)(ab == __builtin_inff())) ? 1.0f : r;
    r = ((int)(b == 0.0f) | (int)(a == 1.0f)) ? 1.0f : r;
    return r;
}
DI float f_bf16_round(float x) {
    __bf16 h = (__bf16)x;
    return (float)h;
}

template <uint32_t U> DI float un_op(float x) {
    if constexpr (U == U_SQRT) return f_sqrt(x);
    else if constexpr (U == U_ABS) return __builtin_fabsf(x);
    else if constexpr (U == U_LOG) return f_log2(x) * LN2;
    else if constexpr (U == U_EXP) return f_exp(x);
    else if constexpr (U == U_ROUND) return __builtin_rintf(x);
    else if constexpr (U == U_FLOOR) return __builtin_floorf(x);
    else if constexpr (U == U_ISFINITE) return (__builtin_fabsf(x) < __builtin_inff()) ? 1.0f : 0.0f;
    else if constexpr (U == U_NEG) return -x;
    else if constexpr (U == U_RSQRT) return f_rsq(x);
    else if constexpr (U == U_RCP) return f_rcp(x);
    else if constexpr (U == U_TANH) return f_tanh(x);
    else if constexpr (U == U_ERF) return f_erf(x);
    else if constexpr (U == U_SIGMOID) return f_sigmoid(x);
    else if constexpr (U == U_SQUARE) return x * x;
    else if constexpr (U == U_GELU_TANH) return f_gelu_tanh(x);
    else if constexpr (U == U_GELU_ERF) return f_gelu_erf(x);
    else if constexpr (U == U_SILU) return f_silu(x);
    else if constexpr (U == U_CAST_BF16) return f_bf16_round(x);
    else return x;
}

template <uint32_t B> DI float bin_op(float a, float b) {
    if constexpr (B == B_NONE) return b;
    else if constexpr (B == B_ADD) return a + b;
    else if constexpr (B == B_SUB) return a - b;
    else if constexpr (B == B_RSUB) return b - a;
    else if constexpr (B == B_MUL) return a * b;
    else if constexpr (B == B_DIV) return a * f_rcp(b);
    else if constexpr (B == B_RDIV) return b * f_rcp(a);
    else if constexpr (B == B_MIN) return f_minp(a, b);
    else if constexpr (B == B_MAX) return f_maxp(a, b);
    else if constexpr (B == B_POW) return f_pow(a, b);
    else if constexpr (B == B_RPOW) return f_pow(b, a);
    else if constexpr (B == B_EQ) return a == b ? 1.0f : 0.0f;
    else if constexpr (B == B_NE) return a != b ? 1.0f : 0.0f;
    else if constexpr (B == B_LT) return a < b ? 1.0f : 0.0f;
    else if constexpr (B == B_LE) return a <= b ? 1.0f : 0.0f;
    else if constexpr (B == B_GT) return a > b ? 1.0f : 0.0f;
    else if constexpr (B == B_GE) return a >= b ? 1.0f : 0.0f;
    // exp of a difference: the difference is exact to one rounding, so the plain product with
    // log2(e) keeps the relative error below |a - b| * 2^-24 (5e-6 at the overflow threshold)
    else if constexpr (B == B_EXPSUB) return f_exp2((a - b) * LOG2E);
    else if constexpr (B == B_REXPSUB) return f_exp2((b - a) * LOG2E);
    else return a;
}

// scalar (one value) versions selected at run time; used for the row-scalar registers
DI float un_dyn(uint32_t u, float x) {
    switch (u) {
#define C(U) case U: return un_op<U>(x);
        C(U_SQRT) C(U_ABS) C(U_LOG) C(U_EXP) C(U_ROUND) C(U_FLOOR) C(U_ISFINITE) C(U_NEG) C(U_RSQRT)
        C(U_RCP) C(U_TANH) C(U_ERF) C(U_SIGMOID) C(U_SQUARE) C(U_GELU_TANH) C(U_GELU_ERF) C(U_SILU)
        C(U_CAST_BF16)
#undef C
        default: return x;
    }
}
DI float bin_dyn(uint32_t b, float x, float y) {
    switch (b) {
#define C(B) case B: return bin_op<B>(x, y);
        C(B_NONE) C(B_ADD) C(B_SUB) C(B_RSUB) C(B_MUL) C(B_DIV) C(B_RDIV) C(B_MIN) C(B_MAX) C(B_POW)
        C(B_RPOW) C(B_EQ) C(B_NE) C(B_LT) C(B_LE) C(B_GT) C(B_GE) C(B_EXPSUB) C(B_REXPSUB)
#undef C
        default: return x;
    }
}

// ------------------------------------------------------------------------------------------
// A tile register is a struct of K fp32 per lane.  Helpers below touch it only through constant
// element indices and never choose between two registers at run time (the interpreter's switch
// does that, in the kernel body), so every register is split into K independent scalar VGPRs and
// an instruction updates its destination in place.
// ------------------------------------------------------------------------------------------
typedef float f32x4 __attribute__((ext_vector_type(4)));
// (held as groups of four consecutive registers: a 16-byte load or store moves a whole group without copies)
template <int K> struct Tile { f32x4 q[K / 4]; };
#define TV(T, I) ((T).q[(I) >> 2][(I) & 3])
template <int K> DI void tile_zero(Tile<K> &t) { sfor<K / 4>([&]<int Q>() LI { t.q[Q] = f32x4{0.0f, 0.0f, 0.0f, 0.0f}; }); }

template <int K, uint32_t U> DI void tile_un(Tile<K> &a) {
    sfor<K>([&]<int I>() LI { TV(a, I) = un_op<U>(TV(a, I)); });
}
template <int K, uint32_t B> DI void tile_bin(Tile<K> &a, const Tile<K> &b) {
    sfor<K>([&]<int I>() LI { TV(a, I) = bin_op<B>(TV(a, I), TV(b, I)); });
}
template <int K, uint32_t B> DI void tile_bins(Tile<K> &a, float s) {
    sfor<K>([&]<int I>() LI { TV(a, I) = bin_op<B>(TV(a, I), s); });
}

template <int K> DI void tile_un_dispatch(Tile<K> &a, uint32_t u) {
    switch (u) {
#define C(U) case U: tile_un<K, U>(a); break;
        C(U_SQRT) C(U_ABS) C(U_LOG) C(U_EXP) C(U_ROUND) C(U_FLOOR) C(U_ISFINITE) C(U_NEG) C(U_RSQRT)
        C(U_RCP) C(U_TANH) C(U_ERF) C(U_SIGMOID) C(U_SQUARE) C(U_GELU_TANH) C(U_GELU_ERF) C(U_SILU)
        C(U_CAST_BF16)
#undef C
        default: break;
    }
}
template <int K> DI void tile_bin_dispatch(Tile<K> &a, const Tile<K> &b, uint32_t op) {
    switch (op) {
#define C(B) case B: tile_bin<K, B>(a, b); break;
        C(B_NONE) C(B_ADD) C(B_SUB) C(B_RSUB) C(B_MUL) C(B_DIV) C(B_RDIV) C(B_MIN) C(B_MAX) C(B_POW)
        C(B_RPOW) C(B_EQ) C(B_NE) C(B_LT) C(B_LE) C(B_GT) C(B_GE) C(B_EXPSUB) C(B_REXPSUB)
#undef C
        default: break;
    }
}
template <int K> DI void tile_bins_dispatch(Tile<K> &a, float s, uint32_t op) {
    switch (op) {
#define C(B) case B: tile_bins<K, B>(a, s); break;
        C(B_NONE) C(B_ADD) C(B_SUB) C(B_RSUB) C(B_MUL) C(B_DIV) C(B_RDIV) C(B_MIN) C(B_MAX) C(B_POW)
        C(B_RPOW) C(B_EQ) C(B_NE) C(B_LT) C(B_LE) C(B_GT) C(B_GE) C(B_EXPSUB) C(B_REXPSUB)
#undef C
        default: break;
    }
}

// ------------------------------------------------------------------------------------------
// cross-lane reduction inside a wave with DPP / ds_swizzle / readlane; `width` (lanes per
// row, a power of two up to 64) is wave-uniform.  The combination order is fixed, so results
// are bitwise reproducible.
// ------------------------------------------------------------------------------------------
template <uint32_t R> DI float red_comb(float a, float b) {
    if constexpr (R == R_MAX) return f_maxp(a, b);
    else if constexpr (R == R_MIN) return f_minp(a, b);
    else return a + b;
}
template <uint32_t R> DI float red_ident() {
    if constexpr (R == R_MAX) return -__builtin_inff();
    else if constexpr (R == R_MIN) return __builtin_inff();
    else return 0.0f;
}
template <int CTRL> DI float dpp_mov(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
template <uint32_t R> DI float swap16(float v) {   // combine with lane ^ 16
    return red_comb<R>(v, __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F)));
}
template <uint32_t R> DI float wave_allreduce(float v, uint32_t width) {
    if (width == 64) {          // the common case, free of branches: the row spans the whole wave
        v = red_comb<R>(v, dpp_mov<0xB1>(v));                             // quad_perm [1,0,3,2]
        v = red_comb<R>(v, dpp_mov<0x4E>(v));                             // quad_perm [2,3,0,1]
        v = red_comb<R>(v, dpp_mov<0x141>(v));                            // row_half_mirror
        v = red_comb<R>(v, dpp_mov<0x140>(v));                            // row_mirror
        v = swap16<R>(v);
        float lo = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
        float hi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
        return red_comb<R>(lo, hi);
    }
    if (width >= 2) v = red_comb<R>(v, dpp_mov<0xB1>(v));
    if (width >= 4) v = red_comb<R>(v, dpp_mov<0x4E>(v));
    if (width >= 8) v = red_comb<R>(v, dpp_mov<0x141>(v));
    if (width >= 16) v = red_comb<R>(v, dpp_mov<0x140>(v));
    if (width >= 32) v = swap16<R>(v);
    return v;
}

// ------------------------------------------------------------------------------------------
// per-tile geometry
// ------------------------------------------------------------------------------------------
struct Geo {
    // wave-uniform
    uint64_t colbase;     // first column of the tile
    uint32_t ncols;       // valid columns of the tile
    uint32_t GV;          // G * V: column distance between two chunks of one lane
    uint32_t nvec;        // chunks per lane
    uint32_t nact;        // nvec * V
    uint32_t part_slot;   // chunk slot that holds the ragged last chunk, or ~0u
    uint32_t part_lane;   // lane (within the row group) that owns it
    uint32_t part_col;    // its first column (relative to colbase)
    uint32_t part_n;      // its number of valid elements
    uint32_t ragged;      // some lane has invalid columns inside live chunks: reductions must mask
    // per lane
    uint32_t i1, i2, i3;  // decomposition of the lane's row index over the outer dims
    uint32_t lanecol;     // first column of the lane's chunk 0, relative to colbase: V times the lane's index within the row group
    uint32_t rowok;       // 1 when the lane's row lies inside the tensor
};

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));
typedef u32x4 u32x4_a2 __attribute__((aligned(2)));
typedef f32x4 f32x4_a4 __attribute__((aligned(4)));
#define GLOBAL_AS __attribute__((address_space(1)))
typedef const GLOBAL_AS char *gcptr;   // global memory, read
typedef GLOBAL_AS char *gptr;          // global memory, write

DI float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
DI float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xFFFF0000u); }
DI uint32_t pack_bf16x2(float a, float b) {
    typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
    typedef float f2 __attribute__((ext_vector_type(2)));
    f2 v = {a, b};
    bf2 h = __builtin_convertvector(v, bf2);
    return __builtin_bit_cast(uint32_t, h);
}
DI uint16_t pack_bf16(float a) {
    __bf16 h = (__bf16)a;
    return __builtin_bit_cast(uint16_t, h);
}

// element offset of the lane's row for a tensor with outer strides s1..s3
DI int64_t row_offset(const Geo &g, int64_t s1, int64_t s2, int64_t s3) {
    return (int64_t)g.i1 * s1 + (int64_t)g.i2 * s2 + (int64_t)g.i3 * s3;
}

// Predicated stores.  The interpreter loop must not contain a branch that differs between the
// lanes of a wave: with only wave-uniform branches the compiler keeps the dispatch as plain scalar
// jumps and updates registers in place.  Loads therefore clamp the address of an invalid lane to
// a valid one (its data is never used), and stores switch the invalid lanes off in EXEC inside
// one assembly statement.  (The compiler does not look inside the statement, so the wait state that this
// chip wants between a store of more than 8 bytes and an instruction that overwrites the stored registers is
// written out: the s_nop after the restored EXEC mask.)
DI void st_b128(gptr p, f32x4 v, bool ok) {
    const uint64_t m = __builtin_amdgcn_ballot_w64(ok);
    uint64_t sv;
    asm volatile("s_and_saveexec_b64 %0, %1\n\tglobal_store_dwordx4 %2, %3, off nt\n\ts_mov_b64 exec, %0\n\ts_nop 0"
                 : "=&s"(sv) : "s"(m), "v"(p), "v"(v) : "memory", "scc");
}
DI void st_b32(gptr p, float v, bool ok) {
    const uint64_t m = __builtin_amdgcn_ballot_w64(ok);
    uint64_t sv;
    asm volatile("s_and_saveexec_b64 %0, %1\n\tglobal_store_dword %2, %3, off nt\n\ts_mov_b64 exec, %0\n\ts_nop 0"
                 : "=&s"(sv) : "s"(m), "v"(p), "v"(v) : "memory", "scc");
}
DI void st_b16(gptr p, uint32_t v, bool ok) {
    const uint64_t m = __builtin_amdgcn_ballot_w64(ok);
    uint64_t sv;
    asm volatile("s_and_saveexec_b64 %0, %1\n\tglobal_store_short %2, %3, off nt\n\ts_mov_b64 exec, %0\n\ts_nop 0"
                 : "=&s"(sv) : "s"(m), "v"(p), "v"(v) : "memory", "scc");
}

// Loading the lane's part of a tile has two halves, so that the loads of several tensors are in flight
// together: request_inplace issues every whole chunk straight into the destination tile register (no staging
// registers: fp32 chunks land where their elements live, a bf16 chunk of 8 elements = 16 bytes lands in the
// upper half of the register), and finish_tile, called once all loads of a group of load records have been
// issued, widens the bf16 bits in place and fetches the chunk a ragged row ends in.
// DT: 0 = fp32, 1 = bf16.  V = chunk width.  `rowp` points at column `colbase` of the lane's row in this tensor
// (row 0 for a lane whose row is outside the tensor).  A chunk that lies beyond the tile's columns reads the
// tile's chunk 0 instead: the value is never stored and reductions mask it.  Dtype, chunk width and cache hint
// are fixed at compile time, so the request needs no per-piece scalar arithmetic.  NT: the data is read once,
// hint the caches accordingly.
typedef f32x4 f32x4_a2 __attribute__((aligned(2)));
template <bool NT> DI f32x4 ld_b128(gcptr q) {
    const GLOBAL_AS f32x4_a2 *src = (const GLOBAL_AS f32x4_a2 *)q;
    if constexpr (NT) return __builtin_nontemporal_load(src);
    else return *src;
}

template <int K, int DT, int V, bool NT> DI void request_inplace(Tile<K> &t, gcptr rowp, const Geo &g) {
    constexpr int ES = DT == 0 ? 4 : 2;
    if constexpr (K >= V) {
        constexpr int NJ = K / V;
        if (g.ncols >= (uint32_t)V) {       // wave-uniform: the tile has at least one whole chunk
            sfor<NJ>([&]<int J>() LI {
                const uint32_t c0 = g.lanecol + (uint32_t)J * g.GV;
                const uint32_t cc = c0 + V <= g.ncols ? c0 : 0u;
                gcptr q = rowp + (uint64_t)cc * ES;
                if constexpr (DT == 0) {
                    sfor<V / 4>([&]<int H>() LI { t.q[J * (V / 4) + H] = ld_b128<NT>(q + 16 * H); });
                } else {
                    t.q[K / 8 + J] = ld_b128<NT>(q);        // raw bits, widened by finish_tile
                }
            });
        }
    }
}
template <int K> DI void request_dispatch(Tile<K> &t, uint32_t dt, uint32_t V, bool nt, gcptr rowp, const Geo &g) {
    if (nt) {
        if (dt == 0) {
            if (V == 4) request_inplace<K, 0, 4, true>(t, rowp, g);
            else request_inplace<K, 0, 8, true>(t, rowp, g);
        } else {
            request_inplace<K, 1, 8, true>(t, rowp, g);
        }
    } else {
        if (dt == 0) {
            if (V == 4) request_inplace<K, 0, 4, false>(t, rowp, g);
            else request_inplace<K, 0, 8, false>(t, rowp, g);
        } else {
            request_inplace<K, 1, 8, false>(t, rowp, g);
        }
    }
}

// The second half.  bf16: chunk J sits as raw bits in group K/8 + J and becomes the eight values of groups
// 2J and 2J + 1; going through the chunks in ascending order never overwrites bits that are still to be read
// (2J + 1 <= K/8 + J for every J < K/8, and the last chunk is read before its own group is written).
template <int K, int DT, int V> DI void finish_tile(Tile<K> &t, gcptr rowp, const Geo &g) {
    constexpr int ES = DT == 0 ? 4 : 2;
    if constexpr (K < V) tile_zero<K>(t);
    if constexpr (K >= V) {
        constexpr int NJ = K / V;
        if (g.ncols < (uint32_t)V) {        // narrower than one chunk: only the ragged part below
            tile_zero<K>(t);
        } else if constexpr (DT == 1) {
            sfor<NJ>([&]<int J>() LI {
                const u32x4 r = __builtin_bit_cast(u32x4, t.q[K / 8 + J]);
                const uint32_t w0 = r.x, w1 = r.y, w2 = r.z, w3 = r.w;
                t.q[2 * J] = f32x4{bf16_lo(w0), bf16_hi(w0), bf16_lo(w1), bf16_hi(w1)};
                t.q[2 * J + 1] = f32x4{bf16_lo(w2), bf16_hi(w2), bf16_lo(w3), bf16_hi(w3)};
            });
        }
        if (g.part_slot != ~0u) {   // wave-uniform: this tile ends inside a chunk
            // its elements are read one by one by every lane of the row (one of them keeps them); an element
            // beyond the row reads element 0 again
            const bool own = g.lanecol == g.part_lane * (uint32_t)V;
            float pv[V];
            sfor<V>([&]<int E>() LI {
                const uint32_t e = (uint32_t)E < g.part_n ? (uint32_t)E : 0u;       // wave-uniform
                gcptr q = rowp + (uint64_t)(g.part_col + e) * ES;
                if constexpr (DT == 0) pv[E] = *(const GLOBAL_AS float *)q;
                else pv[E] = bf16_lo(*(const GLOBAL_AS uint16_t *)q);
            });
            sfor<NJ>([&]<int J>() LI {
                if ((uint32_t)J == g.part_slot) {       // wave-uniform
                    sfor<V>([&]<int E>() LI {
                        const bool ok = own && (uint32_t)E < g.part_n;
                        // (the empty statement keeps this a select between two values: a select between
                        // two register-array elements would be turned into a select of their addresses,
                        // which forces both arrays into memory)
                        float x = pv[E];
                        asm volatile("" : "+v"(x));
                        TV(t, J * V + E) = ok ? x : TV(t, J * V + E);
                    });
                }
            });
        }
    }
}
template <int K> DI void finish_dispatch(Tile<K> &t, uint32_t dt, uint32_t V, gcptr rowp, const Geo &g) {
    if (dt == 0) {
        if (V == 4) finish_tile<K, 0, 4>(t, rowp, g);
        else finish_tile<K, 0, 8>(t, rowp, g);
    } else {
        finish_tile<K, 1, 8>(t, rowp, g);
    }
}

// The streaming reduction along the penultimate axis keeps several rows of one tensor in flight per wave and
// combines them into an accumulating register: it stages a row's raw bits in registers of its own (only the
// variants with at most 8 elements per lane run it).
template <int K> struct Raw {
    f32x4 q[K / 4];     // the whole chunks, 16 bytes per piece
    uint32_t pv[8];     // the elements of the chunk the row ends in (raw bits), requested alongside
};
template <int K, int DT, int V, bool NT> DI void request_staged(Raw<K> &raw, gcptr rowp, const Geo &g) {
    constexpr int ES = DT == 0 ? 4 : 2;
    if constexpr (K >= V) {
        constexpr int NJ = K / V;
        if (g.ncols >= (uint32_t)V) {
            sfor<NJ>([&]<int J>() LI {
                const uint32_t c0 = g.lanecol + (uint32_t)J * g.GV;
                const uint32_t cc = c0 + V <= g.ncols ? c0 : 0u;
                gcptr q = rowp + (uint64_t)cc * ES;
                constexpr int PIECES = DT == 0 ? V / 4 : 1;
                sfor<PIECES>([&]<int H>() LI { raw.q[J * PIECES + H] = ld_b128<NT>(q + 16 * H); });
            });
        }
        if (g.part_slot != ~0u) {
            sfor<V>([&]<int E>() LI {
                const uint32_t e = (uint32_t)E < g.part_n ? (uint32_t)E : 0u;
                gcptr q = rowp + (uint64_t)(g.part_col + e) * ES;
                if constexpr (DT == 0) raw.pv[E] = *(const GLOBAL_AS uint32_t *)q;
                else raw.pv[E] = *(const GLOBAL_AS uint16_t *)q;
            });
        }
    }
}
template <int K> DI void request_staged_dispatch(Raw<K> &raw, uint32_t dt, uint32_t V, bool nt, gcptr rowp, const Geo &g) {
    if (nt) {
        if (dt == 0) {
            if (V == 4) request_staged<K, 0, 4, true>(raw, rowp, g);
            else request_staged<K, 0, 8, true>(raw, rowp, g);
        } else {
            request_staged<K, 1, 8, true>(raw, rowp, g);
        }
    } else {
        if (dt == 0) {
            if (V == 4) request_staged<K, 0, 4, false>(raw, rowp, g);
            else request_staged<K, 0, 8, false>(raw, rowp, g);
        } else {
            request_staged<K, 1, 8, false>(raw, rowp, g);
        }
    }
}
// t = B(t, staged row), element by element as the pieces are widened; elements outside the row keep their value
template <int K, int DT, int V, uint32_t B> DI void combine_staged(Tile<K> &t, const Raw<K> &raw, const Geo &g) {
    if constexpr (K >= V) {
        constexpr int NJ = K / V;
        if (g.ncols >= (uint32_t)V) {
            const bool masked = g.ragged != 0;       // wave-uniform
            auto chunk = [&]<int J>(bool whole) LI {
                float x[V];
                if constexpr (DT == 0) {
                    sfor<V / 4>([&]<int H>() LI {
                        const f32x4 r = raw.q[J * (V / 4) + H];
                        x[4 * H + 0] = r.x; x[4 * H + 1] = r.y; x[4 * H + 2] = r.z; x[4 * H + 3] = r.w;
                    });
                } else {
                    const u32x4 r = __builtin_bit_cast(u32x4, raw.q[J]);
                    const uint32_t w0 = r.x, w1 = r.y, w2 = r.z, w3 = r.w;
                    x[0] = bf16_lo(w0); x[1] = bf16_hi(w0); x[2] = bf16_lo(w1); x[3] = bf16_hi(w1);
                    x[4] = bf16_lo(w2); x[5] = bf16_hi(w2); x[6] = bf16_lo(w3); x[7] = bf16_hi(w3);
                }
                sfor<V>([&]<int E>() LI {
                    const float y = bin_op<B>(TV(t, J * V + E), x[E]);
                    TV(t, J * V + E) = whole ? y : TV(t, J * V + E);
                });
            };
            if (!masked) {
                sfor<NJ>([&]<int J>() LI { chunk.template operator()<J>(true); });
            } else {
                sfor<NJ>([&]<int J>() LI { chunk.template operator()<J>(g.lanecol + (uint32_t)J * g.GV + V <= g.ncols); });
            }
        }
        if (g.part_slot != ~0u) {
            const bool own = g.lanecol == g.part_lane * (uint32_t)V;
            float pv[V];
            sfor<V>([&]<int E>() LI {
                const uint32_t bits = raw.pv[E];
                if constexpr (DT == 0) pv[E] = __builtin_bit_cast(float, bits);
                else pv[E] = bf16_lo(bits);
            });
            sfor<NJ>([&]<int J>() LI {
                if ((uint32_t)J == g.part_slot) {
                    sfor<V>([&]<int E>() LI {
                        const bool ok = own && (uint32_t)E < g.part_n;
                        float x = pv[E];
                        asm volatile("" : "+v"(x));
                        x = bin_op<B>(TV(t, J * V + E), x);
                        TV(t, J * V + E) = ok ? x : TV(t, J * V + E);
                    });
                }
            });
        }
    }
}
template <int K, uint32_t B> DI void combine_staged_dispatch(Tile<K> &t, const Raw<K> &raw, uint32_t dt, uint32_t V, const Geo &g) {
    if (dt == 0) {
        if (V == 4) combine_staged<K, 0, 4, B>(t, raw, g);
        else combine_staged<K, 0, 8, B>(t, raw, g);
    } else {
        combine_staged<K, 1, 8, B>(t, raw, g);
    }
}

template <int K, int DT, int V> DI void store_tile(const Tile<K> &t, gptr rowp, const Geo &g) {
    constexpr int ES = DT == 0 ? 4 : 2;
    if constexpr (K >= V) {
        constexpr int NJ = K / V;
        const uint32_t lanecol = g.lanecol;
        if (g.ncols >= (uint32_t)V) {
            sfor<NJ>([&]<int J>() LI {
                const uint32_t c0 = lanecol + (uint32_t)J * g.GV;
                const bool ok = g.rowok && c0 + V <= g.ncols;
                gptr q = rowp + (uint64_t)c0 * ES;
                if constexpr (DT == 0) {
                    sfor<V / 4>([&]<int H>() LI { st_b128(q + 16 * H, t.q[J * (V / 4) + H], ok); });
                } else {
                    const f32x4 lo = t.q[2 * J], hi = t.q[2 * J + 1];
                    const u32x4 r = {pack_bf16x2(lo.x, lo.y), pack_bf16x2(lo.z, lo.w), pack_bf16x2(hi.x, hi.y), pack_bf16x2(hi.z, hi.w)};
                    st_b128(q, __builtin_bit_cast(f32x4, r), ok);
                }
            });
        }
        if (g.part_slot != ~0u) {
            const bool own = g.rowok && g.lanecol == g.part_lane * (uint32_t)V;
            sfor<NJ>([&]<int J>() LI {
                if ((uint32_t)J == g.part_slot) {
                    sfor<V>([&]<int E>() LI {
                        if ((uint32_t)E < g.part_n) {       // wave-uniform
                            gptr q = rowp + (uint64_t)(g.part_col + E) * ES;
                            if constexpr (DT == 0) st_b32(q, TV(t, J * V + E), own);
                            else st_b16(q, (uint32_t)pack_bf16(TV(t, J * V + E)), own);
                        }
                    });
                }
            });
        }
    }
}
template <int K> DI void store_dispatch(const Tile<K> &t, uint32_t dt, uint32_t V, gptr rowp, const Geo &g) {
    if (dt == 0) {
        if (V == 4) store_tile<K, 0, 4>(t, rowp, g);
        else store_tile<K, 0, 8>(t, rowp, g);
    } else {
        store_tile<K, 1, 8>(t, rowp, g);
    }
}

// ---- wide rows ------------------------------------------------------------------------------------
// When a row is held by at least one whole wave (G >= 64), everything about the row is the same for all lanes
// of a wave: its index, its offsets in every tensor, whether it exists.  The wide instantiation of the kernel
// does that arithmetic once per wave on the scalar unit and addresses memory as a scalar row base plus a 32-bit
// lane offset (the form of the load / store instruction that takes a scalar base), so that a memory record
// costs a handful of scalar instructions and one vector instruction per chunk for the offset.
typedef const GLOBAL_AS char *gcptr_u;      // (a wave-uniform pointer)
struct Wide {
    uint32_t i1, i2, i3;    // the wave's row, decomposed over the outer dims (wave-uniform)
    uint32_t rowok;         // the wave's row lies inside the tensor
};

// byte offset of chunk J of this lane from the row base; a chunk beyond the tile's columns reads chunk 0 instead
template <int V, int ES> DI uint32_t chunk_off(const Geo &g, uint32_t lanecol, int J) {
    const uint32_t c0 = lanecol + (uint32_t)J * g.GV;
    const uint32_t cc = c0 + V <= g.ncols ? c0 : 0u;
    return cc * ES;
}
template <int K, int DT, int V, bool NT> DI void issue_wide(Tile<K> &t, const char *rowbase, const uint32_t (&vo)[K / V]) {
    constexpr int NJ = K / V;
    sfor<NJ>([&]<int J>() LI {
        gcptr q = (gcptr)(rowbase + (uint64_t)vo[J]);
        if constexpr (DT == 0) {
            sfor<V / 4>([&]<int H>() LI { t.q[J * (V / 4) + H] = ld_b128<NT>(q + 16 * H); });
        } else {
            t.q[K / 8 + J] = ld_b128<NT>(q);
        }
    });
}
// The offsets are computed before the destination register is selected: inside the selected case nothing but
// the load instructions may write a register, or the compiler would compute addresses in the registers the
// load is about to overwrite, which costs a wait for every load still in flight into them.
#define DVM_ISSUE_WIDE(DT, V, NT)                                                                   \
    {                                                                                               \
        uint32_t vo[K / V];                                                                         \
        sfor<K / V>([&]<int J>() LI { vo[J] = chunk_off<V, (DT == 0 ? 4 : 2)>(g, g.lanecol, J); }); \
        _Pragma("unroll") for (int j_ = 0; j_ < K / V; ++j_) asm volatile("" : "+v"(vo[j_]));       \
        if (ra == SRC_ACC) {                                                                        \
            issue_wide<K, DT, V, NT>(acc, rowbase, vo);                                             \
        } else {                                                                                    \
            DVM_WITH_R(ra, rr, (issue_wide<K, DT, V, NT>(rr, rowbase, vo)))                         \
        }                                                                                           \
    }

// full tile (no ragged chunk, every chunk inside the row), row inside the tensor: plain 16-byte stores
template <int K, int DT, int V> DI void store_wide_full(const Tile<K> &t, char *rowbase, const Geo &g) {
    constexpr int ES = DT == 0 ? 4 : 2;
    constexpr int NJ = K / V;
    sfor<NJ>([&]<int J>() LI {
        if (J == 0 || (uint32_t)(J * V) < g.nact) {        // wave-uniform: chunk slots the tile uses
            const uint32_t vo = (g.lanecol + (uint32_t)J * g.GV) * ES;
            GLOBAL_AS char *q = (GLOBAL_AS char *)(rowbase + (uint64_t)vo);
            if constexpr (DT == 0) {
                sfor<V / 4>([&]<int H>() LI { __builtin_nontemporal_store(t.q[J * (V / 4) + H], (GLOBAL_AS f32x4 *)(q + 16 * H)); });
            } else {
                const f32x4 lo = t.q[2 * J], hi = t.q[2 * J + 1];
                const u32x4 r = {pack_bf16x2(lo.x, lo.y), pack_bf16x2(lo.z, lo.w), pack_bf16x2(hi.x, hi.y), pack_bf16x2(hi.z, hi.w)};
                __builtin_nontemporal_store(__builtin_bit_cast(f32x4, r), (GLOBAL_AS f32x4 *)q);
            }
        }
    });
}
template <int K> DI void store_wide_full_dispatch(const Tile<K> &t, uint32_t dt, uint32_t V, char *rowbase, const Geo &g) {
    if (dt == 0) {
        if (V == 4) store_wide_full<K, 0, 4>(t, rowbase, g);
        else if constexpr (K >= 8) store_wide_full<K, 0, 8>(t, rowbase, g);
    } else {
        if constexpr (K >= 8) store_wide_full<K, 1, 8>(t, rowbase, g);
    }
}

// in-lane part of a row reduction over the accumulator.  When the tile is ragged, a chunk of a lane
// is either wholly inside the row, wholly outside, or the one chunk the row ends in: whole chunks
// are reduced unmasked and selected per chunk, only the last chunk is masked element by element.
template <int K, uint32_t R, int V> DI float lane_reduce_ragged(const Tile<K> &a, const Geo &g) {
    float v = red_ident<R>();
    if constexpr (K >= V) {
        constexpr int NJ = K / V;
        constexpr uint32_t RC = R == R_SUMSQ ? R_SUM : R;      // how partial results combine
        sfor<NJ>([&]<int J>() LI {
            if (J == 0 || (uint32_t)(J * V) < g.nact) {        // wave-uniform
                float c = red_ident<R>();
                sfor<V>([&]<int E>() LI {
                    if constexpr (R == R_SUMSQ) c = f_fma(TV(a, J * V + E), TV(a, J * V + E), c);
                    else c = red_comb<R>(c, TV(a, J * V + E));
                });
                const bool whole = g.lanecol + (uint32_t)J * g.GV + V <= g.ncols;
                v = red_comb<RC>(v, whole ? c : red_ident<R>());
            }
        });
        if (g.part_slot != ~0u) {
            const bool own = g.lanecol == g.part_lane * (uint32_t)V;
            sfor<NJ>([&]<int J>() LI {
                if ((uint32_t)J == g.part_slot) {              // wave-uniform
                    sfor<V>([&]<int E>() LI {
                        const bool ok = own && (uint32_t)E < g.part_n;
                        if constexpr (R == R_SUMSQ) {
                            const float x = ok ? TV(a, J * V + E) : 0.0f;
                            v = f_fma(x, x, v);
                        } else {
                            v = red_comb<R>(v, ok ? TV(a, J * V + E) : red_ident<R>());
                        }
                    });
                }
            });
        }
    }
    return v;
}
template <int K, uint32_t R> DI float lane_reduce(const Tile<K> &a, const Geo &g, uint32_t V) {
    float v = red_ident<R>();
    if (!g.ragged) {
        sfor<K / 4>([&]<int Q>() LI {
            if (Q == 0 || (uint32_t)(Q * 4) < g.nact) {
                sfor<4>([&]<int E>() LI {
                    if constexpr (R == R_SUMSQ) v = f_fma(TV(a, Q * 4 + E), TV(a, Q * 4 + E), v);
                    else v = red_comb<R>(v, TV(a, Q * 4 + E));
                });
            }
        });
    } else if (V == 8) {
        v = lane_reduce_ragged<K, R, 8>(a, g);
    } else {
        v = lane_reduce_ragged<K, R, 4>(a, g);
    }
    return v;
}

// the two halves apart (a row longer than a tile is reduced tile after tile within the lane, then once across the lanes)
template <int K> DI float lane_reduce_dispatch(const Tile<K> &a, const Geo &g, uint32_t V, uint32_t kind) {
    switch (kind) {
        case R_MAX: return lane_reduce<K, R_MAX>(a, g, V);
        case R_MIN: return lane_reduce<K, R_MIN>(a, g, V);
        case R_SUMSQ: return lane_reduce<K, R_SUMSQ>(a, g, V);
        default: return lane_reduce<K, R_SUM>(a, g, V);
    }
}
DI float wave_allreduce_dispatch(float v, uint32_t kind, uint32_t width) {
    switch (kind) {
        case R_MAX: return wave_allreduce<R_MAX>(v, width);
        case R_MIN: return wave_allreduce<R_MIN>(v, width);
        default: return wave_allreduce<R_SUM>(v, width);
    }
}
template <int K> DI float reduce_dispatch(const Tile<K> &a, const Geo &g, uint32_t V, uint32_t kind, uint32_t width) {
    switch (kind) {
        case R_MAX: return wave_allreduce<R_MAX>(lane_reduce<K, R_MAX>(a, g, V), width);
        case R_MIN: return wave_allreduce<R_MIN>(lane_reduce<K, R_MIN>(a, g, V), width);
        case R_SUMSQ: return wave_allreduce<R_SUM>(lane_reduce<K, R_SUMSQ>(a, g, V), width);
        default: return wave_allreduce<R_SUM>(lane_reduce<K, R_SUM>(a, g, V), width);
    }
}

// Every record starts on a 16-byte boundary and is 4 or 8 words long, so one scalar 128-bit load
// fetches a whole record (the view forms take a second one).  The record after the current one is
// requested before the current handler runs, so that the scalar-cache latency of decoding overlaps
// the vector work (the pipelining of decode and execute of Section 4.3).  The prefetch may reach
// past the code body: it stays inside the kernel-argument struct.
typedef uint32_t u32x4s __attribute__((ext_vector_type(4)));
DI u32x4s fetch4(const uint32_t *code, uint32_t pc) {
    return *(const u32x4s *)__builtin_assume_aligned(code + pc, 16);
}
// the same with a byte offset: one scalar load with a register offset, no 64-bit address arithmetic
DI u32x4s fetch4b(const uint32_t *code, uint32_t byte_off) {
    return *(const u32x4s *)__builtin_assume_aligned((const char *)code + (uint64_t)byte_off, 16);
}

DI float pick_s(float s0, float s1, float s2, float s3, uint32_t i) {
    float v = s0;
    v = i == 1 ? s1 : v;
    v = i == 2 ? s2 : v;
    v = i == 3 ? s3 : v;
    return v;
}

// unsigned division by an invariant divisor with a precomputed multiplier and two shifts
// (Granlund & Montgomery, "Division by invariant integers using multiplication", 32-bit case)
DI uint32_t magic_div(uint32_t n, uint32_t m, uint32_t sh) {
    uint32_t t = __umulhi(m, n);
    return (t + ((n - t) >> (sh & 0xFF))) >> (sh >> 8);
}
DI uint32_t sdiv_u(uint32_t n, uint32_t m, uint32_t sh) {   // the same on wave-uniform values
    uint32_t t = (uint32_t)(((uint64_t)m * n) >> 32);
    return (t + ((n - t) >> (sh & 0xFF))) >> (sh >> 8);
}

// Where a tile of a segment sits.  Columns (wave-uniform): first column and width of column tile
// `tile_c`, and which chunk the row ends in.  Rows: the lane's row decomposed over the outer
// iteration dims; `rp` is the row of the tile this lane holds.
DI void tile_cols(Geo &gt, const uint32_t *sh, uint32_t tile_c, uint32_t G, uint32_t V) {
    const uint32_t TC = sh[S_TC];
    const uint64_t D0 = (uint64_t)sh[S_D0LO] | ((uint64_t)sh[S_D0HI] << 32);
    gt.colbase = (uint64_t)tile_c * TC;
    const uint64_t rem = D0 - gt.colbase;
    gt.ncols = rem < TC ? (uint32_t)rem : TC;
    const uint32_t full_chunks = V == 8 ? gt.ncols >> 3 : gt.ncols >> 2;      // V is 4 or 8
    gt.part_n = gt.ncols - full_chunks * V;
    gt.part_slot = ~0u;
    gt.part_lane = 0;
    gt.part_col = full_chunks * V;
    if (gt.part_n != 0) {
        gt.part_slot = __builtin_amdgcn_readfirstlane(full_chunks / G);
        gt.part_lane = full_chunks - gt.part_slot * G;
    }
    // rows never mix in a reduction, so only invalid columns inside live chunks need a mask
    gt.ragged = gt.ncols != gt.nact * G;
}
DI void tile_rows_at(Geo &gt, const uint32_t *sh, uint32_t row, bool ok) {
    gt.rowok = ok;
    const uint32_t rowc = gt.rowok ? row : 0;
    gt.i1 = rowc; gt.i2 = 0; gt.i3 = 0;
    const uint32_t D1 = sh[S_D1];
    if (D1 != 0) {
        const uint32_t q = magic_div(rowc, sh[S_M1], sh[S_SH1]);
        gt.i1 = rowc - q * D1;
        gt.i2 = q;
        const uint32_t D2 = sh[S_D2];
        if (D2 != 0) {
            const uint32_t q2 = magic_div(q, sh[S_M2], sh[S_SH2]);
            gt.i2 = q - q2 * D2;
            gt.i3 = q2;
        }
    }
}
DI void tile_rows(Geo &gt, const uint32_t *sh, uint32_t tile_r, uint32_t rp, uint32_t tid, uint32_t RP, uint32_t seg_threads) {
    const uint32_t row = tile_r * RP + rp;
    tile_rows_at(gt, sh, row, (row < sh[S_NROWS]) && (rp < RP) && (tid < seg_threads));
}

// ------------------------------------------------------------------------------------------
// row-invariant operands kept in LDS
// ------------------------------------------------------------------------------------------
#define LDS_AS __attribute__((address_space(3)))
// Copy the first `d0` elements of the tensor at `src` (dtype dt) into an LDS image of n16 16-byte pieces, zero behind
// the row's end.  All `nthreads` threads of the workgroup take part; every branch is wave-uniform (a thread
// past the last piece copies the last piece once more).
DI void lds_copy_row(LDS_AS char *dst, uint32_t n16, gcptr src, uint64_t d0, uint32_t dt, uint32_t tid, uint32_t nthreads) {
    const uint32_t es = dt == 0 ? 4u : 2u;
    const uint32_t epp = 16u / es;                        // elements per piece
    const bool aligned = (((uint64_t)(uintptr_t)src) & 15u) == 0;
    for (uint32_t base = 0; base < n16; base += nthreads) {
        const uint32_t want = base + tid;
        const uint32_t i = want < n16 ? want : n16 - 1;
        const uint64_t e0 = (uint64_t)i * epp;
        const bool whole = aligned && e0 + epp <= d0;
        u32x4 v;
        if (__builtin_amdgcn_ballot_w64(!whole) == 0) {     // the usual case: this wave's pieces all lie inside the row
            v = *(const GLOBAL_AS u32x4 *)(src + (uint64_t)i * 16u);
        } else {
            uint32_t wds[4] = {0u, 0u, 0u, 0u};
            if (dt == 0) {
                sfor<4>([&]<int E>() LI {
                    const uint64_t e = e0 + E;
                    const uint32_t x = *(const GLOBAL_AS uint32_t *)(src + (e < d0 ? e : 0) * 4u);
                    wds[E] = e < d0 ? x : 0u;
                });
            } else {
                sfor<8>([&]<int E>() LI {
                    const uint64_t e = e0 + E;
                    const uint32_t x = *(const GLOBAL_AS uint16_t *)(src + (e < d0 ? e : 0) * 2u);
                    wds[E / 2] |= (e < d0 ? x : 0u) << (16 * (E & 1));
                });
            }
            v = u32x4{wds[0], wds[1], wds[2], wds[3]};
        }
        *(LDS_AS u32x4 *)(dst + (size_t)i * 16u) = v;
    }
}
// Element E (0..V-1) of a chunk of an LDS image held as raw 16-byte pieces: r0 (and r1 for fp32 chunks of eight).
template <int E> DI float lds_elem(const u32x4 &r0, const u32x4 &r1, bool bf16) {
    if (bf16) {
        const uint32_t w = r0[E / 2];
        return (E & 1) ? bf16_hi(w) : bf16_lo(w);
    }
    return __builtin_bit_cast(float, E < 4 ? r0[E & 3] : r1[E & 3]);
}
// acc = acc * s [* A] [+ B] chunk by chunk, A and B read from their LDS images (V = 4: fp32 images; V = 8: bf16 or
// fp32, per image).  A chunk of this lane that lies beyond the image (the lane holds fewer live chunks than
// others) reads the image's first chunk: its result is never stored and reductions mask it.
template <int K, int V, bool HASA, bool HASB>
DI void lds_fma(Tile<K> &acc, float s, const LDS_AS char *pa, const LDS_AS char *pb, bool a_bf16, bool b_bf16, uint32_t lanecol, const Geo &g) {
    if constexpr (K >= V) {
        constexpr int NJ = K / V;
        const uint32_t ncols_pad = (g.ncols + (uint32_t)V - 1u) / (uint32_t)V * (uint32_t)V;
        const uint32_t esa = (V == 8 && a_bf16) ? 2u : 4u, esb = (V == 8 && b_bf16) ? 2u : 4u;
        sfor<NJ>([&]<int J>() LI {
            if ((uint32_t)J < g.nvec) {         // wave-uniform
                const uint32_t c0 = lanecol + (uint32_t)J * g.GV;
                const uint32_t cc = c0 + V <= ncols_pad ? c0 : 0u;
                u32x4 a0 = {0u, 0u, 0u, 0u}, a1 = a0, b0 = a0, b1 = a0;
                if constexpr (HASA) {
                    a0 = *(const LDS_AS u32x4 *)(pa + cc * esa);
                    if (V == 8 && !a_bf16) a1 = *(const LDS_AS u32x4 *)(pa + cc * esa + 16u);
                }
                if constexpr (HASB) {
                    b0 = *(const LDS_AS u32x4 *)(pb + cc * esb);
                    if (V == 8 && !b_bf16) b1 = *(const LDS_AS u32x4 *)(pb + cc * esb + 16u);
                }
                sfor<V>([&]<int E>() LI {
                    const float t = TV(acc, J * V + E) * s;
                    if constexpr (HASA && HASB) TV(acc, J * V + E) = f_fma(t, lds_elem<E>(a0, a1, V == 8 && a_bf16), lds_elem<E>(b0, b1, V == 8 && b_bf16));
                    else if constexpr (HASA) TV(acc, J * V + E) = t * lds_elem<E>(a0, a1, V == 8 && a_bf16);
                    else TV(acc, J * V + E) = t + lds_elem<E>(b0, b1, V == 8 && b_bf16);
                });
            }
        });
    }
}

// ------------------------------------------------------------------------------------------
// the interpreter
// ------------------------------------------------------------------------------------------
// Run STMT with `RR` naming tile register number IDX (a wave-uniform value): one switch case per
// register, so that every case references its register statically.
#define DVM_WITH_R(IDX, RR, STMT)                                        \
    switch (IDX) {                                                       \
        case 0: { Tile<K> &RR = r0; STMT; } break;                         \
        case 1: if constexpr (NR > 1) { Tile<K> &RR = r1; STMT; } break;   \
        case 2: if constexpr (NR > 2) { Tile<K> &RR = r2; STMT; } break;   \
        case 3: if constexpr (NR > 3) { Tile<K> &RR = r3; STMT; } break;   \
        case 4: if constexpr (NR > 4) { Tile<K> &RR = r4; STMT; } break;   \
        case 5: if constexpr (NR > 5) { Tile<K> &RR = r5; STMT; } break;   \
        default: break;                                                  \
    }
#define DVM_WITH_R2(IDX, RR, STMT)                                       \
    switch (IDX) {                                                       \
        case 0: { Tile<K> &RR = r0; STMT; } break;                         \
        case 1: if constexpr (NR > 1) { Tile<K> &RR = r1; STMT; } break;   \
        case 2: if constexpr (NR > 2) { Tile<K> &RR = r2; STMT; } break;   \
        case 3: if constexpr (NR > 3) { Tile<K> &RR = r3; STMT; } break;   \
        case 4: if constexpr (NR > 4) { Tile<K> &RR = r4; STMT; } break;   \
        case 5: if constexpr (NR > 5) { Tile<K> &RR = r5; STMT; } break;   \
        default: break;                                                  \
    }
#define DVM_GET_S(I) pick_s(s0, s1, s2, s3, (I))
#define DVM_SET_S(I, VAL)                   \
    do {                                    \
        const uint32_t si_ = (I);           \
        const float sv_ = (VAL);            \
        s0 = si_ == 0 ? sv_ : s0;           \
        s1 = si_ == 1 ? sv_ : s1;           \
        s2 = si_ == 2 ? sv_ : s2;           \
        s3 = si_ == 3 ? sv_ : s3;           \
    } while (0)
#define DVM_I64(LO, HI) ((int64_t)((uint64_t)(LO) | ((uint64_t)(HI) << 32)))

// The handlers that use the tile geometry must see it through values the optimiser cannot trace
// back across iterations; otherwise it hoists their address arithmetic and lane masks into the
// tile prologue and executes them for every tile, used or not.  The empty assembly statements pin
// each value to its register at no cost.  Handlers that work on registers only skip all of this.
#define DVM_GEO()                                                                                             \
    asm volatile("" : "+v"(gt.i1), "+v"(gt.i2), "+v"(gt.i3), "+v"(gt.lanecol), "+v"(gt.rowok));   \
    Geo g = gt;                                                                                               \
    {                                                                                                         \
        uint32_t cb_lo = __builtin_amdgcn_readfirstlane((uint32_t)gt.colbase);                                \
        uint32_t cb_hi = __builtin_amdgcn_readfirstlane((uint32_t)(gt.colbase >> 32));                        \
        g.ncols = __builtin_amdgcn_readfirstlane(gt.ncols);                                                   \
        g.GV = __builtin_amdgcn_readfirstlane(gt.GV);                                                         \
        g.nvec = __builtin_amdgcn_readfirstlane(gt.nvec);                                                     \
        g.nact = __builtin_amdgcn_readfirstlane(gt.nact);                                                     \
        g.part_slot = __builtin_amdgcn_readfirstlane(gt.part_slot);                                           \
        g.part_lane = __builtin_amdgcn_readfirstlane(gt.part_lane);                                           \
        g.part_col = __builtin_amdgcn_readfirstlane(gt.part_col);                                             \
        g.part_n = __builtin_amdgcn_readfirstlane(gt.part_n);                                                 \
        g.ragged = __builtin_amdgcn_readfirstlane(gt.ragged);                                                 \
        asm volatile("" : "+s"(cb_lo), "+s"(cb_hi), "+s"(g.ncols), "+s"(g.GV), "+s"(g.nvec), "+s"(g.nact));   \
        asm volatile("" : "+s"(g.part_slot), "+s"(g.part_lane), "+s"(g.part_col), "+s"(g.part_n), "+s"(g.ragged)); \
        g.colbase = (uint64_t)cb_lo | ((uint64_t)cb_hi << 32);                                                \
    }

// CRED: the instantiation that also runs segments which reduce along the penultimate axis (unit loop,
// accumulate and combine records).  Programs without such a segment run the plain instantiation, whose
// tile loop carries none of that bookkeeping (it costs scalar registers the interpreter loop has none
// to spare of: 5-10 % on short tiles).
// WIDE: the instantiation for launches in which every segment spreads a row over at least one whole wave (see
// "wide rows" above); the other instantiations take any geometry.
template <int K, int NR, int MAXT, int WAVES, bool CRED, bool WIDE>
__global__ void __launch_bounds__(MAXT) __attribute__((amdgpu_waves_per_eu(WAVES))) dvm_vm_kernel(const KArgs args) {
    static_assert(!(CRED && WIDE), "the instantiation for reductions along the penultimate axis is the general one");
    __shared__ float red_lds[2][16];
    // (sized by the launch: 1 KiB per wave of the widest segment that reduces along the penultimate axis, else nothing)
    extern __shared__ __align__(16) float comb_lds[];

    // the register file of one lane: accumulator, tile registers, row-scalar registers
    Tile<K> acc, r0, r1, r2, r3, r4, r5;
    tile_zero<K>(acc); tile_zero<K>(r0); tile_zero<K>(r1); tile_zero<K>(r2);
    tile_zero<K>(r3); tile_zero<K>(r4); tile_zero<K>(r5);
    float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;

    const uint32_t tid = threadIdx.x;
    const uint32_t wave = __builtin_amdgcn_readfirstlane(tid) >> 6;
    const uint32_t bid = blockIdx.x;
    const uint32_t ngrid = gridDim.x;
    uint32_t red_par = 0;
    uint32_t n_sync = 0;                    // grid-wide synchronisation points passed so far
    uint32_t rot = 0;                       // first workgroup of the next segment's tiles (rotating assignment)
    const uint32_t *code = args.code;
    // the launch's tensor addresses, one per lane: a memory record reads the one it needs with a single lane read
    // (the index is wave-uniform) instead of a scalar load whose latency it would have to wait for
    uint32_t tp_lo, tp_hi;
    {
        const uint64_t mine = args.tensors[tid & (DVM_MAX_TENSORS - 1)];
        tp_lo = (uint32_t)mine;
        tp_hi = (uint32_t)(mine >> 32);
    }
    // A batched launch runs the whole program once per set of tensors, the sets one after the other; the workgroups
    // pass from one set to the next without waiting for each other (the sets are independent).
    for (uint32_t set = 0; set < args.n_sets; ++set) {
    if (args.sets != 0) {
        const uint32_t slot = tid & (DVM_MAX_TENSORS - 1);
        const uint32_t idx = set * args.n_tensors + (slot < args.n_tensors ? slot : 0u);
        const uint64_t mine = ((const GLOBAL_AS uint64_t *)args.sets)[idx];
        tp_lo = (uint32_t)mine;
        tp_hi = (uint32_t)(mine >> 32);
    }
#define DVM_TENSOR(IDX)                                                                                  \
    ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)tp_lo, (int)(IDX)) |                             \
     ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)tp_hi, (int)(IDX)) << 32))

    uint32_t seg = 0;                       // word offset of the current segment
    for (uint32_t si = 0; si < args.nseg; ++si) {
        const uint32_t *sh = &code[seg];
        const uint32_t seg_words = sh[S_WORDS];
        if (si < args.seg_first) {          // (a segment of an earlier launch of this program)
            seg += seg_words;
            continue;
        }
        const uint32_t code_size = sh[S_CODESIZE];
        const uint32_t M = sh[S_NTILES];
        const uint32_t geom = sh[S_GEOM];
        const uint32_t G = geom & 0xFFFF, V = (geom >> 16) & 0xFF, nvec = geom >> 24;
        const uint32_t RP = sh[S_RP] & 0xFFFF, seg_threads = sh[S_RP] >> 16;
        const uint32_t tbase = sh[S_TBASE];
        const uint32_t body = seg + SH_WORDS;
        const uint32_t body_end = body + code_size;

        Geo gt;
        gt.GV = G * V;
        gt.nvec = nvec;
        gt.nact = nvec * V;
        const uint32_t rp = tid / G;            // row of the tile held by this lane
        gt.lanecol = (tid - rp * G) * V;
        const uint32_t gw = G >> 6;             // waves per row when a row spans waves
        const uint32_t width = G < 64 ? G : 64;
        const uint32_t w0i = gw > 1 ? (wave / gw) * gw : wave;   // first wave of this lane's row

        // The prologue of this segment overwrites the LDS images the previous one may still be reading
        if (sh[S_FLAGS] & SF_LDS) __syncthreads();

        // A segment that depends on earlier ones of this launch waits here (Section 5.1, temporal stacking of
        // dependent operators).  Release: this workgroup's stores are complete and visible to the device.
        if (sh[S_FLAGS] & (SF_SYNC_WG | SF_SYNC_GRID)) {
            // every wave: its own stores have left the wave (they sit in this compute unit's caches or beyond)
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __syncthreads();
            if (sh[S_FLAGS] & SF_SYNC_GRID) {
                // every workgroup of the launch arrives once per such point; the grid was sized to be resident as a
                // whole, so all arrive; should the machine be shared and some never start, the bounded wait ends
                // with the status word set and this workgroup leaves the kernel.  One wave per workgroup makes
                // the workgroup's stores visible to the device (the caches it has to write back and, afterwards,
                // invalidate are shared by all its waves) and waits.
                ++n_sync;
                if (wave == 0) {
                    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
                    uint32_t ok = 1;
                    if (tid == 0) {
                        GLOBAL_AS uint32_t *wsp = (GLOBAL_AS uint32_t *)args.ws;
                        __hip_atomic_fetch_add(&wsp[WS_ARRIVED], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
                        const uint32_t target = n_sync * ngrid;
                        for (uint32_t spins = 0; __hip_atomic_load(&wsp[WS_ARRIVED], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT) < target; ++spins) {
                            if (spins >= args.spin_limit || __hip_atomic_load(&wsp[WS_STATUS], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                                __hip_atomic_store(&wsp[WS_STATUS], WS_STATUS_GAVE_UP, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                ok = 0;
                                break;
                            }
                            __builtin_amdgcn_s_sleep(8);
                        }
                        red_lds[0][0] = __builtin_bit_cast(float, ok);
                    }
                    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                }
                __syncthreads();
                const uint32_t go = __builtin_bit_cast(uint32_t, red_lds[0][0]);
                __syncthreads();
                if (go == 0) return;
            } else {
                // (lines of the buffer that this compute unit cached before the producer wrote them must go)
                if (wave == 0) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
                __syncthreads();
            }
        }

        // Algorithm 2: m = ceil(M / N); this workgroup runs tiles [m*id, min(M, m*(id+1))).  In a
        // spatially stacked launch N and id count the workgroups of this segment's share only.
        uint32_t sbid = bid, sgrid = ngrid;
        if (args.rotate != 0) {
            sbid = bid >= rot ? bid - rot : bid + ngrid - rot;
            rot += M % ngrid;
            if (rot >= ngrid) rot -= ngrid;
        }
        if (sh[S_NWG] != 0) {
            sbid = bid - sh[S_WG0];
            sgrid = sh[S_NWG];
            if (sbid >= sgrid) {        // (unsigned: also true for workgroups below the share)
                seg += seg_words;
                continue;
            }
        }
        const uint32_t m = (M + sgrid - 1) / sgrid;
        const uint64_t t_lo64 = (uint64_t)m * sbid;
        uint32_t t_lo = t_lo64 < M ? (uint32_t)t_lo64 : M;
        uint32_t t_hi = (M - t_lo) < m ? M : t_lo + m;
        uint32_t t_step = 1;
        // Interleaved assignment: workgroup id runs tiles id, id + N, id + 2N, ...  At any moment the resident
        // workgroups then work on one contiguous stretch of the tensors, which the memory system of this
        // machine serves measurably faster than N streams that are far apart (the blocked ranges).
        if (sh[S_FLAGS] & SF_INTERLEAVED) {
            t_lo = sbid < M ? sbid : M;
            t_hi = M;
            t_step = sgrid;
        }

        const uint32_t nct = sh[S_NCT];
        if (nct <= 1) tile_cols(gt, sh, 0, G, V);
        // A segment that reduces along the penultimate axis counts units (outer index, column tile) in M;
        // the workgroup walks the `inner` rows of a unit RP at a time, one row per wave and step (rin),
        // accumulating in tile registers, and runs the epilogue records after the last step.  Other
        // segments: one step per tile.
        // A segment over rows longer than a tile (SF_LONGROW) counts rows in M; the workgroup passes over a row once per
        // reduction and once more for the rest (lr_phase), each pass column tile after column tile (lr_c): a pass runs
        // the records from the start of the body up to its reduction, skipping the reductions whose value is final and
        // every store; the last pass runs to the end and stores.
        const bool longrow = (sh[S_FLAGS] & SF_LONGROW) != 0;
        const uint32_t n_red = longrow ? sh[S_NCTSH] : 0u;
        uint32_t lr_phase = 0, lr_c = 0;
        float racc = 0.0f;                  // the lane's part of the reduction of the current pass
        uint32_t rin = 0;
        for (uint32_t tile = t_lo; tile < t_hi;) {
            const uint32_t *shl = sh;
            uint32_t this_end = body_end;
            if constexpr (CRED) {
                const uint32_t inner = shl[S_INNER];
                uint32_t tile_r0 = tile;
                if (nct > 1) {          // (a single column tile was placed once, before the loop)
                    tile_r0 = sdiv_u(tile, shl[S_NCTM], shl[S_NCTSH]);
                    if (rin == 0) tile_cols(gt, shl, tile - tile_r0 * nct, G, V);      // the steps of a unit share its columns
                }
                if (inner != 0) {
                    const uint32_t r = rin * RP + rp;
                    tile_rows_at(gt, shl, tile_r0 * inner + r, (r < inner) && (rp < RP) && (tid < seg_threads));
                    if ((rin + 1) * RP < inner && !(shl[S_FLAGS] & SF_CSTREAM)) this_end = body + shl[S_EPILOG];
                } else {
                    tile_rows(gt, shl, tile_r0, rp, tid, RP, seg_threads);
                }
            } else {
                // tile prologue: where this tile sits, which of its lanes and chunks are valid
                uint32_t tile_r = tile;
                if (longrow) {
                    tile_cols(gt, sh, lr_c, G, V);
                } else if (nct > 1) {   // (a single column tile was placed once, before the loop)
                    tile_r = sdiv_u(tile, sh[S_NCTM], sh[S_NCTSH]);
                    tile_cols(gt, sh, tile - tile_r * nct, G, V);
                }
                tile_rows(gt, sh, tile_r, rp, tid, RP, seg_threads);
            }
            Wide wd;
            if constexpr (WIDE) {       // all lanes of a wave hold the same row: its place as wave-uniform values
                wd.i1 = __builtin_amdgcn_readfirstlane(gt.i1);
                wd.i2 = __builtin_amdgcn_readfirstlane(gt.i2);
                wd.i3 = __builtin_amdgcn_readfirstlane(gt.i3);
                wd.rowok = __builtin_amdgcn_readfirstlane(gt.rowok);
            }

            // the first tile of this workgroup also runs the prologue records (pinned operands)
            // (its second part runs again when the second outer index of the tile's first or last row
            // differs from that of the previous tile: an operand pinned there varies with that index only)
            uint32_t first = body;
            uint32_t red_idx = 0;           // reductions met so far in this pass over the records
            if (tile != t_lo || rin != 0) {
                first = body + shl[S_PROLOG];
                if (shl[S_PROLOGA] != shl[S_PROLOG]) {
                    const uint32_t m1 = shl[S_M1], sh1 = shl[S_SH1];
                    const uint32_t ra = tile * RP;          // prologues exist in row mode only: tile = row tile
                    const uint32_t rb = ra - t_step * RP;   // first row of the tile this workgroup ran before
                    const bool crossed = sdiv_u(ra, m1, sh1) != sdiv_u(rb, m1, sh1) ||
                                         sdiv_u(ra + RP - 1, m1, sh1) != sdiv_u(rb + RP - 1, m1, sh1);
                    if (crossed) first = body + shl[S_PROLOGA];
                }
            }
            // (the program counter is a byte offset into the code)
            u32x4s nw = fetch4b(code, first * 4);
            for (uint32_t pcb = first * 4; pcb < this_end * 4;) {
                const u32x4s cw = nw;
                // (elements are copied to scalars first: bit-casting a vector element directly is miscompiled)
                const uint32_t w = cw.x, cw1 = cw.y, cw2 = cw.z, cw3 = cw.w;
                const uint32_t op = w & 0xFF, a = (w >> 16) & 0xFF, b = w >> 24;
                const uint32_t cur = pcb >> 2;
                pcb += (w >> 6) & 0x3FCu;       // record length in words, times four
                nw = fetch4b(code, pcb);
                switch (op) {
                    case I_LOAD:
                    case I_VLOAD: {
                        // A run of consecutive load records is one group: first every record of the run issues its
                        // requests (all of them are then in flight together, each into its own destination
                        // register), then a second walk over the same records finishes them (bf16 widening in
                        // place, the chunk a ragged row ends in).
                        if constexpr (WIDE) {
                            Geo g = gt;
                            uint32_t gp = cur;
                            u32x4s rw = cw;
                            const bool slow_finish = g.part_slot != ~0u || g.ncols < V;
                            uint32_t widen = 0;             // bit r + 1: register r (bit 0: ACC) holds raw bf16 bits
                            for (;;) {
                                asm volatile("" : "+v"(g.lanecol));
                                const uint32_t r0w = rw.x, w1 = rw.y, r2w = rw.z, r3w = rw.w;
                                const uint32_t rop = r0w & 0xFF, ra = (r0w >> 16) & 0xFF;
                                const uint32_t ti = w1 & 0xFF, dt = (w1 >> 8) & 0xFF;
                                int64_t off = (int64_t)wd.i1 * DVM_I64(r2w, r3w) + (int64_t)g.colbase;
                                if (rop == I_VLOAD) {
                                    const u32x4s hw = fetch4(code, gp + 4);
                                    const uint32_t h0 = hw.x, h1 = hw.y, h2 = hw.z, h3 = hw.w;
                                    off += (int64_t)wd.i2 * DVM_I64(h0, h1) + (int64_t)wd.i3 * DVM_I64(h2, h3);
                                }
                                const char *rowbase = (const char *)DVM_TENSOR(tbase + ti) + off * (dt == 0 ? 4 : 2);
                                if (g.ncols >= V) {
                                    if ((w1 >> 16) & MF_STREAM) {
                                        if (dt != 0) { if constexpr (K >= 8) DVM_ISSUE_WIDE(1, 8, true) }
                                        else if (V == 4) DVM_ISSUE_WIDE(0, 4, true)
                                        else { if constexpr (K >= 8) DVM_ISSUE_WIDE(0, 8, true) }
                                    } else {
                                        if (dt != 0) { if constexpr (K >= 8) DVM_ISSUE_WIDE(1, 8, false) }
                                        else if (V == 4) DVM_ISSUE_WIDE(0, 4, false)
                                        else { if constexpr (K >= 8) DVM_ISSUE_WIDE(0, 8, false) }
                                    }
                                }
                                if (dt != 0) widen |= ra == SRC_ACC ? 1u : 2u << ra;
                                gp += (r0w >> 8) & 0xFF;
                                if (gp >= this_end) break;
                                rw = fetch4(code, gp);
                                const uint32_t nop = rw.x & 0xFF;
                                if (nop != I_LOAD && nop != I_VLOAD) break;
                            }
                            if (slow_finish) {          // ragged rows: walk the records again (row address for the last chunk)
                                for (uint32_t fp = cur; fp < gp;) {
                                    asm volatile("" : "+v"(g.lanecol));
                                    const u32x4s fw = fetch4(code, fp);
                                    const uint32_t r0w = fw.x, w1 = fw.y, r2w = fw.z, r3w = fw.w;
                                    const uint32_t rop = r0w & 0xFF, ra = (r0w >> 16) & 0xFF;
                                    const uint32_t ti = w1 & 0xFF, dt = (w1 >> 8) & 0xFF;
                                    int64_t off = (int64_t)wd.i1 * DVM_I64(r2w, r3w) + (int64_t)g.colbase;
                                    if (rop == I_VLOAD) {
                                        const u32x4s hw = fetch4(code, fp + 4);
                                        const uint32_t h0 = hw.x, h1 = hw.y, h2 = hw.z, h3 = hw.w;
                                        off += (int64_t)wd.i2 * DVM_I64(h0, h1) + (int64_t)wd.i3 * DVM_I64(h2, h3);
                                    }
                                    gcptr rowp = (gcptr)((const char *)DVM_TENSOR(tbase + ti) + off * (dt == 0 ? 4 : 2));
                                    if (ra == SRC_ACC) {
                                        finish_dispatch<K>(acc, dt, V, rowp, g);
                                    } else {
                                        DVM_WITH_R(ra, rr, (finish_dispatch<K>(rr, dt, V, rowp, g)))
                                    }
                                    fp += (r0w >> 8) & 0xFF;
                                }
                            } else if (widen != 0) {    // full rows: only the bf16 registers need their second half
                                if constexpr (K >= 8) {
                                    if (widen & 1u) finish_tile<K, 1, 8>(acc, nullptr, g);
                                    if (widen & 2u) finish_tile<K, 1, 8>(r0, nullptr, g);
                                    if constexpr (NR > 1) if (widen & 4u) finish_tile<K, 1, 8>(r1, nullptr, g);
                                    if constexpr (NR > 2) if (widen & 8u) finish_tile<K, 1, 8>(r2, nullptr, g);
                                    if constexpr (NR > 3) if (widen & 16u) finish_tile<K, 1, 8>(r3, nullptr, g);
                                    if constexpr (NR > 4) if (widen & 32u) finish_tile<K, 1, 8>(r4, nullptr, g);
                                    if constexpr (NR > 5) if (widen & 64u) finish_tile<K, 1, 8>(r5, nullptr, g);
                                }
                            }
                            pcb = gp * 4;
                            nw = fetch4b(code, pcb);
                            break;
                        }
                        DVM_GEO()
                        uint32_t gp = cur;              // word offset of the record being issued
                        u32x4s rw = cw;
                        bool finish = g.part_slot != ~0u || g.ncols < V;
                        for (;;) {
                            // (the lane's column is made opaque once per record: otherwise the chunk addresses of every
                            // dtype and chunk width are computed ahead of the loop and held in registers throughout)
                            asm volatile("" : "+v"(g.lanecol));
                            const uint32_t r0w = rw.x, w1 = rw.y, r2w = rw.z, r3w = rw.w;
                            const uint32_t rop = r0w & 0xFF, ra = (r0w >> 16) & 0xFF;
                            const uint32_t ti = w1 & 0xFF, dt = (w1 >> 8) & 0xFF;
                            int64_t off = (int64_t)g.i1 * DVM_I64(r2w, r3w) + (int64_t)g.colbase;
                            if (rop == I_VLOAD) {
                                const u32x4s hw = fetch4(code, gp + 4);
                                const uint32_t h0 = hw.x, h1 = hw.y, h2 = hw.z, h3 = hw.w;
                                off += (int64_t)g.i2 * DVM_I64(h0, h1) + (int64_t)g.i3 * DVM_I64(h2, h3);
                            }
                            const uint32_t es = dt == 0 ? 4 : 2;
                            gcptr rowp = (gcptr)DVM_TENSOR(tbase + ti) + off * es;
                            const bool nt = ((w1 >> 16) & MF_STREAM) != 0;
                            if (ra == SRC_ACC) {
                                request_dispatch<K>(acc, dt, V, nt, rowp, g);
                            } else {
                                DVM_WITH_R(ra, rr, (request_dispatch<K>(rr, dt, V, nt, rowp, g)))
                            }
                            finish |= dt != 0;
                            gp += (r0w >> 8) & 0xFF;
                            if (gp >= this_end) break;
                            rw = fetch4(code, gp);
                            const uint32_t nop = rw.x & 0xFF;
                            if (nop != I_LOAD && nop != I_VLOAD) break;
                        }
                        if (finish) {
                            for (uint32_t fp = cur; fp < gp;) {
                                asm volatile("" : "+v"(g.lanecol));
                                const u32x4s fw = fetch4(code, fp);
                                const uint32_t r0w = fw.x, w1 = fw.y, r2w = fw.z, r3w = fw.w;
                                const uint32_t rop = r0w & 0xFF, ra = (r0w >> 16) & 0xFF;
                                const uint32_t ti = w1 & 0xFF, dt = (w1 >> 8) & 0xFF;
                                gcptr rowp = nullptr;
                                if (g.part_slot != ~0u) {       // (only the ragged chunk needs the address again)
                                    int64_t off = (int64_t)g.i1 * DVM_I64(r2w, r3w) + (int64_t)g.colbase;
                                    if (rop == I_VLOAD) {
                                        const u32x4s hw = fetch4(code, fp + 4);
                                        const uint32_t h0 = hw.x, h1 = hw.y, h2 = hw.z, h3 = hw.w;
                                        off += (int64_t)g.i2 * DVM_I64(h0, h1) + (int64_t)g.i3 * DVM_I64(h2, h3);
                                    }
                                    rowp = (gcptr)DVM_TENSOR(tbase + ti) + off * (dt == 0 ? 4 : 2);
                                }
                                if (ra == SRC_ACC) {
                                    finish_dispatch<K>(acc, dt, V, rowp, g);
                                } else {
                                    DVM_WITH_R(ra, rr, (finish_dispatch<K>(rr, dt, V, rowp, g)))
                                }
                                fp += (r0w >> 8) & 0xFF;
                            }
                        }
                        pcb = gp * 4;                   // resume behind the group
                        nw = fetch4b(code, pcb);
                        break;
                    }
                    case I_STORE:
                    case I_VSTORE: {
                        if (longrow && lr_phase != n_red) break;    // (only the last pass over a long row stores)
                        if constexpr (WIDE) {
                            if (gt.part_slot == ~0u && gt.ragged == 0 && gt.ncols >= V) {   // a full tile: plain stores
                                if (wd.rowok) {
                                    Geo g = gt;
                                    asm volatile("" : "+v"(g.lanecol));
                                    const uint32_t w1 = cw1;
                                    const uint32_t ti = w1 & 0xFF, dt = (w1 >> 8) & 0xFF;
                                    int64_t off = (int64_t)wd.i1 * DVM_I64(cw2, cw3) + (int64_t)g.colbase;
                                    if (op == I_VSTORE) {
                                        const u32x4s hw = fetch4(code, cur + 4);
                                        const uint32_t h0 = hw.x, h1 = hw.y, h2 = hw.z, h3 = hw.w;
                                        off += (int64_t)wd.i2 * DVM_I64(h0, h1) + (int64_t)wd.i3 * DVM_I64(h2, h3);
                                    }
                                    char *rowbase = (char *)DVM_TENSOR(tbase + ti) + off * (dt == 0 ? 4 : 2);
                                    if (a == SRC_ACC) {
                                        if (b != 0) tile_bins<K, B_MUL>(acc, DVM_GET_S(b - 1));
                                        store_wide_full_dispatch<K>(acc, dt, V, rowbase, g);
                                    } else {
                                        DVM_WITH_R(a, rr, store_wide_full_dispatch<K>(rr, dt, V, rowbase, g))
                                    }
                                }
                                break;
                            }
                        }
                        DVM_GEO()
                        const uint32_t w1 = cw1;
                        const uint32_t ti = w1 & 0xFF, dt = (w1 >> 8) & 0xFF;
                        int64_t off = (int64_t)g.i1 * DVM_I64(cw2, cw3) + (int64_t)g.colbase;
                        if (op == I_VSTORE) {
                            const u32x4s hw = fetch4(code, cur + 4);
                            const uint32_t h0 = hw.x, h1 = hw.y, h2 = hw.z, h3 = hw.w;
                            off += (int64_t)g.i2 * DVM_I64(h0, h1) + (int64_t)g.i3 * DVM_I64(h2, h3);
                        }
                        const uint32_t es = dt == 0 ? 4 : 2;
                        gptr base = (gptr)DVM_TENSOR(tbase + ti);
                        gptr rowp = base + off * es;
                        if (a == SRC_ACC) {
                            // (b: a row scalar to multiply by first; the accumulator's value is dead afterwards)
                            if (b != 0) tile_bins<K, B_MUL>(acc, DVM_GET_S(b - 1));
                            store_dispatch<K>(acc, dt, V, rowp, g);
                        } else {
                            DVM_WITH_R(a, rr, store_dispatch<K>(rr, dt, V, rowp, g))
                        }
                        break;
                    }
                    case I_LOADS: {
                        DVM_GEO()
                        const uint32_t w1 = cw1;
                        const uint32_t ti = w1 & 0xFF, dt = (w1 >> 8) & 0xFF;
                        const u32x4s hw = fetch4(code, cur + 4);
                        const uint32_t h0 = hw.x, h1 = hw.y, h2 = hw.z, h3 = hw.w;
                        const int64_t off = row_offset(g, DVM_I64(cw2, cw3), DVM_I64(h0, h1), DVM_I64(h2, h3));
                        gcptr base = (gcptr)DVM_TENSOR(tbase + ti);
                        float v;       // a lane outside the tensor reads row 0: valid memory, value unused
                        if (dt == 0) v = *(const GLOBAL_AS float *)(base + off * 4);
                        else v = bf16_lo(*(const GLOBAL_AS uint16_t *)(base + off * 2));
                        DVM_SET_S(a, v);
                        break;
                    }
                    case I_STORES: {
                        if (longrow && (lr_phase != n_red || lr_c != 0)) break;     // (once per row, in its last pass)
                        DVM_GEO()
                        const uint32_t w1 = cw1;
                        const uint32_t ti = w1 & 0xFF, dt = (w1 >> 8) & 0xFF;
                        const u32x4s hw = fetch4(code, cur + 4);
                        const uint32_t h0 = hw.x, h1 = hw.y, h2 = hw.z, h3 = hw.w;
                        const int64_t off = row_offset(g, DVM_I64(cw2, cw3), DVM_I64(h0, h1), DVM_I64(h2, h3));
                        gptr base = (gptr)DVM_TENSOR(tbase + ti);
                        const float v = DVM_GET_S(a);
                        const bool ok = g.rowok && g.lanecol == 0 && g.colbase == 0;
                        if (dt == 0) st_b32(base + off * 4, v, ok);
                        else st_b16(base + off * 2, (uint32_t)pack_bf16(v), ok);
                        break;
                    }
                    case I_MOVRA:
                        DVM_WITH_R(a, rr, rr = acc)
                        break;
                    case I_MOVAR:
                        DVM_WITH_R(a, rr, acc = rr)
                        break;
                    case I_UN:
                        tile_un_dispatch<K>(acc, b);
                        break;
                    case I_BIN:
                        if (a < SRC_S0) {
                            DVM_WITH_R(a, rr, tile_bin_dispatch<K>(acc, rr, b))
                        } else if (a == SRC_ACC) {
                            const Tile<K> t = acc;
                            tile_bin_dispatch<K>(acc, t, b);
                        } else {
                            const float s = a == SRC_IMM ? __builtin_bit_cast(float, cw1) : DVM_GET_S(a - SRC_S0);
                            tile_bins_dispatch<K>(acc, s, b);
                        }
                        break;
                    case I_CACC: if constexpr (CRED) {      // the first step of a unit starts the accumulator, the others combine into it
                        // (a wave whose row lies past the end of the unit contributes nothing)
                        const bool ok = gt.rowok;
                        if (rin == 0) {
                            const float ident = b == R_SUM ? 0.0f : (b == R_MAX ? -__builtin_inff() : __builtin_inff());
                            DVM_WITH_R(a, rr, sfor<K>([&]<int I>() LI { TV(rr, I) = ok ? TV(acc, I) : ident; }))
                        } else if (b == R_SUM) {
                            DVM_WITH_R(a, rr, sfor<K>([&]<int I>() LI { TV(rr, I) = ok ? TV(rr, I) + TV(acc, I) : TV(rr, I); }))
                        } else if (b == R_MAX) {
                            DVM_WITH_R(a, rr, sfor<K>([&]<int I>() LI { TV(rr, I) = ok ? f_maxp(TV(rr, I), TV(acc, I)) : TV(rr, I); }))
                        } else {
                            DVM_WITH_R(a, rr, sfor<K>([&]<int I>() LI { TV(rr, I) = ok ? f_minp(TV(rr, I), TV(acc, I)) : TV(rr, I); }))
                        }
                    }
                        break;
                    case I_CSTREAM: if constexpr (CRED && K <= 8) {      // (the encoder emits it for these variants only)
                        // this wave's share of the unit's rows (every RP-th, starting at its own), U rows in flight:
                        // all their loads are issued before the first is combined into the accumulator
                        DVM_GEO()
                        const uint32_t w1 = cw1;
                        const uint32_t ti = w1 & 0xFF, dt = (w1 >> 8) & 0xFF;
                        const bool nt = ((w1 >> 16) & MF_STREAM) != 0;
                        const int64_t st1 = DVM_I64(cw2, cw3);
                        const u32x4s hw = fetch4(code, cur + 4);
                        const uint32_t h0 = hw.x, h1 = hw.y, h2 = hw.z, h3 = hw.w;
                        const uint32_t es = dt == 0 ? 4 : 2;
                        // (a wave without a valid first row decomposed row 0: in bounds, and it combines nothing)
                        const int64_t off0 = (int64_t)g.i2 * DVM_I64(h0, h1) + (int64_t)g.i3 * DVM_I64(h2, h3) + (int64_t)g.colbase;
                        gcptr base = (gcptr)DVM_TENSOR(tbase + ti);
                        const uint32_t inner_n = sh[S_INNER];
                        const float ident = b == R_SUM ? 0.0f : (b == R_MAX ? -__builtin_inff() : __builtin_inff());
                        constexpr int U = K <= 4 ? 6 : 4;       // (as many as the registers hold)
                        DVM_WITH_R(a, rr, {
                            sfor<K>([&]<int I>() LI { TV(rr, I) = ident; });
                            if (wave < RP) {
                                for (uint32_t r = wave; r < inner_n; r += RP * U) {
                                    Raw<K> raw[U];
                                    sfor<U>([&]<int J>() LI {
                                        const uint32_t ru = r + (uint32_t)J * RP;
                                        const uint32_t rc = ru < inner_n ? ru : r;      // past the end: read row r again, unused
                                        request_staged_dispatch<K>(raw[J], dt, V, nt, base + (off0 + (int64_t)rc * st1) * es, g);
                                    });
                                    sfor<U>([&]<int J>() LI {
                                        if (r + (uint32_t)J * RP < inner_n) {
                                            if (b == R_SUM) combine_staged_dispatch<K, B_ADD>(rr, raw[J], dt, V, g);
                                            else if (b == R_MAX) combine_staged_dispatch<K, B_MAX>(rr, raw[J], dt, V, g);
                                            else combine_staged_dispatch<K, B_MIN>(rr, raw[J], dt, V, g);
                                        }
                                    });
                                }
                            }
                        })
                    }
                        break;
                    case I_CCOMB:       // every wave ends up with the combination, taken in wave order; the first wave stores
                        if constexpr (CRED) if (sh[S_INNER] != 0 && RP > 1) {
                            uint32_t lane = tid & 63u;
                            asm volatile("" : "+v"(lane));      // (keeps the LDS addresses out of the registers that live across the loop)
                            DVM_WITH_R(a, rr, sfor<K / 4>([&]<int Q>() LI {
                                if (wave < RP) {
                                    float *mine = &comb_lds[(wave * 64u + lane) * 4u];
                                    mine[0] = TV(rr, 4 * Q); mine[1] = TV(rr, 4 * Q + 1); mine[2] = TV(rr, 4 * Q + 2); mine[3] = TV(rr, 4 * Q + 3);
                                }
                                __syncthreads();
                                float c0 = comb_lds[lane * 4u], c1 = comb_lds[lane * 4u + 1], c2 = comb_lds[lane * 4u + 2], c3 = comb_lds[lane * 4u + 3];
                                for (uint32_t o = 1; o < RP; ++o) {
                                    const float *p = &comb_lds[(o * 64u + lane) * 4u];
                                    if (b == R_SUM) { c0 += p[0]; c1 += p[1]; c2 += p[2]; c3 += p[3]; }
                                    else if (b == R_MAX) { c0 = f_maxp(c0, p[0]); c1 = f_maxp(c1, p[1]); c2 = f_maxp(c2, p[2]); c3 = f_maxp(c3, p[3]); }
                                    else { c0 = f_minp(c0, p[0]); c1 = f_minp(c1, p[1]); c2 = f_minp(c2, p[2]); c3 = f_minp(c3, p[3]); }
                                }
                                __syncthreads();
                                TV(rr, 4 * Q) = c0; TV(rr, 4 * Q + 1) = c1; TV(rr, 4 * Q + 2) = c2; TV(rr, 4 * Q + 3) = c3;
                            }))
                            gt.rowok = (rp == 0) && (tid < seg_threads);
                        }
                        break;
                    case I_SEL:         // every pair of registers gets its own copy of the loop: no tile is copied
                        DVM_WITH_R(a, xa, DVM_WITH_R2(b, xb, sfor<K>([&]<int I>() LI { TV(acc, I) = TV(acc, I) != 0.0f ? TV(xa, I) : TV(xb, I); })))
                        break;
                    case I_FMA: {
                        const float s = cw1 != 0 ? DVM_GET_S(cw1 - 1) : 1.0f;
                        if constexpr (NR <= 4) {        // one loop per (multiplier, addend) pair of registers
                            if (cw1 == 0) {
                                DVM_WITH_R(a, xa, DVM_WITH_R2(b, xb, sfor<K>([&]<int I>() LI { TV(acc, I) = f_fma(TV(acc, I), TV(xa, I), TV(xb, I)); })))
                            } else if (b == FMA_NO_ADDEND) {
                                DVM_WITH_R(a, xa, sfor<K>([&]<int I>() LI { TV(acc, I) = TV(acc, I) * s * TV(xa, I); }))
                            } else {
                                DVM_WITH_R(a, xa, DVM_WITH_R2(b, xb, sfor<K>([&]<int I>() LI { TV(acc, I) = f_fma(TV(acc, I) * s, TV(xa, I), TV(xb, I)); })))
                            }
                        } else {                        // many registers: the pairs would multiply the code size
                            if (cw1 != 0) tile_bins<K, B_MUL>(acc, s);
                            DVM_WITH_R(a, xa, (tile_bin<K, B_MUL>(acc, xa)))
                            if (b != FMA_NO_ADDEND) {
                                DVM_WITH_R(b, xb, (tile_bin<K, B_ADD>(acc, xb)))
                            }
                        }
                        break;
                    }
                    case I_LDSCOPY: {
                        // every thread of the workgroup copies 16-byte pieces of the tensor's only row into the image;
                        // pieces that reach beyond the row's end are put together element by element, zero-filled
                        const uint32_t ti = cw1 & 0xFF, dt = (cw1 >> 8) & 0xFF;
                        gcptr src = (gcptr)DVM_TENSOR(tbase + ti);
                        const uint64_t D0 = (uint64_t)sh[S_D0LO] | ((uint64_t)sh[S_D0HI] << 32);
                        lds_copy_row((LDS_AS char *)comb_lds + cw2, cw3 >> 4, src, D0, dt, tid, blockDim.x);
                        if (b != 0) __syncthreads();
                        break;
                    }
                    case I_LFMA: {
                        const float s = cw1 != 0 ? DVM_GET_S(cw1 - 1) : 1.0f;
                        const uint32_t la = a & 0xF, lb = a >> 4;
                        const LDS_AS char *pa = (const LDS_AS char *)comb_lds + cw2;
                        const LDS_AS char *pb = (const LDS_AS char *)comb_lds + cw3;
                        const uint32_t lc = gt.lanecol;
                        if (V == 4) {
                            if (la != LFMA_NONE && lb != LFMA_NONE) lds_fma<K, 4, true, true>(acc, s, pa, pb, false, false, lc, gt);
                            else if (la != LFMA_NONE) lds_fma<K, 4, true, false>(acc, s, pa, pb, false, false, lc, gt);
                            else lds_fma<K, 4, false, true>(acc, s, pa, pb, false, false, lc, gt);
                        } else {
                            if constexpr (K >= 8) {
                                if (la != LFMA_NONE && lb != LFMA_NONE) lds_fma<K, 8, true, true>(acc, s, pa, pb, (b & 1u) != 0, (b & 2u) != 0, lc, gt);
                                else if (la != LFMA_NONE) lds_fma<K, 8, true, false>(acc, s, pa, pb, (b & 1u) != 0, false, lc, gt);
                                else lds_fma<K, 8, false, true>(acc, s, pa, pb, false, (b & 2u) != 0, lc, gt);
                            }
                        }
                        break;
                    }
                    case I_RED: {
                        if (longrow) {
                            const uint32_t mine = red_idx++;
                            if (mine < lr_phase) break;         // its value is final: S[a] holds it
                        }
                        DVM_GEO()
                        float v;
                        if (longrow) {
                            // this pass's reduction: the lane's part of this column tile joins those of the tiles before;
                            // after the row's last tile the lanes (and waves) are combined as for a short row
                            const float part = lane_reduce_dispatch<K>(acc, g, V, b);
                            racc = lr_c == 0 ? part : (b == R_MAX ? f_maxp(racc, part) : (b == R_MIN ? f_minp(racc, part) : racc + part));
                            pcb = this_end * 4;                 // the pass ends here
                            if (lr_c + 1 < nct) break;
                            v = wave_allreduce_dispatch(racc, b, width);
                        } else {
                            v = reduce_dispatch<K>(acc, g, V, b, width);
                        }
                        if (gw > 1) {
                            // a row spans gw waves: exchange the per-wave results through LDS.  Two
                            // buffers alternate, so one barrier per reduction is enough.
                            red_lds[red_par][wave & 15] = v;     // every lane of the wave holds the same value
                            __syncthreads();
                            v = red_lds[red_par][w0i & 15];
                            for (uint32_t i = 1; i < gw; ++i) {
                                const float o = red_lds[red_par][(w0i + i) & 15];
                                v = b == R_MAX ? f_maxp(v, o) : (b == R_MIN ? f_minp(v, o) : v + o);
                            }
                            red_par ^= 1;
                        }
                        // the row-scalar ops folded into this record: U(v * scale + shift)
                        v = f_fma(v, __builtin_bit_cast(float, cw2), __builtin_bit_cast(float, cw3));
                        if (cw1 != U_NONE) v = un_dyn(cw1, v);
                        DVM_SET_S(a, v);
                        break;
                    }
                    case I_SOP: {
                        const uint32_t w1 = cw1;
                        const uint32_t kind = w1 & 0xFF, srck = (w1 >> 8) & 0xFF, c = (w1 >> 16) & 0xFF;
                        const float x = DVM_GET_S(b);
                        float r;
                        if (kind >= SOP_UNARY) {
                            r = un_dyn(kind - SOP_UNARY, x);
                        } else {
                            const float y = srck == 1 ? __builtin_bit_cast(float, cw2) : DVM_GET_S(c);
                            r = bin_dyn(kind, x, y);
                        }
                        DVM_SET_S(a, r);
                        break;
                    }
                    default:
                        break;
                }
            }
            if constexpr (CRED) {   // next step of this unit, or the next tile
                const uint32_t inner = sh[S_INNER];
                if (inner == 0 || (rin + 1) * RP >= inner || (sh[S_FLAGS] & SF_CSTREAM)) { rin = 0; tile += t_step; } else { ++rin; }
            } else if (longrow) {
                if (++lr_c == nct) {
                    lr_c = 0;
                    if (++lr_phase > n_red) { lr_phase = 0; tile += t_step; }
                }
            } else {
                tile += t_step;
            }
        }
        seg += seg_words;
    }
    }   // (sets)
}

// ------------------------------------------------------------------------------------------
// interpreter variants and host side
// ------------------------------------------------------------------------------------------
// X(K, NR, largest workgroup, resident waves per SIMD the register allocation aims for).  Every
// variant is compiled in a translation unit of its own (this file with -DDVM_VARIANT_K=.. etc.),
// which defines the kernel and a launcher; the translation unit without those macros holds the
// host side.  The build script reads this list.
#define DVM_VARIANT_LIST(X) \
    X(4, 2, 1024, 8) X(4, 6, 1024, 8) X(8, 2, 1024, 7) X(8, 6, 512, 4) \
    X(16, 2, 1024, 6) X(16, 4, 512, 4) X(16, 6, 512, 3) X(32, 2, 256, 4) X(32, 4, 256, 2) X(64, 1, 256, 3)

// (the variants also built as the instantiation that runs reductions along the penultimate axis)
#define DVM_CRED_VARIANT_LIST(X) \
    X(4, 2, 1024, 4) X(4, 6, 1024, 4) X(8, 2, 1024, 4) X(8, 6, 512, 4) X(16, 6, 512, 3) X(32, 2, 256, 3) X(32, 4, 256, 2)

#define DVM_LAUNCHER_NAME_(K, NR) dvm_vm_launch_##K##_##NR
#define DVM_LAUNCHER_NAME(K, NR) DVM_LAUNCHER_NAME_(K, NR)
#define DVM_CRED_LAUNCHER_NAME_(K, NR) dvm_vm_launch_c_##K##_##NR
#define DVM_CRED_LAUNCHER_NAME(K, NR) DVM_CRED_LAUNCHER_NAME_(K, NR)
#define DVM_WIDE_LAUNCHER_NAME_(K, NR) dvm_vm_launch_w_##K##_##NR
#define DVM_WIDE_LAUNCHER_NAME(K, NR) DVM_WIDE_LAUNCHER_NAME_(K, NR)

}  // namespace

#ifdef DVM_VARIANT_K
// ---- one interpreter variant: kernel instantiation + launcher ---------------------------------
// launcher(grid, block, lds_bytes, stream, kargs, blocks_per_cu): blocks_per_cu null: launch; else only report how
// many workgroups of this size one compute unit holds at a time.  Returns the hipError_t of the calls it made.
#if defined(DVM_VARIANT_CRED)
#define DVM_THIS_LAUNCHER DVM_CRED_LAUNCHER_NAME(DVM_VARIANT_K, DVM_VARIANT_NR)
#define DVM_THIS_KERNEL dvm_vm_kernel<DVM_VARIANT_K, DVM_VARIANT_NR, DVM_VARIANT_MAXT, DVM_VARIANT_WAVES, true, false>
#elif defined(DVM_VARIANT_WIDE)
#define DVM_THIS_LAUNCHER DVM_WIDE_LAUNCHER_NAME(DVM_VARIANT_K, DVM_VARIANT_NR)
#define DVM_THIS_KERNEL dvm_vm_kernel<DVM_VARIANT_K, DVM_VARIANT_NR, DVM_VARIANT_MAXT, DVM_VARIANT_WAVES, false, true>
#else
#define DVM_THIS_LAUNCHER DVM_LAUNCHER_NAME(DVM_VARIANT_K, DVM_VARIANT_NR)
#define DVM_THIS_KERNEL dvm_vm_kernel<DVM_VARIANT_K, DVM_VARIANT_NR, DVM_VARIANT_MAXT, DVM_VARIANT_WAVES, false, false>
#endif
extern "C" int DVM_THIS_LAUNCHER(unsigned grid, unsigned block, unsigned lds_bytes, void *stream, const void *kargs, int *blocks_per_cu) {
    if (blocks_per_cu) return (int)hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, DVM_THIS_KERNEL, (int)block, lds_bytes);
    hipLaunchKernelGGL((DVM_THIS_KERNEL), dim3(grid), dim3(block), lds_bytes, (hipStream_t)stream, *(const KArgs *)kargs);
    return (int)hipGetLastError();
}
#else
// ---- host side: dvm_run ---------------------------------------------------------------------
#define X(K, NR, MAXT, W) extern "C" int DVM_LAUNCHER_NAME(K, NR)(unsigned, unsigned, unsigned, void *, const void *, int *);
DVM_VARIANT_LIST(X)
#undef X
#define X(K, NR, MAXT, W) extern "C" int DVM_WIDE_LAUNCHER_NAME(K, NR)(unsigned, unsigned, unsigned, void *, const void *, int *);
DVM_VARIANT_LIST(X)
#undef X
#define X(K, NR, MAXT, W) extern "C" int DVM_CRED_LAUNCHER_NAME(K, NR)(unsigned, unsigned, unsigned, void *, const void *, int *);
DVM_CRED_VARIANT_LIST(X)
#undef X

// The workspace of dvm_run_static: one array per device, in the library's own image, so that the entry point
// needs no allocation.  In host code the array's name is only a handle for hipGetSymbolAddress; the device
// address it yields (per device) is what kernels and fills get.
static __device__ __align__(256) unsigned char scratch[DVM_STATIC_WORKSPACE_BYTES];

namespace {

typedef int (*vm_launch_t)(unsigned, unsigned, unsigned, void *, const void *, int *);
struct VariantEntry { int K, NR; vm_launch_t launch; };
#define X(K, NR, MAXT, W) {K, NR, DVM_LAUNCHER_NAME(K, NR)},
const VariantEntry g_variants[] = {DVM_VARIANT_LIST(X)};
#undef X
#define X(K, NR, MAXT, W) {K, NR, DVM_WIDE_LAUNCHER_NAME(K, NR)},
const VariantEntry g_wide_variants[] = {DVM_VARIANT_LIST(X)};
#undef X
#define X(K, NR, MAXT, W) {K, NR, DVM_CRED_LAUNCHER_NAME(K, NR)},
const VariantEntry g_cred_variants[] = {DVM_CRED_VARIANT_LIST(X)};
#undef X

thread_local int t_last_hip_error = 0;

constexpr int MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];

// Look up this device's copy of `scratch` (once per device; the device must be current for the lookup).
int scratch_setup(int device) {
    if (device < 0 || device >= MAX_DEVICES) return dvm_set_error(DVM_E_ARGS, "device index out of range");
    if (g_scratch_ptr[device].load(std::memory_order_acquire)) return DVM_OK;
    int cur = -1;
    hipError_t e = hipGetDevice(&cur);
    if (e == hipSuccess && cur != device) e = hipSetDevice(device);
    void *ptr = nullptr;
    if (e == hipSuccess) e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
    if (cur >= 0 && cur != device) {
        const hipError_t e2 = hipSetDevice(cur);
        if (e == hipSuccess) e = e2;
    }
    if (e != hipSuccess || !ptr) {
        t_last_hip_error = (int)e;
        return dvm_set_error(DVM_E_HIP, e != hipSuccess ? hipGetErrorString(e) : "hipGetSymbolAddress returned no address");
    }
    g_scratch_ptr[device].store(ptr, std::memory_order_release);
    return DVM_OK;
}

// clears the synchronisation area of a launch's workspace (a kernel rather than a memset node, so that the
// clearing may be captured into a HIP graph with the launch it precedes)
__global__ void dvm_ws_clear(uint32_t *ws) {
    if (threadIdx.x < WS_SYNC_WORDS) ws[threadIdx.x] = 0;
}

}  // namespace

extern "C" int dvm_last_hip_error(void) { return t_last_hip_error; }

extern "C" int dvm_ctx_query_device(int hip_device, int *n_cu) {
    hipDeviceProp_t prop;
    hipError_t e = hipGetDeviceProperties(&prop, hip_device);
    if (e != hipSuccess) {
        t_last_hip_error = (int)e;
        return DVM_E_HIP;
    }
    *n_cu = prop.multiProcessorCount;
    return scratch_setup(hip_device);
}

namespace {

// Workgroups of `block` threads and `lds_bytes` that one compute unit holds at a time, per launcher; asked of the
// runtime once and remembered (a handful of combinations occur).
struct OccEntry { vm_launch_t launch; uint32_t block, lds_bytes; int per_cu; };
constexpr int OCC_SLOTS = 64;
OccEntry g_occ[OCC_SLOTS];
std::atomic<int> g_occ_n{0};
std::mutex g_occ_mu;

int resident_per_cu(vm_launch_t launch, uint32_t block, uint32_t lds_bytes, int *per_cu) {
    const int n = g_occ_n.load(std::memory_order_acquire);
    for (int i = 0; i < n; ++i)
        if (g_occ[i].launch == launch && g_occ[i].block == block && g_occ[i].lds_bytes == lds_bytes) { *per_cu = g_occ[i].per_cu; return 0; }
    int v = 0;
    const int e = launch(0, block, lds_bytes, nullptr, nullptr, &v);
    if (e != 0) return e;
    std::lock_guard<std::mutex> lock(g_occ_mu);
    const int m = g_occ_n.load(std::memory_order_relaxed);
    if (m < OCC_SLOTS) {
        g_occ[m] = OccEntry{launch, block, lds_bytes, v};
        g_occ_n.store(m + 1, std::memory_order_release);
    }
    *per_cu = v;
    return 0;
}

struct Batch { int n_sets; void *table; size_t table_bytes; };     // device memory for the sets' address table
int run_impl(const dvm_ctx *ctx, const void *bytecode, size_t len, void *const *tensors_in, int n_tensors, void *hip_stream, bool static_ws,
             const Batch *batch);

}  // namespace

extern "C" int dvm_run(const dvm_ctx *ctx, const void *bytecode, size_t len, void *const *tensors, int n_tensors,
                       void *hip_stream) {
    return run_impl(ctx, bytecode, len, tensors, n_tensors, hip_stream, false, nullptr);
}

extern "C" int dvm_run_static(const dvm_ctx *ctx, const void *bytecode, size_t len, void *const *tensors, int n_tensors,
                              void *hip_stream) {
    return run_impl(ctx, bytecode, len, tensors, n_tensors, hip_stream, true, nullptr);
}

extern "C" int dvm_run_batched(const dvm_ctx *ctx, const void *bytecode, size_t len, void *const *tensor_sets, int n_tensors, int n_sets,
                               void *table, size_t table_bytes, void *hip_stream) {
    if (n_sets < 1 || n_tensors < 1 || !table) return dvm_set_error(DVM_E_ARGS, "dvm_run_batched: at least one set of at least one tensor, and a table buffer");
    if (((uintptr_t)table & 7) || table_bytes < (size_t)n_sets * (size_t)n_tensors * 8)
        return dvm_set_error(DVM_E_ARGS, "dvm_run_batched: the table buffer holds n_sets * n_tensors addresses of 8 bytes, 8-byte aligned");
    const Batch b{n_sets, table, table_bytes};
    return run_impl(ctx, bytecode, len, tensor_sets, n_tensors, hip_stream, false, &b);
}

namespace {

// One set of tensors against the bytecode's tensor table: no null pointer, the alignment the bytecode was encoded
// for, equal pointers where it names two entries as the same buffer, and no overlap between a buffer one segment
// writes and a buffer of another segment unless the bytecode orders them.
int check_tensor_set(const uint32_t *w, const uint8_t *seg_of, void *const *tensors) {
    const uint32_t ntens = w[PH_NTENS];
    uint64_t addr_of[DVM_MAX_TENSORS], size_of[DVM_MAX_TENSORS];
    for (uint32_t i = 0; i < ntens; ++i) {
        const uint32_t *te = w + PH_WORDS_N + i * TT_WORDS;
        const uint32_t info = te[TT_INFO];
        const uint64_t align = 1ull << ((info >> 16) & 0xFF);
        const uint64_t addr = (uint64_t)(uintptr_t)tensors[i];
        if (addr == 0) return dvm_set_error(DVM_E_ARGS, "dvm_run: null tensor pointer");
        if (addr & (align - 1)) return dvm_set_error(DVM_E_ALIGN, "dvm_run: tensor pointer below the alignment the bytecode was encoded for");
        if ((info >> 24) != 0 && addr != (uint64_t)(uintptr_t)tensors[(info >> 24) - 1])
            return dvm_set_error(DVM_E_ARGS, "dvm_run: two entries the bytecode names as the same buffer got different pointers");
        addr_of[i] = addr;
        size_of[i] = (uint64_t)te[TT_BYTES_LO] | ((uint64_t)te[TT_BYTES_HI] << 32);
    }
    if (w[PH_NSEG] > 1) {
        for (uint32_t i = 0; i < ntens; ++i) {
            const uint32_t ii = w[PH_WORDS_N + i * TT_WORDS + TT_INFO];
            if (ii & TI_WORKSPACE) continue;
            uint32_t root_i = i;
            while (w[PH_WORDS_N + root_i * TT_WORDS + TT_INFO] >> 24) root_i = (w[PH_WORDS_N + root_i * TT_WORDS + TT_INFO] >> 24) - 1;
            for (uint32_t j = 0; j < i; ++j) {
                const uint32_t ij = w[PH_WORDS_N + j * TT_WORDS + TT_INFO];
                if (seg_of[i] == seg_of[j] || !((ii | ij) & TI_OUTPUT)) continue;
                if (addr_of[i] >= addr_of[j] + size_of[j] || addr_of[j] >= addr_of[i] + size_of[i]) continue;
                uint32_t root_j = j;
                while (w[PH_WORDS_N + root_j * TT_WORDS + TT_INFO] >> 24) root_j = (w[PH_WORDS_N + root_j * TT_WORDS + TT_INFO] >> 24) - 1;
                if (root_i != root_j)
                    return dvm_set_error(DVM_E_ARGS, "dvm_run: a buffer one stacked part writes overlaps a buffer of another part "
                                                     "and the bytecode does not order them (dvm_stack_dependent)");
            }
        }
    }
    return DVM_OK;
}

int run_impl(const dvm_ctx *ctx, const void *bytecode, size_t len, void *const *tensors_in, int n_tensors, void *hip_stream, bool static_ws,
             const Batch *batch) {
    if (!ctx || !bytecode || (!tensors_in && n_tensors > 0)) return dvm_set_error(DVM_E_ARGS, "dvm_run: null argument");
    if (dvm_ctx_device(ctx) < 0) return dvm_set_error(DVM_E_ARGS, "dvm_run: context was created without a device");
    int st = dvm_validate(bytecode, len);
    if (st != DVM_OK) return st;
    const uint32_t *w = (const uint32_t *)bytecode;
    const uint32_t ntens = w[PH_NTENS];
    // dvm_run_static: the library's own array stands in for the workspace entry, which the caller leaves out
    void *tensors_full[DVM_MAX_TENSORS];
    void *const *tensors = tensors_in;
    if (static_ws && ntens > 0 && (w[PH_WORDS_N + (ntens - 1) * TT_WORDS + TT_INFO] & TI_WORKSPACE)) {
        if ((uint32_t)n_tensors + 1 != ntens) return dvm_set_error(DVM_E_ARGS, "dvm_run_static: pass the bytecode's tensors without its workspace");
        const uint32_t *te = w + PH_WORDS_N + (ntens - 1) * TT_WORDS;
        if (te[TT_BYTES_HI] != 0 || te[TT_BYTES_LO] > DVM_STATIC_WORKSPACE_BYTES)
            return dvm_set_error(DVM_E_LIMIT, "dvm_run_static: the launch needs a workspace beyond DVM_STATIC_WORKSPACE_BYTES; use dvm_run with a workspace of the caller's");
        st = scratch_setup(dvm_ctx_device(ctx));
        if (st != DVM_OK) return st;
        for (int i = 0; i < n_tensors; ++i) tensors_full[i] = tensors_in[i];
        tensors_full[n_tensors] = g_scratch_ptr[dvm_ctx_device(ctx)].load(std::memory_order_acquire);
        tensors = tensors_full;
        ++n_tensors;
    }
    if ((uint32_t)n_tensors != ntens) return dvm_set_error(DVM_E_ARGS, "dvm_run: tensor count does not match the bytecode");
    const uint32_t segs_off = PH_WORDS_N + ntens * TT_WORDS;
    const uint32_t seg_words = w[PH_WORDS] - segs_off;
    if (seg_words > (uint32_t)CODE_WORDS) return dvm_set_error(DVM_E_LIMIT, "dvm_run: bytecode exceeds the kernel-argument budget");

    if (w[PH_GRID] == 0) return DVM_OK;   // an empty iteration space: nothing to launch, pointers may be null

    KArgs ka;
    memcpy(ka.code, w + segs_off, (size_t)seg_words * 4);
    ka.ws = 0;
    for (uint32_t i = 0; i < ntens; ++i) {
        ka.tensors[i] = (uint64_t)(uintptr_t)tensors[i];
        if (w[PH_WORDS_N + i * TT_WORDS + TT_INFO] & TI_WORKSPACE) {
            ka.ws = ka.tensors[i];                      // the synchronisation area
            ka.tensors[i] += DVM_WORKSPACE_BYTES;       // segments that name the workspace as a tensor see its data area
        }
    }
    ka.sets = 0;
    ka.n_sets = 1;
    ka.n_tensors = ntens;
    ka.rotate = 0;
    ka.seg_first = 0;
    ka.nseg = w[PH_NSEG];
    ka.spin_limit = (uint32_t)dvm_ctx_sync_limit(ctx);

    const int K = (int)(w[PH_VARIANT] & 0xFF), NR = (int)((w[PH_VARIANT] >> 8) & 0xFF);
    uint32_t grid = w[PH_GRID];
    const uint32_t block = w[PH_BLOCK];
    // A segment that reduces along the penultimate axis needs the instantiation that runs such segments,
    // and LDS for the combination across waves: four floats per lane of every participating wave
    uint32_t lds_bytes = 0;
    bool cred = false, wide = true;     // wide: every segment spreads a row over whole waves
    bool grid_sync = false, wg_sync = false, longrow = false;
    uint8_t seg_of[DVM_MAX_TENSORS];    // the segment a tensor belongs to
    memset(seg_of, 0xFF, sizeof(seg_of));
    for (uint32_t s = 0, at = segs_off; s < w[PH_NSEG]; ++s) {
        const uint32_t *sh = w + at;
        const uint32_t rp = sh[S_RP] & 0xFFFF;
        cred |= sh[S_INNER] != 0;
        wide &= (sh[S_GEOM] & 0xFFFF) >= 64;
        grid_sync |= (sh[S_FLAGS] & SF_SYNC_GRID) != 0;
        wg_sync |= (sh[S_FLAGS] & SF_SYNC_WG) != 0;
        longrow |= (sh[S_FLAGS] & SF_LONGROW) != 0;
        if (sh[S_INNER] != 0 && rp > 1 && rp * 64u * 16u > lds_bytes) lds_bytes = rp * 64u * 16u;
        if (sh[S_FLAGS] & SF_LDS)           // the images the prologue copies into LDS
            for (uint32_t pc = SH_WORDS; pc < SH_WORDS + sh[S_PROLOGA]; pc += (sh[pc] >> 8) & 0xFF)
                if ((sh[pc] & 0xFF) == I_LDSCOPY && sh[pc + 2] + sh[pc + 3] > lds_bytes) lds_bytes = sh[pc + 2] + sh[pc + 3];
        for (uint32_t t = 0; t < sh[S_NTENS]; ++t) seg_of[sh[S_TBASE] + t] = (uint8_t)s;
        at += sh[S_WORDS];
    }
    // Segments of one launch run without order between them unless the bytecode says otherwise: see check_tensor_set
    const int n_sets = batch ? batch->n_sets : 1;
    for (int k = 0; k < n_sets; ++k) {
        st = check_tensor_set(w, seg_of, tensors + (size_t)k * ntens);
        if (st != DVM_OK) return st;
    }
    if (batch) {
        if (grid_sync || ka.ws != 0) return dvm_set_error(DVM_E_UNSUPPORTED, "dvm_run_batched: bytecode with a workspace runs one set at a time");
        // the sets' addresses travel through the caller's table buffer (copied on the launch's stream)
        const hipError_t ce = hipMemcpyAsync(batch->table, tensors, (size_t)n_sets * ntens * 8, hipMemcpyHostToDevice, (hipStream_t)hip_stream);
        if (ce != hipSuccess) {
            t_last_hip_error = (int)ce;
            return dvm_set_error(DVM_E_HIP, hipGetErrorString(ce));
        }
        ka.sets = (uint64_t)(uintptr_t)batch->table;
        ka.n_sets = (uint32_t)n_sets;
    }
    // Several segments, or several sets: the tiles of each are dealt out from where the one before stopped.  (Not
    // when a segment relies on its producer's assignment of tiles to workgroups, nor when the segments own shares
    // of the workgroups.)
    ka.rotate = (w[PH_NSEG] > 1 || n_sets > 1) && !wg_sync && (w[PH_TYPE] & 0xFFFF) != KT_STACK_SPATIAL ? 1u : 0u;
    if (cred && longrow)
        return dvm_set_error(DVM_E_UNSUPPORTED, "dvm_run: a launch holds both a reduction along the penultimate axis and rows longer than a tile");
    vm_launch_t launch = nullptr;
    if (cred) {
        for (const VariantEntry &v : g_cred_variants)
            if (v.K == K && v.NR == NR) launch = v.launch;
    } else if (wide) {
        for (const VariantEntry &v : g_wide_variants)
            if (v.K == K && v.NR == NR) launch = v.launch;
    } else {
        for (const VariantEntry &v : g_variants)
            if (v.K == K && v.NR == NR) launch = v.launch;
    }
    if (!launch) return dvm_set_error(DVM_E_BADCODE, "dvm_run: no interpreter variant for this bytecode");
    hipError_t e;
    if (grid_sync) {
        // every workgroup waits for all the others: the whole grid has to be resident at once
        int per_cu = 0, n_cu = 0;
        e = (hipError_t)resident_per_cu(launch, block, lds_bytes, &per_cu);
        if (e != hipSuccess) {
            t_last_hip_error = (int)e;
            return dvm_set_error(DVM_E_HIP, hipGetErrorString(e));
        }
        dvm_ctx_planner_get(ctx, &n_cu, nullptr);
        // (the parts were planned one by one, some for interpreter variants that hold more waves than the
        // launch's common one: the interpreter deals the tiles out over whatever grid it finds itself in)
        if (per_cu < 1 || n_cu < 1)
            return dvm_set_error(DVM_E_UNSUPPORTED, "dvm_run: the device holds no workgroup of this launch's size");
        if ((uint64_t)grid > (uint64_t)per_cu * (uint64_t)n_cu) grid = (uint32_t)per_cu * (uint32_t)n_cu;
        hipLaunchKernelGGL(dvm_ws_clear, dim3(1), dim3(64), 0, (hipStream_t)hip_stream, (uint32_t *)(uintptr_t)ka.ws);
    }
    // A launch whose segments (and sets) deal their tiles out in rotation keeps as many workgroups busy as it has
    // tiles in all: the grid grows from what the largest segment alone asked for to that, up to what the device holds
    // at once (short segments of many sets then run side by side instead of one after the other on a few workgroups).
    if (ka.rotate != 0 && !grid_sync) {
        uint64_t total = 0;
        for (uint32_t s = 0, at = segs_off; s < w[PH_NSEG]; ++s) {
            total += w[at + S_NTILES];
            at += w[at + S_WORDS];
        }
        total *= (uint64_t)n_sets;
        if (total > grid) {
            int per_cu = 0, n_cu = 0;
            e = (hipError_t)resident_per_cu(launch, block, lds_bytes, &per_cu);
            if (e != hipSuccess) {
                t_last_hip_error = (int)e;
                return dvm_set_error(DVM_E_HIP, hipGetErrorString(e));
            }
            dvm_ctx_planner_get(ctx, &n_cu, nullptr);
            const uint64_t cap = (uint64_t)(per_cu > 0 ? per_cu : 1) * (uint64_t)(n_cu > 0 ? n_cu : 1);
            const uint64_t want = total < cap ? total : cap;
            if (want > grid) grid = (uint32_t)want;
        }
    }
    // one kernel launch per run of segments up to the next one that asks for a launch of its own
    for (uint32_t first = 0; first < w[PH_NSEG];) {
        uint32_t end = first + 1;
        for (uint32_t s = 0, at = segs_off; s < w[PH_NSEG]; ++s) {
            if (s > first && s == end && !(w[at + S_FLAGS] & SF_NEW_LAUNCH)) ++end;
            at += w[at + S_WORDS];
        }
        ka.seg_first = first;
        ka.nseg = end;
        e = (hipError_t)launch(grid, block, lds_bytes, hip_stream, &ka, nullptr);
        if (e != hipSuccess) {
            t_last_hip_error = (int)e;
            return dvm_set_error(DVM_E_HIP, hipGetErrorString(e));
        }
        first = end;
    }
    return DVM_OK;
}

}  // namespace

extern "C" int dvm_workspace_status(const void *workspace, void *hip_stream, int *gave_up) {
    if (!workspace || !gave_up) return dvm_set_error(DVM_E_ARGS, "dvm_workspace_status: null argument");
    uint32_t word = 0;
    hipError_t e = hipMemcpyAsync(&word, (const uint32_t *)workspace + WS_STATUS, 4, hipMemcpyDeviceToHost, (hipStream_t)hip_stream);
    if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)hip_stream);
    if (e != hipSuccess) {
        t_last_hip_error = (int)e;
        return dvm_set_error(DVM_E_HIP, hipGetErrorString(e));
    }
    *gave_up = word != 0;
    return DVM_OK;
}
#endif  // host side
