// Bytecode layout shared by the host encoder and the device interpreter.
//
// A program is a header followed by one code body per meta-kernel (Section 4.2, "Bytecode
// encoding": the header carries the kernel type, the code size and the total number of tiles;
// the body holds one record per operation with its instruction id, its length, the destination
// and source tile registers, and extras).  The paper's format figure is not reproduced in its
// text, so the field widths below are this implementation's own: little-endian 32-bit words,
// every record a whole number of words, unused bits zero (which makes equal inputs give equal
// bytes).
//
//   program  := PH_WORDS header words | n_tensors * TT_WORDS tensor-table words | segment*
//   segment  := SH_WORDS header words | body (S_CODESIZE words of instruction records)
//   record   := word0 = op | len<<8 | a<<16 | b<<24, then len-1 operand words; len is 4 or 8: every
//               record starts on a 16-byte boundary so that one scalar load fetches it whole
//
// The tile registers are the interpreter's local memory: an accumulator ACC and NR tile
// registers R0.. of K fp32 elements per lane each, and NS row-scalar registers S0.. (one value
// per row, replicated on the lanes that hold the row).
#ifndef DVM_BYTECODE_H
#define DVM_BYTECODE_H

#include <stdint.h>

namespace dvmbc {

constexpr uint32_t MAGIC   = 0x314D5644u;   // "DVM1"
constexpr uint32_t VERSION = 1;

// kernel types (Section 4.2: a meta-kernel on the vector path, or a stacking-based kernel)
constexpr uint32_t KT_META  = 0;            // printed as "vmain.v"
constexpr uint32_t KT_STACK = 1;            // temporally stacked meta-kernels, "vstack.t"
constexpr uint32_t KT_STACK_SPATIAL = 2;    // spatially stacked: every segment runs on its own share of the workgroups, "vstack.s"

// ---- program header -------------------------------------------------------------------------
enum : int {
    PH_MAGIC = 0,
    PH_TYPE,        // kernel type | VERSION << 16
    PH_WORDS,       // length of the whole program in words
    PH_NSEG,        // number of segments (meta-kernels)
    PH_BLOCK,       // threads per workgroup of the launch
    PH_GRID,        // workgroups of the launch: the N of Algorithm 2
    PH_VARIANT,     // interpreter variant: K | NR << 8; bits 16-23: tile registers the program uses + 1 (0: not noted)
    PH_NTENS,       // tensors of the launch
    PH_WORDS_COUNT
};
constexpr int PH_WORDS_N = PH_WORDS_COUNT;

// tensor table entry
enum : int {
    TT_INFO = 0,    // dtype | is_output << 8 | is_workspace << 9 | log2(assumed pointer alignment in bytes) << 16
    TT_BYTES_LO,    // minimum size of the buffer in bytes
    TT_BYTES_HI,
    TT_WORDS
};

// ---- segment header -------------------------------------------------------------------------
enum : int {
    S_WORDS = 0,    // header + body, in words
    S_CODESIZE,     // body size in words (the paper's CodeSize)
    S_NTILES,       // total number of tiles M of this meta-kernel
    S_GEOM,         // G (lanes per row, u16) | V (elements per chunk, u8) << 16 | nvec << 24
    S_RP,           // rows per tile (u16) | active threads (u16) << 16
    S_NCT,          // column tiles per row
    S_TC,           // tile width in elements
    S_D0LO, S_D0HI, // row length in elements
    S_NROWS,        // number of rows (product of the outer iteration dims)
    S_D1, S_M1, S_SH1,   // outer dim 1 and the multiply-shift constants that divide by it
    S_D2, S_M2, S_SH2,   // outer dim 2
    S_NCTM, S_NCTSH,     // multiply-shift constants that divide by S_NCT
    S_TBASE,        // index of this segment's first tensor in the launch's tensor list
    S_NTENS,        // tensors of this segment
    S_FLAGS,        // SF_*
    S_IMASK,        // bit op -> the instruction id occurs in the body (for the disassembler)
    S_PROLOG,       // words at the start of the body that do not run for every tile: the prologue (pinned operands)
    S_PROLOGA,      // the first S_PROLOGA words of the prologue run once per workgroup only; the rest of it runs
                    // again whenever the index of the second outer dim (row / S_D1) differs from the previous tile's
    S_WG0, S_NWG,   // spatial stacking: this segment runs on workgroups [S_WG0, S_WG0 + S_NWG) only (S_NWG 0: on all)
    S_INNER,        // reduction along the penultimate axis: its extent `size` (0: the segment has none).  Then
                    // S_NTILES counts units of work (outer index, column tile); a workgroup visits the `size`
                    // rows of a unit S_RP at a time (one row per wave), so a tile register can accumulate over
                    // them; I_CCOMB combines the waves' registers
    S_EPILOG,       // body words that run for every row of a unit; the records after them (the epilogue) run
                    // after the last row of the unit only (= S_CODESIZE when there is no epilogue)
    SH_WORDS
};
static_assert(SH_WORDS % 4 == 0, "segment header must keep records 16-byte aligned");
// The workspace of a launch (a tensor of its own, the last of the launch, flagged in the tensor table): device memory
// the caller lends to the launch.  Its first words are the synchronisation area; dvm_run clears it before the launch.
constexpr uint32_t TI_OUTPUT = 1u << 8, TI_WORKSPACE = 1u << 9;
enum : int { WS_ARRIVED = 0, WS_STATUS = 1, WS_SYNC_WORDS = 16 };      // (64 bytes)
constexpr uint32_t WS_STATUS_GAVE_UP = 1;   // a workgroup's bounded wait ran out: the launch's results are incomplete
constexpr int LEN_REC = 4;              // length of every record except the view forms
constexpr uint32_t SF_WGSYNC  = 1u;     // rows span several waves: reductions use the barrier
constexpr uint32_t SF_RAGGED  = 2u;     // some tile has invalid rows or columns: mask reductions
constexpr uint32_t SF_CSTREAM = 4u;     // reducing segment whose per-row part is I_CSTREAM records only: one step per unit
constexpr uint32_t SF_INTERLEAVED = 8u; // workgroup id runs tiles id, id + N, id + 2N, ... instead of Algorithm 2's blocked range
// A stacked meta-kernel that reads what an earlier meta-kernel of the same launch wrote (Section 5.1: temporal
// stacking does not require independent operators) starts behind a synchronisation point:
constexpr uint32_t SF_LONGROW = 256u;    // rows longer than a tile with reductions along them: S_NTILES counts rows, S_NCT the column tiles
                                         // of a row, S_NCTSH the reductions in the body; the workgroup passes over the row once
                                         // per reduction (accumulating it tile after tile) and once more for the stores
constexpr uint32_t SF_NEW_LAUNCH = 128u; // dvm_run starts a kernel launch of its own at this segment: everything before it is complete and
                                         // visible (the cheapest device-wide order on a chip whose second-level caches are
                                         // not coherent with each other; used where the data handed over is small)
constexpr uint32_t SF_LDS = 64u;        // the prologue copies row-invariant tensors into LDS: the workgroup synchronises around it
constexpr uint32_t SF_SYNC_WG   = 16u;  // its producer ran with the same tile-to-workgroup assignment over the same rows: a
                                        // workgroup reads only rows it wrote itself, so it waits for its own stores only
constexpr uint32_t SF_SYNC_GRID = 32u;  // any other dependence: every workgroup of the launch has finished the segments before
                                        // (an arrival counter in the launch's workspace; the wait is bounded and gives up
                                        // through the workspace's status word)

// ---- instruction ids --------------------------------------------------------------------------
enum : uint32_t {
    I_NOP = 0,
    I_LOAD,      // contiguous rows, one row stride     a = dst (b = 0).  Consecutive load records form a group: the
                 // interpreter issues the requests of all of them before it waits for the first
    I_VLOAD,     // view load: three outer strides      (Table 1: ViewLoad)
    I_LOADS,     // one value per row -> S[a]
    I_STORE,     // a = src register; b != 0: multiply ACC by S[b-1] first   (Table 1: Store)
    I_VSTORE,    //                                     (Table 1: ViewStore)
    I_STORES,    // S[a] -> one value per row
    I_MOVRA,     // R[a] = ACC                          (Table 1: Copy)
    I_MOVAR,     // ACC = R[a]
    I_UN,        // ACC = U_b(ACC)
    I_BIN,       // ACC = B_b(ACC, src a)               src: R, S (Table 1: Broadcast of a row value), ACC, IMM
    I_SEL,       // ACC = ACC != 0 ? R[a] : R[b]        (Table 1: Select)
    I_RED,       // S[a] = post(R_b over the row of ACC); word1 = U_post, word2 = scale, word3 = shift:
                 // post(x) = U_post(x * scale + shift), the row-scalar ops that directly follow a
                 // reduction folded into its record.  When a row spans several waves the handler
                 // synchronises the workgroup between the per-wave part and the combination.
    I_SOP,       // S[a] = op(S[b], S[c] | imm)
    I_FMA,       // ACC = ACC * s * R[a] + R[b]: adjacent multiplies and an add fused into one record.  word1 = 0: s = 1,
                 // else s = S[word1 - 1]; b = FMA_NO_ADDEND: nothing is added
    I_CACC,      // R[a] = first row of the unit ? ACC : R_b(R[a], ACC): accumulates a reduction along the
                 // penultimate axis (Table 1: Sum / Max / Min over [M, size, N] with N > 1)
    I_CCOMB,     // epilogue only: combine R[a] over the waves of the workgroup with R_b (each wave accumulated its
                 // own share of the unit's rows), through LDS; afterwards only the first wave stores
    I_CSTREAM,   // R[a] = R_b over the rows of the unit that fall to this wave, of a tensor (memory record with three
                 // strides): the whole per-row part of a segment that only reduces input tensors along the
                 // penultimate axis (SF_CSTREAM), with several rows in flight per wave instead of one per step
    I_LDSCOPY,   // prologue only: copy a row-invariant tensor (every outer stride 0) into the workgroup's LDS, as it
                 // lies in memory, zero-filled up to the tile width.  word1 = tensor | dtype << 8, word2 = byte offset
                 // of the image in LDS, word3 = its size in bytes (a multiple of 16); b != 0: the workgroup
                 // synchronises afterwards (set on the last copy of a prologue)
    I_LFMA,      // ACC = ACC [* S] [* La] [+ Lb] with La, Lb LDS images (the multiply-add is fused when both are there).
                 // a = La | Lb << 4 as image numbers (LFMA_NONE: absent), b = bit 0: La is bf16, bit 1: Lb is bf16;
                 // word1 = 0 or S index + 1, word2 / word3 = byte offsets of La / Lb in LDS
    I_COUNT
};
constexpr uint32_t LFMA_NONE = 0xF;
constexpr int LDS_SLOTS = 4;                    // LDS images per segment
constexpr uint32_t LDS_IMAGE_MAX_BYTES = 65536; // all images of a segment together

// memory record: word1 = tensor | dtype << 8 | flags << 16 ; then strides as int64 (lo, hi)
constexpr int LEN_LOAD  = 4;            // word0, word1, s1
constexpr int LEN_VLOAD = 8;            // word0, word1, s1, s2, s3
constexpr uint32_t MF_ALIGNED16 = 1u;   // every chunk of this tensor starts on a 16-byte boundary
constexpr uint32_t MF_STREAM    = 8u;   // load only: every element of the tensor is read exactly once by the
                                        // launch (no broadcast over an iterated dim): bypass-style cache hint

// source / destination selectors
constexpr uint32_t SRC_R0  = 0;         // 0 .. NR-1
constexpr uint32_t SRC_S0  = 16;        // 16 .. 16+NS-1
constexpr uint32_t SRC_ACC = 32;
constexpr uint32_t SRC_IMM = 33;
constexpr int NS = 4;                   // row-scalar registers
constexpr uint32_t FMA_NO_ADDEND = 0xFF;

// binary ops B_*
enum : uint32_t {
    B_NONE = 0, B_ADD, B_SUB, B_RSUB, B_MUL, B_DIV, B_RDIV, B_MIN, B_MAX, B_POW, B_RPOW,
    B_EQ, B_NE, B_LT, B_LE, B_GT, B_GE,
    B_EXPSUB, B_REXPSUB,    // exp(a - b), exp(b - a): the encoder's fusion of a subtraction feeding an exponential
    B_COUNT
};
// unary ops U_*
enum : uint32_t {
    U_NONE = 0, U_SQRT, U_ABS, U_LOG, U_EXP, U_ROUND, U_FLOOR, U_ISFINITE, U_NEG, U_RSQRT, U_RCP,
    U_TANH, U_ERF, U_SIGMOID, U_SQUARE, U_GELU_TANH, U_GELU_ERF, U_SILU, U_CAST_BF16, U_COUNT
};
// reductions R_*
enum : uint32_t { R_SUM = 0, R_MAX, R_MIN, R_SUMSQ, R_COUNT };

// I_SOP: word1 = kind | srckind << 8 | c << 16 ; word2 = immediate.  kind < 64: B_kind(S[b], x);
// kind >= 64: U_(kind-64)(S[b]).  srckind 0: x = S[c]; 1: x = immediate.
constexpr int LEN_SOP = 4;
constexpr uint32_t SOP_UNARY = 64;

inline uint32_t w0(uint32_t op, uint32_t len, uint32_t a, uint32_t b) {
    return op | (len << 8) | (a << 16) | (b << 24);
}

// interpreter variants compiled into the library: elements per lane per tile register (K),
// number of tile registers (NR), largest workgroup, and resident waves per SIMD (from the
// compiled kernels' register use; 4 SIMDs per compute unit).
// `cred`: also built as the instantiation that runs reductions along the penultimate axis.
struct Variant { int K, NR, max_threads, waves_per_simd; bool cred; };
constexpr Variant VARIANTS[] = {
    { 4, 2, 1024, 8, true}, { 4, 6, 1024, 8, true},
    { 8, 2, 1024, 7, true}, { 8, 6,  512, 4, true},
    {16, 2, 1024, 6, false}, {16, 4,  512, 4, false}, {16, 6,  512, 3, true},
    {32, 2,  256, 4, true}, {32, 4,  256, 2, true},
    {64, 1,  256, 3, false},
};
constexpr int N_VARIANTS = sizeof(VARIANTS) / sizeof(VARIANTS[0]);

}  // namespace dvmbc
#endif
