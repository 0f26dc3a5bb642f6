// kernels.h -- argument blocks and launch descriptions shared by the device code (kernels.hip)
// and the chain runtime (chain.hip).  gfx950 only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pgk {

enum Op : int { kAdd = 0, kMul = 1, kGelu = 2, kRmsNorm = 3, kGemv = 4, kScaleBiasRelu = 5 };
enum DType : int { kF32 = 0, kBF16 = 1 };

// One argument block per kernel, passed by value as the kernel's single parameter.  An operand
// whose bit is set in the kernel's IND template mask holds the address of a pointer-table slot
// instead of the tensor's address: the kernel loads the tensor pointer from it before anything
// else (the dereference prologue of Parameter Indirection, paper Sec. 4 "Kernel generation").
struct EwArgs {          // ADD / MUL / GELU
    void* out;
    const void* a;
    const void* b;
    long long n;
    long long m;
};
struct RmsArgs {
    void* out;
    const void* x;
    const void* g;
    int rows;
    int cols;
    float eps;
};
struct GemvArgs {
    void* out;
    const void* W;
    const void* h;
    int rows;
    int n;
    int cols;
    int row_groups;      // matrix-core form only: the grid is (column blocks) x (row groups); from Launch
};
struct SbrArgs {
    void* out;
    const void* x;
    const void* s;
    const void* b;
    long long n;
    unsigned inner;
    unsigned channels;
};

// Batched multi-tensor copy: the destination side is static and lives in device memory, the
// source pointers change every replay and travel in the argument block.
constexpr int kCopyMaxSrc = 448;           // 448 * 8 B + header < 4 KB of kernel arguments
constexpr unsigned kCopyChunkBytes = 8192;   // bytes of one tensor handled by one workgroup: 256 lanes x 2 x 16 B
struct CopyTensor { void* dst; unsigned long long bytes; };
struct CopyChunk { unsigned tensor; unsigned len; unsigned long long off; };
struct CopyArgs {
    const CopyChunk* chunks;     // [dev] chunk list, offset to this launch's first chunk
    const CopyTensor* tensors;   // [dev] per-tensor destination and size
    int src_base;                // tensor index of src[0]
    int n_chunks;
    const void* src[kCopyMaxSrc];
};

// Pointer-table writer: the pointers ride in the argument block, one wave stores them.
constexpr int kTableMaxPtrs = 480;
struct TableArgs {
    const void** table;          // [dev]
    int base;
    int n;
    const void* ptr[kTableMaxPtrs];
};

// ---- merged dispatches --------------------------------------------------------------------------------
// A captured graph need not spend one dispatch per kernel.  A run of consecutive kernels of a chain that
// all work element for element on the same n elements -- add / mul / GELU, and RMSNorm over rows of
// exactly 256 x 16 bytes -- goes out as ONE dispatch.  The tensor is cut into units of 256 lanes x 16
// bytes (lane t owns vector t of a unit; an RMSNorm row is one unit), one workgroup per unit.  The lane
// runs the kernels one after the other, each with its stand-alone arithmetic and its one rounding to
// the storage type, stores its output unless a later kernel of the run overwrites it, and hands the stored bits on to the next kernel in
// registers when that kernel reads the same buffer element for element -- so the run costs one trip
// to memory, not one per kernel.  Operands that no kernel of the run produces are fetched up front.
constexpr int kMergeMaxPhases = 4;        // kernels per merged dispatch
constexpr int kMergeSlots = 3;            // outputs a lane keeps in registers for later kernels of the run
constexpr unsigned kMergeFromMemory = 255;

struct MergePhase {
    void* out;
    const void* in0;        // ADD / MUL / GELU: a; RMSNORM: x
    const void* in1;        // ADD / MUL: b; RMSNORM: gain
    unsigned m;             // ADD / MUL: period of b
    float eps;              // RMSNORM
    // op | src0 << 8 | src1 << 16 | dst << 24: the kernel (kAdd, kMul, kGelu, kRmsNorm), the register slot
    // each operand is taken from (or kMergeFromMemory), the slot that keeps the output
    unsigned meta;
    unsigned ind;           // bit 0 / 1: in0 / in1 hold the address of a pointer-table slot
};
struct MergedArgs {
    unsigned n;             // elements every kernel of the run produces (a whole number of 16-byte vectors)
    int n_phase;
    MergePhase ph[kMergeMaxPhases];   // entries from n_phase on: meta says "operands from slots", nothing is fetched
};

// The same idea for a GEMV followed by element-for-element kernels over its outputs (GELU of the result,
// the residual add, an input add): they ride in the GEMV's dispatch as an epilogue.  After the wave's
// reduction every lane holds the finished sums; lane e of a wave takes output e (row e >> 1 of h, column
// j0 + (e & 1)), rounds it to the storage type as the GEMV's own store would, and runs the following
// kernels on that one element, operands fetched while the weights were in flight.  No workgroup needs
// another's results, so nothing has to be waited for.
constexpr int kEpiMaxPhases = 3;
constexpr unsigned kEpiStore = 1u << 8;   // MergePhase::ind: this kernel's output is stored (no later kernel of the run overwrites it)
// And the RMSNorm in front of the GEMV can ride along as a prologue: every workgroup of the GEMV needs the
// whole normalised vector anyway, so each one normalises the rows itself (the stand-alone kernel's
// arithmetic, lane t holding vector t of a row -- exactly where the GEMV wants h in LDS) while its
// weights are on their way, and workgroup 0 stores the result where the RMSNorm kernel would have.
// A kernel of the epilogue may update the normalised stream in place (the residual add does); the
// runtime then lets it write a shadow copy of that buffer instead, so that no workgroup can read an
// element another one has already replaced (chain.hip: versions).
constexpr unsigned kEpiHeadStore = 1u << 16;    // GemvEpiArgs::head: store the GEMV's result
constexpr unsigned kEpiPrologue = 1u << 17;     // h is not loaded but computed: RMSNorm of x with gain and eps
constexpr unsigned kEpiXSlot = 1u << 18, kEpiGainSlot = 1u << 19;   // x / gain are pointer-table slots
constexpr unsigned kEpiStoreH = 1u << 20;       // workgroup 0 stores the normalised rows to g.h
struct GemvEpiArgs {
    GemvArgs g;             // with a prologue g.h is where the normalised rows are stored, not read
    unsigned head;          // bit 0 / 1: W / h are pointer-table slots; bits 8-15: slot that keeps the GEMV's result; bits 16-20 above
    int n_epi;
    const void* x;          // prologue: [rows, cols] to normalise
    const void* gain;       // prologue: [cols]
    float eps;
    int reserved;
    MergePhase ph[kEpiMaxPhases];   // m: period of in1 (rows * n = element for element)
};

struct Launch {
    const void* fn = nullptr;        // host-side kernel handle
    hipFunction_t mod_fn = nullptr;  // the same kernel as a module function, resolved on first launch
    unsigned arg_bytes = 0;          // size of the kernel's argument block
    dim3 grid{1, 1, 1};
    dim3 block{1, 1, 1};
    unsigned gemm_row_groups = 0;    // GEMV on the matrix cores: goes into GemvArgs::row_groups (0 = other kernels)
};

struct Shape {
    long long n = 0, m = 0, rows = 1, cols = 0, inner = 0;
};

// Kernel instantiation and launch shape for (op, dtype, mask of indirected operands, shape).  The
// choice depends on the shape alone, never on the mask or on pointer values, so the direct and the
// indirect form of a kernel run the same schedule.  False if there is no such kernel.
bool plan(int op, int dtype, int ind_mask, const Shape& shape, Launch* out);
const void* copy_kernel();
const void* table_kernel();
// Can this kernel be part of a merged dispatch?  From op, dtype and shape alone.  On success *n_out is
// the number of elements it produces (all kernels of a run must agree on it and on the dtype).
// whole_vectors: n must be a whole number of 16-byte vectors (runs of one workgroup per unit; a GEMV's
// epilogue works element by element and takes any n).
bool merge_candidate(int op, int dtype, const Shape& shape, bool whole_vectors, long long* n_out);
// Runs over small fp32 tensors work one element (4 bytes) per lane instead of a 16-byte vector: such
// kernels are bound by their dispatch, not by bytes, and one element per lane is what lets the fp32 GELU
// (evaluated in fp64, a few hundred instructions) ride along.  No RMSNorm in such a run (its row is a unit
// of 256 lanes x 16 bytes).
constexpr long long kMergeNarrowMax = 16384;        // elements
bool merge_narrow(int dtype, long long n);
const void* merged_kernel(int dtype, bool narrow);
// Is this a GEMV shape an epilogue form exists for?  bf16, rows of 2048 columns: up to 4 rows of h (the
// shape k_gemv_shared<bf16, ., 2, rows> serves; n >= 1024), or 5 rows and more (the matrix-core forms
// plan() picks for such rows; n >= 32).  *n_out = rows * n.
bool merge_head(int op, int dtype, const Shape& shape, long long* n_out);
// The epilogue form for that many rows of h; launched with the grid and row groups plan() gives the plain
// GEMV of the same shape.  A prologue exists up to kPrologueMaxRows rows (null otherwise).
// Up to two tiles of 16 rows, one per workgroup, fill the 256 CUs once; beyond, two workgroups share a CU and each
// normalises its tile, which costs more than the dispatch it saves (decode chain at 48 rows: 1261 -> 1336 us).
constexpr int kPrologueMaxRows = 32;
const void* gemv_epilogue_kernel(int rows_of_h, bool with_prologue);

}  // namespace pgk
