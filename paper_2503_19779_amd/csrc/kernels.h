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

}  // namespace pgk
