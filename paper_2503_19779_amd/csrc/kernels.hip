// kernels.hip -- the chain's device code for gfx950 (wave64): elementwise add / mul / GELU,
// RMSNorm, GEMV, per-channel scale + bias + ReLU, the batched multi-tensor copy and the
// pointer-table writer.
//
// Every compute kernel exists in a direct form (operands are tensor addresses) and in indirect
// forms (an operand is the address of a pointer-table slot that the kernel dereferences first;
// paper, Sec. 3 "Parameter Indirection" and Sec. 4 "Kernel generation": the body is unchanged,
// only a dereference prologue is added).  All forms of a kernel are instantiations of one body
// with one launch shape, so every replay mode computes bit-identical results.
//
// The chain's kernels are short (a few microseconds), so their cost is latency, not throughput:
// each shape class gets its own small instantiation (picked on the host from the shape alone, never
// from a pointer value), all loads are issued before the first use, and work is spread over lanes
// rather than looped inside one.  A misaligned external tensor changes only how a 16-byte vector is
// fetched (element loads instead of one vector load), never which lane adds what in which order, so
// results do not depend on alignment either.
//
// The translation unit is built with -ffp-contract=off: fused multiply-adds appear only where
// written.
#include "kernels.h"

#include <cstddef>

namespace pgk {
namespace {

constexpr int kBlock = 256;   // threads per workgroup = 4 waves of 64

#define PG_GLOBAL __attribute__((address_space(1)))
#define PG_CONSTANT __attribute__((address_space(4)))

// ---- operand resolution -------------------------------------------------------------------
template <bool IND>
__device__ __forceinline__ const void* resolve(const void* p) {
    if constexpr (IND) {
        // uniform address: one scalar load.  What a slot holds is a tensor in global memory; saying so lets the
        // compiler use global loads where it would otherwise fall back to generic ones (which also count as LDS operations)
        return (const void*)(const void PG_GLOBAL*)*reinterpret_cast<const uintptr_t*>(p);
    } else {
        return p;
    }
}

__device__ __forceinline__ bool aligned_to(const void* p, unsigned bytes) {
    return (reinterpret_cast<uintptr_t>(p) & (bytes - 1u)) == 0;
}

// ---- storage formats ------------------------------------------------------------------------
// Two fp32 values to a packed pair of bf16: round to nearest, ties to even, NaN stays a quiet NaN.
// One gfx950 conversion instruction instead of a dozen integer ones: these kernels are latency
// bound, every instruction on the path from the last load to the store counts.
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
typedef float v2f __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned pack2_bf16(float lo, float hi) {
    v2f x;
    x.x = lo;
    x.y = hi;
    return __builtin_bit_cast(unsigned, __builtin_convertvector(x, v2bf));
}
__device__ __forceinline__ unsigned f32_to_bf16(float f) { return pack2_bf16(f, 0.f) & 0xffffu; }

typedef unsigned short bf16_t;

// A "vector" is VB bytes (16 or 4) = NV elements, carried in NW 32-bit words.
template <typename T, int VB> struct Vec;
template <int VB> struct Vec<float, VB> {
    static constexpr int NV = VB / 4, NW = VB / 4;
    static __device__ __forceinline__ void unpack(const unsigned* w, float* f) {
#pragma unroll
        for (int i = 0; i < NV; i++) f[i] = __uint_as_float(w[i]);
    }
    static __device__ __forceinline__ void pack(const float* f, unsigned* w) {
#pragma unroll
        for (int i = 0; i < NV; i++) w[i] = __float_as_uint(f[i]);
    }
};
template <int VB> struct Vec<bf16_t, VB> {
    static constexpr int NV = VB / 2, NW = VB / 4;
    static __device__ __forceinline__ void unpack(const unsigned* w, float* f) {
#pragma unroll
        for (int i = 0; i < NW; i++) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ void pack(const float* f, unsigned* w) {
#pragma unroll
        for (int i = 0; i < NW; i++) w[i] = pack2_bf16(f[2 * i], f[2 * i + 1]);
    }
};

__device__ __forceinline__ unsigned load_raw(const float* p) { return *reinterpret_cast<const unsigned*>(p); }
__device__ __forceinline__ unsigned load_raw(const bf16_t* p) { return *p; }
template <typename T> __device__ __forceinline__ float from_raw(unsigned r) {
    return __uint_as_float(sizeof(T) == 4 ? r : r << 16);
}
__device__ __forceinline__ float load_elem(const float* p) { return *p; }
__device__ __forceinline__ float load_elem(const bf16_t* p) { return __uint_as_float((unsigned)*p << 16); }
__device__ __forceinline__ void store_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void store_elem(bf16_t* p, float v) { *p = (bf16_t)f32_to_bf16(v); }

typedef unsigned v4u __attribute__((ext_vector_type(4)));

// Fetch one vector of VB bytes as words.  AL: the address is VB-aligned; otherwise the same bytes
// arrive through element-sized loads (a tensor is always element aligned).  Loads only: nothing here
// consumes the data, so a caller can issue many of these before the first wait.
template <typename T, int VB, bool AL, bool NT = false>
__device__ __forceinline__ void load_vec(const T* p, unsigned* w) {
    constexpr int NW = VB / 4;
    if constexpr (AL) {
        if constexpr (VB == 16) {
            v4u t;
            if constexpr (NT) t = __builtin_nontemporal_load(reinterpret_cast<const v4u*>(p));
            else t = *reinterpret_cast<const v4u*>(p);
            w[0] = t.x; w[1] = t.y; w[2] = t.z; w[3] = t.w;
        } else {
            w[0] = *reinterpret_cast<const unsigned*>(p);
        }
    } else if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int i = 0; i < NW; i++) w[i] = reinterpret_cast<const unsigned*>(p)[i];
    } else {
#pragma unroll
        for (int i = 0; i < NW; i++)
            w[i] = (unsigned)reinterpret_cast<const unsigned short*>(p)[2 * i] |
                   ((unsigned)reinterpret_cast<const unsigned short*>(p)[2 * i + 1] << 16);
    }
}

// The same fetch through a pointer that says "global memory" outright.  A tensor address that reached the
// kernel through a pointer-table slot or a run-time choice is a generic pointer to the compiler; generic
// loads are slower and are counted as LDS operations as well, so a wait for LDS would wait for them too.
template <typename T, bool AL, bool NT = false>
__device__ __forceinline__ void load_vec_global(const T* p, unsigned* w) {
    if constexpr (AL) {
        v4u t;
        if constexpr (NT) t = __builtin_nontemporal_load((const v4u PG_GLOBAL*)(uintptr_t)p);
        else t = *(const v4u PG_GLOBAL*)(uintptr_t)p;
        w[0] = t.x; w[1] = t.y; w[2] = t.z; w[3] = t.w;
    } else if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int i = 0; i < 4; i++) w[i] = ((const unsigned PG_GLOBAL*)(uintptr_t)p)[i];
    } else {
        const unsigned short PG_GLOBAL* q = (const unsigned short PG_GLOBAL*)(uintptr_t)p;
#pragma unroll
        for (int i = 0; i < 4; i++) w[i] = (unsigned)q[2 * i] | ((unsigned)q[2 * i + 1] << 16);
    }
}
// The 4-byte vector (one fp32 or two bf16 elements) through a global pointer.
template <typename T, bool AL>
__device__ __forceinline__ void load_vec4_global(const T* p, unsigned* w) {
    if constexpr (sizeof(T) == 4 || AL) w[0] = *(const unsigned PG_GLOBAL*)(uintptr_t)p;
    else {
        const unsigned short PG_GLOBAL* q = (const unsigned short PG_GLOBAL*)(uintptr_t)p;
        w[0] = (unsigned)q[0] | ((unsigned)q[1] << 16);
    }
}
template <typename T>
__device__ __forceinline__ unsigned load_raw_global(const T* p) {
    if constexpr (sizeof(T) == 4) return *(const unsigned PG_GLOBAL*)(uintptr_t)p;
    else return *(const unsigned short PG_GLOBAL*)(uintptr_t)p;
}
// Element i of a tensor whose address is the same in every lane: the address stays in scalar registers and
// the load takes the lane's offset beside it, with no vector arithmetic on 64-bit addresses.
template <typename T>
__device__ __forceinline__ unsigned load_raw_global_at(const T* base, unsigned i) {
    if constexpr (sizeof(T) == 4) return ((const unsigned PG_GLOBAL*)(uintptr_t)base)[i];
    else return ((const unsigned short PG_GLOBAL*)(uintptr_t)base)[i];
}
__device__ __forceinline__ void store_vec_global(void* p, const unsigned* w) {
    v4u t;
    t.x = w[0]; t.y = w[1]; t.z = w[2]; t.w = w[3];
    *(v4u PG_GLOBAL*)(uintptr_t)p = t;
}
// A pointer-table slot, or the tensor address itself: decided at run time (the merged kernels; the
// stand-alone ones decide at compile time, resolve<IND>).  The slot is read as constant memory -- nothing
// writes the table while a graph runs -- which makes it a scalar load that no vector-memory wait covers.
__device__ __forceinline__ const void* resolve_rt(const void* p, unsigned is_slot) {
    return is_slot ? *(const void* const PG_CONSTANT*)(uintptr_t)p : p;
}

// Rows of `cols` elements in 16-byte vectors: nfull = cols / NV full vectors, then (RAGGED shapes
// only) one partial vector.  Fetching is split in two so that all loads of a kernel can be in flight
// together: row_vec_issue loads vector min(v, nfull-1) -- always inside the row, no branch -- and
// row_vec_finish unpacks it, zeroes it if v lies beyond the full vectors, and reads the partial
// vector's elements one by one.
template <typename T, bool AL, bool NT = false>
__device__ __forceinline__ void row_vec_issue(const T* row, int nfull, int v, unsigned* w) {
    constexpr int NV = Vec<T, 16>::NV;
    const int vc = v < nfull ? v : nfull - 1;
    load_vec<T, 16, AL, NT>(row + (size_t)vc * NV, w);
}
// Words of vector v after the fact: zero beyond the full vectors, and (RAGGED) the partial vector
// read element by element.
template <typename T, bool RAGGED>
__device__ __forceinline__ void row_vec_fix(const T* row, int cols, int nfull, int v, unsigned* w) {
    constexpr int NV = Vec<T, 16>::NV;
    if (v >= nfull) {
#pragma unroll
        for (int i = 0; i < 4; i++) w[i] = 0u;
        if constexpr (RAGGED) {
            if (v == nfull) {
                const int left = cols - nfull * NV;
#pragma unroll
                for (int i = 0; i < NV; i++) {
                    if (i < left) {
                        const unsigned r = load_raw(row + (size_t)nfull * NV + i);
                        if constexpr (sizeof(T) == 4) w[i] = r;
                        else w[i / 2] |= r << (16 * (i & 1));
                    }
                }
            }
        }
    }
}
template <typename T, bool RAGGED>
__device__ __forceinline__ void row_vec_finish(const T* row, int cols, int nfull, int v, unsigned* w, float* f) {
    row_vec_fix<T, RAGGED>(row, cols, nfull, v, w);
    Vec<T, 16>::unpack(w, f);
}

// acc += sum of the products of two vectors' elements, in element order.  bf16: one packed
// two-element dot product (fp32 accumulate) per word; fp32: one fused multiply-add per element.
template <typename T>
__device__ __forceinline__ float dot_acc(const unsigned* a, const unsigned* b, float acc) {
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int i = 0; i < 4; i++) acc = __builtin_fmaf(__uint_as_float(a[i]), __uint_as_float(b[i]), acc);
    } else {
#pragma unroll
        for (int i = 0; i < 4; i++)
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(v2bf, a[i]), __builtin_bit_cast(v2bf, b[i]), acc, false);
    }
    return acc;
}

template <int VB>
__device__ __forceinline__ void store_vec(void* p, const unsigned* w) {
    if constexpr (VB == 16) {
        v4u t;
        t.x = w[0]; t.y = w[1]; t.z = w[2]; t.w = w[3];
        *reinterpret_cast<v4u*>(p) = t;
    } else {
        *reinterpret_cast<unsigned*>(p) = w[0];
    }
}

// ---- wave64 reduction -----------------------------------------------------------------------
// Butterfly over the 16 lanes of a DPP row, then the four row sums are read out and added in a
// fixed order.  Every lane performs the same additions on the same values, so all lanes hold the
// same bits.  Needs all 64 lanes active.
template <int CTRL>
__device__ __forceinline__ float dpp_add(float v) {
    int t = __builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, false);
    return v + __int_as_float(t);
}
__device__ __forceinline__ float wave_sum(float v) {
    v = dpp_add<0xB1>(v);    // quad_perm [1,0,3,2]: lane ^ 1
    v = dpp_add<0x4E>(v);    // quad_perm [2,3,0,1]: lane ^ 2
    v = dpp_add<0x141>(v);   // row_half_mirror: the other quad of each 8
    v = dpp_add<0x140>(v);   // row_mirror: the other half of each 16
    float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    return ((r0 + r1) + r2) + r3;
}

// Workgroup barrier for an exchange through LDS only: waits for this wave's LDS operations, not for its
// outstanding global stores (which __syncthreads would, at about a microsecond apiece).
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// ---- elementwise ----------------------------------------------------------------------------
// GELU(a) = a * Phi(a) with Phi(a) = erfc(-a / sqrt 2) / 2 (keeps relative accuracy in the left
// tail).  For fp32 tensors it is evaluated in fp64 and rounded once, so that the result is the
// correctly rounded one except within ~1e-16 of a rounding boundary: an fp32 erfc is a few ulp off,
// and a chain of multiplies and cancelling adds amplifies that beyond 1e-5.  For bf16 tensors fp32
// is far more than the 8 stored bits need, and the library erfcf (a few hundred instructions over
// several branches, which a wave of mixed values all takes) made large GELU kernels ALU-bound at a
// quarter of the HBM rate; gelu_bf16 below is branch-free and about 40 instructions.
//
// erfc(z), z >= 0, as (1 - u) * exp(-z^2 + u * Q(u)) with u = z / (2 + z) in [0, 1): the exponent's
// second term is log(erfc(z) exp(z^2) (1 + z/2)), smooth in u and zero at u = 0, so that erfc(0) = 1
// comes out exactly and tiny inputs give a/2 exactly.  Q: degree 9, a Chebyshev fit on z <= 9.7
// (beyond, a * Phi(a) is below the smallest normal number), max error 8e-9 in the exponent.  z^2 is
// taken with its rounding error (one fma), the exponential as 2^k * exp2(r) with |r| <= 0.51 after a
// two-constant reduction, so the relative error stays near 2e-7 into the tail.  Checked against the
// fp64 definition on every finite bf16 input: the bf16 result is the correctly rounded one for all
// of them (the closest any exact value comes to a rounding boundary is 8e-7, at a = -0.336).
__device__ __forceinline__ float gelu_bf16(float a) {
    const float x = a * -0.70710678118654752440f;
    const float z = __builtin_fminf(__builtin_fabsf(x), 14.0f);      // erfc(14) = 0 in fp32; keeps z * z finite (and a NaN out of the exponent)
    const float u = z * __builtin_amdgcn_rcpf(2.0f + z);
    const float t = 1.0f - u;
    float p = -0.153892517f;
    p = __builtin_fmaf(p, u, 0.49560681f);
    p = __builtin_fmaf(p, u, -0.509543419f);
    p = __builtin_fmaf(p, u, 0.182105958f);
    p = __builtin_fmaf(p, u, -0.144903973f);
    p = __builtin_fmaf(p, u, 0.072065711f);
    p = __builtin_fmaf(p, u, 0.19142893f);
    p = __builtin_fmaf(p, u, 0.161542267f);
    p = __builtin_fmaf(p, u, -0.303239733f);
    p = __builtin_fmaf(p, u, -1.25675833f);
    p = p * u;
    const float s = z * z, e = __builtin_fmaf(z, z, -s);               // z^2 = s + e exactly
    constexpr float kLog2e = 1.4426950408889634f, kLn2Hi = 0.693145751953125f, kLn2Lo = 1.42860682030941723212e-6f;
    const float kf = __builtin_rintf((p - s) * kLog2e);
    float r = __builtin_fmaf(kf, -kLn2Hi, -s);
    r = r + p;
    r = r - e;
    r = __builtin_fmaf(kf, -kLn2Lo, r);
    const float v = __builtin_ldexpf(t * __builtin_amdgcn_exp2f(r * kLog2e), (int)kf);
    const float erfc_x = x < 0.f ? 2.0f - v : v;
    return (0.5f * a) * erfc_x;      // a NaN comes back through this product; -inf * 0 = NaN as in the definition
}

template <int OP, bool WIDE>
__device__ __forceinline__ float ew_apply(float a, float b) {
    if constexpr (OP == kAdd) {
        return a + b;
    } else if constexpr (OP == kMul) {
        return a * b;
    } else if constexpr (WIDE) {
        const double x = (double)a;
        return (float)((0.5 * x) * erfc(x * -0.70710678118654752440));
    } else {
        return gelu_bf16(a);
    }
}

// Each lane owns U vectors of VB bytes, 256 lanes apart; one block also does the n % NV trailing
// elements.  `o` may alias `a` (in place): a lane reads what it later overwrites.  AL: a (and b,
// when it is read by vectors) are VB-aligned.
// `bid`: the index of the block of 256 lanes this call plays (blockIdx.x in the stand-alone kernel).
template <typename T, int OP, int VB, int U, typename IdxT, bool AL>
__device__ __forceinline__ void ew_body(const T* a, const T* b, T* o, IdxT n, IdxT m, bool b_vec, unsigned bid) {
    using V = Vec<T, VB>;
    constexpr int NV = V::NV, NW = V::NW;
    constexpr bool kBinary = (OP != kGelu);
    constexpr bool kWide = sizeof(T) == 4;
    const IdxT nvec = n / NV;
    const IdxT base = (IdxT)bid * (kBlock * U) + threadIdx.x;
    unsigned wa[U][NW], wb[U][NW], rb[U][NV];
#pragma unroll
    for (int u = 0; u < U; u++) {
        const IdxT v = base + (IdxT)u * kBlock;
        if (v < nvec) {
            load_vec<T, VB, AL>(a + v * NV, wa[u]);
            if constexpr (kBinary) {
                const IdxT i0 = v * NV;
                if (b_vec) {
                    load_vec<T, VB, AL>(b + ((m == n) ? i0 : i0 % m), wb[u]);
                } else {
#pragma unroll
                    for (int e = 0; e < NV; e++) rb[u][e] = load_raw(b + (i0 + e) % m);
                }
            }
        }
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
        const IdxT v = base + (IdxT)u * kBlock;
        if (v < nvec) {
            float fa[NV], fb[NV], fo[NV];
            unsigned wo[NW];
            V::unpack(wa[u], fa);
            if constexpr (kBinary) {
                if (b_vec) V::unpack(wb[u], fb);
                else
#pragma unroll
                    for (int e = 0; e < NV; e++) fb[e] = from_raw<T>(rb[u][e]);
            }
#pragma unroll
            for (int e = 0; e < NV; e++) fo[e] = ew_apply<OP, kWide>(fa[e], kBinary ? fb[e] : 0.f);
            V::pack(fo, wo);
            store_vec<VB>(o + v * NV, wo);
        }
    }
    if constexpr (NV > 1) {
        if (bid == nvec / (kBlock * U)) {   // the block that would own vector index nvec
            const IdxT i = nvec * NV + threadIdx.x;
            if (threadIdx.x < NV && i < n) {
                const float fb1 = kBinary ? load_elem(b + (i % m)) : 0.f;
                store_elem(o + i, ew_apply<OP, kWide>(load_elem(a + i), fb1));
            }
        }
    }
}

template <typename T, int OP, int IND, int VB, int U, typename IdxT>
__global__ __launch_bounds__(kBlock) void k_elementwise(EwArgs p) {
    constexpr bool kBinary = (OP != kGelu);
    constexpr int NV = Vec<T, VB>::NV;
    const T* a = static_cast<const T*>(resolve<(IND & 1) != 0>(p.a));
    const T* b = kBinary ? static_cast<const T*>(resolve<(IND & 2) != 0>(p.b)) : nullptr;
    T* o = static_cast<T*>(p.out);
    const IdxT n = (IdxT)p.n, m = (IdxT)p.m;
    const bool b_vec = kBinary && (m % NV) == 0;      // then a vector of b never wraps around the period
    const bool al = aligned_to(a, VB) && (!b_vec || aligned_to(b, VB));
    if (__builtin_expect(al, 1)) ew_body<T, OP, VB, U, IdxT, true>(a, b, o, n, m, b_vec, blockIdx.x);
    else ew_body<T, OP, VB, U, IdxT, false>(a, b, o, n, m, b_vec, blockIdx.x);
}

// ---- per-channel scale + bias + ReLU on [N, C, inner] ---------------------------------------
__device__ __forceinline__ float sbr_apply(float x, float s, float b) {
    const float v = __builtin_fmaf(x, s, b);
    return v > 0.f ? v : 0.f;
}

// VEC: inner is a multiple of the 16-byte vector, so a vector never straddles two channels.
template <typename T, bool VEC, int U, typename IdxT, bool AL>
__device__ __forceinline__ void sbr_body(const T* x, const T* s, const T* b, T* o, IdxT n, unsigned inner, unsigned channels) {
    using V = Vec<T, 16>;
    constexpr int NV = VEC ? V::NV : 1;
    const IdxT nvec = n / NV;      // n is a multiple of inner, hence of NV
    const IdxT base = (IdxT)blockIdx.x * (kBlock * U) + threadIdx.x;
    unsigned wx[U][4], rs[U], rbv[U];
#pragma unroll
    for (int u = 0; u < U; u++) {
        const IdxT v = base + (IdxT)u * kBlock;
        if (v < nvec) {
            if constexpr (VEC) load_vec<T, 16, AL>(x + v * NV, wx[u]);
            else wx[u][0] = load_raw(x + v);
            const unsigned c = (unsigned)(((v * NV) / inner) % channels);
            rs[u] = load_raw(s + c);
            rbv[u] = load_raw(b + c);
        }
    }
#pragma unroll
    for (int u = 0; u < U; u++) {
        const IdxT v = base + (IdxT)u * kBlock;
        if (v < nvec) {
            const float fs = from_raw<T>(rs[u]), fb = from_raw<T>(rbv[u]);
            if constexpr (VEC) {
                float fx[V::NV], fo[V::NV];
                unsigned wo[V::NW];
                V::unpack(wx[u], fx);
#pragma unroll
                for (int e = 0; e < V::NV; e++) fo[e] = sbr_apply(fx[e], fs, fb);
                V::pack(fo, wo);
                store_vec<16>(o + v * NV, wo);
            } else {
                store_elem(o + v, sbr_apply(from_raw<T>(wx[u][0]), fs, fb));
            }
        }
    }
}

template <typename T, int IND, bool VEC, int U, typename IdxT>
__global__ __launch_bounds__(kBlock) void k_scale_bias_relu(SbrArgs p) {
    const T* x = static_cast<const T*>(resolve<(IND & 1) != 0>(p.x));
    const T* s = static_cast<const T*>(resolve<(IND & 2) != 0>(p.s));
    const T* b = static_cast<const T*>(resolve<(IND & 4) != 0>(p.b));
    T* o = static_cast<T*>(p.out);
    if (!VEC || aligned_to(x, 16)) sbr_body<T, VEC, U, IdxT, true>(x, s, b, o, (IdxT)p.n, p.inner, p.channels);
    else sbr_body<T, VEC, U, IdxT, false>(x, s, b, o, (IdxT)p.n, p.inner, p.channels);
}

// ---- RMSNorm: one workgroup per row ------------------------------------------------------------
// Each thread keeps its VPT vectors of x and of the gain in registers (all fetched up front), sums
// squares with fused multiply-adds, a wave64 shuffle reduction follows, the four wave sums are
// staged through LDS and added in a fixed order by every thread.  VPT = 0 is the long-row form: it
// loops and reads x a second time.
template <typename T, bool RAGGED>
__device__ __forceinline__ void rms_store(T* o, int cols, int nfull, int v, bool al_o, const float* fo) {
    constexpr int NV = Vec<T, 16>::NV;
    if (v < nfull && (al_o || !RAGGED)) {
        unsigned w[4];
        Vec<T, 16>::pack(fo, w);
        store_vec<16>(o + (size_t)v * NV, w);
    } else if constexpr (RAGGED) {
        const int left = cols - v * NV;
#pragma unroll
        for (int e = 0; e < NV; e++)
            if (e < left) store_elem(o + (size_t)v * NV + e, fo[e]);
    }
}

template <typename T, int VPT, bool RAGGED, bool AL>
__device__ __forceinline__ void rms_body(const T* x, const T* g, T* o, int cols, float eps, bool al_o, float* part) {
    constexpr int NV = Vec<T, 16>::NV;
    const int tid = threadIdx.x;
    const int nfull = cols / NV;
    float acc = 0.f;
    if constexpr (VPT > 0) {
        unsigned wx[VPT][4], wg[VPT][4];
        float fx[VPT][NV], fg[VPT][NV];
        if (!RAGGED || nfull > 0) {
#pragma unroll
            for (int u = 0; u < VPT; u++) {
                row_vec_issue<T, AL>(x, nfull, tid + u * kBlock, wx[u]);
                row_vec_issue<T, AL>(g, nfull, tid + u * kBlock, wg[u]);
            }
        }
#pragma unroll
        for (int u = 0; u < VPT; u++) {
            row_vec_finish<T, RAGGED>(x, cols, nfull, tid + u * kBlock, wx[u], fx[u]);
#pragma unroll
            for (int e = 0; e < NV; e++) acc = __builtin_fmaf(fx[u][e], fx[u][e], acc);
        }
        acc = wave_sum(acc);
        if ((tid & 63) == 0) part[tid >> 6] = acc;
        __syncthreads();
        const float total = ((part[0] + part[1]) + part[2]) + part[3];
        const float scale = 1.0f / sqrtf(total / (float)cols + eps);
#pragma unroll
        for (int u = 0; u < VPT; u++) {
            float fo[NV];
            row_vec_finish<T, RAGGED>(g, cols, nfull, tid + u * kBlock, wg[u], fg[u]);
#pragma unroll
            for (int e = 0; e < NV; e++) fo[e] = (fx[u][e] * scale) * fg[u][e];
            rms_store<T, RAGGED>(o, cols, nfull, tid + u * kBlock, al_o, fo);
        }
    } else {
        const int nvec = (cols + NV - 1) / NV;
        for (int v = tid; v < nvec; v += kBlock) {
            unsigned w[4];
            float f[NV];
            if (!RAGGED || nfull > 0) row_vec_issue<T, AL>(x, nfull, v, w);
            row_vec_finish<T, RAGGED>(x, cols, nfull, v, w, f);
#pragma unroll
            for (int e = 0; e < NV; e++) acc = __builtin_fmaf(f[e], f[e], acc);
        }
        acc = wave_sum(acc);
        if ((tid & 63) == 0) part[tid >> 6] = acc;
        __syncthreads();
        const float total = ((part[0] + part[1]) + part[2]) + part[3];
        const float scale = 1.0f / sqrtf(total / (float)cols + eps);
        for (int v = tid; v < nvec; v += kBlock) {
            unsigned w[4], w2[4];
            float f[NV], fgv[NV], fo[NV];
            if (!RAGGED || nfull > 0) {
                row_vec_issue<T, AL>(x, nfull, v, w);
                row_vec_issue<T, AL>(g, nfull, v, w2);
            }
            row_vec_finish<T, RAGGED>(x, cols, nfull, v, w, f);
            row_vec_finish<T, RAGGED>(g, cols, nfull, v, w2, fgv);
#pragma unroll
            for (int e = 0; e < NV; e++) fo[e] = (f[e] * scale) * fgv[e];
            rms_store<T, RAGGED>(o, cols, nfull, v, al_o, fo);
        }
    }
}

// one row by one workgroup of 256 lanes; x0 / o0: the first row
template <typename T, int VPT, bool RAGGED>
__device__ __forceinline__ void rms_row(const T* x0, const T* g, T* o0, int cols, float eps, size_t row, float* part) {
    const T* x = x0 + row * cols;
    T* o = o0 + row * cols;
    // rows of an aligned buffer stay aligned when cols is a multiple of the vector; else check this row
    const bool al = aligned_to(x, 16) && aligned_to(g, 16);
    const bool al_o = aligned_to(o, 16);
    if (__builtin_expect(al, 1)) rms_body<T, VPT, RAGGED, true>(x, g, o, cols, eps, al_o, part);
    else rms_body<T, VPT, RAGGED, false>(x, g, o, cols, eps, al_o, part);
}

template <typename T, int IND, int VPT, bool RAGGED>
__global__ __launch_bounds__(kBlock) void k_rmsnorm(RmsArgs p) {
    const T* x = static_cast<const T*>(resolve<(IND & 1) != 0>(p.x));
    const T* g = static_cast<const T*>(resolve<(IND & 2) != 0>(p.g));
    __shared__ float part[kBlock / 64];
    rms_row<T, VPT, RAGGED>(x, g, static_cast<T*>(p.out), p.cols, p.eps, blockIdx.x, part);
}

// ---- GEMV ------------------------------------------------------------------------------------------
// Ask for every kernel argument in one batch of scalar loads.  Left alone, the compiler fetches `n`
// for the early-exit test first and the pointers only behind it: two dependent trips to the kernel
// argument buffer (cold in the scalar cache at every launch) before the first weight load goes out,
// about 0.4 us on a 3 us kernel.
__device__ __forceinline__ void args_up_front(const GemvArgs& p) {
    asm volatile("" ::"s"(p.out), "s"(p.W), "s"(p.h), "s"(p.rows), "s"(p.n), "s"(p.cols), "s"(p.row_groups));
}

// Memory-bound: every weight is read exactly once.  One wave computes R output columns (R weight
// rows): per chunk of 4 * 64 vectors of the row it issues all R * 4 weight loads (non-temporal:
// streamed, no reuse) and the 4 loads of its slice of h before the first multiply, accumulates in
// fp32 in a fixed order, and reduces across the wave.  No MFMA: at batch 1 there is no reuse to
// feed a matrix core.  Row-shape classes RS (from cols alone): 0 = cols is a whole number of
// chunks (no bounds handling at all), 1 = a whole number of vectors, 2 = ragged.
constexpr int kGemvChunk = 4;   // vectors per lane per chunk

template <typename T, int RS, bool AL, bool NT>
__device__ __forceinline__ void gemv_issue(const T* row, int nfull, int v, unsigned* w) {
    constexpr int NV = Vec<T, 16>::NV;
    if constexpr (RS == 0) load_vec<T, 16, AL, NT>(row + (size_t)v * NV, w);
    else row_vec_issue<T, AL, NT>(row, nfull, v, w);
}
template <typename T, int RS>
__device__ __forceinline__ void gemv_fix(const T* row, int cols, int nfull, int v, unsigned* w) {
    if constexpr (RS != 0) row_vec_fix<T, RS == 2>(row, cols, nfull, v, w);
}

template <typename T, int R, int RS, bool AL>
__device__ __forceinline__ void gemv_body(const T* W, const T* h, T* y, int n, int cols, int j0, int lane) {
    constexpr int NV = Vec<T, 16>::NV;
    const int nfull = cols / NV;
    const int nvec = (cols + NV - 1) / NV;
    float acc[R];
    const T* wrow[R];
#pragma unroll
    for (int r = 0; r < R; r++) {
        acc[r] = 0.f;
        wrow[r] = W + (size_t)((j0 + r < n) ? j0 + r : n - 1) * cols;   // a ragged last group re-reads the last row
    }
    for (int v0 = 0; v0 < nvec; v0 += 64 * kGemvChunk) {
        unsigned ww[R][kGemvChunk][4], wh[kGemvChunk][4];
        if (RS != 2 || nfull > 0) {
#pragma unroll
            for (int r = 0; r < R; r++)
#pragma unroll
                for (int u = 0; u < kGemvChunk; u++) gemv_issue<T, RS, AL, true>(wrow[r], nfull, v0 + u * 64 + lane, ww[r][u]);
#pragma unroll
            for (int u = 0; u < kGemvChunk; u++) gemv_issue<T, RS, AL, false>(h, nfull, v0 + u * 64 + lane, wh[u]);
        }
#pragma unroll
        for (int u = 0; u < kGemvChunk; u++) gemv_fix<T, RS>(h, cols, nfull, v0 + u * 64 + lane, wh[u]);
#pragma unroll
        for (int r = 0; r < R; r++)
#pragma unroll
            for (int u = 0; u < kGemvChunk; u++) {
                gemv_fix<T, RS>(wrow[r], cols, nfull, v0 + u * 64 + lane, ww[r][u]);
                acc[r] = dot_acc<T>(ww[r][u], wh[u], acc[r]);
            }
    }
#pragma unroll
    for (int r = 0; r < R; r++) {
        const float s = wave_sum(acc[r]);
        if (lane == 0 && j0 + r < n) store_elem(y + j0 + r, s);
    }
}

template <typename T, int IND, int R, int RS>
__global__ __launch_bounds__(kBlock) void k_gemv(GemvArgs p) {
    args_up_front(p);
    const T* W = static_cast<const T*>(resolve<(IND & 1) != 0>(p.W));
    const T* h = static_cast<const T*>(resolve<(IND & 2) != 0>(p.h));
    T* y = static_cast<T*>(p.out);
    const int lane = threadIdx.x & 63;
    const int j0 = (blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6)) * R;
    if (j0 >= p.n) return;   // whole wave leaves together
    // row starts of W stay aligned only if cols is a multiple of the vector
    const bool al = RS != 2 && aligned_to(W, 16) && aligned_to(h, 16);
    if (__builtin_expect(al, 1)) gemv_body<T, R, RS, true>(W, h, y, p.n, p.cols, j0, lane);
    else gemv_body<T, R, RS, false>(W, h, y, p.n, p.cols, j0, lane);
}

// The same for rows of exactly one chunk (2048 bf16 or 1024 fp32 columns -- the decode chain's shape)
// and one or two rows of h: instead of every wave fetching all of h, lane t of the workgroup fetches
// vector t of each row once and the four waves share it through LDS.  That takes 12 KB (one row of h)
// or 24 KB (two) of cache traffic per workgroup off the load path the weights come in by (3.16 ->
// 3.07 us per launch at 2048 x 2048, one row); h is asked for before the weights, so the exchange is
// over long before the first weight arrives.  Same lanes, same products, same order as gemv_body and
// gemvb_body: the results are bit-identical.
static_assert(kBlock == 64 * kGemvChunk, "one vector of h per lane of the workgroup");
// `after_issue()` runs once every weight load of the wave has been asked for (the epilogue form of the
// kernel fetches its own operands there: every instruction in front of the weight loads delays the whole
// kernel -- asking for the epilogue's operands first, so that they would be back before the weights,
// measured 0.17 us slower per launch); sums[r][rr] receives the finished dot products, the same bits in
// every lane.
// GLOBAL: W and h reached the kernel as generic pointers (through a run-time choice); fetch them with loads
// that say "global memory" outright.
// PRO: h is not loaded but computed here -- `h` points at the rows x to normalise, `gain` and `eps` are
// RMSNorm's; the arithmetic is rms_body's for a row of one vector per lane (fused multiply-add sum of
// squares in element order, wave_sum, the four wave sums added in a fixed order through LDS,
// 1 / sqrt(mean + eps), (x * scale) * gain, one rounding), and lane t's vector of the result goes where
// lane t's vector of h would have gone.  hstore != nullptr: this workgroup also stores the rows there.
// (eps by reference: the epilogue kernel reads it from its arguments inside the hook.)
template <typename T, int R, int RB, bool AL, bool GLOBAL, bool PRO, class Hook>
__device__ __forceinline__ void gemv_sums_shared(const T* W, const T* h, int n, int j0, int lane, int tid, v4u* hs /* [RB][kBlock] */,
                                                 Hook after_issue, float (*sums)[RB],
                                                 const T* gain = nullptr, const float& eps = 0.f, T* hstore = nullptr, float* part = nullptr) {
    constexpr int NV = Vec<T, 16>::NV;
    constexpr int kCols = 64 * kGemvChunk * NV;
    unsigned hv[RB][4], ww[R][kGemvChunk][4], wh[RB][kGemvChunk][4], wg[4];
#pragma unroll
    for (int rr = 0; rr < RB; rr++) {
        if constexpr (GLOBAL) load_vec_global<T, AL, false>(h + (size_t)rr * kCols + (size_t)tid * NV, hv[rr]);
        else load_vec<T, 16, AL, false>(h + (size_t)rr * kCols + (size_t)tid * NV, hv[rr]);
    }
    if constexpr (PRO) load_vec_global<T, AL, false>(gain + (size_t)tid * NV, wg);
    __builtin_amdgcn_sched_barrier(0);   // h first: loads come back in the order they were issued
#pragma unroll
    for (int r = 0; r < R; r++) {
        const T* wrow = W + (size_t)((j0 + r < n) ? j0 + r : n - 1) * kCols;   // a ragged last group re-reads the last row
#pragma unroll
        for (int u = 0; u < kGemvChunk; u++) {
            if constexpr (GLOBAL) load_vec_global<T, AL, true>(wrow + (size_t)(u * 64 + lane) * NV, ww[r][u]);
            else load_vec<T, 16, AL, true>(wrow + (size_t)(u * 64 + lane) * NV, ww[r][u]);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
    after_issue();
    if constexpr (PRO) {
        float fg[NV];
        Vec<T, 16>::unpack(wg, fg);
        // every row's sum of squares first, then one barrier for all rows (a row of partial sums per row of x)
#pragma unroll
        for (int rr = 0; rr < RB; rr++) {
            float fx[NV];
            Vec<T, 16>::unpack(hv[rr], fx);
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < NV; e++) acc = __builtin_fmaf(fx[e], fx[e], acc);
            acc = wave_sum(acc);
            if ((tid & 63) == 0) part[rr * (kBlock / 64) + (tid >> 6)] = acc;
        }
        lds_barrier();
#pragma unroll
        for (int rr = 0; rr < RB; rr++) {
            float fx[NV], fo[NV];
            Vec<T, 16>::unpack(hv[rr], fx);
            const float* prow = part + rr * (kBlock / 64);
            const float total = ((prow[0] + prow[1]) + prow[2]) + prow[3];
            const float scale = 1.0f / sqrtf(total / (float)kCols + eps);
#pragma unroll
            for (int e = 0; e < NV; e++) fo[e] = (fx[e] * scale) * fg[e];
            Vec<T, 16>::pack(fo, hv[rr]);
        }
    }
#pragma unroll
    for (int rr = 0; rr < RB; rr++) {
        v4u t;
        t.x = hv[rr][0]; t.y = hv[rr][1]; t.z = hv[rr][2]; t.w = hv[rr][3];
        hs[rr * kBlock + tid] = t;
    }
    __syncthreads();      // every wave of the workgroup gets here: none leaves early
    if constexpr (PRO) {  // after the barrier, which would otherwise wait for these stores
        if (hstore)
#pragma unroll
            for (int rr = 0; rr < RB; rr++) store_vec_global(hstore + (size_t)rr * kCols + (size_t)tid * NV, hv[rr]);
    }
#pragma unroll
    for (int rr = 0; rr < RB; rr++)
#pragma unroll
        for (int u = 0; u < kGemvChunk; u++) {
            const v4u t = hs[rr * kBlock + u * 64 + lane];
            wh[rr][u][0] = t.x; wh[rr][u][1] = t.y; wh[rr][u][2] = t.z; wh[rr][u][3] = t.w;
        }
    float acc[R][RB];
#pragma unroll
    for (int r = 0; r < R; r++)
#pragma unroll
        for (int rr = 0; rr < RB; rr++) {
            acc[r][rr] = 0.f;
#pragma unroll
            for (int u = 0; u < kGemvChunk; u++) acc[r][rr] = dot_acc<T>(ww[r][u], wh[rr][u], acc[r][rr]);
        }
#pragma unroll
    for (int rr = 0; rr < RB; rr++)
#pragma unroll
        for (int r = 0; r < R; r++) sums[r][rr] = wave_sum(acc[r][rr]);
}

template <typename T, int R, int RB, bool AL>
__device__ __forceinline__ void gemv_body_shared(const T* W, const T* h, T* y, int n, int j0, int lane, int tid, v4u* hs /* [RB][kBlock] */) {
    float sums[R][RB];
    gemv_sums_shared<T, R, RB, AL, false, false>(W, h, n, j0, lane, tid, hs, [] {}, sums);
#pragma unroll
    for (int rr = 0; rr < RB; rr++)
#pragma unroll
        for (int r = 0; r < R; r++)
            if (lane == 0 && j0 + r < n) store_elem(y + (size_t)rr * n + j0 + r, sums[r][rr]);
}

// RB = rows of h: 1 to 4
template <typename T, int IND, int R, int RB>
__global__ __launch_bounds__(kBlock) void k_gemv_shared(GemvArgs p) {
    args_up_front(p);
    const T* W = static_cast<const T*>(resolve<(IND & 1) != 0>(p.W));
    const T* h = static_cast<const T*>(resolve<(IND & 2) != 0>(p.h));
    T* y = static_cast<T*>(p.out);
    __shared__ v4u hs[RB * kBlock];
    const int tid = threadIdx.x, lane = tid & 63;
    const int j0 = (blockIdx.x * (kBlock / 64) + (tid >> 6)) * R;
    const bool al = aligned_to(W, 16) && aligned_to(h, 16);
    if (__builtin_expect(al, 1)) gemv_body_shared<T, R, RB, true>(W, h, y, p.n, j0, lane, tid, hs);
    else gemv_body_shared<T, R, RB, false>(W, h, y, p.n, j0, lane, tid, hs);
}

// Batched (rows > 1) on the vector units: one wave per R output columns, as in the one-row kernel;
// the R weight chunks stay in registers while the rows of h (from cache) stream past them,
// RB rows at a time (RB = 2 when there are only two rows: a clamped row would be loaded and summed
// for nothing).
template <typename T, int R, int RB, int RS, bool AL>
__device__ __forceinline__ void gemvb_body(const T* W, const T* h, T* y, int rows, int n, int cols, int j0, int lane) {
    constexpr int NV = Vec<T, 16>::NV;
    const int nfull = cols / NV;
    const int nvec = (cols + NV - 1) / NV;
    const T* wrow[R];
#pragma unroll
    for (int r = 0; r < R; r++) wrow[r] = W + (size_t)((j0 + r < n) ? j0 + r : n - 1) * cols;   // a ragged last group re-reads the last row
    for (int r0 = 0; r0 < rows; r0 += RB) {
        float acc[R][RB];
        const T* hrow[RB];
#pragma unroll
        for (int rr = 0; rr < RB; rr++) {
#pragma unroll
            for (int r = 0; r < R; r++) acc[r][rr] = 0.f;
            hrow[rr] = h + (size_t)((r0 + rr < rows) ? r0 + rr : rows - 1) * cols;
        }
        for (int v0 = 0; v0 < nvec; v0 += 64 * kGemvChunk) {
            unsigned ww[R][kGemvChunk][4], wh[RB][kGemvChunk][4];
            if (RS != 2 || nfull > 0) {
#pragma unroll
                for (int r = 0; r < R; r++)
#pragma unroll
                    for (int u = 0; u < kGemvChunk; u++) gemv_issue<T, RS, AL, true>(wrow[r], nfull, v0 + u * 64 + lane, ww[r][u]);
#pragma unroll
                for (int rr = 0; rr < RB; rr++)
#pragma unroll
                    for (int u = 0; u < kGemvChunk; u++) gemv_issue<T, RS, AL, false>(hrow[rr], nfull, v0 + u * 64 + lane, wh[rr][u]);
            }
#pragma unroll
            for (int r = 0; r < R; r++)
#pragma unroll
                for (int u = 0; u < kGemvChunk; u++) gemv_fix<T, RS>(wrow[r], cols, nfull, v0 + u * 64 + lane, ww[r][u]);
#pragma unroll
            for (int rr = 0; rr < RB; rr++)
#pragma unroll
                for (int u = 0; u < kGemvChunk; u++) {
                    gemv_fix<T, RS>(hrow[rr], cols, nfull, v0 + u * 64 + lane, wh[rr][u]);
#pragma unroll
                    for (int r = 0; r < R; r++) acc[r][rr] = dot_acc<T>(ww[r][u], wh[rr][u], acc[r][rr]);
                }
        }
#pragma unroll
        for (int rr = 0; rr < RB; rr++)
#pragma unroll
            for (int r = 0; r < R; r++) {
                const float s = wave_sum(acc[r][rr]);
                if (lane == 0 && r0 + rr < rows && j0 + r < n) store_elem(y + (size_t)(r0 + rr) * n + j0 + r, s);
            }
    }
}

template <typename T, int IND, int R, int RB, int RS>
__global__ __launch_bounds__(kBlock) void k_gemv_batched(GemvArgs p) {
    args_up_front(p);
    const T* W = static_cast<const T*>(resolve<(IND & 1) != 0>(p.W));
    const T* h = static_cast<const T*>(resolve<(IND & 2) != 0>(p.h));
    T* y = static_cast<T*>(p.out);
    const int lane = threadIdx.x & 63;
    const int j0 = (blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6)) * R;
    if (j0 >= p.n) return;
    const bool al = RS != 2 && aligned_to(W, 16) && aligned_to(h, 16);
    if (__builtin_expect(al, 1)) gemvb_body<T, R, RB, RS, true>(W, h, y, p.rows, p.n, p.cols, j0, lane);
    else gemvb_body<T, R, RB, RS, false>(W, h, y, p.rows, p.n, p.cols, j0, lane);
}

// Batched bf16 with whole 16-byte vectors per row: y[rows, n] = h[rows, cols] * W[n, cols]^T is a
// dense contraction once rows > 1, so it goes to the matrix cores (v_mfma_f32_16x16x32_bf16, fp32
// accumulate).  Still weight-streaming bound up to rows ~ 128: every weight is read once from HBM.
//   - a workgroup owns 16 output columns and one group of 16-row tiles of h; the grid is
//     (column blocks) x (row groups), column block fastest, so that the row groups of one column
//     block land on the same XCD (workgroups go to the 8 XCDs round-robin) and all but the first find
//     the weights in its L2;
//   - its 4 waves split K: of every 8 consecutive 32-wide K-steps wave w takes steps 2w and 2w+1 (128
//     contiguous bytes of each row), 16 steps per 2048 columns;
//   - a fragment (A: lane l holds row l & 15, B: column l & 15; the 8 consecutive k's of chunk l >> 4
//     of a step) read straight from global memory would touch 16 rows x 64 bytes per instruction, all
//     4 KB apart: half cache lines, one cache channel (measured: 0.3 - 1.1 us slower per launch).
//     Instead each wave loads its own K-slices of 16 rows -- a tile of h, or the weights of the 16
//     columns -- row by row (one row = 8 x 128 contiguous bytes per instruction) and transposes them
//     through its private slice of LDS into fragment order.  The weight fragments stay in registers
//     when cols <= 2048 (SINGLE) and are re-read per tile (from cache) otherwise; the next tile's rows
//     of h are in flight while the matrix cores work on this one.  LDS slot (lane of the load) holds 16 rows x 16 bytes and is padded to 272
//     bytes so that 16 consecutive lanes hit all banks.  74 KB of LDS per workgroup: two fit a CU, and
//     one's staging overlaps the other's multiplies;
//   - rows beyond the batch re-read the last row and are never stored;
//   - per tile the 4 waves' partial sums meet in LDS and are added in a fixed order; lane l of a tile
//     holds column (l & 15), rows 4 * (l >> 4) .. + 3.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int kMmSteps = 16;        // K-steps per wave per super-chunk (4 waves x 16 steps x 32 = 2048 columns)
constexpr int kMmSlotBytes = 272;   // 16 rows x 16 B + 16 B of padding
constexpr int kMmWaveLds = 64 * kMmSlotBytes;   // one wave's staging area: one tile, 64 slots
constexpr int kMmMaxRowGroups = 4;
constexpr int kMmWideRows = 81;     // rows from which the 32-column form is used (measured: the 16-column form is faster up to 5 tiles of rows, slower from 6)

// k offset of the 16-byte chunk that lane `l` of wave `wave` loads from a row (super-chunk at step s0);
// the same chunk is fragment step l >> 2, k-chunk l & 3 of that wave.
__device__ __forceinline__ int mm_k0(int s0, int wave, int l) {
    return (s0 + (l >> 3) * 8 + wave * 2 + ((l >> 2) & 1)) * 32 + (l & 3) * 8;
}

// 16 rows of a row-major matrix (a tile of h, or the weights of 16 output columns), this wave's
// K-slices: one row per instruction; rows beyond the matrix repeat its last row
template <bool FULL, bool AL, int NR = 16>
__device__ __forceinline__ void mm_load_rows(const bf16_t* h, int rows, int cols, int r0, int s0, int wave, int lane, unsigned (*g)[4]) {
    const int k0 = mm_k0(s0, wave, lane);
    const int koff = (FULL || k0 < cols) ? k0 : 0;      // an out-of-range chunk is read from column 0 and zeroed on both sides later
#pragma unroll
    for (int r = 0; r < NR; r++) {
        const int R = r0 + r < rows ? r0 + r : rows - 1;
        load_vec_global<bf16_t, AL, false>(h + (size_t)R * cols + koff, g[r]);     // global outright: see load_vec_global
    }
}

// LDS operations of one wave execute in order: these writes cannot overtake the previous tile's reads
template <int NR = 16>
__device__ __forceinline__ void mm_stage(char* lds /* this wave's */, int lane, const unsigned (*g)[4]) {
#pragma unroll
    for (int r = 0; r < NR; r++) {
        v4u t;
        t.x = g[r][0]; t.y = g[r][1]; t.z = g[r][2]; t.w = g[r][3];
        *reinterpret_cast<v4u*>(lds + lane * kMmSlotBytes + r * 16) = t;
    }
}

// fragment (step i, k-chunk lane >> 4, row or column lane & 15) of the tile staged in `lds`
__device__ __forceinline__ void mm_read_frags(const char* lds, int lane, v4u* f) {
#pragma unroll
    for (int i = 0; i < kMmSteps; i++)
        f[i] = *reinterpret_cast<const v4u*>(lds + (i * 4 + (lane >> 4)) * kMmSlotBytes + (lane & 15) * 16);
}
// chunks beyond cols are zeroed on both sides (the loads fetched column 0 in their place): zeroing the
// weight side alone would turn an Inf or NaN of h[:, 0:8] into NaN in every output (0 * Inf)
template <bool FULL>
__device__ __forceinline__ void mm_zero_tail(v4u* b, int cols, int s0, int wave, int kq) {
    if constexpr (!FULL) {
#pragma unroll
        for (int i = 0; i < kMmSteps; i++)      // cols is a multiple of 8: a chunk is all in or all out
            if ((s0 + (i >> 1) * 8 + wave * 2 + (i & 1)) * 32 + kq * 8 >= cols) b[i] = v4u{0u, 0u, 0u, 0u};
    }
}
__device__ __forceinline__ void mm_mfma(const v4u* a, const v4u* b, f32x4& acc) {
#pragma unroll
    for (int i = 0; i < kMmSteps; i++)
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[i]), acc, 0, 0, 0);
}

// What becomes of a finished tile.  All four waves share the output stage: a lane is given NE consecutive
// rows of one column -- begin(r, j, ok) before the partial sums are exchanged (or earlier), put(k, v) for
// each of its sums, end().
// MmStore: the stand-alone kernels -- each sum is rounded and stored.
template <int NE>
struct MmStore {
    static constexpr bool kEarly = false;
    bf16_t* y;
    int rows, n;
    size_t at = 0;
    int r = 0;
    bool col_ok = false;
    __device__ __forceinline__ void prepare() {}
    __device__ __forceinline__ void begin(int r_, int j, bool ok) { r = r_; col_ok = ok; at = (size_t)r_ * n + j; }
    __device__ __forceinline__ void put(int k, float v) { if (col_ok && r + k < rows) store_elem(y + at + (size_t)k * n, v); }
    __device__ __forceinline__ void end() {}
};
// MmEpilogue: the kernels that follow the GEMV in the chain, element for element, ride along (kernels.h,
// GemvEpiArgs): prepare() reads their table out of the kernel arguments and resolves pointer-table slots --
// the bodies call it once their weight loads are on their way, as k_gemv_epilogue does, so that nothing but
// the first 64 bytes of the arguments stands between the start of the kernel and those loads; begin() asks
// for the operands, so that they arrive while the tile is staged and multiplied and the partial sums are
// exchanged; end() plays the kernels on the lane's outputs, rounding to bf16 after each as the stand-alone
// kernels do, with the GELU as the only branch.
// EARLY (the narrow forms, whose few loads leave the operands' latency exposed): begin() comes right behind the
// weight loads and always issues the same number of loads -- an operand that comes from a register slot is
// fetched from the GEMV's own output buffer instead and ignored -- so that every wait on the rows and weights
// knows exactly how many younger loads are outstanding.  Otherwise the loads are conditional, which the compiler
// cannot count (a wait for an older load placed behind them would wait for more than it needs), and begin() comes
// once the rows and weights of the tile have been taken out of their registers, in front of the multiplies.
template <int NE, bool EARLY>
struct MmEpilogue {
    static constexpr bool kEarly = EARLY;
    static constexpr int P = kEpiMaxPhases;
    bf16_t* y;
    int rows, n;
    unsigned head;
    int n_epi;
    const void PG_CONSTANT* ka;   // the kernel-argument segment (a GemvEpiArgs)
    float eps = 0.f;              // the prologue's, read with the table
    const bf16_t* q0[P];        // operand addresses, pointer-table slots resolved; null: comes from a register slot
    const bf16_t* q1[P];
    bf16_t* outs[P];
    unsigned ms[P], metas[P], inds[P];
    bool plain = true;          // EARLY: no operand has a broadcast period
    bool decoder = false;       // the kernels are GELU of the GEMV's result, then one or two adds with an operand from memory
    // per call
    unsigned idx[NE];
    bool ok[NE];
    unsigned ld0[P][NE], ld1[P][NE];
    float v[NE];
    __device__ __forceinline__ void prepare() {
        static_assert(P == 3, "the argument batch names every phase");
        using SlotPtr = const void* const PG_CONSTANT*;
        const void* a0[P];
        const void* a1[P];
        {   // through the segment's address made opaque: otherwise the compiler moves these loads (invariant
            // memory) to the top of the kernel, in front of the weight loads
            const GemvEpiArgs PG_CONSTANT* kp = (const GemvEpiArgs PG_CONSTANT*)ka;
            asm volatile("" : "+s"(kp));
            eps = kp->eps;
#pragma unroll
            for (int i = 0; i < P; i++) {
                a0[i] = kp->ph[i].in0; a1[i] = kp->ph[i].in1; outs[i] = static_cast<bf16_t*>(kp->ph[i].out);
                ms[i] = kp->ph[i].m; metas[i] = kp->ph[i].meta; inds[i] = kp->ph[i].ind;
            }
            asm volatile("" : "+s"(eps),
                              "+s"(a0[0]), "+s"(a1[0]), "+s"(outs[0]), "+s"(ms[0]), "+s"(metas[0]), "+s"(inds[0]),
                              "+s"(a0[1]), "+s"(a1[1]), "+s"(outs[1]), "+s"(ms[1]), "+s"(metas[1]), "+s"(inds[1]),
                              "+s"(a0[2]), "+s"(a1[2]), "+s"(outs[2]), "+s"(ms[2]), "+s"(metas[2]), "+s"(inds[2]));
        }
        bool f0[P], f1[P], s0[P], s1[P];
        unsigned any = 0;
#pragma unroll
        for (int i = 0; i < P; i++) {
            const unsigned mt = metas[i];
            f0[i] = ((mt >> 8) & 0xffu) == kMergeFromMemory;
            f1[i] = (mt & 0xffu) != kGelu && ((mt >> 16) & 0xffu) == kMergeFromMemory;
            s0[i] = f0[i] && (inds[i] & 1u);
            s1[i] = f1[i] && (inds[i] & 2u);
            any |= (f0[i] ? inds[i] & 1u : 0u) | (f1[i] ? inds[i] & 2u : 0u);
        }
        any = __builtin_amdgcn_readfirstlane(any);
        asm volatile("" : "+s"(any));       // keeps what follows behind the weight loads
        {   // the decoder block's tail, recognised here so that end() runs it straight through (see k_gemv_epilogue)
            auto add_of = [](unsigned mt, unsigned q) {
                const unsigned a = (mt >> 8) & 0xffu, b = (mt >> 16) & 0xffu;
                return (mt & 0xffu) == (unsigned)kAdd && ((a == q && b == kMergeFromMemory) || (a == kMergeFromMemory && b == q));
            };
            const unsigned hq = (head >> 8) & 0xffu, d0 = metas[0] >> 24, d1 = metas[1] >> 24;
            decoder = (n_epi == 2 || n_epi == 3) && (metas[0] & 0xffu) == (unsigned)kGelu && ((metas[0] >> 8) & 0xffu) == hq &&
                      add_of(metas[1], d0) && (n_epi == 2 || add_of(metas[2], d1));
        }
        if (any) {                           // some operand is a pointer-table slot: all in one batch, without branches
            auto slot_addr = [&](const void* q, bool is_slot) -> SlotPtr { return is_slot ? (SlotPtr)(uintptr_t)q : (SlotPtr)ka; };
            SlotPtr at0[P], at1[P];
            const void* t0[P];
            const void* t1[P];
#pragma unroll
            for (int i = 0; i < P; i++) { at0[i] = slot_addr(a0[i], s0[i]); at1[i] = slot_addr(a1[i], s1[i]); }
#pragma unroll
            for (int i = 0; i < P; i++) { t0[i] = *at0[i]; t1[i] = *at1[i]; }
            asm volatile("" : "+s"(t0[0]), "+s"(t1[0]), "+s"(t0[1]), "+s"(t1[1]), "+s"(t0[2]), "+s"(t1[2]));
#pragma unroll
            for (int i = 0; i < P; i++) {
                if (s0[i]) a0[i] = t0[i];
                if (s1[i]) a1[i] = t1[i];
            }
        }
        if constexpr (EARLY) {
            const unsigned total = (unsigned)rows * (unsigned)n;
            plain = true;
#pragma unroll
            for (int i = 0; i < P; i++) {
                q0[i] = f0[i] ? static_cast<const bf16_t*>(a0[i]) : y;
                q1[i] = f1[i] ? static_cast<const bf16_t*>(a1[i]) : y;
                ms[i] = f1[i] ? ms[i] : total;
                plain = plain && ms[i] == total;
            }
        } else {
#pragma unroll
            for (int i = 0; i < P; i++) {
                q0[i] = f0[i] ? static_cast<const bf16_t*>(a0[i]) : nullptr;
                q1[i] = f1[i] ? static_cast<const bf16_t*>(a1[i]) : nullptr;
#pragma unroll
                for (int k = 0; k < NE; k++) ld0[i][k] = ld1[i][k] = 0u;
            }
        }
    }
    __device__ __forceinline__ void begin(int r, int j, bool col_ok) {
        const unsigned total = (unsigned)rows * (unsigned)n;
#pragma unroll
        for (int e = 0; e < NE; e++) {
            ok[e] = col_ok && r + e < rows;
            idx[e] = ok[e] ? (unsigned)(r + e) * (unsigned)n + (unsigned)j : 0u;
        }
        if constexpr (EARLY) {
            if (__builtin_expect(plain, 1)) {      // the usual case, one branch for all
#pragma unroll
                for (int i = 0; i < P; i++)
#pragma unroll
                    for (int e = 0; e < NE; e++) {
                        ld0[i][e] = load_raw_global_at(q0[i], idx[e]);
                        ld1[i][e] = load_raw_global_at(q1[i], idx[e]);
                    }
            } else {
#pragma unroll
                for (int i = 0; i < P; i++)
#pragma unroll
                    for (int e = 0; e < NE; e++) {
                        ld0[i][e] = load_raw_global_at(q0[i], idx[e]);
                        ld1[i][e] = load_raw_global_at(q1[i], idx[e] % ms[i]);
                    }
            }
        } else {
#pragma unroll
            for (int i = 0; i < P; i++) {
                if (i < n_epi && q0[i]) {
#pragma unroll
                    for (int e = 0; e < NE; e++) ld0[i][e] = load_raw_global_at(q0[i], idx[e]);
                }
                if (i < n_epi && q1[i]) {
                    const unsigned m = ms[i];
#pragma unroll
                    for (int e = 0; e < NE; e++) ld1[i][e] = load_raw_global_at(q1[i], m == total ? idx[e] : idx[e] % m);
                }
            }
        }
    }
    __device__ __forceinline__ void put(int e, float sum) { v[e] = sum; }
    __device__ __forceinline__ void end() {
        unsigned bits[NE];
        float slot[kMergeSlots][NE];
        __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0): every operand, before the first store (see k_gemv_epilogue)
#pragma unroll
        for (int e = 0; e < NE; e++) {
            bits[e] = f32_to_bf16(v[e]);
            if (ok[e] && (head & kEpiHeadStore)) *(unsigned short PG_GLOBAL*)(uintptr_t)(y + idx[e]) = (unsigned short)bits[e];
        }
        if (__builtin_expect(decoder, 1)) {
            // the same kernels with the same arithmetic and roundings, operands known: GELU of the GEMV's rounded result,
            // then each add takes the value before it and its operand from memory, in the order its descriptor names
            const bool mf1 = ((metas[1] >> 8) & 0xffu) == kMergeFromMemory, mf2 = ((metas[2] >> 8) & 0xffu) == kMergeFromMemory;
#pragma unroll
            for (int e = 0; e < NE; e++) {
                float val = ew_apply<kGelu, false>(from_raw<bf16_t>(bits[e]), 0.f);
                unsigned b = f32_to_bf16(val);
                if (ok[e] && (inds[0] & kEpiStore)) *(unsigned short PG_GLOBAL*)(uintptr_t)(outs[0] + idx[e]) = (unsigned short)b;
                val = from_raw<bf16_t>(b);
                {
                    const float fa = mf1 ? from_raw<bf16_t>(ld0[1][e]) : val, fb = mf1 ? val : from_raw<bf16_t>(ld1[1][e]);
                    b = f32_to_bf16(ew_apply<kAdd, false>(fa, fb));
                    if (ok[e] && (inds[1] & kEpiStore)) *(unsigned short PG_GLOBAL*)(uintptr_t)(outs[1] + idx[e]) = (unsigned short)b;
                    val = from_raw<bf16_t>(b);
                }
                if (n_epi == 3) {
                    const float fa = mf2 ? from_raw<bf16_t>(ld0[2][e]) : val, fb = mf2 ? val : from_raw<bf16_t>(ld1[2][e]);
                    b = f32_to_bf16(ew_apply<kAdd, false>(fa, fb));
                    if (ok[e] && (inds[2] & kEpiStore)) *(unsigned short PG_GLOBAL*)(uintptr_t)(outs[2] + idx[e]) = (unsigned short)b;
                }
            }
            return;
        }
        {
            const unsigned dst = (head >> 8) & 0xffu;
#pragma unroll
            for (int q = 0; q < kMergeSlots; q++)
#pragma unroll
                for (int e = 0; e < NE; e++) slot[q][e] = dst == (unsigned)q ? from_raw<bf16_t>(bits[e]) : 0.f;
        }
#pragma unroll
        for (int i = 0; i < P; i++) {
            if (i >= n_epi) break;
            const unsigned mt = metas[i], ind = inds[i];
            const unsigned op = mt & 0xffu, src0 = (mt >> 8) & 0xffu, src1 = (mt >> 16) & 0xffu, dst = mt >> 24;
            float fa[NE], fb[NE], fo[NE];
#pragma unroll
            for (int e = 0; e < NE; e++) {
                fa[e] = from_raw<bf16_t>(ld0[i][e]);
                fb[e] = from_raw<bf16_t>(ld1[i][e]);
#pragma unroll
                for (int q = 0; q < kMergeSlots; q++) {
                    if (src0 == (unsigned)q) fa[e] = slot[q][e];
                    if (src1 == (unsigned)q) fb[e] = slot[q][e];
                }
            }
            if (op == kGelu) {
#pragma unroll
                for (int e = 0; e < NE; e++) fo[e] = ew_apply<kGelu, false>(fa[e], 0.f);
            } else {
#pragma unroll
                for (int e = 0; e < NE; e++) {
                    const float sum = ew_apply<kAdd, false>(fa[e], fb[e]), prod = ew_apply<kMul, false>(fa[e], fb[e]);
                    fo[e] = op == kAdd ? sum : prod;
                }
            }
#pragma unroll
            for (int e = 0; e < NE; e++) {
                bits[e] = f32_to_bf16(fo[e]);
                if (ok[e] && (ind & kEpiStore)) *(unsigned short PG_GLOBAL*)(uintptr_t)(outs[i] + idx[e]) = (unsigned short)bits[e];
#pragma unroll
                for (int q = 0; q < kMergeSlots; q++)
                    if (dst == (unsigned)q) slot[q][e] = from_raw<bf16_t>(bits[e]);
            }
        }
    }
};

// where the output stage of the 16-column forms puts a lane: wave w takes row w of the four that an
// accumulator lane holds
template <int NC = 16, class Emit>
__device__ __forceinline__ void mm_emit_begin(Emit& emit, int n, int r0, int j0, int wave, int lane) {
    emit.begin(r0 + (lane >> 4) * 4 + wave, j0 + (lane & 15), j0 + (lane & 15) < n && (NC == 16 || (lane & 15) < NC));
}
// sum the 4 waves' partial tiles in a fixed order and hand rows r0 .. r0 + 15 of the 16 columns at j0 to `emit`
// (mm_emit_begin has been called for this tile)
template <class Emit>
__device__ __forceinline__ void mm_reduce_store(float* red, f32x4 acc, Emit& emit, int wave, int lane) {
    // A matrix-core result may not be read by an LDS write until the instruction has drained (up to
    // 19 wait states for the longest forms).  The compiler inserts those itself inside a block, but
    // it was seen to omit them when the last multiply of a K loop and this write sit in different
    // blocks (loop exit): the write then stored a stale accumulator.  32 idle cycles, tied to `acc`
    // so that they stay between the two, make it independent of that.
    asm volatile("s_nop 15\n\ts_nop 15" : "+v"(acc));
    float* dst = red + ((size_t)wave * 64 + lane) * 4;
    dst[0] = acc.x; dst[1] = acc.y; dst[2] = acc.z; dst[3] = acc.w;
    __syncthreads();
    {
        const int e = wave;
        const float p0 = red[((size_t)0 * 64 + lane) * 4 + e], p1 = red[((size_t)1 * 64 + lane) * 4 + e];
        const float p2 = red[((size_t)2 * 64 + lane) * 4 + e], p3 = red[((size_t)3 * 64 + lane) * 4 + e];
        emit.put(0, ((p0 + p1) + p2) + p3);
    }
    __syncthreads();      // `red` is free again
    emit.end();
}

// mm_rmsnorm_rows is defined with the narrow form below
template <int NRH>
__device__ __forceinline__ void mm_rmsnorm_rows(unsigned (*g)[4], const unsigned* wg, float eps, bf16_t* hstore, int rows, int wave, int lane, float* scratch);

// PRO (SINGLE, FULL, one tile of rows per workgroup -- rows < kMmWideRows): h points at the rows to normalise,
// the workgroups of column block 0 store the normalised rows to hstore (see mm_rmsnorm_rows).
template <bool FULL, bool SINGLE, bool AL, bool PRO = false, class Emit>
__device__ __forceinline__ void gemm_mfma_body(const bf16_t* W, const bf16_t* h, Emit& emit, int rows, int n, int cols, int row_groups,
                                               char* stage /* LDS: 4 x kMmWaveLds */, float* red /* LDS: [4 waves][64 lanes][4] */,
                                               const bf16_t* gain = nullptr, const float& eps = 0.f /* read by emit.prepare() */, bf16_t* hstore = nullptr) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kq = lane >> 4;
    const int ncb = (n + 15) / 16;
    const int cb = blockIdx.x % ncb, rg = blockIdx.x / ncb;
    const int ntiles = (rows + 15) / 16, per = (ntiles + row_groups - 1) / row_groups;
    const int t0 = rg * per, t1 = (t0 + per < ntiles) ? t0 + per : ntiles;
    if (t0 >= t1) return;                                  // whole workgroup: nothing waits on it
    const int j0 = cb * 16;
    char* lds = stage + wave * kMmWaveLds;
    unsigned g[16][4], gw[16][4];
    v4u a[kMmSteps], b[kMmSteps];
    if constexpr (SINGLE) {
        // The h rows (from L2) are asked for before the weights (from HBM): loads return in order, so
        // the tile is staged and its fragments are back in registers while the weights are still on
        // their way; then the same LDS slice takes the weights.  The weight fragments stay in registers
        // for all tiles of the workgroup, and a later tile's rows are in flight across the multiplies
        // of the one before.
        mm_load_rows<FULL, AL>(h, rows, cols, t0 * 16, 0, wave, lane, g);
        unsigned wg[4] = {0u, 0u, 0u, 0u};
        if constexpr (PRO) load_vec_global<bf16_t, AL, false>(gain + mm_k0(0, wave, lane), wg);   // before the weights: loads come back in order
        mm_load_rows<FULL, AL>(W, n, cols, j0, 0, wave, lane, gw);
        emit.prepare();                                      // the epilogue's table right behind the weight loads
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        if constexpr (PRO) {
            static_assert(FULL && SINGLE, "the prologue exists for rows of 2048 columns");
            bf16_t* tile_store = (hstore && cb == 0) ? hstore + (size_t)t0 * 16 * (32 * 4 * kMmSteps) : nullptr;
            mm_rmsnorm_rows<16>(g, wg, eps, tile_store, rows - t0 * 16, wave, lane, reinterpret_cast<float*>(stage));
            lds_barrier();        // the sums are read: the staging area takes the rows now
        }
        mm_stage(lds, lane, g);
        mm_read_frags(lds, lane, a);
        mm_zero_tail<FULL>(a, cols, 0, wave, kq);
        if (t1 - t0 > 1) mm_load_rows<FULL, AL>(h, rows, cols, (t0 + 1) * 16, 0, wave, lane, g);
        mm_stage(lds, lane, gw);
        mm_read_frags(lds, lane, b);
        mm_zero_tail<FULL>(b, cols, 0, wave, kq);
        __builtin_amdgcn_sched_barrier(0);   // all fragment reads before the first multiply, not one LDS latency per pair
        mm_emit_begin(emit, n, t0 * 16, j0, wave, lane);
        mm_mfma(a, b, acc);
        mm_reduce_store(red, acc, emit, wave, lane);
#pragma unroll 1
        for (int t = t0 + 1; t < t1; t++) {
            acc = f32x4{0.f, 0.f, 0.f, 0.f};
            mm_stage(lds, lane, g);
            if (t + 1 < t1) mm_load_rows<FULL, AL>(h, rows, cols, (t + 1) * 16, 0, wave, lane, g);
            mm_read_frags(lds, lane, a);
            mm_zero_tail<FULL>(a, cols, 0, wave, kq);
            __builtin_amdgcn_sched_barrier(0);
            mm_emit_begin(emit, n, t * 16, j0, wave, lane);
            mm_mfma(a, b, acc);
            mm_reduce_store(red, acc, emit, wave, lane);
        }
    } else {
        emit.prepare();
#pragma unroll 1
        for (int t = t0; t < t1; t++) {
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
            for (int s0 = 0; s0 * 32 < cols; s0 += 4 * kMmSteps) {
                mm_load_rows<FULL, AL>(h, rows, cols, t * 16, s0, wave, lane, g);
                mm_load_rows<FULL, AL>(W, n, cols, j0, s0, wave, lane, gw);
                mm_stage(lds, lane, g);
                mm_read_frags(lds, lane, a);
                mm_zero_tail<FULL>(a, cols, s0, wave, kq);
                mm_stage(lds, lane, gw);
                mm_read_frags(lds, lane, b);
                mm_zero_tail<FULL>(b, cols, s0, wave, kq);
                __builtin_amdgcn_sched_barrier(0);
                mm_mfma(a, b, acc);
            }
            mm_emit_begin(emit, n, t * 16, j0, wave, lane);
            mm_reduce_store(red, acc, emit, wave, lane);
        }
    }
}

// Narrow form for one tile of rows (rows <= 16) and cols <= 2048: 8 output columns per workgroup, so
// that 2048 columns make 256 workgroups and every CU pulls weights (a loads-only kernel takes in the
// same bytes 0.35 us faster from 256 CUs than from 128); half of each multiply is idle, which costs
// nothing here.  Only the 8 weight rows are loaded and staged: fragment columns 8-15 are whatever the
// slot held before and their results are never stored.  NRH = 8 (4) when rows <= 8 (4): the absent
// rows of the tile are not loaded either.  With two tiles of rows (8 columns x 2 tiles = 512
// workgroups, measured) it loses to the 16-column form: 5.7 against 4.9 us at 32 rows.
// RMSNorm of the rows the narrow form has just loaded, as a prologue (FULL, 2048 columns): lane (wave, l)
// holds 16-byte chunk c of every row, where c runs over all 256 chunks of a row across the workgroup, but
// not in lane order.  The stand-alone kernel's sums must be reproduced bit for bit: per chunk the fused
// sum of squares in element order (any lane can do that); then the stand-alone kernel's reduction, which
// is a tree of fixed shape over the chunk sums in chunk order -- wave_sum adds neighbours, then pairs of
// pairs, of quads, of eights (a floating-point add does not care which operand is which), then the four
// sixteens in order, and the four wave sums in order.  Here the chunk sums go to LDS in chunk order and
// the workgroup's 16 * NRH subtrees of sixteen leaves are spread over its lanes, one each; lane r < NRH
// then finishes row r (four sixteens per wave sum, four wave sums) and turns the total into the row's
// scale; every lane scales its own chunks: (x * scale) * gain, one rounding.  `scratch`: NRH * 336 + NRH
// floats of LDS that nothing else uses until the rows are staged.  hstore: this workgroup also stores the rows.
template <int NRH>
__device__ __forceinline__ void mm_rmsnorm_rows(unsigned (*g)[4], const unsigned* wg /* the lane's chunk of the gain */, float eps, bf16_t* hstore,
                                                int rows, int wave, int lane, float* scratch) {
    constexpr int kCols = 32 * 4 * kMmSteps;
    constexpr int kRow = 256 + 64;             // a row of chunk sums, 8 floats of padding after every 32: the lanes of a wave hold
                                               // chunks 32 apart, which would otherwise all fall into the same eight banks
    const int tid = wave * 64 + lane;
    const int k0 = mm_k0(0, wave, lane);
    float* sq = scratch;                       // [NRH][kRow]: chunk sums in chunk order
    float* six = scratch + NRH * kRow;         // [NRH][16]: sums of sixteen chunks
    float* scale = six + NRH * 16;             // [NRH]
    auto at = [](int c) { return c + 8 * (c >> 5); };
    float fx[NRH][8];
#pragma unroll
    for (int r = 0; r < NRH; r++) {
        Vec<bf16_t, 16>::unpack(g[r], fx[r]);
        float acc = 0.f;
#pragma unroll
        for (int e = 0; e < 8; e++) acc = __builtin_fmaf(fx[r][e], fx[r][e], acc);
        sq[r * kRow + at(k0 >> 3)] = acc;
    }
    lds_barrier();
    if (tid < 16 * NRH) {                      // subtree tid: row tid / 16, chunks 16 * (tid % 16) .. + 15
        const f32x4* leaf = reinterpret_cast<const f32x4*>(sq + (tid >> 4) * kRow + at((tid & 15) * 16));
        const f32x4 l0 = leaf[0], l1 = leaf[1], l2 = leaf[2], l3 = leaf[3];
        const float q0 = (l0.x + l0.y) + (l0.z + l0.w), q1 = (l1.x + l1.y) + (l1.z + l1.w);
        const float q2 = (l2.x + l2.y) + (l2.z + l2.w), q3 = (l3.x + l3.y) + (l3.z + l3.w);
        six[tid] = (q0 + q1) + (q2 + q3);
    }
    lds_barrier();
    if (tid < NRH) {
        const f32x4* sx = reinterpret_cast<const f32x4*>(six + tid * 16);
        float wsum[4];
#pragma unroll
        for (int w = 0; w < 4; w++) wsum[w] = ((sx[w].x + sx[w].y) + sx[w].z) + sx[w].w;
        const float total = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
        scale[tid] = 1.0f / sqrtf(total / (float)kCols + eps);
    }
    lds_barrier();
    float fg[8];
    Vec<bf16_t, 16>::unpack(wg, fg);
#pragma unroll
    for (int r = 0; r < NRH; r++) {
        float fo[8];
        const float sc = scale[r];
#pragma unroll
        for (int e = 0; e < 8; e++) fo[e] = (fx[r][e] * sc) * fg[e];
        Vec<bf16_t, 16>::pack(fo, g[r]);
    }
    if (hstore) {
#pragma unroll
        for (int r = 0; r < NRH; r++)
            if (r < rows) store_vec_global(hstore + (size_t)r * kCols + k0, g[r]);
    }
}

template <bool FULL, bool AL, int NRH, bool PRO = false, class Emit>
__device__ __forceinline__ void gemm_mfma_narrow_body(const bf16_t* W, const bf16_t* h, Emit& emit, int rows, int n, int cols,
                                                      char* stage, float* red, const bf16_t* gain = nullptr, const float& eps = 0.f /* read by emit.prepare() */,
                                                      bf16_t* hstore = nullptr) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int kq = lane >> 4;
    const int j0 = blockIdx.x * 8, r0 = 0;
    char* lds = stage + wave * kMmWaveLds;
    unsigned g[NRH][4], gw[8][4];
    v4u a[kMmSteps], b[kMmSteps];
    mm_load_rows<FULL, AL, NRH>(h, rows, cols, r0, 0, wave, lane, g);      // with a prologue: the rows to normalise
    unsigned wg[4] = {0u, 0u, 0u, 0u};
    if constexpr (PRO) load_vec_global<bf16_t, AL, false>(gain + mm_k0(0, wave, lane), wg);   // before the weights: loads come back in order
    mm_load_rows<FULL, AL, 8>(W, n, cols, j0, 0, wave, lane, gw);
    emit.prepare();                                          // the epilogue's table right behind the weight loads
    if constexpr (Emit::kEarly) mm_emit_begin<8>(emit, n, r0, j0, wave, lane);
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if constexpr (PRO) {
        static_assert(FULL, "the prologue exists for rows of 2048 columns");
        static_assert((NRH * 336 + NRH) * sizeof(float) <= 4 * kMmWaveLds, "the prologue's sums fit the staging area");
        mm_rmsnorm_rows<NRH>(g, wg, eps, hstore, rows, wave, lane, reinterpret_cast<float*>(stage));
        lds_barrier();        // the sums are read: the staging area takes the rows now
    }
    mm_stage<NRH>(lds, lane, g);
    mm_read_frags(lds, lane, a);
    mm_zero_tail<FULL>(a, cols, 0, wave, kq);
    mm_stage<8>(lds, lane, gw);
    mm_read_frags(lds, lane, b);
    mm_zero_tail<FULL>(b, cols, 0, wave, kq);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (!Emit::kEarly) mm_emit_begin<8>(emit, n, r0, j0, wave, lane);
    mm_mfma(a, b, acc);
    mm_reduce_store(red, acc, emit, wave, lane);
}

template <int IND, bool FULL, int NRH>
__global__ __launch_bounds__(kBlock, 2) void k_gemm_mfma_bf16_narrow(GemvArgs p) {
    const bf16_t* W = static_cast<const bf16_t*>(resolve<(IND & 1) != 0>(p.W));
    const bf16_t* h = static_cast<const bf16_t*>(resolve<(IND & 2) != 0>(p.h));
    bf16_t* y = static_cast<bf16_t*>(p.out);
    MmStore<1> emit{y, p.rows, p.n};
    __shared__ __attribute__((aligned(16))) char stage[4 * kMmWaveLds];
    __shared__ float red[4 * 64 * 4];
    const bool al = aligned_to(W, 16) && aligned_to(h, 16);
    if (__builtin_expect(al, 1)) gemm_mfma_narrow_body<FULL, true, NRH>(W, h, emit, p.rows, p.n, p.cols, stage, red);
    else gemm_mfma_narrow_body<FULL, false, NRH>(W, h, emit, p.rows, p.n, p.cols, stage, red);
}

// Wide form for many rows and cols == 2048: 32 output columns per workgroup, i.e. two sets of weight
// fragments and two accumulators against every staged tile of h, which halves the h traffic per
// output (the bound once there are many rows).  One workgroup per CU (the fragments of 32 columns do not fit
// the register budget of two), waves 0 and 1 each finish one 16-column half.
template <bool AL, class Emit>
__device__ __forceinline__ void gemm_mfma_wide_body(const bf16_t* W, const bf16_t* h, Emit& emit, int rows, int n, int cols, int row_groups,
                                                    char* stage, float* red /* LDS: [2 halves][4 waves][64 lanes][4] */) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ncb = (n + 31) / 32;
    const int cb = blockIdx.x % ncb, rg = blockIdx.x / ncb;
    const int ntiles = (rows + 15) / 16, per = (ntiles + row_groups - 1) / row_groups;
    const int t0 = rg * per, t1 = (t0 + per < ntiles) ? t0 + per : ntiles;
    if (t0 >= t1) return;
    const int j0 = cb * 32;
    char* lds = stage + wave * kMmWaveLds;
    unsigned g[16][4], gw0[16][4], gw1[16][4];
    v4u a[kMmSteps], b0[kMmSteps], b1[kMmSteps];
    mm_load_rows<true, AL>(h, rows, cols, t0 * 16, 0, wave, lane, g);
    mm_load_rows<true, AL>(W, n, cols, j0, 0, wave, lane, gw0);
    mm_load_rows<true, AL>(W, n, cols, j0 + 16, 0, wave, lane, gw1);
    emit.prepare();      // the epilogue's table right behind the weight loads
    mm_stage(lds, lane, g);
    mm_read_frags(lds, lane, a);
    if (t1 - t0 > 1) mm_load_rows<true, AL>(h, rows, cols, (t0 + 1) * 16, 0, wave, lane, g);
    mm_stage(lds, lane, gw0);
    mm_read_frags(lds, lane, b0);
    mm_stage(lds, lane, gw1);
    mm_read_frags(lds, lane, b1);
    for (int t = t0;;) {
        f32x4 acc0 = {0.f, 0.f, 0.f, 0.f}, acc1 = {0.f, 0.f, 0.f, 0.f};
        __builtin_amdgcn_sched_barrier(0);
        // output stage: wave w finishes rows 2 * (w >> 1), + 1 of each accumulator lane's four, in 16-column half w & 1
        emit.begin(t * 16 + (lane >> 4) * 4 + (wave >> 1) * 2, j0 + (wave & 1) * 16 + (lane & 15), j0 + (wave & 1) * 16 + (lane & 15) < n);
#pragma unroll
        for (int i = 0; i < kMmSteps; i++) {
            acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b0[i]), acc0, 0, 0, 0);
            acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b1[i]), acc1, 0, 0, 0);
        }
        asm volatile("s_nop 15\n\ts_nop 15" : "+v"(acc0), "+v"(acc1));   // see mm_reduce_store
        float* d0 = red + ((size_t)(0 * 4 + wave) * 64 + lane) * 4;
        float* d1 = red + ((size_t)(1 * 4 + wave) * 64 + lane) * 4;
        d0[0] = acc0.x; d0[1] = acc0.y; d0[2] = acc0.z; d0[3] = acc0.w;
        d1[0] = acc1.x; d1[1] = acc1.y; d1[2] = acc1.z; d1[3] = acc1.w;
        __syncthreads();
        {
            const float* src = red + (size_t)(wave & 1) * 4 * 64 * 4;
#pragma unroll
            for (int k = 0; k < 2; k++) {
                const int e = (wave >> 1) * 2 + k;
                const float p0 = src[((size_t)0 * 64 + lane) * 4 + e], p1 = src[((size_t)1 * 64 + lane) * 4 + e];
                const float p2 = src[((size_t)2 * 64 + lane) * 4 + e], p3 = src[((size_t)3 * 64 + lane) * 4 + e];
                emit.put(k, ((p0 + p1) + p2) + p3);
            }
        }
        __syncthreads();
        emit.end();
        if (++t >= t1) break;
        mm_stage(lds, lane, g);
        if (t + 1 < t1) mm_load_rows<true, AL>(h, rows, cols, (t + 1) * 16, 0, wave, lane, g);
        mm_read_frags(lds, lane, a);
    }
}

template <int IND>
__global__ __launch_bounds__(kBlock, 1) void k_gemm_mfma_bf16_wide(GemvArgs p) {
    const bf16_t* W = static_cast<const bf16_t*>(resolve<(IND & 1) != 0>(p.W));
    const bf16_t* h = static_cast<const bf16_t*>(resolve<(IND & 2) != 0>(p.h));
    bf16_t* y = static_cast<bf16_t*>(p.out);
    MmStore<2> emit{y, p.rows, p.n};
    __shared__ __attribute__((aligned(16))) char stage[4 * kMmWaveLds];
    __shared__ float red[2 * 4 * 64 * 4];
    const bool al = aligned_to(W, 16) && aligned_to(h, 16);
    if (__builtin_expect(al, 1)) gemm_mfma_wide_body<true>(W, h, emit, p.rows, p.n, p.cols, p.row_groups, stage, red);
    else gemm_mfma_wide_body<false>(W, h, emit, p.rows, p.n, p.cols, p.row_groups, stage, red);
}

template <int IND, bool FULL, bool SINGLE>
__global__ __launch_bounds__(kBlock, 2) void k_gemm_mfma_bf16(GemvArgs p) {
    const bf16_t* W = static_cast<const bf16_t*>(resolve<(IND & 1) != 0>(p.W));
    const bf16_t* h = static_cast<const bf16_t*>(resolve<(IND & 2) != 0>(p.h));
    bf16_t* y = static_cast<bf16_t*>(p.out);
    MmStore<1> emit{y, p.rows, p.n};
    __shared__ __attribute__((aligned(16))) char stage[4 * kMmWaveLds];
    __shared__ float red[4 * 64 * 4];
    const bool al = aligned_to(W, 16) && aligned_to(h, 16);   // rows keep the alignment: cols is a multiple of 8
    if (__builtin_expect(al, 1)) gemm_mfma_body<FULL, SINGLE, true>(W, h, emit, p.rows, p.n, p.cols, p.row_groups, stage, red);
    else gemm_mfma_body<FULL, SINGLE, false>(W, h, emit, p.rows, p.n, p.cols, p.row_groups, stage, red);
}

// The matrix-core forms with an elementwise epilogue (kernels.h, GemvEpiArgs; no prologue): the same bodies,
// with MmEpilogue in place of the plain store.  Only for rows of 2048 columns.  FORM 0: narrow, 8 rows of h
// loaded; 1: narrow, 16; 2: 16 columns per workgroup, one pass over K; 3: wide.
template <int FORM, bool PRO = false>
__global__ __launch_bounds__(kBlock, (FORM == 3 || PRO) ? 1 : 2) void k_gemm_mfma_epilogue(GemvEpiArgs p) {
    static_assert(!PRO || FORM <= 2, "a prologue exists for the forms with one tile of rows per workgroup");
    // As in k_gemv_epilogue: the first 64 bytes of the arguments hold everything that is needed before the
    // loads of h and the weights can go out, and only those are waited for here, in one batch of scalar loads;
    // the epilogue's table and eps are read once the weights are on their way (MmEpilogue::prepare).
    static_assert(offsetof(GemvEpiArgs, gain) + sizeof(void*) == 64, "what the kernel needs first sits in the first 64 bytes");
    const void* Wa = p.g.W;
    const void* ha = p.g.h;
    bf16_t* y = static_cast<bf16_t*>(p.g.out);
    int rows = p.g.rows, n = p.g.n, cols = p.g.cols, row_groups = p.g.row_groups;
    unsigned head = p.head;
    int n_epi = p.n_epi;
    const void* xa = p.x;
    const void* ga = p.gain;
    asm volatile("" : "+s"(Wa), "+s"(ha), "+s"(y), "+s"(rows), "+s"(n), "+s"(cols), "+s"(row_groups), "+s"(head), "+s"(n_epi), "+s"(xa), "+s"(ga));
    const void PG_CONSTANT* const ka = (const void PG_CONSTANT*)__builtin_amdgcn_kernarg_segment_ptr();   // a readable address for a load whose result is not used
    using SlotPtr = const void* const PG_CONSTANT*;
    auto slot_addr = [&](const void* q, bool is_slot) -> SlotPtr { return is_slot ? (SlotPtr)(uintptr_t)q : (SlotPtr)ka; };
    // with a prologue the GEMV's input is computed from x and the gain; p.g.h is where the normalised rows are stored
    if (head & (1u | (PRO ? kEpiXSlot | kEpiGainSlot : 2u))) {      // some operand is a pointer-table slot: all in one batch, without branches
        const bool sw = head & 1u, sh = head & (PRO ? kEpiXSlot : 2u), sg = PRO && (head & kEpiGainSlot);
        SlotPtr aw = slot_addr(Wa, sw), ah = slot_addr(PRO ? xa : ha, sh), ag = slot_addr(ga, sg);
        const void* tw = *aw;
        const void* th = *ah;
        const void* tg = PRO ? *ag : nullptr;
        asm volatile("" : "+s"(tw), "+s"(th), "+s"(tg));
        if (sw) Wa = tw;
        if (sh) { if (PRO) xa = th; else ha = th; }
        if (sg) ga = tg;
    }
    const bf16_t* W = static_cast<const bf16_t*>(Wa);
    const bf16_t* h = static_cast<const bf16_t*>(PRO ? xa : ha);
    const bf16_t* gain = PRO ? static_cast<const bf16_t*>(ga) : nullptr;
    // the narrow forms have one workgroup per column block: the first stores; the 16-column form picks its column block 0 itself
    bf16_t* hstore = (PRO && (head & kEpiStoreH) && (FORM == 2 || blockIdx.x == 0)) ? static_cast<bf16_t*>(const_cast<void*>(ha)) : nullptr;
    __shared__ __attribute__((aligned(16))) char stage[4 * kMmWaveLds];
    __shared__ float red[(FORM == 3 ? 2 : 1) * 4 * 64 * 4];
    MmEpilogue<FORM == 3 ? 2 : 1, FORM <= 1> emit;
    emit.y = y; emit.rows = rows; emit.n = n; emit.head = head; emit.n_epi = n_epi; emit.ka = ka;
    const bool al = aligned_to(W, 16) && aligned_to(h, 16) && (!PRO || aligned_to(gain, 16));
    if constexpr (FORM == 0) {
        if (__builtin_expect(al, 1)) gemm_mfma_narrow_body<true, true, 8, PRO>(W, h, emit, rows, n, cols, stage, red, gain, emit.eps, hstore);
        else gemm_mfma_narrow_body<true, false, 8, PRO>(W, h, emit, rows, n, cols, stage, red, gain, emit.eps, hstore);
    } else if constexpr (FORM == 1) {
        if (__builtin_expect(al, 1)) gemm_mfma_narrow_body<true, true, 16, PRO>(W, h, emit, rows, n, cols, stage, red, gain, emit.eps, hstore);
        else gemm_mfma_narrow_body<true, false, 16, PRO>(W, h, emit, rows, n, cols, stage, red, gain, emit.eps, hstore);
    } else if constexpr (FORM == 2) {
        if (__builtin_expect(al, 1)) gemm_mfma_body<true, true, true, PRO>(W, h, emit, rows, n, cols, row_groups, stage, red, gain, emit.eps, hstore);
        else gemm_mfma_body<true, true, false, PRO>(W, h, emit, rows, n, cols, row_groups, stage, red, gain, emit.eps, hstore);
    } else {
        if (__builtin_expect(al, 1)) gemm_mfma_wide_body<true>(W, h, emit, rows, n, cols, row_groups, stage, red);
        else gemm_mfma_wide_body<false>(W, h, emit, rows, n, cols, row_groups, stage, red);
    }
}

// ---- merged dispatches ------------------------------------------------------------------------------
// Same arithmetic as the stand-alone kernels, element for element: ew_apply for add / mul / GELU;
// RMSNorm as rms_body does it for a row of exactly one vector per lane (fused multiply-add sum of
// squares in element order, wave_sum, the four wave sums added in a fixed order through LDS,
// 1 / sqrt(mean + eps), (x * scale) * gain); one rounding to the storage type per kernel (pack), and
// what a later kernel of the run is handed in registers is exactly the stored bits.
// One workgroup per unit, straight-line: all operand fetches of the run first (unrolled: their registers
// need static indices; a lane beyond the tensor re-reads the last vector and never stores, so there is
// no per-lane branch and all fetches are in flight together), then ONE copy of the arithmetic in a loop
// over the kernels that picks its operands out of the fetched vectors and the register slots with
// conditional moves (one copy of the GELU and of the RMSNorm reduction for up to four kernels; an
// unrolled form with every operand choice resolved at run time by branches was slower: a taken branch
// costs a one-wave-per-SIMD kernel about as much as a dozen arithmetic instructions).

template <typename T, int VB, bool AL>
__device__ __forceinline__ void merged_body(const MergedArgs& p, const T* const* in0, const T* const* in1, float* part) {
    using V = Vec<T, VB>;
    constexpr int NV = V::NV, NW = VB / 4;
    auto fetch = [](const T* q, unsigned* w) {
        if constexpr (VB == 16) load_vec_global<T, AL>(q, w);
        else load_vec4_global<T, AL>(q, w);
    };
    constexpr bool kWide = sizeof(T) == 4;
    constexpr int P = kMergeMaxPhases;
    const unsigned tid = threadIdx.x;
    // the run's table, once, in scalar registers (read inside the loop below it would be indexed memory)
    T* outs[P];
    unsigned metas[P], inds[P];
    float epss[P];
#pragma unroll
    for (int i = 0; i < P; i++) {
        outs[i] = static_cast<T*>(p.ph[i].out);
        metas[i] = p.ph[i].meta;
        inds[i] = p.ph[i].ind;
        epss[i] = p.ph[i].eps;
    }
    const unsigned n = p.n, nvec = n / NV;
    const unsigned v = blockIdx.x * kBlock + tid;
    const bool act = v < nvec;
    const unsigned i0 = (act ? v : nvec - 1) * NV;
    unsigned ld0[P][NW], ld1[P][NW];
#pragma unroll
    for (int i = 0; i < P; i++) {
        const unsigned mt = metas[i], op = mt & 0xffu;
        if (((mt >> 8) & 0xffu) == kMergeFromMemory) {
            fetch(in0[i] + i0, ld0[i]);
        } else {
#pragma unroll
            for (int k = 0; k < NW; k++) ld0[i][k] = 0u;
        }
        if (op != kGelu && ((mt >> 16) & 0xffu) == kMergeFromMemory) {
            const unsigned m = p.ph[i].m;
            if (op == kRmsNorm || m % NV == 0) {
                // RMSNorm: a row is one unit, lane t holds vector t of the gain; add / mul: a vector of b never wraps around the period
                fetch(in1[i] + (op == kRmsNorm ? tid * NV : (m == n ? i0 : i0 % m)), ld1[i]);
            } else {
#pragma unroll
                for (int k = 0; k < NW; k++) ld1[i][k] = 0u;
#pragma unroll
                for (int e = 0; e < NV; e++) {                     // the raw bits, element by element
                    const unsigned r = load_raw_global(in1[i] + (i0 + e) % m);
                    if constexpr (sizeof(T) == 4) ld1[i][e] = r;
                    else ld1[i][e / 2] |= r << (16 * (e & 1));
                }
            }
        } else {
#pragma unroll
            for (int k = 0; k < NW; k++) ld1[i][k] = 0u;
        }
    }
    unsigned slot[kMergeSlots][NW];
#pragma unroll
    for (int q = 0; q < kMergeSlots; q++)
#pragma unroll
        for (int k = 0; k < NW; k++) slot[q][k] = 0u;
    const int n_phase = p.n_phase;
    // All fetches have been asked for together; wait for them here, once.  Left to the compiler, the wait
    // sits at the head of the loop below and then also waits, every time round, for the store of the
    // kernel before (loads and stores of a wave share one counter): a microsecond per kernel.
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
    {   // A chain -- every kernel takes the result of the one before it (the first: memory) and, if it has a second
        // operand, takes that from memory; no RMSNorm -- is played straight through: the choice of the operation is
        // the only thing left to decide per kernel (the operand, slot and table selection of the general loop below
        // and its taken branches cost a one-wave-per-SIMD kernel more than the arithmetic).  Same operations, same
        // order, same roundings.
        bool chain = n_phase >= 1;
        unsigned prev = kMergeFromMemory;
#pragma unroll
        for (int i = 0; i < P; i++) {
            const unsigned mt = metas[i], op = mt & 0xffu;
            const bool in = i < n_phase;
            chain = chain && (!in || (op != (unsigned)kRmsNorm && ((mt >> 8) & 0xffu) == prev && (op == (unsigned)kGelu || ((mt >> 16) & 0xffu) == kMergeFromMemory)));
            prev = mt >> 24;
        }
        if (chain) {
            unsigned w[NW];
#pragma unroll
            for (int k = 0; k < NW; k++) w[k] = ld0[0][k];
#pragma unroll
            for (int i = 0; i < P; i++) {
                if (i >= n_phase) break;
                const unsigned op = metas[i] & 0xffu;
                float fa[NV], fb[NV], fo[NV];
                V::unpack(w, fa);
                V::unpack(ld1[i], fb);
                if (op == (unsigned)kGelu) {
                    if constexpr (!kWide || VB == 4) {
#pragma unroll
                        for (int e = 0; e < NV; e++) fo[e] = ew_apply<kGelu, kWide>(fa[e], 0.f);
                    } else {
#pragma unroll
                        for (int e = 0; e < NV; e++) fo[e] = fa[e];      // never planned: the fp32 GELU rides only one element per lane
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < NV; e++) {
                        const float sum = ew_apply<kAdd, kWide>(fa[e], fb[e]), prod = ew_apply<kMul, kWide>(fa[e], fb[e]);
                        fo[e] = op == (unsigned)kAdd ? sum : prod;
                    }
                }
                V::pack(fo, w);
                if (act && (inds[i] & kEpiStore)) {
                    if constexpr (VB == 16) store_vec_global(outs[i] + i0, w);
                    else *(unsigned PG_GLOBAL*)(uintptr_t)(outs[i] + i0) = w[0];
                }
            }
            return;
        }
    }
#pragma unroll 1
    for (int i = 0; i < n_phase; i++) {
        // this kernel's entry of the table and its fetched operands: uniform selects, no indexing
        T* out = outs[0];
        unsigned mt = metas[0];
        unsigned ind = inds[0];
        float eps = epss[0];
        unsigned wa[NW], wb[NW], wo[NW];
#pragma unroll
        for (int k = 0; k < NW; k++) { wa[k] = ld0[0][k]; wb[k] = ld1[0][k]; }
#pragma unroll
        for (int j = 1; j < P; j++)
            if (i == j) {
                out = outs[j]; mt = metas[j]; ind = inds[j]; eps = epss[j];
#pragma unroll
                for (int k = 0; k < NW; k++) { wa[k] = ld0[j][k]; wb[k] = ld1[j][k]; }
            }
        const unsigned op = mt & 0xffu, src0 = (mt >> 8) & 0xffu, src1 = (mt >> 16) & 0xffu, dst = mt >> 24;
#pragma unroll
        for (int q = 0; q < kMergeSlots; q++) {
            if (src0 == (unsigned)q)
#pragma unroll
                for (int k = 0; k < NW; k++) wa[k] = slot[q][k];
            if (src1 == (unsigned)q)
#pragma unroll
                for (int k = 0; k < NW; k++) wb[k] = slot[q][k];
        }
        float fa[NV], fb[NV], fo[NV];
        V::unpack(wa, fa);
        V::unpack(wb, fb);
        if (VB == 16 && op == kRmsNorm) {      // a row is one unit of 256 lanes x 16 bytes: never in the narrow form
            float acc = 0.f;
#pragma unroll
            for (int e = 0; e < NV; e++) acc = __builtin_fmaf(fa[e], fa[e], acc);
            acc = wave_sum(acc);
            if ((tid & 63) == 0) part[tid >> 6] = acc;
            lds_barrier();
            const float total = ((part[0] + part[1]) + part[2]) + part[3];
            lds_barrier();                                         // `part` is free for a later RMSNorm of the run
            const float scale = 1.0f / sqrtf(total / (float)(kBlock * NV) + eps);
#pragma unroll
            for (int e = 0; e < NV; e++) fo[e] = (fa[e] * scale) * fb[e];
        } else if (op == kAdd) {
#pragma unroll
            for (int e = 0; e < NV; e++) fo[e] = ew_apply<kAdd, kWide>(fa[e], fb[e]);
        } else if (op == kMul) {
#pragma unroll
            for (int e = 0; e < NV; e++) fo[e] = ew_apply<kMul, kWide>(fa[e], fb[e]);
        } else {
            if constexpr (!kWide || VB == 4) {                     // fp32 GELU (evaluated in fp64): one element per lane only
#pragma unroll
                for (int e = 0; e < NV; e++) fo[e] = ew_apply<kGelu, kWide>(fa[e], 0.f);
            } else {
#pragma unroll
                for (int e = 0; e < NV; e++) fo[e] = fa[e];
            }
        }
        V::pack(fo, wo);
        if (act && (ind & kEpiStore)) {      // not stored: a later kernel of the run overwrites it, and nothing reads memory in between
            if constexpr (VB == 16) store_vec_global(out + i0, wo);
            else *(unsigned PG_GLOBAL*)(uintptr_t)(out + i0) = wo[0];
        }
#pragma unroll
        for (int q = 0; q < kMergeSlots; q++)
            if (dst == (unsigned)q)
#pragma unroll
                for (int k = 0; k < NW; k++) slot[q][k] = wo[k];
    }
}

template <typename T, int VB>
__global__ __launch_bounds__(kBlock) void k_merged(MergedArgs p) {
    constexpr int P = kMergeMaxPhases;
    __shared__ float part[kBlock / 64];
    // operand addresses, once, before any store of this kernel: pointer-table slots are read with scalar loads
    const T* in0[P];
    const T* in1[P];
    bool al = true;
#pragma unroll
    for (int i = 0; i < P; i++) {
        in0[i] = in1[i] = nullptr;
        const unsigned mt = p.ph[i].meta;
        if (((mt >> 8) & 0xffu) == kMergeFromMemory) {
            in0[i] = static_cast<const T*>(resolve_rt(p.ph[i].in0, p.ph[i].ind & 1));
            al = al && aligned_to(in0[i], VB);
        }
        if ((mt & 0xffu) != kGelu && ((mt >> 16) & 0xffu) == kMergeFromMemory) {
            in1[i] = static_cast<const T*>(resolve_rt(p.ph[i].in1, p.ph[i].ind & 2));
            al = al && aligned_to(in1[i], VB);
        }
    }
    if (__builtin_expect(al, 1)) merged_body<T, VB, true>(p, in0, in1, part);
    else merged_body<T, VB, false>(p, in0, in1, part);
}

// GEMV with an elementwise epilogue: k_gemv_shared's body, then lane e of each wave plays output e through
// the kernels that follow (see kernels.h).  bf16 only.
template <int RB, bool PRO>
__global__ __launch_bounds__(kBlock) void k_gemv_epilogue(GemvEpiArgs p) {
    constexpr int P = kEpiMaxPhases;
    // The GEMV's own arguments first, in one batch of scalar loads (see args_up_front): nothing else stands
    // between the start of the kernel and the weight loads.  The epilogue's table is read once those are on
    // their way (`fetch`), and kept in scalar registers from then on.
    // The first 64 bytes of the arguments hold everything that is needed before the weight loads can go out,
    // and only those are waited for here, in one batch of scalar loads (see args_up_front; the start of the
    // argument buffer arrives in under 0.1 us, the lines behind it take 0.3 us more).  The epilogue's table
    // and eps are read once the weights are on their way (`fetch`).
    static_assert(offsetof(GemvEpiArgs, gain) + sizeof(void*) == 64, "what the kernel needs first sits in the first 64 bytes");
    const void* Wa = p.g.W;
    const void* ha = p.g.h;
    bf16_t* y = static_cast<bf16_t*>(p.g.out);
    int n = p.g.n;
    unsigned head = p.head;
    int n_epi = p.n_epi;
    const void* xa = p.x;
    const void* ga = p.gain;
    asm volatile("" : "+s"(Wa), "+s"(ha), "+s"(y), "+s"(n), "+s"(head), "+s"(n_epi), "+s"(xa), "+s"(ga));
    const void* a0[P];
    const void* a1[P];
    bf16_t* outs[P];
    unsigned ms[P], metas[P], inds[P];
    float eps = 0.f;
    static_assert(P == 3, "the argument batch in fetch names every phase");
    const void PG_CONSTANT* const ka = (const void PG_CONSTANT*)__builtin_amdgcn_kernarg_segment_ptr();   // a readable address for a load whose result is not used
    using SlotPtr = const void* const PG_CONSTANT*;
    auto slot_addr = [&](const void* q, bool is_slot) -> SlotPtr { return is_slot ? (SlotPtr)(uintptr_t)q : (SlotPtr)ka; };
    // with a prologue the GEMV's input is computed from x and the gain; p.g.h is where workgroup 0 stores it
    if (head & (1u | (PRO ? kEpiXSlot | kEpiGainSlot : 2u))) {      // some operand is a pointer-table slot: all in one batch, without branches
        const bool sw = head & 1u, sh = head & (PRO ? kEpiXSlot : 2u), sg = PRO && (head & kEpiGainSlot);
        SlotPtr aw = slot_addr(Wa, sw), ah = slot_addr(PRO ? xa : ha, sh), ag = slot_addr(ga, sg);
        const void* tw = *aw;
        const void* th = *ah;
        const void* tg = PRO ? *ag : nullptr;
        asm volatile("" : "+s"(tw), "+s"(th), "+s"(tg));
        if (sw) Wa = tw;
        if (sh) { if (PRO) xa = th; else ha = th; }
        if (sg) ga = tg;
    }
    const bf16_t* W = static_cast<const bf16_t*>(Wa);
    const bf16_t* h = static_cast<const bf16_t*>(PRO ? xa : ha);
    const bf16_t* gain = PRO ? static_cast<const bf16_t*>(ga) : nullptr;
    bf16_t* hstore = (PRO && (head & kEpiStoreH) && blockIdx.x == 0) ? static_cast<bf16_t*>(const_cast<void*>(ha)) : nullptr;
    __shared__ v4u hs[RB * kBlock];
    __shared__ float part[RB * (kBlock / 64)];
    const int tid = threadIdx.x, lane = tid & 63;
    const int j0 = (blockIdx.x * (kBlock / 64) + (tid >> 6)) * 2;
    unsigned ld0[P], ld1[P];
    bool mine = false;
    unsigned idx = 0;
    bool decoder = false;       // the tail is GELU of the GEMV's result, then one or two adds with an operand from memory
    // The epilogue's operands: asked for once the weights are on their way (pointer-table slots first, with
    // scalar loads, all at once).  Always the same number of loads -- an operand that comes from a register
    // slot is fetched from the GEMV's own output buffer instead and ignored -- so that every wait on the
    // weights knows exactly how many younger loads are outstanding.
    auto fetch = [&] {
        {   // the rest of the arguments, through the kernel-argument segment's address made opaque: otherwise the
            // compiler moves these loads (invariant memory) to the top of the kernel, in front of the weight loads
            const GemvEpiArgs PG_CONSTANT* kp = (const GemvEpiArgs PG_CONSTANT*)ka;
            asm volatile("" : "+s"(kp));
            eps = kp->eps;
#pragma unroll
            for (int i = 0; i < P; i++) {
                a0[i] = kp->ph[i].in0; a1[i] = kp->ph[i].in1; outs[i] = static_cast<bf16_t*>(kp->ph[i].out);
                ms[i] = kp->ph[i].m; metas[i] = kp->ph[i].meta; inds[i] = kp->ph[i].ind;
            }
            asm volatile("" : "+s"(eps),
                              "+s"(a0[0]), "+s"(a1[0]), "+s"(outs[0]), "+s"(ms[0]), "+s"(metas[0]), "+s"(inds[0]),
                              "+s"(a0[1]), "+s"(a1[1]), "+s"(outs[1]), "+s"(ms[1]), "+s"(metas[1]), "+s"(inds[1]),
                              "+s"(a0[2]), "+s"(a1[2]), "+s"(outs[2]), "+s"(ms[2]), "+s"(metas[2]), "+s"(inds[2]));
        }
        mine = lane < 2 * RB && j0 + (lane & 1) < n;
        idx = mine ? (unsigned)(lane >> 1) * (unsigned)n + (unsigned)(j0 + (lane & 1)) : 0u;
        const unsigned total = (unsigned)RB * (unsigned)n;
        bool f0[P], f1[P], s0[P], s1[P];
        unsigned any = 0;
#pragma unroll
        for (int i = 0; i < P; i++) {
            const unsigned mt = metas[i];
            f0[i] = ((mt >> 8) & 0xffu) == kMergeFromMemory;
            f1[i] = (mt & 0xffu) != kGelu && ((mt >> 16) & 0xffu) == kMergeFromMemory;
            s0[i] = f0[i] && (inds[i] & 1u);
            s1[i] = f1[i] && (inds[i] & 2u);
            any |= (f0[i] ? inds[i] & 1u : 0u) | (f1[i] ? inds[i] & 2u : 0u);
        }
        any = __builtin_amdgcn_readfirstlane(any);
        asm volatile("" : "+s"(any));       // keeps what follows behind the weight loads
        {   // the decoder block's tail, recognised here (scalar arithmetic under the weights' latency) so that the
            // tail itself runs it straight through, without the operand and slot selection of the general form
            auto add_of = [](unsigned mt, unsigned q) {
                const unsigned a = (mt >> 8) & 0xffu, b = (mt >> 16) & 0xffu;
                return (mt & 0xffu) == (unsigned)kAdd && ((a == q && b == kMergeFromMemory) || (a == kMergeFromMemory && b == q));
            };
            const unsigned hq = (head >> 8) & 0xffu, d0 = metas[0] >> 24, d1 = metas[1] >> 24;
            decoder = (n_epi == 2 || n_epi == 3) && (metas[0] & 0xffu) == (unsigned)kGelu && ((metas[0] >> 8) & 0xffu) == hq &&
                      add_of(metas[1], d0) && (n_epi == 2 || add_of(metas[2], d1));
        }
        if (any) {
            SlotPtr at0[P], at1[P];
            const void* t0[P];
            const void* t1[P];
#pragma unroll
            for (int i = 0; i < P; i++) { at0[i] = slot_addr(a0[i], s0[i]); at1[i] = slot_addr(a1[i], s1[i]); }
#pragma unroll
            for (int i = 0; i < P; i++) { t0[i] = *at0[i]; t1[i] = *at1[i]; }
            asm volatile("" : "+s"(t0[0]), "+s"(t1[0]), "+s"(t0[1]), "+s"(t1[1]), "+s"(t0[2]), "+s"(t1[2]));
#pragma unroll
            for (int i = 0; i < P; i++) {
                if (s0[i]) a0[i] = t0[i];
                if (s1[i]) a1[i] = t1[i];
            }
        }
        const bf16_t* q0[P];
        const bf16_t* q1[P];
        unsigned mm[P];
        bool plain = true;      // no operand has a broadcast period: the usual case, one branch for all
#pragma unroll
        for (int i = 0; i < P; i++) {
            q0[i] = f0[i] ? static_cast<const bf16_t*>(a0[i]) : y;
            q1[i] = f1[i] ? static_cast<const bf16_t*>(a1[i]) : y;
            mm[i] = f1[i] ? ms[i] : total;
            plain = plain && mm[i] == total;
        }
        if (__builtin_expect(plain, 1)) {
#pragma unroll
            for (int i = 0; i < P; i++) {
                ld0[i] = load_raw_global_at(q0[i], idx);
                ld1[i] = load_raw_global_at(q1[i], idx);
            }
        } else {
#pragma unroll
            for (int i = 0; i < P; i++) {
                ld0[i] = load_raw_global_at(q0[i], idx);
                ld1[i] = load_raw_global_at(q1[i], idx % mm[i]);
            }
        }
    };
    float sums[2][RB];
    if (__builtin_expect(aligned_to(W, 16) && aligned_to(h, 16) && (!PRO || aligned_to(gain, 16)), 1))
        gemv_sums_shared<bf16_t, 2, RB, true, true, PRO>(W, h, n, j0, lane, tid, hs, fetch, sums, gain, eps, hstore, part);
    else
        gemv_sums_shared<bf16_t, 2, RB, false, true, PRO>(W, h, n, j0, lane, tid, hs, fetch, sums, gain, eps, hstore, part);
    float v = sums[0][0];
#pragma unroll
    for (int rr = 0; rr < RB; rr++)
#pragma unroll
        for (int r = 0; r < 2; r++)
            if (lane == rr * 2 + r) v = sums[r][rr];
    unsigned bits = f32_to_bf16(v);
    // The epilogue's operands have been on their way since before the weights were used; claim them all now,
    // before the first store of the tail.  Loads and stores complete in one queue, in order, so a wait for
    // an operand placed after a store would wait for that store to be acknowledged as well.
    __builtin_amdgcn_s_waitcnt(0x0F70);      // vmcnt(0)
    if (mine && (head & kEpiHeadStore)) *(unsigned short PG_GLOBAL*)(uintptr_t)(y + idx) = (unsigned short)bits;
    float slot[kMergeSlots];
#pragma unroll
    for (int q = 0; q < kMergeSlots; q++) slot[q] = 0.f;
    {
        const unsigned dst = (head >> 8) & 0xffu;
#pragma unroll
        for (int q = 0; q < kMergeSlots; q++)
            if (dst == (unsigned)q) slot[q] = from_raw<bf16_t>(bits);
    }
    if (__builtin_expect(decoder, 1)) {
        // the same kernels with the same arithmetic and roundings, operands known: GELU of the GEMV's rounded result,
        // then each add takes the value before it and its operand from memory, in the order its descriptor names
        const bool st = mine;
        float val = ew_apply<kGelu, false>(from_raw<bf16_t>(bits), 0.f);
        bits = f32_to_bf16(val);
        if (st && (inds[0] & kEpiStore)) *(unsigned short PG_GLOBAL*)(uintptr_t)(outs[0] + idx) = (unsigned short)bits;
        val = from_raw<bf16_t>(bits);
        {
            const bool mem_first = ((metas[1] >> 8) & 0xffu) == kMergeFromMemory;
            const float fa = mem_first ? from_raw<bf16_t>(ld0[1]) : val, fb = mem_first ? val : from_raw<bf16_t>(ld1[1]);
            bits = f32_to_bf16(ew_apply<kAdd, false>(fa, fb));
            if (st && (inds[1] & kEpiStore)) *(unsigned short PG_GLOBAL*)(uintptr_t)(outs[1] + idx) = (unsigned short)bits;
            val = from_raw<bf16_t>(bits);
        }
        if (n_epi == 3) {
            const bool mem_first = ((metas[2] >> 8) & 0xffu) == kMergeFromMemory;
            const float fa = mem_first ? from_raw<bf16_t>(ld0[2]) : val, fb = mem_first ? val : from_raw<bf16_t>(ld1[2]);
            bits = f32_to_bf16(ew_apply<kAdd, false>(fa, fb));
            if (st && (inds[2] & kEpiStore)) *(unsigned short PG_GLOBAL*)(uintptr_t)(outs[2] + idx) = (unsigned short)bits;
        }
        return;
    }
    // Unrolled, with the one big choice (GELU or not) as the only branch inside a phase: a taken branch costs
    // this one-wave-per-SIMD tail more than a dozen arithmetic instructions.
#pragma unroll
    for (int i = 0; i < P; i++) {
        if (i >= n_epi) break;
        const unsigned mt = metas[i], ind = inds[i];
        const unsigned op = mt & 0xffu, src0 = (mt >> 8) & 0xffu, src1 = (mt >> 16) & 0xffu, dst = mt >> 24;
        float fa = from_raw<bf16_t>(ld0[i]), fb = from_raw<bf16_t>(ld1[i]);
#pragma unroll
        for (int q = 0; q < kMergeSlots; q++) {
            if (src0 == (unsigned)q) fa = slot[q];
            if (src1 == (unsigned)q) fb = slot[q];
        }
        float fo;
        if (op == kGelu) {
            fo = ew_apply<kGelu, false>(fa, 0.f);
        } else {
            const float sum = ew_apply<kAdd, false>(fa, fb), prod = ew_apply<kMul, false>(fa, fb);
            fo = op == kAdd ? sum : prod;
        }
        bits = f32_to_bf16(fo);
        if (mine && (ind & kEpiStore)) *(unsigned short PG_GLOBAL*)(uintptr_t)(outs[i] + idx) = (unsigned short)bits;
#pragma unroll
        for (int q = 0; q < kMergeSlots; q++)
            if (dst == (unsigned)q) slot[q] = from_raw<bf16_t>(bits);
    }
}

// ---- batched multi-tensor copy -----------------------------------------------------------------
// One workgroup per chunk (<= kCopyChunkBytes of one tensor): every lane issues its two 128-bit
// non-temporal loads, then its two stores, and the workgroup is done -- measured on the log-uniform
// size mix, many short-lived workgroups with two vectors in flight per lane beat fewer, longer ones
// (6.2 against 5.2 TB/s).  Destinations are placeholders the library laid out itself (256-byte
// aligned, chunk offsets multiples of the chunk size), so only the source alignment varies: sources
// that are not 16-byte aligned fall back to 4-byte or 2-byte moves.
constexpr int kCopyUnroll = 2;
static_assert(kCopyChunkBytes == kBlock * kCopyUnroll * 16, "one pass of the workgroup covers one chunk");

__global__ __launch_bounds__(kBlock) void k_copy(CopyArgs p) {
    const CopyChunk c = p.chunks[blockIdx.x];
    const CopyTensor t = p.tensors[c.tensor];
    const char* __restrict__ src = static_cast<const char*>(p.src[c.tensor - p.src_base]) + c.off;
    char* __restrict__ dst = static_cast<char*>(t.dst) + c.off;
    const unsigned len = c.len;
    const unsigned tid = threadIdx.x;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) == 0) {
        const v4u* s16 = reinterpret_cast<const v4u*>(src);
        v4u* d16 = reinterpret_cast<v4u*>(dst);
        const unsigned nvec = len >> 4;
        for (unsigned v0 = 0; v0 < nvec; v0 += kBlock * kCopyUnroll) {
            v4u r[kCopyUnroll];
#pragma unroll
            for (int u = 0; u < kCopyUnroll; u++) {
                const unsigned v = v0 + u * kBlock + tid;
                if (v < nvec) r[u] = __builtin_nontemporal_load(s16 + v);
            }
#pragma unroll
            for (int u = 0; u < kCopyUnroll; u++) {
                const unsigned v = v0 + u * kBlock + tid;
                if (v < nvec) __builtin_nontemporal_store(r[u], d16 + v);
            }
        }
        const unsigned i = (nvec << 4) + tid;
        if (i < len) dst[i] = src[i];
    } else if ((reinterpret_cast<uintptr_t>(src) & 3u) == 0) {
        const unsigned* s4 = reinterpret_cast<const unsigned*>(src);
        unsigned* d4 = reinterpret_cast<unsigned*>(dst);
        const unsigned nw = len >> 2;
        for (unsigned v = tid; v < nw; v += kBlock) d4[v] = s4[v];
        const unsigned i = (nw << 2) + tid;
        if (i < len) dst[i] = src[i];
    } else {
        // tensors are aligned to their element size, so a source that is not 4-byte aligned holds
        // 2-byte elements and has an even length
        const unsigned short* s2 = reinterpret_cast<const unsigned short*>(src);
        unsigned short* d2 = reinterpret_cast<unsigned short*>(dst);
        const unsigned nh = len >> 1;
        for (unsigned v = tid; v < nh; v += kBlock) d2[v] = s2[v];
    }
}

// ---- pointer-table writer ------------------------------------------------------------------------
__global__ __launch_bounds__(64) void k_table_write(TableArgs p) {
    for (int i = threadIdx.x; i < p.n; i += 64) p.table[p.base + i] = p.ptr[i];
}

// ---- host side: pick the instantiation and the launch shape from the kernel's shape alone ----------
#define PG_FN(...) reinterpret_cast<const void*>(&__VA_ARGS__)

unsigned blocks_for(long long n, long long per_block) {
    const long long g = (n + per_block - 1) / per_block;
    return (unsigned)(g < 1 ? 1 : g);
}

template <typename T, int OP, int VB, int U, typename IdxT>
const void* ew_by_ind(int ind) {
    switch (ind) {
    case 0: return PG_FN(k_elementwise<T, OP, 0, VB, U, IdxT>);
    case 1: return PG_FN(k_elementwise<T, OP, 1, VB, U, IdxT>);
    case 2: if constexpr (OP != kGelu) return PG_FN(k_elementwise<T, OP, 2, VB, U, IdxT>); else return nullptr;
    case 3: if constexpr (OP != kGelu) return PG_FN(k_elementwise<T, OP, 3, VB, U, IdxT>); else return nullptr;
    default: return nullptr;
    }
}

// Shape classes: (4-byte vectors, 1 per lane) for small GELUs, whose cost is the arithmetic a lane
// does in sequence; (16-byte, 1 per lane) for short tensors; (16-byte, 4 per lane) for long ones,
// with 64-bit indices beyond 2^31 elements.
template <typename T, int OP>
bool plan_ew_t(int ind, long long n, Launch* out) {
    constexpr int NV16 = 16 / (int)sizeof(T), NV4 = 4 / (int)sizeof(T);
    const long long bytes = n * (long long)sizeof(T);
    const bool narrow = OP == kGelu && n <= (1ll << 20);
    out->block = dim3(kBlock);
    if (narrow) {
        out->fn = ew_by_ind<T, OP, 4, 1, unsigned>(ind);
        out->grid = dim3(blocks_for(n, (long long)kBlock * NV4));
    } else if (bytes <= (4ll << 20)) {
        out->fn = ew_by_ind<T, OP, 16, 1, unsigned>(ind);
        out->grid = dim3(blocks_for(n, (long long)kBlock * NV16));
    } else if (n < (1ll << 31)) {
        out->fn = ew_by_ind<T, OP, 16, 4, unsigned>(ind);
        out->grid = dim3(blocks_for(n, (long long)kBlock * 4 * NV16));
    } else {
        out->fn = ew_by_ind<T, OP, 16, 4, unsigned long long>(ind);
        out->grid = dim3(blocks_for(n, (long long)kBlock * 4 * NV16));
    }
    return out->fn != nullptr;
}

template <typename T>
bool plan_ew(int op, int ind, long long n, Launch* out) {
    switch (op) {
    case kAdd: return plan_ew_t<T, kAdd>(ind, n, out);
    case kMul: return plan_ew_t<T, kMul>(ind, n, out);
    case kGelu: return plan_ew_t<T, kGelu>(ind, n, out);
    default: return false;
    }
}

template <typename T, int VPT, bool RAGGED>
const void* rms_by_ind(int ind) {
    switch (ind) {
    case 0: return PG_FN(k_rmsnorm<T, 0, VPT, RAGGED>);
    case 1: return PG_FN(k_rmsnorm<T, 1, VPT, RAGGED>);
    case 2: return PG_FN(k_rmsnorm<T, 2, VPT, RAGGED>);
    case 3: return PG_FN(k_rmsnorm<T, 3, VPT, RAGGED>);
    default: return nullptr;
    }
}

template <typename T>
bool plan_rms(int ind, int rows, int cols, Launch* out) {
    constexpr int NV = 16 / (int)sizeof(T);
    const int nvec = (cols + NV - 1) / NV;
    const bool ragged = (cols % NV) != 0;
    if (nvec <= kBlock) out->fn = ragged ? rms_by_ind<T, 1, true>(ind) : rms_by_ind<T, 1, false>(ind);
    else if (nvec <= 4 * kBlock) out->fn = ragged ? rms_by_ind<T, 4, true>(ind) : rms_by_ind<T, 4, false>(ind);
    else out->fn = ragged ? rms_by_ind<T, 0, true>(ind) : rms_by_ind<T, 0, false>(ind);
    out->grid = dim3((unsigned)rows);
    out->block = dim3(kBlock);
    return out->fn != nullptr;
}

template <typename T, int R, int RS>
const void* gemv_by_ind(int ind) {
    switch (ind) {
    case 0: return PG_FN(k_gemv<T, 0, R, RS>);
    case 1: return PG_FN(k_gemv<T, 1, R, RS>);
    case 2: return PG_FN(k_gemv<T, 2, R, RS>);
    case 3: return PG_FN(k_gemv<T, 3, R, RS>);
    default: return nullptr;
    }
}
template <typename T, int R, int RB, int RS>
const void* gemvb_by_ind(int ind) {
    switch (ind) {
    case 0: return PG_FN(k_gemv_batched<T, 0, R, RB, RS>);
    case 1: return PG_FN(k_gemv_batched<T, 1, R, RB, RS>);
    case 2: return PG_FN(k_gemv_batched<T, 2, R, RB, RS>);
    case 3: return PG_FN(k_gemv_batched<T, 3, R, RB, RS>);
    default: return nullptr;
    }
}

template <typename T, int RB>
const void* gemv_shared_by_ind(int ind) {
    switch (ind) {
    case 0: return PG_FN(k_gemv_shared<T, 0, 2, RB>);
    case 1: return PG_FN(k_gemv_shared<T, 1, 2, RB>);
    case 2: return PG_FN(k_gemv_shared<T, 2, 2, RB>);
    case 3: return PG_FN(k_gemv_shared<T, 3, 2, RB>);
    default: return nullptr;
    }
}

template <typename T, int RS>
bool plan_gemv_rs(int ind, int rows, int n, int cols, Launch* out) {
    out->block = dim3(kBlock);
    const bool one_chunk = RS == 0 && cols == 64 * kGemvChunk * (16 / (int)sizeof(T));   // the forms that share h through LDS
    if (rows == 1 && n >= 1024) {
        // two weight rows per wave once there are enough rows to fill the chip with half the waves
        out->fn = one_chunk ? gemv_shared_by_ind<T, 1>(ind) : gemv_by_ind<T, 2, RS>(ind);
        out->grid = dim3(blocks_for(n, (kBlock / 64) * 2));
    } else if (rows == 1) {
        out->fn = gemv_by_ind<T, 1, RS>(ind);
        out->grid = dim3(blocks_for(n, kBlock / 64));
    } else if (n >= 1024) {
        if (one_chunk && rows <= 4) out->fn = rows == 2 ? gemv_shared_by_ind<T, 2>(ind) : rows == 3 ? gemv_shared_by_ind<T, 3>(ind) : gemv_shared_by_ind<T, 4>(ind);
        else out->fn = rows == 2 ? gemvb_by_ind<T, 2, 2, RS>(ind) : gemvb_by_ind<T, 2, 4, RS>(ind);
        out->grid = dim3(blocks_for(n, (kBlock / 64) * 2));
    } else {
        out->fn = rows == 2 ? gemvb_by_ind<T, 1, 2, RS>(ind) : gemvb_by_ind<T, 1, 4, RS>(ind);
        out->grid = dim3(blocks_for(n, kBlock / 64));
    }
    return out->fn != nullptr;
}

template <bool FULL, bool SINGLE>
const void* gemm_by_ind(int ind) {
    switch (ind) {
    case 0: return PG_FN(k_gemm_mfma_bf16<0, FULL, SINGLE>);
    case 1: return PG_FN(k_gemm_mfma_bf16<1, FULL, SINGLE>);
    case 2: return PG_FN(k_gemm_mfma_bf16<2, FULL, SINGLE>);
    case 3: return PG_FN(k_gemm_mfma_bf16<3, FULL, SINGLE>);
    default: return nullptr;
    }
}

template <bool FULL, int NRH>
const void* gemm_narrow_by_ind(int ind) {
    switch (ind) {
    case 0: return PG_FN(k_gemm_mfma_bf16_narrow<0, FULL, NRH>);
    case 1: return PG_FN(k_gemm_mfma_bf16_narrow<1, FULL, NRH>);
    case 2: return PG_FN(k_gemm_mfma_bf16_narrow<2, FULL, NRH>);
    case 3: return PG_FN(k_gemm_mfma_bf16_narrow<3, FULL, NRH>);
    default: return nullptr;
    }
}

template <typename T>
bool plan_gemv(int ind, int rows, int n, int cols, Launch* out) {
    constexpr int NV = 16 / (int)sizeof(T);
    if constexpr (sizeof(T) == 2) {
        // A dense contraction: matrix cores from 5 rows on, and for 3 and 4 rows where the narrow form
        // applies and the vector form that shares h through LDS does not (measured at 2048 x 2048, us
        // per launch at 2 / 3 / 4 rows: vector with shared h 3.3 / 3.5 / 3.7, narrow matrix-core form
        // 3.9 / 4.0 / 4.0, vector with h per wave 3.8 / 4.4 / 4.5).
        const bool narrow_ok = rows <= 16 && cols <= 32 * 4 * kMmSteps && n >= 16;
        const bool shared_ok = rows <= 4 && n >= 1024 && cols == 64 * kGemvChunk * NV;
        if (cols % 8 == 0 && (rows > 4 || (rows >= 3 && narrow_ok && !shared_ok))) {
            out->block = dim3(kBlock);
            // row groups of 16-row tiles: enough workgroups to fill the chip twice over at most
            const int ntiles = (rows + 15) / 16;
            out->gemm_row_groups = (unsigned)(ntiles < kMmMaxRowGroups ? ntiles : kMmMaxRowGroups);
            out->grid = dim3(blocks_for(n, 16) * out->gemm_row_groups);
            constexpr int kSuper = 32 * 4 * kMmSteps;   // columns one pass of the 4 waves covers
            if (cols == kSuper && rows >= kMmWideRows && n >= 32) {
                out->grid = dim3(blocks_for(n, 32) * out->gemm_row_groups);
                switch (ind) {
                case 0: out->fn = PG_FN(k_gemm_mfma_bf16_wide<0>); break;
                case 1: out->fn = PG_FN(k_gemm_mfma_bf16_wide<1>); break;
                case 2: out->fn = PG_FN(k_gemm_mfma_bf16_wide<2>); break;
                case 3: out->fn = PG_FN(k_gemm_mfma_bf16_wide<3>); break;
                default: out->fn = nullptr;
                }
            } else if (narrow_ok) {
                out->grid = dim3(blocks_for(n, 8));
                const int nrh = rows <= 4 ? 4 : rows <= 8 ? 8 : 16;
                out->fn = cols == kSuper ? (nrh == 4 ? gemm_narrow_by_ind<true, 4>(ind) : nrh == 8 ? gemm_narrow_by_ind<true, 8>(ind) : gemm_narrow_by_ind<true, 16>(ind))
                                         : (nrh == 4 ? gemm_narrow_by_ind<false, 4>(ind) : nrh == 8 ? gemm_narrow_by_ind<false, 8>(ind) : gemm_narrow_by_ind<false, 16>(ind));
            } else if (cols == kSuper) out->fn = gemm_by_ind<true, true>(ind);
            else if (cols < kSuper) out->fn = gemm_by_ind<false, true>(ind);
            else if (cols % kSuper == 0) out->fn = gemm_by_ind<true, false>(ind);
            else out->fn = gemm_by_ind<false, false>(ind);
            return out->fn != nullptr;
        }
    }
    if (cols % (64 * kGemvChunk * NV) == 0) return plan_gemv_rs<T, 0>(ind, rows, n, cols, out);
    if (cols % NV == 0) return plan_gemv_rs<T, 1>(ind, rows, n, cols, out);
    return plan_gemv_rs<T, 2>(ind, rows, n, cols, out);
}

template <typename T, bool VEC, int U, typename IdxT>
const void* sbr_by_ind(int ind) {
    switch (ind) {
    case 0: return PG_FN(k_scale_bias_relu<T, 0, VEC, U, IdxT>);
    case 1: return PG_FN(k_scale_bias_relu<T, 1, VEC, U, IdxT>);
    case 2: return PG_FN(k_scale_bias_relu<T, 2, VEC, U, IdxT>);
    case 3: return PG_FN(k_scale_bias_relu<T, 3, VEC, U, IdxT>);
    case 4: return PG_FN(k_scale_bias_relu<T, 4, VEC, U, IdxT>);
    case 5: return PG_FN(k_scale_bias_relu<T, 5, VEC, U, IdxT>);
    case 6: return PG_FN(k_scale_bias_relu<T, 6, VEC, U, IdxT>);
    case 7: return PG_FN(k_scale_bias_relu<T, 7, VEC, U, IdxT>);
    default: return nullptr;
    }
}

template <typename T>
bool plan_sbr(int ind, long long n, long long inner, Launch* out) {
    constexpr int NV = 16 / (int)sizeof(T);
    const bool vec = (inner % NV) == 0;
    const long long units = vec ? n / NV : n;
    out->block = dim3(kBlock);
    if (n >= (1ll << 31)) {
        out->fn = vec ? sbr_by_ind<T, true, 4, unsigned long long>(ind) : sbr_by_ind<T, false, 4, unsigned long long>(ind);
        out->grid = dim3(blocks_for(units, kBlock * 4));
    } else if (units <= 16384) {
        out->fn = vec ? sbr_by_ind<T, true, 1, unsigned>(ind) : sbr_by_ind<T, false, 1, unsigned>(ind);
        out->grid = dim3(blocks_for(units, kBlock));
    } else {
        out->fn = vec ? sbr_by_ind<T, true, 4, unsigned>(ind) : sbr_by_ind<T, false, 4, unsigned>(ind);
        out->grid = dim3(blocks_for(units, kBlock * 4));
    }
    return out->fn != nullptr;
}

template <typename T>
bool plan_t(int op, int ind, const Shape& s, Launch* out) {
    switch (op) {
    case kAdd: case kMul: case kGelu: return plan_ew<T>(op, ind, s.n, out);
    case kRmsNorm: return plan_rms<T>(ind, (int)s.rows, (int)s.cols, out);
    case kGemv: return plan_gemv<T>(ind, (int)s.rows, (int)s.n, (int)s.cols, out);
    case kScaleBiasRelu: return plan_sbr<T>(ind, s.n, s.inner, out);
    default: return false;
    }
}

}  // namespace

bool plan(int op, int dtype, int ind_mask, const Shape& shape, Launch* out) {
    switch (op) {
    case kAdd: case kMul: case kGelu: out->arg_bytes = sizeof(EwArgs); break;
    case kRmsNorm: out->arg_bytes = sizeof(RmsArgs); break;
    case kGemv: out->arg_bytes = sizeof(GemvArgs); break;
    case kScaleBiasRelu: out->arg_bytes = sizeof(SbrArgs); break;
    default: return false;
    }
    out->mod_fn = nullptr;
    out->gemm_row_groups = 0;
    if (dtype == kF32) return plan_t<float>(op, ind_mask, shape, out);
    if (dtype == kBF16) return plan_t<bf16_t>(op, ind_mask, shape, out);
    return false;
}
bool merge_candidate(int op, int dtype, const Shape& s, bool whole_vectors, long long* n_out) {
    if (dtype != kF32 && dtype != kBF16) return false;
    const int nv = dtype == kF32 ? 4 : 8;
    long long n = 0;
    if (op == kAdd || op == kMul || op == kGelu) {
        if (s.m <= 0) return false;
        n = s.n;
        // fp32 GELU is evaluated in fp64: mergeable only where the run works one element per lane (small tensors)
        if (op == kGelu && dtype == kF32 && !merge_narrow(dtype, n)) return false;
    } else if (op == kRmsNorm) {
        if (s.cols != (long long)kBlock * nv) return false;   // a row must be exactly one unit
        n = s.rows * s.cols;
    } else {
        return false;
    }
    if (n <= 0 || (whole_vectors && !merge_narrow(dtype, n) && n % nv != 0) || n > (1ll << 31)) return false;
    *n_out = n;
    return true;
}

bool merge_narrow(int dtype, long long n) { return dtype == kF32 && n > 0 && n <= kMergeNarrowMax; }

bool merge_head(int op, int dtype, const Shape& s, long long* n_out) {
    if (op != kGemv || dtype != kBF16 || s.cols != 64 * kGemvChunk * 8 || s.rows < 1) return false;
    if (s.rows <= 4) {
        // exactly the shapes plan_gemv gives to k_gemv_shared<bf16, IND, 2, rows>
        if (s.n < 1024) return false;
    } else {
        // the matrix-core forms plan_gemv picks for rows of 2048 columns: narrow (up to 16 rows), 16 columns per
        // workgroup, wide (from kMmWideRows rows); element indices are kept in 32 bits
        if (s.n < 32 || s.rows * s.n > (1ll << 31)) return false;
    }
    *n_out = s.rows * s.n;
    return true;
}

static_assert(kPrologueMaxRows < kMmWideRows, "a prologue exists only where a workgroup owns one tile of rows");
const void* gemv_epilogue_kernel(int rows_of_h, bool with_prologue) {
    if (rows_of_h > 4) {
        if (with_prologue) {
            if (rows_of_h <= 8) return reinterpret_cast<const void*>(&k_gemm_mfma_epilogue<0, true>);
            if (rows_of_h <= 16) return reinterpret_cast<const void*>(&k_gemm_mfma_epilogue<1, true>);
            if (rows_of_h <= kPrologueMaxRows) return reinterpret_cast<const void*>(&k_gemm_mfma_epilogue<2, true>);
            return nullptr;
        }
        if (rows_of_h <= 8) return reinterpret_cast<const void*>(&k_gemm_mfma_epilogue<0>);
        if (rows_of_h <= 16) return reinterpret_cast<const void*>(&k_gemm_mfma_epilogue<1>);
        if (rows_of_h < kMmWideRows) return reinterpret_cast<const void*>(&k_gemm_mfma_epilogue<2>);
        return reinterpret_cast<const void*>(&k_gemm_mfma_epilogue<3>);
    }
    switch (rows_of_h * 2 + (with_prologue ? 1 : 0)) {
    case 2: return reinterpret_cast<const void*>(&k_gemv_epilogue<1, false>);
    case 3: return reinterpret_cast<const void*>(&k_gemv_epilogue<1, true>);
    case 4: return reinterpret_cast<const void*>(&k_gemv_epilogue<2, false>);
    case 5: return reinterpret_cast<const void*>(&k_gemv_epilogue<2, true>);
    case 6: return reinterpret_cast<const void*>(&k_gemv_epilogue<3, false>);
    case 7: return reinterpret_cast<const void*>(&k_gemv_epilogue<3, true>);
    case 8: return reinterpret_cast<const void*>(&k_gemv_epilogue<4, false>);
    case 9: return reinterpret_cast<const void*>(&k_gemv_epilogue<4, true>);
    default: return nullptr;
    }
}

const void* merged_kernel(int dtype, bool narrow) {
    if (dtype == kF32) return narrow ? reinterpret_cast<const void*>(&k_merged<float, 4>) : reinterpret_cast<const void*>(&k_merged<float, 16>);
    if (dtype == kBF16 && !narrow) return reinterpret_cast<const void*>(&k_merged<bf16_t, 16>);
    return nullptr;
}

const void* copy_kernel() { return reinterpret_cast<const void*>(&k_copy); }
const void* table_kernel() { return reinterpret_cast<const void*>(&k_table_write); }

}  // namespace pgk
