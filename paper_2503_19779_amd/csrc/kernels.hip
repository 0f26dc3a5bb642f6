// kernels.hip -- the chain's device code for gfx950 (wave64): elementwise add / mul / GELU,
// RMSNorm, GEMV, per-channel scale + bias + ReLU, the batched multi-tensor copy and the
// pointer-table writer.
//
// Every compute kernel exists in a direct form (operands are tensor addresses) and in indirect
// forms (an operand is the address of a pointer-table slot that the kernel dereferences first;
// paper, Sec. 3 "Parameter Indirection" and Sec. 4 "Kernel generation": the body is unchanged,
// only a dereference prologue is added).  All forms of a kernel are instantiations of one body
// with one launch shape, so every replay mode computes bit-identical results.  The translation
// unit is built with -ffp-contract=off: fused multiply-adds appear only where written.
#include "kernels.h"

namespace pgk {
namespace {

constexpr int kBlock = 256;   // threads per workgroup = 4 waves of 64
constexpr int kUnroll = 4;    // 16-byte vectors per thread kept in flight

// ---- operand resolution -------------------------------------------------------------------
template <bool IND>
__device__ __forceinline__ const void* resolve(const void* p) {
    if constexpr (IND) {
        return *reinterpret_cast<const void* const*>(p);   // uniform address: one scalar load
    } else {
        return p;
    }
}

__device__ __forceinline__ bool aligned16(const void* p) {
    return (reinterpret_cast<uintptr_t>(p) & 15u) == 0;
}

// ---- storage formats ------------------------------------------------------------------------
__device__ __forceinline__ float bf16_to_f32(unsigned b) { return __uint_as_float(b << 16); }

// round to nearest, ties to even; NaN stays a quiet NaN
__device__ __forceinline__ unsigned f32_to_bf16(float f) {
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    u += 0x7fffu + ((u >> 16) & 1u);
    return u >> 16;
}

typedef unsigned short bf16_t;

template <typename T> struct Fmt;
template <> struct Fmt<float> {
    static constexpr int N = 4;   // elements per 16-byte vector
    static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
        f[0] = __uint_as_float(r.x); f[1] = __uint_as_float(r.y);
        f[2] = __uint_as_float(r.z); f[3] = __uint_as_float(r.w);
    }
    static __device__ __forceinline__ uint4 pack(const float* f) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Fmt<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(const uint4& r, float* f) {
        f[0] = __uint_as_float(r.x << 16); f[1] = __uint_as_float(r.x & 0xffff0000u);
        f[2] = __uint_as_float(r.y << 16); f[3] = __uint_as_float(r.y & 0xffff0000u);
        f[4] = __uint_as_float(r.z << 16); f[5] = __uint_as_float(r.z & 0xffff0000u);
        f[6] = __uint_as_float(r.w << 16); f[7] = __uint_as_float(r.w & 0xffff0000u);
    }
    static __device__ __forceinline__ uint4 pack(const float* f) {
        return make_uint4(f32_to_bf16(f[0]) | (f32_to_bf16(f[1]) << 16), f32_to_bf16(f[2]) | (f32_to_bf16(f[3]) << 16),
                          f32_to_bf16(f[4]) | (f32_to_bf16(f[5]) << 16), f32_to_bf16(f[6]) | (f32_to_bf16(f[7]) << 16));
    }
    static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = (bf16_t)f32_to_bf16(v); }
};

template <typename T> __device__ __forceinline__ uint4 ld16(const T* p) { return *reinterpret_cast<const uint4*>(p); }
template <typename T> __device__ __forceinline__ void st16(T* p, const uint4& v) { *reinterpret_cast<uint4*>(p) = v; }

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

// ---- elementwise ----------------------------------------------------------------------------
// GELU(a) = a * Phi(a) with Phi(a) = erfc(-a / sqrt 2) / 2 (keeps relative accuracy in the left
// tail).  For fp32 tensors it is evaluated in fp64 and rounded once, so that the result is the
// correctly rounded one except within ~1e-16 of a rounding boundary: an fp32 erfc is a few ulp off,
// and a chain of multiplies and cancelling adds amplifies that beyond 1e-5.  For bf16 tensors fp32
// is far more than the 8 stored bits need.
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
        return (0.5f * a) * erfcf(a * -0.70710678118654752440f);
    }
}

template <typename T, int OP, typename IdxT>
__device__ __forceinline__ void ew_body(const T* a, const T* __restrict__ b, T* o, IdxT n, IdxT m) {   // o may alias a
    constexpr int N = Fmt<T>::N;
    constexpr bool kBinary = (OP != kGelu);
    const bool vec_ok = aligned16(a) && aligned16(o) && (!kBinary || (aligned16(b) && (m % N) == 0));
    if (vec_ok) {
        const IdxT nvec = n / N;
        const IdxT base = (IdxT)blockIdx.x * (kBlock * kUnroll) + threadIdx.x;
        uint4 ra[kUnroll], rb[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; u++) {
            const IdxT v = base + (IdxT)u * kBlock;
            if (v < nvec) {
                ra[u] = ld16(a + v * N);
                if constexpr (kBinary) {
                    const IdxT bi = (m == n) ? v * N : (v * N) % m;
                    rb[u] = ld16(b + bi);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; u++) {
            const IdxT v = base + (IdxT)u * kBlock;
            if (v < nvec) {
                float fa[N], fb[N], fo[N];
                Fmt<T>::unpack(ra[u], fa);
                if constexpr (kBinary) Fmt<T>::unpack(rb[u], fb);
#pragma unroll
                for (int e = 0; e < N; e++) fo[e] = ew_apply<OP, sizeof(T) == 4>(fa[e], kBinary ? fb[e] : 0.f);
                st16(o + v * N, Fmt<T>::pack(fo));
            }
        }
        if (blockIdx.x == nvec / (kBlock * kUnroll)) {   // fewer than N trailing elements: the block that owns vector index nvec
            const IdxT i = nvec * N + threadIdx.x;
            if (i < n) {
                const float fb1 = kBinary ? Fmt<T>::load(b + (i % m)) : 0.f;
                Fmt<T>::store(o + i, ew_apply<OP, sizeof(T) == 4>(Fmt<T>::load(a + i), fb1));
            }
        }
    } else {
        const IdxT tile = (IdxT)kBlock * kUnroll * N;
        const IdxT start = (IdxT)blockIdx.x * tile;
        const IdxT end = (n - start < tile) ? n : start + tile;
        for (IdxT i = start + threadIdx.x; i < end; i += kBlock) {
            const float fb1 = kBinary ? Fmt<T>::load(b + (i % m)) : 0.f;
            Fmt<T>::store(o + i, ew_apply<OP, sizeof(T) == 4>(Fmt<T>::load(a + i), fb1));
        }
    }
}

template <typename T, int OP, int IND>
__global__ __launch_bounds__(kBlock) void k_elementwise(EwArgs p) {
    const T* a = static_cast<const T*>(resolve<(IND & 1) != 0>(p.a));
    const T* b = (OP != kGelu) ? static_cast<const T*>(resolve<(IND & 2) != 0>(p.b)) : nullptr;
    T* o = static_cast<T*>(p.out);
    if (p.n < (1ll << 31)) {
        ew_body<T, OP, unsigned>(a, b, o, (unsigned)p.n, (unsigned)p.m);
    } else {
        ew_body<T, OP, unsigned long long>(a, b, o, (unsigned long long)p.n, (unsigned long long)p.m);
    }
}

// ---- per-channel scale + bias + ReLU on [N, C, inner] ---------------------------------------
__device__ __forceinline__ float sbr_apply(float x, float s, float b) {
    const float v = __builtin_fmaf(x, s, b);
    return v > 0.f ? v : 0.f;
}

template <typename T, typename IdxT>
__device__ __forceinline__ void sbr_body(const T* x /* o may alias x */, const T* __restrict__ s, const T* __restrict__ b, T* o,
                                         IdxT n, unsigned inner, unsigned channels) {
    constexpr int N = Fmt<T>::N;
    const bool vec_ok = aligned16(x) && aligned16(o) && (inner % N) == 0;
    if (vec_ok) {
        const IdxT nvec = n / N;   // n is a multiple of inner, hence of N
        const IdxT base = (IdxT)blockIdx.x * (kBlock * kUnroll) + threadIdx.x;
        uint4 rx[kUnroll];
        float fs[kUnroll], fbv[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; u++) {
            const IdxT v = base + (IdxT)u * kBlock;
            if (v < nvec) {
                rx[u] = ld16(x + v * N);
                const unsigned c = (unsigned)(((v * N) / inner) % channels);
                fs[u] = Fmt<T>::load(s + c);
                fbv[u] = Fmt<T>::load(b + c);
            }
        }
#pragma unroll
        for (int u = 0; u < kUnroll; u++) {
            const IdxT v = base + (IdxT)u * kBlock;
            if (v < nvec) {
                float fx[N], fo[N];
                Fmt<T>::unpack(rx[u], fx);
#pragma unroll
                for (int e = 0; e < N; e++) fo[e] = sbr_apply(fx[e], fs[u], fbv[u]);
                st16(o + v * N, Fmt<T>::pack(fo));
            }
        }
    } else {
        const IdxT tile = (IdxT)kBlock * kUnroll * N;
        const IdxT start = (IdxT)blockIdx.x * tile;
        const IdxT end = (n - start < tile) ? n : start + tile;
        for (IdxT i = start + threadIdx.x; i < end; i += kBlock) {
            const unsigned c = (unsigned)((i / inner) % channels);
            Fmt<T>::store(o + i, sbr_apply(Fmt<T>::load(x + i), Fmt<T>::load(s + c), Fmt<T>::load(b + c)));
        }
    }
}

template <typename T, int IND>
__global__ __launch_bounds__(kBlock) void k_scale_bias_relu(SbrArgs p) {
    const T* x = static_cast<const T*>(resolve<(IND & 1) != 0>(p.x));
    const T* s = static_cast<const T*>(resolve<(IND & 2) != 0>(p.s));
    const T* b = static_cast<const T*>(resolve<(IND & 4) != 0>(p.b));
    T* o = static_cast<T*>(p.out);
    if (p.n < (1ll << 31)) {
        sbr_body<T, unsigned>(x, s, b, o, (unsigned)p.n, p.inner, p.channels);
    } else {
        sbr_body<T, unsigned long long>(x, s, b, o, (unsigned long long)p.n, p.inner, p.channels);
    }
}

// ---- RMSNorm: one workgroup per row ------------------------------------------------------------
// Sum of squares: each thread accumulates its elements with fused multiply-adds, a wave64
// shuffle reduction follows, the four wave sums are staged through LDS and added in a fixed
// order by every thread.  Up to kKeep vectors per thread stay in registers between the two
// passes (hidden <= 8192 for bf16), longer rows are read again.
template <typename T, int IND>
__global__ __launch_bounds__(kBlock) void k_rmsnorm(RmsArgs p) {
    constexpr int N = Fmt<T>::N;
    constexpr int kKeep = 4;
    const int cols = p.cols;
    const size_t row = blockIdx.x;
    const T* __restrict__ x = static_cast<const T*>(resolve<(IND & 1) != 0>(p.x)) + row * cols;
    const T* __restrict__ g = static_cast<const T*>(resolve<(IND & 2) != 0>(p.g));
    T* o = static_cast<T*>(p.out) + row * cols;
    const int tid = threadIdx.x;
    const bool vec_ok = aligned16(x) && aligned16(g) && aligned16(o) && (cols % N) == 0;
    const int nvec = cols / N;
    uint4 keep[kKeep];
    float acc = 0.f;
    if (vec_ok) {
#pragma unroll
        for (int u = 0; u < kKeep; u++) {
            const int v = tid + u * kBlock;
            if (v < nvec) keep[u] = ld16(x + (size_t)v * N);
        }
#pragma unroll
        for (int u = 0; u < kKeep; u++) {
            const int v = tid + u * kBlock;
            if (v < nvec) {
                float f[N];
                Fmt<T>::unpack(keep[u], f);
#pragma unroll
                for (int e = 0; e < N; e++) acc = __builtin_fmaf(f[e], f[e], acc);
            }
        }
        for (int v = tid + kKeep * kBlock; v < nvec; v += kBlock) {
            float f[N];
            Fmt<T>::unpack(ld16(x + (size_t)v * N), f);
#pragma unroll
            for (int e = 0; e < N; e++) acc = __builtin_fmaf(f[e], f[e], acc);
        }
    } else {
        for (int i = tid; i < cols; i += kBlock) {
            const float f = Fmt<T>::load(x + i);
            acc = __builtin_fmaf(f, f, acc);
        }
    }
    acc = wave_sum(acc);
    __shared__ float part[kBlock / 64];
    if ((tid & 63) == 0) part[tid >> 6] = acc;
    __syncthreads();
    const float total = ((part[0] + part[1]) + part[2]) + part[3];
    const float scale = 1.0f / sqrtf(total / (float)cols + p.eps);
    if (vec_ok) {
#pragma unroll
        for (int u = 0; u < kKeep; u++) {
            const int v = tid + u * kBlock;
            if (v < nvec) {
                float f[N], fg[N], fo[N];
                Fmt<T>::unpack(keep[u], f);
                Fmt<T>::unpack(ld16(g + (size_t)v * N), fg);
#pragma unroll
                for (int e = 0; e < N; e++) fo[e] = (f[e] * scale) * fg[e];
                st16(o + (size_t)v * N, Fmt<T>::pack(fo));
            }
        }
        for (int v = tid + kKeep * kBlock; v < nvec; v += kBlock) {
            float f[N], fg[N], fo[N];
            Fmt<T>::unpack(ld16(x + (size_t)v * N), f);
            Fmt<T>::unpack(ld16(g + (size_t)v * N), fg);
#pragma unroll
            for (int e = 0; e < N; e++) fo[e] = (f[e] * scale) * fg[e];
            st16(o + (size_t)v * N, Fmt<T>::pack(fo));
        }
    } else {
        for (int i = tid; i < cols; i += kBlock)
            Fmt<T>::store(o + i, (Fmt<T>::load(x + i) * scale) * Fmt<T>::load(g + i));
    }
}

// ---- GEMV: one wave per output column, rows of h in blocks of kRowBlock ------------------------
// Memory-bound: the weight row is streamed once with 16-byte loads (four per lane in flight for
// 2048 columns), multiplied into fp32 accumulators, and reduced across the wave.  No MFMA: at
// batch 1 there is no reuse to feed a matrix core.
constexpr int kRowBlock = 4;

template <typename T, int IND>
__global__ __launch_bounds__(kBlock) void k_gemv(GemvArgs p) {
    constexpr int N = Fmt<T>::N;
    const T* __restrict__ W = static_cast<const T*>(resolve<(IND & 1) != 0>(p.W));
    const T* __restrict__ h = static_cast<const T*>(resolve<(IND & 2) != 0>(p.h));
    T* y = static_cast<T*>(p.out);
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    if (j >= p.n) return;   // whole wave leaves together
    const int cols = p.cols, rows = p.rows;
    const T* wrow = W + (size_t)j * cols;
    const bool vec_ok = aligned16(W) && aligned16(h) && (cols % N) == 0;
    const int nvec = cols / N;
    for (int r0 = 0; r0 < rows; r0 += kRowBlock) {
        float acc[kRowBlock];
#pragma unroll
        for (int rr = 0; rr < kRowBlock; rr++) acc[rr] = 0.f;
        if (vec_ok) {
            for (int v0 = 0; v0 < nvec; v0 += 64 * kUnroll) {
                uint4 rw[kUnroll];
#pragma unroll
                for (int u = 0; u < kUnroll; u++) {
                    const int v = v0 + u * 64 + lane;
                    if (v < nvec) rw[u] = ld16(wrow + (size_t)v * N);
                }
#pragma unroll
                for (int rr = 0; rr < kRowBlock; rr++) {
                    if (r0 + rr < rows) {
                        const T* hrow = h + (size_t)(r0 + rr) * cols;
                        uint4 rh[kUnroll];
#pragma unroll
                        for (int u = 0; u < kUnroll; u++) {
                            const int v = v0 + u * 64 + lane;
                            if (v < nvec) rh[u] = ld16(hrow + (size_t)v * N);
                        }
#pragma unroll
                        for (int u = 0; u < kUnroll; u++) {
                            const int v = v0 + u * 64 + lane;
                            if (v < nvec) {
                                float fw[N], fh[N];
                                Fmt<T>::unpack(rw[u], fw);
                                Fmt<T>::unpack(rh[u], fh);
#pragma unroll
                                for (int e = 0; e < N; e++) acc[rr] = __builtin_fmaf(fw[e], fh[e], acc[rr]);
                            }
                        }
                    }
                }
            }
        } else {
            for (int i = lane; i < cols; i += 64) {
                const float fw = Fmt<T>::load(wrow + i);
#pragma unroll
                for (int rr = 0; rr < kRowBlock; rr++)
                    if (r0 + rr < rows) acc[rr] = __builtin_fmaf(fw, Fmt<T>::load(h + (size_t)(r0 + rr) * cols + i), acc[rr]);
            }
        }
#pragma unroll
        for (int rr = 0; rr < kRowBlock; rr++) {
            const float s = wave_sum(acc[rr]);
            if (lane == 0 && r0 + rr < rows) Fmt<T>::store(y + (size_t)(r0 + rr) * p.n + j, s);
        }
    }
}

// ---- batched multi-tensor copy -----------------------------------------------------------------
// One workgroup per chunk (<= kCopyChunkBytes of one tensor).  Destinations are placeholders the
// library laid out itself (256-byte aligned, chunk offsets multiples of the chunk size), so only
// the source alignment varies: 16-byte aligned sources take 128-bit loads and stores with eight
// vectors per lane in flight; others fall back to 4-byte or 2-byte moves.
constexpr int kCopyUnroll = 8;
typedef unsigned v4u __attribute__((ext_vector_type(4)));

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

template <typename T, int OP>
const void* ew_variant(int ind) {
    switch (ind) {
    case 0: return reinterpret_cast<const void*>(&k_elementwise<T, OP, 0>);
    case 1: return reinterpret_cast<const void*>(&k_elementwise<T, OP, 1>);
    case 2: return OP == kGelu ? nullptr : reinterpret_cast<const void*>(&k_elementwise<T, OP, 2>);
    case 3: return OP == kGelu ? nullptr : reinterpret_cast<const void*>(&k_elementwise<T, OP, 3>);
    default: return nullptr;
    }
}
template <typename T>
const void* rms_variant(int ind) {
    switch (ind) {
    case 0: return reinterpret_cast<const void*>(&k_rmsnorm<T, 0>);
    case 1: return reinterpret_cast<const void*>(&k_rmsnorm<T, 1>);
    case 2: return reinterpret_cast<const void*>(&k_rmsnorm<T, 2>);
    case 3: return reinterpret_cast<const void*>(&k_rmsnorm<T, 3>);
    default: return nullptr;
    }
}
template <typename T>
const void* gemv_variant(int ind) {
    switch (ind) {
    case 0: return reinterpret_cast<const void*>(&k_gemv<T, 0>);
    case 1: return reinterpret_cast<const void*>(&k_gemv<T, 1>);
    case 2: return reinterpret_cast<const void*>(&k_gemv<T, 2>);
    case 3: return reinterpret_cast<const void*>(&k_gemv<T, 3>);
    default: return nullptr;
    }
}
template <typename T>
const void* sbr_variant(int ind) {
    switch (ind) {
    case 0: return reinterpret_cast<const void*>(&k_scale_bias_relu<T, 0>);
    case 1: return reinterpret_cast<const void*>(&k_scale_bias_relu<T, 1>);
    case 2: return reinterpret_cast<const void*>(&k_scale_bias_relu<T, 2>);
    case 3: return reinterpret_cast<const void*>(&k_scale_bias_relu<T, 3>);
    case 4: return reinterpret_cast<const void*>(&k_scale_bias_relu<T, 4>);
    case 5: return reinterpret_cast<const void*>(&k_scale_bias_relu<T, 5>);
    case 6: return reinterpret_cast<const void*>(&k_scale_bias_relu<T, 6>);
    case 7: return reinterpret_cast<const void*>(&k_scale_bias_relu<T, 7>);
    default: return nullptr;
    }
}

template <typename T>
const void* kernel_for_t(int op, int ind) {
    switch (op) {
    case kAdd: return ew_variant<T, kAdd>(ind);
    case kMul: return ew_variant<T, kMul>(ind);
    case kGelu: return ew_variant<T, kGelu>(ind);
    case kRmsNorm: return rms_variant<T>(ind);
    case kGemv: return gemv_variant<T>(ind);
    case kScaleBiasRelu: return sbr_variant<T>(ind);
    default: return nullptr;
    }
}

}  // namespace

const void* kernel_for(int op, int dtype, int ind_mask) {
    if (dtype == kF32) return kernel_for_t<float>(op, ind_mask);
    if (dtype == kBF16) return kernel_for_t<bf16_t>(op, ind_mask);
    return nullptr;
}
const void* copy_kernel() { return reinterpret_cast<const void*>(&k_copy); }
const void* table_kernel() { return reinterpret_cast<const void*>(&k_table_write); }

static unsigned blocks_for(long long n, long long per_block) {
    long long g = (n + per_block - 1) / per_block;
    return (unsigned)(g < 1 ? 1 : g);
}
void shape_elementwise(int dtype, long long n, dim3* grid, dim3* block) {
    const int N = dtype == kF32 ? 4 : 8;
    *grid = dim3(blocks_for(n, (long long)kBlock * kUnroll * N));
    *block = dim3(kBlock);
}
void shape_sbr(int dtype, long long n, dim3* grid, dim3* block) { shape_elementwise(dtype, n, grid, block); }
void shape_rmsnorm(int rows, dim3* grid, dim3* block) {
    *grid = dim3((unsigned)rows);
    *block = dim3(kBlock);
}
void shape_gemv(int /*rows*/, int n, dim3* grid, dim3* block) {
    *grid = dim3(blocks_for(n, kBlock / 64));
    *block = dim3(kBlock);
}

}  // namespace pgk
