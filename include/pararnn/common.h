// Shared device helpers of the ParaRNN HIP library (gfx950 only).
#pragma once
#include <type_traits>
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace pararnn {

constexpr int kWave = 64;

// Device-side control block at the start of the workspace.
struct Ctrl {
    unsigned int ticket;     // next tile of the running launch
    unsigned int done;       // workgroups that finished the running launch
    unsigned int gmax_bits;  // max |delta| of the running iteration (fp32 bits, >= 0)
    int stop;                // set once the solve has ended; later launches return at once
    int iters;
    int status;
    unsigned int pad[2];
    int h_final;             // bf16 storage: the output already holds the final iterate (no conversion pass needed)
    unsigned int pad2[7];
};

// status values mirrored from pararnn.h (device code does not include it)
constexpr int kStOk = 0, kStNotConverged = 1, kStNonFinite = 5, kStInternal = 7;

// States of a carry record's tag (tag = epoch * 4 + state).
constexpr unsigned int kFlagAgg = 1;   // tile aggregate (A, b) published
constexpr unsigned int kFlagIncl = 2;  // inclusive value (delta at the tile's end) published
// default number of polls of one predecessor before a tile gives up (reports
// kStInternal, uses a zero carry) so that every wave terminates whatever happens:
// a poll is a memory round trip and a sleep, about a microsecond, so this is seconds,
// where a legitimate wait lasts at most the few milliseconds of a launch
constexpr unsigned int kSpinLimit = 1u << 21;

// ---------------------------------------------------------------- bf16 <-> fp32
__device__ __forceinline__ float bf16_to_f32(unsigned short v)
{
    return __uint_as_float(((unsigned int)v) << 16);
}

// round to nearest, ties to even; NaN stays NaN.  gfx950 converts in hardware
// (v_cvt_pk_bf16_f32, two values per instruction).
__device__ __forceinline__ unsigned short f32_to_bf16(float f)
{
    return __builtin_bit_cast(unsigned short, (__bf16)f);
}

// ------------------------------------------------------ vectors of VEC channels
template <int VEC> struct VecF;  // VEC fp32 values, loaded/stored as one access
template <> struct VecF<1> { using type = float; };
template <> struct VecF<2> { using type = float2; };
template <> struct VecF<4> { using type = float4; };
template <int VEC> struct VecH;  // VEC bf16 values
template <> struct VecH<1> { using type = unsigned short; };
template <> struct VecH<2> { using type = unsigned int; };
template <> struct VecH<4> { using type = uint2; };

template <int VEC>
__device__ __forceinline__ void load_vec(const float *p, float (&out)[VEC])
{
    typename VecF<VEC>::type v = *reinterpret_cast<const typename VecF<VEC>::type *>(p);
    const float *f = reinterpret_cast<const float *>(&v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) out[i] = f[i];
}

template <int VEC>
__device__ __forceinline__ void load_vec(const unsigned short *p, float (&out)[VEC])
{
    typename VecH<VEC>::type v = *reinterpret_cast<const typename VecH<VEC>::type *>(p);
    const unsigned short *s = reinterpret_cast<const unsigned short *>(&v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) out[i] = bf16_to_f32(s[i]);
}

template <int VEC>
__device__ __forceinline__ void store_vec(float *p, const float (&in)[VEC])
{
    typename VecF<VEC>::type v;
    float *f = reinterpret_cast<float *>(&v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) f[i] = in[i];
    *reinterpret_cast<typename VecF<VEC>::type *>(p) = v;
}

template <int VEC>
__device__ __forceinline__ void store_vec(unsigned short *p, const float (&in)[VEC])
{
    typename VecH<VEC>::type v;
    unsigned short *s = reinterpret_cast<unsigned short *>(&v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) s[i] = f32_to_bf16(in[i]);
    *reinterpret_cast<typename VecH<VEC>::type *>(p) = v;
}

// Raw (unconverted) vectors of VEC storage elements: loads are kept in this
// form and widened only where they are used, so that a batch of loads can be
// in flight together.
template <typename T, int VEC> struct RawVec;
template <int VEC> struct RawVec<float, VEC> { using type = typename VecF<VEC>::type; };
template <int VEC> struct RawVec<unsigned short, VEC> { using type = typename VecH<VEC>::type; };

template <typename T, int VEC>
__device__ __forceinline__ typename RawVec<T, VEC>::type load_raw(const T *p)
{
    return *reinterpret_cast<const typename RawVec<T, VEC>::type *>(p);
}

template <typename T, int VEC>
__device__ __forceinline__ typename RawVec<T, VEC>::type zero_raw()
{
    typename RawVec<T, VEC>::type z;
    unsigned char *b = reinterpret_cast<unsigned char *>(&z);
#pragma unroll
    for (unsigned i = 0; i < sizeof(z); ++i) b[i] = 0;
    return z;
}

template <typename T, int VEC>
__device__ __forceinline__ void raw_to_float(const typename RawVec<T, VEC>::type &r, float (&out)[VEC])
{
    const T *e = reinterpret_cast<const T *>(&r);
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        if constexpr (sizeof(T) == 4) out[i] = e[i];
        else out[i] = bf16_to_f32(e[i]);
    }
}

// Buffer-resource accesses: address = resource base (scalar) + per-lane byte
// offset (one VGPR for the whole tile) + scalar byte offset (one SGPR per row),
// so a batch of row loads needs no per-load vector address arithmetic.
typedef __amdgpu_buffer_rsrc_t buf_rsrc;

// Cache-policy bits of a buffer access (gfx950: 1 = sc0, 2 = nt, 16 = sc1).  nt marks a line as
// streamed: it is the first to leave the L2 and does not displace what the memory-side cache holds.
constexpr int kAuxNone = 0, kAuxStream = 2;

__device__ __forceinline__ buf_rsrc make_rsrc(const void *base)
{
    // raw buffer, no swizzle, whole 4 GiB window from base (tiles are far smaller)
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, 0xffffffffu, 0x27000);
}

template <typename T, int VEC, int AUX = kAuxNone>
__device__ __forceinline__ typename RawVec<T, VEC>::type buf_load(buf_rsrc r, unsigned int voff, unsigned int soff)
{
    using R = typename RawVec<T, VEC>::type;
    constexpr int BYTES = sizeof(T) * VEC;
    if constexpr (BYTES == 2) return __builtin_bit_cast(R, __builtin_amdgcn_raw_buffer_load_b16(r, voff, soff, AUX));
    else if constexpr (BYTES == 4) return __builtin_bit_cast(R, __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, AUX));
    else if constexpr (BYTES == 8) return __builtin_bit_cast(R, __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, AUX));
    else return __builtin_bit_cast(R, __builtin_amdgcn_raw_buffer_load_b128(r, voff, soff, AUX));
}

template <typename T, int VEC, int AUX = kAuxNone>
__device__ __forceinline__ void buf_store(buf_rsrc r, unsigned int voff, unsigned int soff, const float (&in)[VEC])
{
    using R = typename RawVec<T, VEC>::type;
    constexpr int BYTES = sizeof(T) * VEC;
    R v;
    T *e = reinterpret_cast<T *>(&v);
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        if constexpr (sizeof(T) == 4) e[i] = in[i];
        else e[i] = f32_to_bf16(in[i]);
    }
    if constexpr (BYTES == 2) __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(unsigned short, v), r, voff, soff, AUX);
    else if constexpr (BYTES == 4) __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(unsigned int, v), r, voff, soff, AUX);
    else if constexpr (BYTES == 8) {
        typedef unsigned int u2 __attribute__((ext_vector_type(2)));
        __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u2, v), r, voff, soff, AUX);
    } else {
        typedef unsigned int u4 __attribute__((ext_vector_type(4)));
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u4, v), r, voff, soff, AUX);
    }
}

// ------------------------------------------------------------------- fast math
// v_exp_f32 / v_rcp_f32 (1 ulp each).  Saturation is exact: exp2 -> 0 or inf,
// rcp(inf) = 0.
__device__ __forceinline__ float fast_sigmoid(float x)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * x));
}

__device__ __forceinline__ float fast_tanh(float x)
{
    // 1 - 2 / (1 + e^{2x}); absolute error ~1e-7 everywhere
    return 1.0f - 2.0f * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(2.8853900817779268f * x));
}

// Folded gate arithmetic, for kernels that evaluate a cell several times on the
// same u (the fused blocks): the gate input u + b is scaled once by the factor
// the exp2-based sigmoid / tanh needs, and the recurrent weights likewise, so
// that a gate costs one FMA, one exp2 and one rcp.  FOLD = false is the plain form.
constexpr float kSigFold = -1.4426950408889634f;    // sigmoid(x) = 1 / (1 + 2^(kSigFold x))
constexpr float kTanhFold = 2.8853900817779268f;    // tanh(x) = 1 - 2 / (1 + 2^(kTanhFold x))
template <bool FOLD> __device__ __forceinline__ float gate_sigmoid(float x)
{
    if constexpr (FOLD) return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(x));
    else return fast_sigmoid(x);
}
template <bool FOLD> __device__ __forceinline__ float gate_tanh(float x)
{
    if constexpr (FOLD) return fmaf(-2.0f, __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(x)), 1.0f);
    else return fast_tanh(x);
}
// w h + u + b, or in folded form wq h + u (u and wq pre-scaled, b inside u)
template <bool FOLD> __device__ __forceinline__ float gate_in(float w, float wq, float h, float u, float b)
{
    if constexpr (FOLD) return fmaf(wq, h, u);
    else return fmaf(w, h, u + b);
}

// Workgroup barrier that orders LDS accesses only: global loads and stores
// issued before it stay in flight (a full __syncthreads() waits for them).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Workgroup barrier for kernels that keep copies from memory into LDS in flight
// (buffer loads with an LDS destination): waits for this wave's own LDS
// instructions only and leaves every vector-memory operation outstanding.  The
// compiler sees an opaque memory clobber, so it moves no memory access across it;
// data another wave wrote to LDS with ordinary LDS instructions before its
// barrier is visible after it.
__device__ __forceinline__ void lds_barrier_keep_vmem()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Maximum of an unsigned value over the 64 lanes of a wave, returned wave-uniform
// (in scalar registers).  Four DPP butterfly steps make every row of 16 lanes
// uniform, then one lane of each row is read.  All lanes must be active.
__device__ __forceinline__ unsigned int wave_max_u32(unsigned int v)
{
    auto dpp = [](unsigned int x, auto ctrl) {
        return (unsigned int)__builtin_amdgcn_update_dpp(0, (int)x, decltype(ctrl)::value, 0xf, 0xf, false);
    };
    v = max(v, dpp(v, std::integral_constant<int, 0xB1>{}));     // quad_perm [1,0,3,2]
    v = max(v, dpp(v, std::integral_constant<int, 0x4E>{}));     // quad_perm [2,3,0,1]
    v = max(v, dpp(v, std::integral_constant<int, 0x141>{}));    // row_half_mirror
    v = max(v, dpp(v, std::integral_constant<int, 0x140>{}));    // row_mirror
    const unsigned int a = __builtin_amdgcn_readlane(v, 0), b = __builtin_amdgcn_readlane(v, 16);
    const unsigned int c = __builtin_amdgcn_readlane(v, 32), d = __builtin_amdgcn_readlane(v, 48);
    return max(max(a, b), max(c, d));
}

// max that keeps a NaN once seen (fmaxf would drop it)
__device__ __forceinline__ float nanmax(float m, float a) { return (a > m || a != a) ? a : m; }

}  // namespace pararnn
