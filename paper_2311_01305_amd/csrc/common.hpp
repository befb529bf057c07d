// Shared device/host helpers of libaweq (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>
#include <mutex>
#include <set>
#include <utility>

#include "aweq.h"

namespace aweq {

constexpr int kWave = 64;
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline int launch_status() { return hipGetLastError() == hipSuccess ? AWEQ_OK : AWEQ_ERR_LAUNCH; }
inline size_t dtype_size(aweq_dtype dt) { return dt == AWEQ_F32 ? 4 : (dt == AWEQ_F16 ? 2 : 1); }

constexpr int kXcdCount = 8;   // workgroup ids are dealt round-robin to the XCDs: id % 8 names the XCD

// ---------------------------------------------------------------- launch helpers (host)
// compute units of the current device, asked once per device
inline int device_cus(int& dev, int& cus)
{
    constexpr int kMaxDev = 64;
    static std::atomic<int> cached[kMaxDev];
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return AWEQ_ERR_LAUNCH;
    cus = cached[dev].load(std::memory_order_relaxed);
    if (cus == 0) {
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return AWEQ_ERR_LAUNCH;
        cached[dev].store(cus, std::memory_order_relaxed);
    }
    return AWEQ_OK;
}

// the dynamic LDS limit of a kernel is raised once per (kernel, device), not per launch
inline int raise_lds_limit(const void* fn, int dev, int bytes)
{
    static std::mutex mu;
    static std::set<std::pair<const void*, int>> done;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count({fn, dev})) return AWEQ_OK;
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) return AWEQ_ERR_LAUNCH;
    done.insert({fn, dev});
    return AWEQ_OK;
}

// K-panel layout of an int8 matrix [rows x K] (the GEMM operands): panel p holds bytes
// 64 p .. 64 p + 63 of every row, rows back to back; columns past K in the last panel are 0.
constexpr int kPanel = 64;
__host__ __device__ inline int64_t panel_count(int64_t K) { return (K + kPanel - 1) / kPanel; }
__host__ __device__ inline int64_t panel_offset(int64_t rows, int64_t r, int64_t k)
{
    return ((k / kPanel) * rows + r) * kPanel + (k % kPanel);
}

// ---------------------------------------------------------------- wavefront primitives
// Butterfly exchanges over the 64-lane wavefront.  Distances 1..8 are DPP modifiers that
// stay inside a row of 16 lanes, distance 16 is a ds_swizzle (no LDS traffic), distance 32
// swaps the two halves of the wavefront.

template <int CTRL>
__device__ __forceinline__ int dpp_mov(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xf, 0xf, false);
}

// value held by the partner lane at butterfly level LVL (0: xor 1 ... 5: xor 32).  Levels
// 2 and 3 use the mirror patterns, which pair the right lanes once levels below are done.
template <int LVL>
__device__ __forceinline__ int partner_bits(int v)
{
    if constexpr (LVL == 0) return dpp_mov<0xB1>(v);        // quad_perm [1,0,3,2]
    else if constexpr (LVL == 1) return dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
    else if constexpr (LVL == 2) return dpp_mov<0x141>(v);  // row_half_mirror
    else if constexpr (LVL == 3) return dpp_mov<0x140>(v);  // row_mirror
    else if constexpr (LVL == 4) return __builtin_amdgcn_ds_swizzle(v, 0x401F);  // xor 16
    else {
        // v_permlane32_swap: r[0] = lanes 0..31 of v in both halves, r[1] = lanes 32..63 in both
        auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
        return (threadIdx.x & 32) ? (int)r[0] : (int)r[1];
    }
}

// value of lane l ^ 8 with no assumption about lower levels (row_ror:8 inside a row of 16)
__device__ __forceinline__ int xor8_bits(int v) { return dpp_mov<0x128>(v); }
__device__ __forceinline__ float xor8(float v) { return __int_as_float(xor8_bits(__float_as_int(v))); }
__device__ __forceinline__ int xor8(int v) { return xor8_bits(v); }

template <int LVL>
__device__ __forceinline__ float partner(float v)
{
    return __int_as_float(partner_bits<LVL>(__float_as_int(v)));
}
template <int LVL>
__device__ __forceinline__ int partner(int v) { return partner_bits<LVL>(v); }
template <int LVL>
__device__ __forceinline__ double partner(double v)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    return __hiloint2double(partner_bits<LVL>(hi), partner_bits<LVL>(lo));
}
template <int LVL>
__device__ __forceinline__ long long partner(long long v)
{
    int lo = (int)(v & 0xffffffffll), hi = (int)(v >> 32);
    lo = partner_bits<LVL>(lo);
    hi = partner_bits<LVL>(hi);
    return ((long long)hi << 32) | (unsigned int)lo;
}

struct OpMin { template <class T> __device__ T operator()(T a, T b) const { return a < b ? a : b; } };
struct OpMax { template <class T> __device__ T operator()(T a, T b) const { return a > b ? a : b; } };
struct OpAdd { template <class T> __device__ T operator()(T a, T b) const { return a + b; } };

// All-reduce over aligned groups of 2^LEVELS lanes (LEVELS = 6: the whole wavefront).
// The mirror levels assume all lower levels ran, which holds because levels run in order.
template <int LEVELS, class T, class Op>
__device__ __forceinline__ T group_allreduce(T v, Op op)
{
    if constexpr (LEVELS > 0) v = op(v, partner<0>(v));
    if constexpr (LEVELS > 1) v = op(v, partner<1>(v));
    if constexpr (LEVELS > 2) v = op(v, partner<2>(v));
    if constexpr (LEVELS > 3) v = op(v, partner<3>(v));
    if constexpr (LEVELS > 4) v = op(v, partner<4>(v));
    if constexpr (LEVELS > 5) v = op(v, partner<5>(v));
    return v;
}

template <class T, class Op>
__device__ __forceinline__ T wave_allreduce(T v, Op op) { return group_allreduce<6>(v, op); }

// Block all-reduce for blocks of NW wavefronts: wavefront results meet in LDS.
// `slot` must hold NW elements of T; contains two barriers, so every thread must call it.
template <int NW, class T, class Op>
__device__ __forceinline__ T block_allreduce(T v, Op op, T* slot)
{
    v = wave_allreduce(v, op);
    const int w = threadIdx.x / kWave;
    __syncthreads();
    if ((threadIdx.x & (kWave - 1)) == 0) slot[w] = v;
    __syncthreads();
    T r = slot[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r = op(r, slot[i]);
    return r;
}

// ------------------------------------------------------------------ quantizer (Eq. 1-2)
// round-half-even to int32, saturated at +-2^30, flagging |q| >= 2^24
__device__ __forceinline__ int rint_sat(float q, uint32_t& st)
{
    float r = rintf(q);
    if (!(fabsf(r) < 16777216.0f)) st |= AWEQ_ST_BIGQUOT;
    r = fminf(fmaxf(r, -1073741824.0f), 1073741824.0f);  // NaN -> -2^30 is never reached for finite input
    return (int)r;
}

// Eq. 2 and the zero point for a slice with extremes lo, hi
__device__ __forceinline__ void qparams(float lo, float hi, int bits, float& step, int& zero, uint32_t& st)
{
    float range = hi - lo;
    float levels = (float)((1 << bits) - 1);
    float sp = range / levels;
    if (!(sp > 0.0f) || isinf(sp)) { sp = 1.0f; st |= AWEQ_ST_DEGENERATE; }
    step = sp;
    zero = -rint_sat(lo / sp, st);
}

// Eq. 1 with a true division
__device__ __forceinline__ int quant_div(float x, float step, int zero, int qmax, uint32_t& st)
{
    int u = rint_sat(x / step, st) + zero;
    return min(max(u, 0), qmax);
}

// Constants of the static int8 activation quantizer (Eq. 1 with b = 8) for the division-free
// paths: `fast` = the exact two-correction quotient is valid for binary16 inputs, `screen` = the
// one-FMA quotient with its distance-to-tie test is (both are explained where they are used, in
// the activation quantizer).
struct ActParams {
    float step, rstep, lo_f, hi_f, thr;
    int zero, zoff;
    bool fast, screen;
};

__device__ __forceinline__ ActParams act_params(const float* act_step, const int32_t* act_zero, bool f16)
{
    ActParams p;
    p.step = *act_step;
    p.zero = *act_zero;
    p.rstep = 1.0f / p.step;
    const uint32_t b = __float_as_uint(p.step);
    const int e = (int)((b >> 23) & 0xff) - 127;
    const uint32_t m = b & 0x7fffffu;
    p.fast = f16 && (b >> 31) == 0 && e >= -60 && e <= 60 && m < 0x7ffff0u && p.zero > -(1 << 23) && p.zero < (1 << 23);
    // screened quotient: |Z| small enough for delta to stay far below 1/2
    const int az = p.zero < 0 ? -p.zero : p.zero;
    p.screen = p.fast && az <= 4096;
    p.thr = 0.5f - ((float)(258 + (az <= 4096 ? az : 0)) * 1.1920928955078125e-07f + 3.0517578125e-05f);
    p.lo_f = (float)(-p.zero);
    p.hi_f = (float)(255 - p.zero);
    p.zoff = p.zero - 128;
    return p;
}

__device__ __forceinline__ void raise_status(uint32_t* status, uint32_t st)
{
    if (status && st) atomicOr(status, st);
}

// 8 binary16 values in one 16-byte register quad
struct alignas(16) Half8 { f16x2 h[4]; };
__device__ __forceinline__ float2 h2f2(f16x2 v) { return make_float2((float)v.x, (float)v.y); }
__device__ __forceinline__ f16x2 hmin2(f16x2 a, f16x2 b) { return __builtin_elementwise_min(a, b); }
__device__ __forceinline__ f16x2 hmax2(f16x2 a, f16x2 b) { return __builtin_elementwise_max(a, b); }
struct alignas(16) Float4 { float f[4]; };

// An fp32 result that is about to be rounded to binary16.  hipcc merges an fp32 multiply and the
// conversion of its product into one v_fma_mixlo_f16, and that instruction rounds the exact
// product once; Eq. 3's fold is defined with two roundings (fp32 product, then the weight's
// type), which differ in about one element per 10^7.  Passing the product through a register
// the compiler cannot see into keeps the two steps apart.
__device__ __forceinline__ float rounded_f32(float v)
{
    asm volatile("" : "+v"(v));
    return v;
}

}  // namespace aweq
