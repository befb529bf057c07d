// Stage 3: asymmetric round-to-nearest weight quantizer (Sec. 2, Eq. 1-2) with the three
// storage formats (int8, packed 4-bit, packed 3-bit).
//
// HBM-bound: each weight is read once and its code written once.  A thread owns "units" of
// 8 consecutive k (16 bytes of binary16, 32 bytes of binary32).  Per-row slices keep the
// whole row in registers between the min/max reduction and the quantization; per-group
// slices are 2^m lanes wide and reduce with DPP butterflies only.
#include "common.hpp"

namespace aweq {

constexpr int kQwBlock = 256;
constexpr int kQwMaxUnits = 12;  // units per thread held in registers: K <= 256 * 8 * 12 = 24576

template <bool F16>
struct Unit;

template <>
struct Unit<true> {
    Half8 raw;
    __device__ __forceinline__ void load(const void* row, int64_t u)
    {
        raw = *reinterpret_cast<const Half8*>(reinterpret_cast<const _Float16*>(row) + u * 8);
    }
    __device__ __forceinline__ void get(float x[8]) const
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float2 f = h2f2(raw.h[i]);
            x[2 * i] = f.x;
            x[2 * i + 1] = f.y;
        }
    }
    // round to binary16 and keep
    __device__ __forceinline__ void set(const float x[8])
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) raw.h[i] = f16x2{(_Float16)x[2 * i], (_Float16)x[2 * i + 1]};
    }
    __device__ __forceinline__ void store(void* row, int64_t u) const
    {
        *reinterpret_cast<Half8*>(reinterpret_cast<_Float16*>(row) + u * 8) = raw;
    }
};

template <>
struct Unit<false> {
    Float4 raw[2];
    __device__ __forceinline__ void load(const void* row, int64_t u)
    {
        const float* p = reinterpret_cast<const float*>(row) + u * 8;
        raw[0] = *reinterpret_cast<const Float4*>(p);
        raw[1] = *reinterpret_cast<const Float4*>(p + 4);
    }
    __device__ __forceinline__ void get(float x[8]) const
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) { x[i] = raw[0].f[i]; x[4 + i] = raw[1].f[i]; }
    }
    __device__ __forceinline__ void set(const float x[8])
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) { raw[0].f[i] = x[i]; raw[1].f[i] = x[4 + i]; }
    }
    __device__ __forceinline__ void store(void* row, int64_t u) const
    {
        float* p = reinterpret_cast<float*>(row) + u * 8;
        *reinterpret_cast<Float4*>(p) = raw[0];
        *reinterpret_cast<Float4*>(p + 4) = raw[1];
    }
};

__device__ __forceinline__ void minmax8(const float x[8], float& lo, float& hi)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) { lo = fminf(lo, x[i]); hi = fmaxf(hi, x[i]); }
}

// Quantise one unit and store its codes in the format of `bits`.  `row_codes` points at the
// start of the row's code bytes, u is the unit index inside the row (bits == 8: the unit sits
// at row_codes + unit_off, which lets the caller pick the layout).  Returns sum (u - 128)
// (meaningful for bits == 8).  For bits == 3 all four lanes of a quad must call this with
// consecutive units (u % 4 == lane % 4).
template <int BITS>
__device__ __forceinline__ int quant_store_unit(const float x[8], float step, int zero, uint8_t* row_codes,
                                                int64_t u, uint32_t& st, int64_t unit_off = -1)
{
    constexpr int qmax = (1 << BITS) - 1;
    int c[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) c[i] = quant_div(x[i], step, zero, qmax, st);
    if constexpr (BITS == 8) {
        int rs = 0;
        uint32_t w0 = 0, w1 = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            w0 |= (uint32_t)((c[i] - 128) & 0xff) << (8 * i);
            w1 |= (uint32_t)((c[4 + i] - 128) & 0xff) << (8 * i);
            rs += c[i] + c[4 + i] - 256;
        }
        *reinterpret_cast<uint2*>(row_codes + (unit_off >= 0 ? unit_off : u * 8)) = make_uint2(w0, w1);
        return rs;
    } else if constexpr (BITS == 4) {
        uint32_t w = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) w |= (uint32_t)c[i] << (4 * i);
        *reinterpret_cast<uint32_t*>(row_codes + u * 4) = w;
        return 0;
    } else {
        // 8 codes = 24 bits; four neighbouring lanes hold 96 bits = three dwords
        uint32_t v = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) v |= (uint32_t)c[i] << (3 * i);
        const uint32_t v0 = (uint32_t)dpp_mov<0x00>((int)v);  // quad_perm [0,0,0,0]
        const uint32_t v1 = (uint32_t)dpp_mov<0x55>((int)v);  // [1,1,1,1]
        const uint32_t v2 = (uint32_t)dpp_mov<0xAA>((int)v);  // [2,2,2,2]
        const uint32_t v3 = (uint32_t)dpp_mov<0xFF>((int)v);  // [3,3,3,3]
        const int q = threadIdx.x & 3;
        const uint32_t d = q == 0 ? (v0 | (v1 << 24)) : (q == 1 ? ((v1 >> 8) | (v2 << 16)) : ((v2 >> 16) | (v3 << 8)));
        if (q < 3) *reinterpret_cast<uint32_t*>(row_codes + (u >> 2) * 12 + q * 4) = d;
        return 0;
    }
}

// ---- one (Step, Z) per row, or one for the tensor (PER_TENSOR: read from step[0]/zero[0]).
// 8-bit codes are the GEMM's weight operand and go out in its K-panel layout.
// FOLD: the row read is the un-equalised W; it is multiplied by s[k] (one fp32 multiply, rounded to
// the weight's type: Eq. 3), written to W_hat and quantised from registers, so W is read once.
template <bool F16, int BITS, bool PER_TENSOR, bool FOLD = false>
__global__ __launch_bounds__(kQwBlock) void quant_weight_row(
    const void* __restrict__ W, int64_t K, int64_t ldw, uint8_t* __restrict__ codes,
    float* __restrict__ step, int32_t* __restrict__ zero, int32_t* __restrict__ rowsum_w, uint32_t* status,
    const float* __restrict__ s = nullptr, void* __restrict__ W_hat = nullptr, int64_t ldwh = 0)
{
    __shared__ float slot_f[kQwBlock / kWave];
    __shared__ int slot_i[kQwBlock / kWave];
    const int64_t n = blockIdx.x;
    const int64_t N = gridDim.x;
    const int64_t units = K / 8;
    const char* row = reinterpret_cast<const char*>(W) + (size_t)n * ldw * (F16 ? 2 : 4);
    uint8_t* row_codes = BITS == 8 ? codes + (size_t)n * kPanel : codes + (size_t)n * (K * BITS / 8);
    uint32_t st = 0;

    Unit<F16> reg[kQwMaxUnits];
    float lo = INFINITY, hi = -INFINITY;
#pragma unroll
    for (int j = 0; j < kQwMaxUnits; ++j) {
        const int64_t u = threadIdx.x + (int64_t)j * kQwBlock;
        if (u < units) {
            reg[j].load(row, u);
            if constexpr (FOLD) {
                float x[8];
                reg[j].get(x);
                const Float4 s0 = *reinterpret_cast<const Float4*>(s + u * 8), s1 = *reinterpret_cast<const Float4*>(s + u * 8 + 4);
#pragma unroll
                for (int i = 0; i < 4; ++i) { x[i] = rounded_f32(x[i] * s0.f[i]); x[4 + i] = rounded_f32(x[4 + i] * s1.f[i]); }
                reg[j].set(x);
                reg[j].store(reinterpret_cast<char*>(W_hat) + (size_t)n * ldwh * (F16 ? 2 : 4), u);
            }
            if constexpr (!PER_TENSOR) {
                float x[8];
                reg[j].get(x);
                minmax8(x, lo, hi);
            }
        }
    }
    float sp;
    int z;
    if constexpr (PER_TENSOR) {
        sp = step[0];
        z = zero[0];
    } else {
        lo = block_allreduce<kQwBlock / kWave>(lo, OpMin(), slot_f);
        hi = block_allreduce<kQwBlock / kWave>(hi, OpMax(), slot_f);
        qparams(lo, hi, BITS, sp, z, st);
        if (threadIdx.x == 0) { step[n] = sp; zero[n] = z; }
    }
    int rs = 0;
#pragma unroll
    for (int j = 0; j < kQwMaxUnits; ++j) {
        const int64_t u = threadIdx.x + (int64_t)j * kQwBlock;
        if (u < units) {
            float x[8];
            reg[j].get(x);
            // unit u of row n in the panel layout: panel u / 8, bytes 8 (u % 8) ..
            rs += quant_store_unit<BITS>(x, sp, z, row_codes, u, st, BITS == 8 ? (u >> 3) * N * kPanel + (u & 7) * 8 : -1);
        }
    }
    if constexpr (BITS == 8) {
        // columns past K in the last panel are zero
        const int64_t u = units + threadIdx.x;
        if (u < panel_count(K) * 8) *reinterpret_cast<uint2*>(row_codes + (u >> 3) * N * kPanel + (u & 7) * 8) = make_uint2(0u, 0u);
    }
    if (BITS == 8 && rowsum_w) {
        rs = block_allreduce<kQwBlock / kWave>(rs, OpAdd(), slot_i);
        if (threadIdx.x == 0) rowsum_w[n] = rs;
    }
    raise_status(status, st);
}

// ---- one (Step, Z) per group of 8 * 2^LEVELS consecutive k inside a row
template <bool F16, int BITS, int LEVELS>
__global__ __launch_bounds__(kQwBlock) void quant_weight_group(
    const void* __restrict__ W, int64_t K, int64_t ldw, uint8_t* __restrict__ codes,
    float* __restrict__ step, int32_t* __restrict__ zero, uint32_t* status)
{
    const int64_t n = blockIdx.y;
    const int64_t units = K / 8;
    const int64_t u = (int64_t)blockIdx.x * kQwBlock + threadIdx.x;
    // K % group == 0 and groups are lane-aligned, so a group is entirely in or out of range
    if (u >= units) return;
    const char* row = reinterpret_cast<const char*>(W) + (size_t)n * ldw * (F16 ? 2 : 4);
    uint8_t* row_codes = codes + (size_t)n * (K * BITS / 8);
    uint32_t st = 0;
    Unit<F16> reg;
    reg.load(row, u);
    float x[8];
    reg.get(x);
    float lo = INFINITY, hi = -INFINITY;
    minmax8(x, lo, hi);
    lo = group_allreduce<LEVELS>(lo, OpMin());
    hi = group_allreduce<LEVELS>(hi, OpMax());
    float sp;
    int z;
    qparams(lo, hi, BITS, sp, z, st);
    quant_store_unit<BITS>(x, sp, z, row_codes, u, st);
    if ((u & ((1 << LEVELS) - 1)) == 0) {
        const int64_t gi = n * (units >> LEVELS) + (u >> LEVELS);
        step[gi] = sp;
        zero[gi] = z;
    }
    raise_status(status, st);
}

// ---- tensor-wide extremes for group = -1: order-preserving unsigned keys + atomics
__device__ __forceinline__ uint32_t float_key(float f)
{
    uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float key_float(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ void tensor_minmax_init(uint32_t* keys)
{
    keys[0] = 0xffffffffu;  // running minimum
    keys[1] = 0u;           // running maximum
}

template <bool F16>
__global__ __launch_bounds__(kQwBlock) void tensor_minmax(const void* __restrict__ W, int64_t N, int64_t K,
                                                          int64_t ldw, uint32_t* keys)
{
    __shared__ float slot[kQwBlock / kWave];
    const int64_t units = K / 8;
    float lo = INFINITY, hi = -INFINITY;
    for (int64_t n = blockIdx.x; n < N; n += gridDim.x) {
        const char* row = reinterpret_cast<const char*>(W) + (size_t)n * ldw * (F16 ? 2 : 4);
        for (int64_t u = threadIdx.x; u < units; u += kQwBlock) {
            Unit<F16> reg;
            reg.load(row, u);
            float x[8];
            reg.get(x);
            minmax8(x, lo, hi);
        }
    }
    lo = block_allreduce<kQwBlock / kWave>(lo, OpMin(), slot);
    hi = block_allreduce<kQwBlock / kWave>(hi, OpMax(), slot);
    if (threadIdx.x == 0) {
        atomicMin(&keys[0], float_key(lo));
        atomicMax(&keys[1], float_key(hi));
    }
}

__global__ void tensor_qparams(const uint32_t* keys, int bits, float* step, int32_t* zero, uint32_t* status)
{
    uint32_t st = 0;
    float sp;
    int z;
    qparams(key_float(keys[0]), key_float(keys[1]), bits, sp, z, st);
    *step = sp;
    *zero = z;
    raise_status(status, st);
}

template <bool F16, int BITS>
static void launch_row(bool per_tensor, const void* W, int64_t N, int64_t K, int64_t ldw, uint8_t* codes,
                       float* step, int32_t* zero, int32_t* rowsum_w, uint32_t* status, hipStream_t st)
{
    if (per_tensor)
        quant_weight_row<F16, BITS, true><<<(unsigned)N, kQwBlock, 0, st>>>(W, K, ldw, codes, step, zero, rowsum_w, status);
    else
        quant_weight_row<F16, BITS, false><<<(unsigned)N, kQwBlock, 0, st>>>(W, K, ldw, codes, step, zero, rowsum_w, status);
}

template <bool F16, int BITS>
static void launch_group(int levels, const void* W, int64_t N, int64_t K, int64_t ldw, uint8_t* codes,
                         float* step, int32_t* zero, uint32_t* status, hipStream_t st)
{
    dim3 grid((unsigned)cdiv(K / 8, kQwBlock), (unsigned)N);
#define AWEQ_LG(L) case L: quant_weight_group<F16, BITS, L><<<grid, kQwBlock, 0, st>>>(W, K, ldw, codes, step, zero, status); break;
    switch (levels) { AWEQ_LG(0) AWEQ_LG(1) AWEQ_LG(2) AWEQ_LG(3) AWEQ_LG(4) AWEQ_LG(5) AWEQ_LG(6) }
#undef AWEQ_LG
}

}  // namespace aweq

using namespace aweq;

extern "C" int aweq_quant_weight(const void* W_hat, aweq_dtype dt, int64_t N, int64_t K, int64_t ldw,
                                 int bits, int group, void* codes, float* step, int32_t* zero,
                                 int32_t* rowsum_w, void* ws, size_t ws_bytes,
                                 uint32_t* status, void* stream)
{
    if (!W_hat || !codes || !step || !zero) return AWEQ_ERR_NULL;
    if (dt != AWEQ_F32 && dt != AWEQ_F16) return AWEQ_ERR_DTYPE;
    if (bits != 8 && bits != 4 && bits != 3) return AWEQ_ERR_BITS;
    if (N <= 0 || K <= 0 || ldw < K || (K % 8) != 0) return AWEQ_ERR_SHAPE;
    if (N > 0x7fffffffll) return AWEQ_ERR_SHAPE;
    if (bits == 3 && (K % 32) != 0) return AWEQ_ERR_ALIGN;
    int levels = -1;
    if (group > 0) {
        for (int l = 0; l <= 6; ++l)
            if (group == (8 << l)) levels = l;
        if (levels < 0 || (K % group) != 0) return AWEQ_ERR_GROUP;
        if (rowsum_w) return AWEQ_ERR_GROUP;  // row sums are defined for per-row / per-tensor int8 only
        if (N > 65535) return AWEQ_ERR_SHAPE;  // rows ride on the grid's y dimension
    } else if (group < -1) {
        return AWEQ_ERR_GROUP;
    } else if (K > (int64_t)kQwBlock * 8 * kQwMaxUnits) {
        return AWEQ_ERR_SHAPE;  // a row must fit the block's registers
    }
    if (!aligned16(W_hat) || ((size_t)ldw * dtype_size(dt)) % 16 != 0 || !aligned16(codes)) return AWEQ_ERR_ALIGN;
    if (group == -1 && (!ws || ws_bytes < 2 * sizeof(uint32_t))) return AWEQ_ERR_WORKSPACE;

    hipStream_t st = as_stream(stream);
    uint8_t* cb = reinterpret_cast<uint8_t*>(codes);
    const bool f16 = dt == AWEQ_F16;
    if (group == -1) {
        uint32_t* keys = reinterpret_cast<uint32_t*>(ws);
        tensor_minmax_init<<<1, 1, 0, st>>>(keys);
        const unsigned g = (unsigned)(N < 2048 ? N : 2048);
        if (f16) tensor_minmax<true><<<g, kQwBlock, 0, st>>>(W_hat, N, K, ldw, keys);
        else tensor_minmax<false><<<g, kQwBlock, 0, st>>>(W_hat, N, K, ldw, keys);
        tensor_qparams<<<1, 1, 0, st>>>(keys, bits, step, zero, status);
    }
#define AWEQ_DISPATCH(F, B)                                                                            \
    if (group > 0) launch_group<F, B>(levels, W_hat, N, K, ldw, cb, step, zero, status, st);           \
    else launch_row<F, B>(group == -1, W_hat, N, K, ldw, cb, step, zero, rowsum_w, status, st);
    if (f16) {
        if (bits == 8) { AWEQ_DISPATCH(true, 8) } else if (bits == 4) { AWEQ_DISPATCH(true, 4) } else { AWEQ_DISPATCH(true, 3) }
    } else {
        if (bits == 8) { AWEQ_DISPATCH(false, 8) } else if (bits == 4) { AWEQ_DISPATCH(false, 4) } else { AWEQ_DISPATCH(false, 3) }
    }
#undef AWEQ_DISPATCH
    return launch_status();
}

// Fold and quantise in one pass over W (per-row quantizer): what aweq_equalize's fold followed by
// aweq_quant_weight with group = 0 produce, with W read once and W_hat not read back.
extern "C" int aweq_fold_quant_weight(const void* W, aweq_dtype dt, int64_t N, int64_t K, int64_t ldw,
                                      const float* s, void* W_hat, int64_t ldwh, int bits, void* codes, float* step,
                                      int32_t* zero, int32_t* rowsum_w, uint32_t* status, void* stream)
{
    if (!W || !s || !W_hat || !codes || !step || !zero) return AWEQ_ERR_NULL;
    if (dt != AWEQ_F32 && dt != AWEQ_F16) return AWEQ_ERR_DTYPE;
    if (bits != 8 && bits != 4 && bits != 3) return AWEQ_ERR_BITS;
    if (N <= 0 || N > 0x7fffffffll || K <= 0 || ldw < K || ldwh < K || (K % 8) != 0) return AWEQ_ERR_SHAPE;
    if (K > (int64_t)kQwBlock * 8 * kQwMaxUnits) return AWEQ_ERR_SHAPE;  // a row must fit the block's registers
    if (bits == 3 && (K % 32) != 0) return AWEQ_ERR_ALIGN;
    if (bits != 8 && rowsum_w) return AWEQ_ERR_BITS;
    if (!aligned16(W) || !aligned16(W_hat) || !aligned16(s) || ((size_t)ldw * dtype_size(dt)) % 16 != 0 ||
        ((size_t)ldwh * dtype_size(dt)) % 16 != 0 || !aligned16(codes))
        return AWEQ_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    uint8_t* cb = reinterpret_cast<uint8_t*>(codes);
#define AWEQ_FQ(F, B) quant_weight_row<F, B, false, true><<<(unsigned)N, kQwBlock, 0, st>>>(W, K, ldw, cb, step, zero, rowsum_w, status, s, W_hat, ldwh)
    if (dt == AWEQ_F16) { if (bits == 8) AWEQ_FQ(true, 8); else if (bits == 4) AWEQ_FQ(true, 4); else AWEQ_FQ(true, 3); }
    else { if (bits == 8) AWEQ_FQ(false, 8); else if (bits == 4) AWEQ_FQ(false, 4); else AWEQ_FQ(false, 3); }
#undef AWEQ_FQ
    return launch_status();
}
