// Stage 5: quantization bias correction (Sec. 3.3).  delta[n] = mean FP output minus mean
// quantised output over the calibration tokens (Eq. 11); the corrected bias is b + delta.
// By linearity both means contract to K-vectors and integer column sums, so this is a
// GEMV over W_hat (HBM-bound, one read of the weight): fp64 accumulation because delta is a
// small difference of two nearly equal means.
#include "common.hpp"

namespace aweq {

constexpr int kBiasBlock = 256;

template <bool F16>
__device__ __forceinline__ void load_w8(const void* row, int64_t u, float x[8])
{
    if constexpr (F16) {
        Half8 v = *reinterpret_cast<const Half8*>(reinterpret_cast<const _Float16*>(row) + u * 8);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float2 f = h2f2(v.h[i]);
            x[2 * i] = f.x;
            x[2 * i + 1] = f.y;
        }
    } else {
        const float* p = reinterpret_cast<const float*>(row) + u * 8;
        Float4 a = *reinterpret_cast<const Float4*>(p), b = *reinterpret_cast<const Float4*>(p + 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) { x[i] = a.f[i]; x[4 + i] = b.f[i]; }
    }
}

// W8A8 (Eq. 11 with the int8 path as the quantised layer):
//   mean_t y[t,n]  = sum_k W_hat[n,k] mu_xhat[k]
//   sum_t  y~[t,n] = Step_x Step_w[n] (colsum_acc[n] - T Z'x rowsum_w[n] - Z'w[n] sum_k colsum_xq[k] + T K Z'x Z'w[n])
// colsum_acc[n] = sum_t acc[t,n] comes from the GEMM, or - by the same linearity, as exact integers -
// from the weight codes: sum_t sum_k xq[t,k] wq[n,k] = sum_k wq[n,k] colsum_xq[k] (wq given, colsum_acc NULL),
// so that calibration does not have to run the forward.
// A block takes kBiasRows output channels at once: mu_xhat and colsum_xq (and their sum over k, which every
// channel needs) are read once per block instead of once per channel.
constexpr int kBiasRows = 8;
template <bool F16>
__global__ __launch_bounds__(kBiasBlock) void bias_w8a8_kernel(
    const void* __restrict__ W_hat, int64_t N, int64_t K, int64_t ldw, const float* __restrict__ mu_xhat, uint64_t count,
    const long long* __restrict__ colsum_acc, const long long* __restrict__ colsum_xq,
    const int32_t* __restrict__ rowsum_w, const float* __restrict__ act_step, const int32_t* __restrict__ act_zero,
    const float* __restrict__ step_w, const int32_t* __restrict__ zero_w, const float* __restrict__ bias_in,
    float* __restrict__ delta, float* __restrict__ bias_out, int enable_bc, const int8_t* __restrict__ wq,
    int w_per_tensor)
{
    __shared__ double slot_d[kBiasBlock / kWave];
    __shared__ long long slot_l[kBiasBlock / kWave];
    const int64_t n0 = (int64_t)blockIdx.x * kBiasRows;
    const int rows = (int)min((int64_t)kBiasRows, N - n0);
    double acc[kBiasRows];
    long long ca[kBiasRows];
#pragma unroll
    for (int r = 0; r < kBiasRows; ++r) { acc[r] = 0.0; ca[r] = 0; }
    long long tot = 0;
    for (int64_t u = threadIdx.x; u < K / 8; u += kBiasBlock) {
        const Float4 m0 = *reinterpret_cast<const Float4*>(mu_xhat + u * 8);
        const Float4 m1 = *reinterpret_cast<const Float4*>(mu_xhat + u * 8 + 4);
        long long cx[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) { cx[i] = colsum_xq[u * 8 + i]; tot += cx[i]; }
#pragma unroll
        for (int r = 0; r < kBiasRows; ++r) {
            if (r >= rows) break;
            const char* row = reinterpret_cast<const char*>(W_hat) + (size_t)(n0 + r) * ldw * (F16 ? 2 : 4);
            float w[8];
            load_w8<F16>(row, u, w);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                acc[r] += (double)w[i] * (double)m0.f[i];
                acc[r] += (double)w[4 + i] * (double)m1.f[i];
            }
            if (wq) {
                // unit u of row n in the K-panel layout: panel u / 8, bytes 8 (u % 8) ..
                const uint2 v = *reinterpret_cast<const uint2*>(wq + ((u >> 3) * N + n0 + r) * kPanel + (u & 7) * 8);
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    ca[r] += (long long)(int8_t)((v.x >> (8 * i)) & 0xff) * cx[i];
                    ca[r] += (long long)(int8_t)((v.y >> (8 * i)) & 0xff) * cx[4 + i];
                }
            }
        }
    }
    tot = block_allreduce<kBiasBlock / kWave>(tot, OpAdd(), slot_l);
    const long long T = (long long)count;
    const long long zx = (long long)*act_zero - 128;
    const double sx = (double)*act_step;
#pragma unroll
    for (int r = 0; r < kBiasRows; ++r) {
        if (r >= rows) break;    // (block-uniform)
        const double a_r = block_allreduce<kBiasBlock / kWave>(acc[r], OpAdd(), slot_d);
        long long c_r = 0;
        if (wq) c_r = block_allreduce<kBiasBlock / kWave>(ca[r], OpAdd(), slot_l);
        if (threadIdx.x == 0) {
            const int64_t n = n0 + r;
            const int64_t pi = w_per_tensor ? 0 : n;   // one (Step, Z) for the tensor, or one per output channel
            const long long zw = (long long)zero_w[pi] - 128;
            const long long a = (wq ? c_r : colsum_acc[n]) - T * zx * (long long)rowsum_w[n] - zw * tot + T * K * zx * zw;
            const double yq = sx * (double)step_w[pi] * (double)a / (double)T;
            const double d = a_r - yq;
            delta[n] = (float)d;
            bias_out[n] = (float)((bias_in ? (double)bias_in[n] : 0.0) + (enable_bc ? d : 0.0));
        }
    }
}

// Weight-only (Eq. 12-15): E[y~ - y] = eps E[x], eps = W~ - W_hat; delta = -eps mu_xhat.
template <bool F16, int BITS>
__global__ __launch_bounds__(kBiasBlock) void bias_wonly_kernel(
    const void* __restrict__ W_hat, int64_t K, int64_t ldw, const float* __restrict__ mu_xhat,
    const uint8_t* __restrict__ codes, int64_t group, const float* __restrict__ step_w,
    const int32_t* __restrict__ zero_w, const float* __restrict__ bias_in, float* __restrict__ delta,
    float* __restrict__ bias_out, int enable_bc)
{
    __shared__ double slot_d[kBiasBlock / kWave];
    const int64_t n = blockIdx.x;
    const char* row = reinterpret_cast<const char*>(W_hat) + (size_t)n * ldw * (F16 ? 2 : 4);
    const uint8_t* crow = codes + (size_t)n * (K * BITS / 8);
    const int64_t g = group > 0 ? group : K;
    const int64_t ng = K / g;
    double acc = 0.0;
    for (int64_t u = threadIdx.x; u < K / 8; u += kBiasBlock) {
        float w[8];
        load_w8<F16>(row, u, w);
        int c[8];
        if constexpr (BITS == 8) {
            // per-row / per-tensor 8-bit codes are stored in the GEMM's K-panel layout
            const uint2 v = group > 0 ? *reinterpret_cast<const uint2*>(crow + u * 8)
                                      : *reinterpret_cast<const uint2*>(codes + ((u >> 3) * (int64_t)gridDim.x + n) * kPanel + (u & 7) * 8);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                c[i] = (int)(int8_t)((v.x >> (8 * i)) & 0xff) + 128;
                c[4 + i] = (int)(int8_t)((v.y >> (8 * i)) & 0xff) + 128;
            }
        } else if constexpr (BITS == 4) {
            const uint32_t v = *reinterpret_cast<const uint32_t*>(crow + u * 4);
#pragma unroll
            for (int i = 0; i < 8; ++i) c[i] = (int)((v >> (4 * i)) & 15u);
        } else {
            const uint8_t* p = crow + u * 3;
            const uint32_t v = (uint32_t)p[0] | ((uint32_t)p[1] << 8) | ((uint32_t)p[2] << 16);
#pragma unroll
            for (int i = 0; i < 8; ++i) c[i] = (int)((v >> (3 * i)) & 7u);
        }
        // the 8 values of a unit share one group (group sizes are multiples of 8)
        const int64_t pi = group < 0 ? 0 : n * ng + (u * 8) / g;
        const float sp = step_w[pi];
        const int z = zero_w[pi];
        const Float4 m0 = *reinterpret_cast<const Float4*>(mu_xhat + u * 8);
        const Float4 m1 = *reinterpret_cast<const Float4*>(mu_xhat + u * 8 + 4);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float wt = (float)(c[i] - z) * sp;
            const double eps = (double)wt - (double)w[i];
            acc += eps * (double)(i < 4 ? m0.f[i] : m1.f[i - 4]);
        }
    }
    acc = block_allreduce<kBiasBlock / kWave>(acc, OpAdd(), slot_d);
    if (threadIdx.x == 0) {
        const double d = -acc;
        delta[n] = (float)d;
        bias_out[n] = (float)((bias_in ? (double)bias_in[n] : 0.0) + (enable_bc ? d : 0.0));
    }
}

}  // namespace aweq

using namespace aweq;

extern "C" int aweq_bias_correct(int mode, const void* W_hat, aweq_dtype dt, int64_t N, int64_t K, int64_t ldw,
                                 const float* mu_xhat, uint64_t count,
                                 const int64_t* colsum_acc, const int64_t* colsum_xq, const int32_t* rowsum_w,
                                 const float* act_step, const int32_t* act_zero,
                                 const void* codes, int bits, int group,
                                 const float* step_w, const int32_t* zero_w,
                                 const float* bias_in, float* delta, float* bias_out, int enable_bc,
                                 uint32_t* status, void* stream)
{
    (void)status;   // this stage meets no numeric condition it would have to report
    if (!W_hat || !mu_xhat || !step_w || !zero_w || !delta || !bias_out) return AWEQ_ERR_NULL;
    if (dt != AWEQ_F32 && dt != AWEQ_F16) return AWEQ_ERR_DTYPE;
    if (N <= 0 || N > 0x7fffffffll || K <= 0 || ldw < K || (K % 8) != 0) return AWEQ_ERR_SHAPE;
    if (!aligned16(W_hat) || ((size_t)ldw * dtype_size(dt)) % 16 != 0 || !aligned16(mu_xhat)) return AWEQ_ERR_ALIGN;
    hipStream_t st = as_stream(stream);
    const bool f16 = dt == AWEQ_F16;
    if (mode == AWEQ_BIAS_W8A8) {
        if (!colsum_xq || !rowsum_w || !act_step || !act_zero) return AWEQ_ERR_NULL;
        if (!colsum_acc && !codes) return AWEQ_ERR_NULL;
        if (count == 0) return AWEQ_ERR_SHAPE;
        // without the GEMM's column sums they are formed from the 8-bit per-row / per-tensor codes (K-panel layout)
        const int8_t* wq = colsum_acc ? nullptr : reinterpret_cast<const int8_t*>(codes);
        if (wq && (bits != 8 || group > 0)) return AWEQ_ERR_BITS;
        if (group != 0 && group != -1) return AWEQ_ERR_GROUP;   // the int8 path has one scale per output channel or per tensor
        const int pt = group == -1;
        if (wq && !aligned16(wq)) return AWEQ_ERR_ALIGN;
        const long long* ca = reinterpret_cast<const long long*>(colsum_acc);
        const long long* cx = reinterpret_cast<const long long*>(colsum_xq);
        if (f16)
            bias_w8a8_kernel<true><<<(unsigned)cdiv(N, kBiasRows), kBiasBlock, 0, st>>>(W_hat, N, K, ldw, mu_xhat, count, ca, cx, rowsum_w, act_step,
                                                                     act_zero, step_w, zero_w, bias_in, delta, bias_out, enable_bc, wq, pt);
        else
            bias_w8a8_kernel<false><<<(unsigned)cdiv(N, kBiasRows), kBiasBlock, 0, st>>>(W_hat, N, K, ldw, mu_xhat, count, ca, cx, rowsum_w, act_step,
                                                                      act_zero, step_w, zero_w, bias_in, delta, bias_out, enable_bc, wq, pt);
    } else if (mode == AWEQ_BIAS_WEIGHT_ONLY) {
        if (!codes) return AWEQ_ERR_NULL;
        if (bits != 8 && bits != 4 && bits != 3) return AWEQ_ERR_BITS;
        if (group < -1 || (group > 0 && ((group % 8) != 0 || (K % group) != 0))) return AWEQ_ERR_GROUP;
        if (!aligned16(codes)) return AWEQ_ERR_ALIGN;
        if (bits == 3 && (K % 32) != 0) return AWEQ_ERR_ALIGN;
        const uint8_t* cb = reinterpret_cast<const uint8_t*>(codes);
#define AWEQ_BW(F, B) bias_wonly_kernel<F, B><<<(unsigned)N, kBiasBlock, 0, st>>>(W_hat, K, ldw, mu_xhat, cb, group, step_w, zero_w, bias_in, delta, bias_out, enable_bc)
        if (f16) { if (bits == 8) AWEQ_BW(true, 8); else if (bits == 4) AWEQ_BW(true, 4); else AWEQ_BW(true, 3); }
        else { if (bits == 8) AWEQ_BW(false, 8); else if (bits == 4) AWEQ_BW(false, 4); else AWEQ_BW(false, 3); }
#undef AWEQ_BW
    } else {
        return AWEQ_ERR_SHAPE;
    }
    return launch_status();
}
