// Stage 2: equalization factors (Sec. 3.2, Eq. 10) and the fold of Eq. 3 (Sec. 3.1).
#include "common.hpp"

namespace aweq {

// K-vector work, one block: s, inv_s, equalised activation range / mean, the static int8
// activation quantizer (Eq. 2 on the range of X_hat), optional prev_scale *= inv_s.
__global__ __launch_bounds__(1024) void equalize_scales(
    const float* __restrict__ xmin, const float* __restrict__ xmax, const double* __restrict__ xsum,
    uint64_t count, const float* __restrict__ wmin, const float* __restrict__ wmax, int64_t K,
    int enable_awe, float* __restrict__ s, float* __restrict__ inv_s, float* __restrict__ prev_scale,
    float* __restrict__ xhat_range, float* __restrict__ mu_xhat, float* __restrict__ act_step,
    int32_t* __restrict__ act_zero, uint32_t* status)
{
    __shared__ float slot[16];
    uint32_t st = 0;
    float lo = INFINITY, hi = -INFINITY;
    for (int64_t k = threadIdx.x; k < K; k += blockDim.x) {
        // the per-channel quantity the scale balances: the channel range (Eq. 10), or - the definition the
        // method replaces (Sec. 1, Sec. 3.2) - the channel's largest magnitude
        const float r_x = enable_awe == AWEQ_SCALE_ABSMAX ? fmaxf(fabsf(xmin[k]), fabsf(xmax[k])) : xmax[k] - xmin[k];
        const float r_w = enable_awe == AWEQ_SCALE_ABSMAX ? fmaxf(fabsf(wmin[k]), fabsf(wmax[k])) : wmax[k] - wmin[k];
        float sk = 1.0f;
        if (enable_awe) {
            if (!(r_x >= 1e-5f) || !(r_w >= 1e-5f)) {
                st |= AWEQ_ST_SCALEGUARD;
            } else {
                const double rx = (double)r_x, rw = (double)r_w;
                sk = (float)(sqrt(rx * rw) / rw);
                if (sk < 1e-4f) { sk = 1e-4f; st |= AWEQ_ST_SCALEGUARD; }
                if (sk > 1e4f) { sk = 1e4f; st |= AWEQ_ST_SCALEGUARD; }
            }
        }
        const float is = 1.0f / sk;
        s[k] = sk;
        inv_s[k] = is;
        if (prev_scale) prev_scale[k] = prev_scale[k] * is;
        if (mu_xhat) mu_xhat[k] = (float)((xsum[k] / (double)count) * (double)is);
        // a correctly rounded multiply by a positive constant is monotone, so the extremes of
        // the equalised column are the scaled extremes of the column
        lo = fminf(lo, xmin[k] * is);
        hi = fmaxf(hi, xmax[k] * is);
    }
    lo = block_allreduce<16>(lo, OpMin(), slot);
    hi = block_allreduce<16>(hi, OpMax(), slot);
    if (threadIdx.x == 0) {
        if (xhat_range) { xhat_range[0] = lo; xhat_range[1] = hi; }
        if (act_step && act_zero) {
            float sp; int z;
            qparams(lo, hi, 8, sp, z, st);
            *act_step = sp;
            *act_zero = z;
        }
    }
    raise_status(status, st);
}

// W_hat[n,k] = W[n,k] * s[k].  Threads own 8 (binary16) or 4 (binary32) columns and walk
// down the rows of their slice, so s stays in registers.
template <bool F16>
__global__ __launch_bounds__(256) void fold_weight(const void* __restrict__ Wv, void* __restrict__ Ov,
                                                   int64_t N, int64_t K, int64_t ldw, int64_t ldwh,
                                                   const float* __restrict__ s, int64_t rows_per_block)
{
    constexpr int E = F16 ? 8 : 4;
    const int64_t col = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * E;
    if (col >= K) return;
    float sc[E];
#pragma unroll
    for (int i = 0; i < E; ++i) sc[i] = s[col + i];
    const int64_t n0 = (int64_t)blockIdx.y * rows_per_block;
    const int64_t n1 = min(N, n0 + rows_per_block);
    for (int64_t n = n0; n < n1; ++n) {
        if constexpr (F16) {
            const _Float16* W = reinterpret_cast<const _Float16*>(Wv);
            _Float16* O = reinterpret_cast<_Float16*>(Ov);
            Half8 v = *reinterpret_cast<const Half8*>(W + n * ldw + col);
            Half8 o;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                float2 f = h2f2(v.h[i]);
                f.x = rounded_f32(f.x * sc[2 * i]);
                f.y = rounded_f32(f.y * sc[2 * i + 1]);
                o.h[i] = f16x2{(_Float16)f.x, (_Float16)f.y};
            }
            *reinterpret_cast<Half8*>(O + n * ldwh + col) = o;
        } else {
            const float* W = reinterpret_cast<const float*>(Wv);
            float* O = reinterpret_cast<float*>(Ov);
            Float4 v = *reinterpret_cast<const Float4*>(W + n * ldw + col);
#pragma unroll
            for (int i = 0; i < 4; ++i) v.f[i] = v.f[i] * sc[i];
            *reinterpret_cast<Float4*>(O + n * ldwh + col) = v;
        }
    }
}

}  // namespace aweq

using namespace aweq;

extern "C" int aweq_equalize(const float* xmin, const float* xmax, const double* xsum, uint64_t count,
                             const float* wmin, const float* wmax, int64_t K, int enable_awe,
                             float* s, float* inv_s,
                             const void* W, void* W_hat, aweq_dtype dt, int64_t N, int64_t ldw, int64_t ldwh,
                             float* prev_scale, float* xhat_range, float* mu_xhat,
                             float* act_step, int32_t* act_zero,
                             uint32_t* status, void* stream)
{
    if (!xmin || !xmax || !wmin || !wmax || !s || !inv_s) return AWEQ_ERR_NULL;
    if (mu_xhat && !xsum) return AWEQ_ERR_NULL;
    if ((act_step == nullptr) != (act_zero == nullptr)) return AWEQ_ERR_NULL;
    if (K <= 0 || (K % 8) != 0) return AWEQ_ERR_SHAPE;
    if (enable_awe < 0 || enable_awe > AWEQ_SCALE_ABSMAX) return AWEQ_ERR_SHAPE;
    if (mu_xhat && count == 0) return AWEQ_ERR_SHAPE;
    if (W) {
        if (!W_hat) return AWEQ_ERR_NULL;
        if (dt != AWEQ_F32 && dt != AWEQ_F16) return AWEQ_ERR_DTYPE;
        if (N <= 0 || ldw < K || ldwh < K) return AWEQ_ERR_SHAPE;
        if (!aligned16(W) || !aligned16(W_hat) || ((size_t)ldw * dtype_size(dt)) % 16 != 0 ||
            ((size_t)ldwh * dtype_size(dt)) % 16 != 0)
            return AWEQ_ERR_ALIGN;
    }
    hipStream_t st = as_stream(stream);
    equalize_scales<<<1, 1024, 0, st>>>(xmin, xmax, xsum, count, wmin, wmax, K, enable_awe, s, inv_s, prev_scale,
                                        xhat_range, mu_xhat, act_step, act_zero, status);
    if (W) {
        const int E = dt == AWEQ_F16 ? 8 : 4;
        const unsigned gx = (unsigned)cdiv(K, 256 * E);
        int64_t slices = cdiv(4096, gx);
        if (slices > N) slices = N;
        const int64_t rpb = cdiv(N, slices);
        dim3 grid(gx, (unsigned)cdiv(N, rpb));
        if (dt == AWEQ_F16)
            fold_weight<true><<<grid, 256, 0, st>>>(W, W_hat, N, K, ldw, ldwh, s, rpb);
        else
            fold_weight<false><<<grid, 256, 0, st>>>(W, W_hat, N, K, ldw, ldwh, s, rpb);
    }
    return launch_status();
}
