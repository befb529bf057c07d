// Diagnostic, not a stage of the method: how fast the matrix cores actually run on this
// machine for a given kind of operand data.  Every wavefront issues back-to-back independent
// v_mfma_i32_32x32x32_i8 (16 accumulators, no memory traffic); one wavefront reports how many
// shader-clock cycles (s_memtime) and 100 MHz reference ticks (s_memrealtime) that took, so
// the caller gets the sustained shader clock under matrix load.
#include "common.hpp"

namespace aweq {

typedef int pv4i __attribute__((ext_vector_type(4)));
typedef int pv16i __attribute__((ext_vector_type(16)));
typedef _Float16 pv8h __attribute__((ext_vector_type(8)));
typedef float pv16f __attribute__((ext_vector_type(16)));

// operand_mode 3: the same loop with v_mfma_f32_32x32x16_f16 on binary16 operands that look like
// activations (unit scale) and de-quantised weights (scale 0.02)
__global__ __launch_bounds__(256) void mfma_clock_probe_f16(int iters, unsigned long long* out)
{
    pv8h a[4], b[4];
    unsigned x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int i = 0; i < 4; ++i)
        for (int c = 0; c < 8; ++c) {
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;
            const float ua = (float)(int)(x & 0xffff) * (1.0f / 32768.0f) - 1.0f;
            x ^= x << 13; x ^= x >> 17; x ^= x << 5;
            const float ub = (float)(int)(x & 0xffff) * (1.0f / 32768.0f) - 1.0f;
            a[i][c] = (_Float16)(2.0f * ua);
            b[i][c] = (_Float16)(0.04f * ub);
        }
    pv16f acc[4][4];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j)
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    float s = 0.0f;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j)
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = c1 - c0;
        out[1] = r1 - r0;
        out[2] = (unsigned long long)__float_as_uint(s);  // keeps the accumulators alive
    }
}

__global__ __launch_bounds__(256) void mfma_clock_probe(int iters, int operand_mode, unsigned long long* out)
{
    pv4i a[4], b[4];
    unsigned x = threadIdx.x * 2654435761u + blockIdx.x * 40503u + 12345u;
    for (int i = 0; i < 4; ++i)
        for (int c = 0; c < 4; ++c) {
            unsigned wa = 0x01010101u, wb = 0x02020202u;  // mode 0: constant bytes
            if (operand_mode != 0) {
                unsigned ra = 0, rb = 0;
                for (int byte = 0; byte < 4; ++byte) {
                    x ^= x << 13; x ^= x >> 17; x ^= x << 5;
                    unsigned va = x & 0xff;
                    x ^= x << 13; x ^= x >> 17; x ^= x << 5;
                    unsigned vb = x & 0xff;
                    if (operand_mode == 2) {  // small signed codes, like equalised activations / weights
                        va = (unsigned)((int)(va % 9) - 4) & 0xff;
                        vb = (unsigned)((int)(vb % 33) - 16) & 0xff;
                    }
                    ra |= va << (8 * byte);
                    rb |= vb << (8 * byte);
                }
                wa = ra; wb = rb;
            }
            a[i][c] = (int)wa;
            b[i][c] = (int)wb;
        }
    pv16i acc[4][4];
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j)
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    const unsigned long long c0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    int s = 0;
    for (int i = 0; i < 4; ++i)
        for (int j = 0; j < 4; ++j)
            for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    const unsigned long long c1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        out[0] = c1 - c0;
        out[1] = r1 - r0;
        out[2] = (unsigned long long)(unsigned)s;  // keeps the accumulators alive
    }
}

}  // namespace aweq

extern "C" int aweq_probe_mfma_clock(int iters, int operand_mode, uint64_t* out, void* stream)
{
    if (!out) return AWEQ_ERR_NULL;
    if (iters <= 0 || iters > (1 << 22) || operand_mode < 0 || operand_mode > 3) return AWEQ_ERR_SHAPE;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return AWEQ_ERR_LAUNCH;
    if (operand_mode == 3)
        aweq::mfma_clock_probe_f16<<<(unsigned)cus, 256, 0, aweq::as_stream(stream)>>>(iters, reinterpret_cast<unsigned long long*>(out));
    else
        aweq::mfma_clock_probe<<<(unsigned)cus, 256, 0, aweq::as_stream(stream)>>>(iters, operand_mode,
                                                                                   reinterpret_cast<unsigned long long*>(out));
    return aweq::launch_status();
}
