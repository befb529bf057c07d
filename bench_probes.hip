// Measurement aids of bench.py (built into libbench_probes.so next to it; not part of libaweq.so
// and not a stage of the method): what this machine delivers with nothing of the method in the way.
//  - bench_probe_mfma_clock: every wavefront issues back-to-back independent matrix instructions
//    (16 accumulators, no memory traffic); one wavefront reports how many shader-clock cycles
//    (s_memtime) and 100 MHz reference ticks (s_memrealtime) that took, so the caller gets the
//    sustained shader clock under matrix load for a given kind of operand data.
//  - bench_probe_stream: bare streaming kernels (16 bytes per lane and load, 8 loads in flight,
//    non-temporal), read only / copy / two bytes read per byte written: the ceiling an HBM-bound
//    pass of that read : write mix can reach here.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace probes {

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
                    } else if (operand_mode == 4) {  // first operand small codes, second operand any byte
                        va = (unsigned)((int)(va % 9) - 4) & 0xff;
                    } else if (operand_mode == 5) {  // the other way round
                        vb = (unsigned)((int)(vb % 9) - 4) & 0xff;
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

typedef int sv4i __attribute__((ext_vector_type(4)));
typedef int sv2i __attribute__((ext_vector_type(2)));
constexpr int kStreamInFlight = 8;

// MODE 0: read `bytes` (the xor of everything read goes to sink so the loads stay); 1: copy `bytes`;
// 2: read `bytes`, write bytes / 2 (8 bytes per lane per 16 read: the mix of a pass that turns
// binary16 values into 8-bit codes).  A block walks its contiguous share in steps of 8 x 4 KiB.
template <int MODE>
__global__ __launch_bounds__(256) void stream_probe(const sv4i* __restrict__ in, void* __restrict__ out, int64_t units,
                                                    int64_t units_per_block, int* __restrict__ sink)
{
    const int64_t u0 = (int64_t)blockIdx.x * units_per_block;
    const int64_t u1 = u0 + units_per_block < units ? u0 + units_per_block : units;
    sv4i x = {0, 0, 0, 0};
    for (int64_t u = u0 + threadIdx.x; u < u1; u += 256 * kStreamInFlight) {
        sv4i v[kStreamInFlight];
#pragma unroll
        for (int j = 0; j < kStreamInFlight; ++j)
            if (u + j * 256 < u1) v[j] = __builtin_nontemporal_load(in + u + j * 256);
#pragma unroll
        for (int j = 0; j < kStreamInFlight; ++j)
            if (u + j * 256 < u1) {
                if constexpr (MODE == 0) x ^= v[j];
                else if constexpr (MODE == 1) __builtin_nontemporal_store(v[j], reinterpret_cast<sv4i*>(out) + u + j * 256);
                else __builtin_nontemporal_store(sv2i{v[j][0] ^ v[j][1], v[j][2] ^ v[j][3]}, reinterpret_cast<sv2i*>(out) + u + j * 256);
            }
    }
    if constexpr (MODE == 0)
        if ((x[0] ^ x[1] ^ x[2] ^ x[3]) == 0x7f3a91c5) *sink = 1;   // practically never: keeps the loads alive
}

}  // namespace probes

// out[3] (device, uint64): shader-clock cycles of one wavefront's loop, 100 MHz reference ticks of the
// same interval, a checksum.  operand_mode 0: constant bytes, 1: uniformly random bytes, 2: small signed
// codes (int8 32x32x32 MFMA, 65536 ops each); 3: the binary16 32x32x16 MFMA (32768 flop each) on
// activation- and weight-like values; 4 / 5: small codes in the first / second int8 operand only, any byte in the other.  One workgroup of four wavefronts per compute unit, iters x 16
// instructions per wavefront.  Returns 0 or a negative number (bad argument / launch refused).
extern "C" int bench_probe_mfma_clock(int iters, int operand_mode, uint64_t* out, void* stream)
{
    if (!out || iters <= 0 || iters > (1 << 22) || operand_mode < 0 || operand_mode > 5) return -1;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return -2;
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    if (operand_mode == 3)
        probes::mfma_clock_probe_f16<<<(unsigned)cus, 256, 0, st>>>(iters, reinterpret_cast<unsigned long long*>(out));
    else
        probes::mfma_clock_probe<<<(unsigned)cus, 256, 0, st>>>(iters, operand_mode, reinterpret_cast<unsigned long long*>(out));
    return hipGetLastError() == hipSuccess ? 0 : -2;
}

// mode 0 / 1 / 2 as above; in: `bytes` readable (a multiple of 16), out: bytes (mode 1) or bytes / 2
// (mode 2) writable, sink: one int; `blocks` workgroups of 256 lanes share the range contiguously.
extern "C" int bench_probe_stream(int mode, const void* in, void* out, int64_t bytes, int blocks, int* sink, void* stream)
{
    if (!in || !sink || (mode != 0 && !out) || mode < 0 || mode > 2 || bytes <= 0 || (bytes % 16) != 0 || blocks <= 0) return -1;
    const int64_t units = bytes / 16;
    int64_t upb = (units + blocks - 1) / blocks;
    upb = (upb + 256 * probes::kStreamInFlight - 1) / (256 * probes::kStreamInFlight) * (256 * probes::kStreamInFlight);
    const unsigned grid = (unsigned)((units + upb - 1) / upb);
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    const probes::sv4i* src = reinterpret_cast<const probes::sv4i*>(in);
    if (mode == 0) probes::stream_probe<0><<<grid, 256, 0, st>>>(src, out, units, upb, sink);
    else if (mode == 1) probes::stream_probe<1><<<grid, 256, 0, st>>>(src, out, units, upb, sink);
    else probes::stream_probe<2><<<grid, 256, 0, st>>>(src, out, units, upb, sink);
    return hipGetLastError() == hipSuccess ? 0 : -2;
}
