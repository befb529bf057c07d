// Helpers of the C ABI: workspace sizes, error names, the K-panel layout converters.
#include "common.hpp"

namespace aweq {
size_t stats_ws_bytes_export(int64_t rows, int64_t K);
size_t quant_act_ws_bytes(int64_t T, int64_t K);
}

extern "C" size_t aweq_workspace_size(aweq_op op, int64_t rows, int64_t K, int64_t N)
{
    if (rows <= 0 || K <= 0) return 0;
    switch (op) {
    case AWEQ_OP_CALIB_STATS: return aweq::stats_ws_bytes_export(rows, K);
    case AWEQ_OP_QUANT_WEIGHT: return 16;  // tensor-wide extremes for group = -1
    case AWEQ_OP_WONLY_GEMM: return N > 0 ? (size_t)N * (size_t)K * 2 : 0;  // the binary16 weight
    case AWEQ_OP_QUANT_ACT: return aweq::quant_act_ws_bytes(rows, K);  // per-slice column sums, per-chunk row sums
    case AWEQ_OP_W8A8_GEMM: {
        // stage 4a's partial sums (aweq_w8a8_gemm on float input), or the keys and sums of the output
        // statistics (aweq_w8a8_gemm_fused): the larger of the two serves both
        const size_t qa = aweq::quant_act_ws_bytes(rows, K), fs = N > 0 ? (size_t)N * 16 : 0;
        return qa > fs ? qa : fs;
    }
    case AWEQ_OP_EQUALIZE:
    case AWEQ_OP_BIAS_CORRECT:
    default: return 0;
    }
}

extern "C" const char* aweq_status_string(int code)
{
    switch (code) {
    case AWEQ_OK: return "AWEQ_OK";
    case AWEQ_ERR_NULL: return "AWEQ_ERR_NULL";
    case AWEQ_ERR_SHAPE: return "AWEQ_ERR_SHAPE";
    case AWEQ_ERR_DTYPE: return "AWEQ_ERR_DTYPE";
    case AWEQ_ERR_BITS: return "AWEQ_ERR_BITS";
    case AWEQ_ERR_GROUP: return "AWEQ_ERR_GROUP";
    case AWEQ_ERR_ALIGN: return "AWEQ_ERR_ALIGN";
    case AWEQ_ERR_WORKSPACE: return "AWEQ_ERR_WORKSPACE";
    case AWEQ_ERR_LAUNCH: return "AWEQ_ERR_LAUNCH";
    default: return "AWEQ_ERR_UNKNOWN";
    }
}

namespace aweq {
// one thread per 8-byte unit of the panel buffer: unit id = (panel * rows + r) * 8 + c
__global__ void pack_panels_kernel(const int8_t* __restrict__ src, int64_t rows, int64_t K, int64_t ld,
                                   int8_t* __restrict__ panels, int64_t units)
{
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= units) return;
    const int c = (int)(id & 7);
    const int64_t pr = id >> 3, p = pr / rows, r = pr % rows;
    const int64_t k = p * kPanel + c * 8;
    uint2 v = make_uint2(0u, 0u);
    if (k < K) v = *reinterpret_cast<const uint2*>(src + r * ld + k);
    *reinterpret_cast<uint2*>(panels + id * 8) = v;
}
// one thread per 8-byte unit of the row-major matrix
__global__ void unpack_panels_kernel(const int8_t* __restrict__ panels, int64_t rows, int64_t K,
                                     int8_t* __restrict__ dst, int64_t ld, int64_t units)
{
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= units) return;
    const int64_t upr = K / 8, r = id / upr, u = id % upr;
    *reinterpret_cast<uint2*>(dst + r * ld + u * 8) =
        *reinterpret_cast<const uint2*>(panels + ((u >> 3) * rows + r) * kPanel + (u & 7) * 8);
}
static int check_panels(const void* a, const void* b, int64_t rows, int64_t K, int64_t ld)
{
    if (!a || !b) return AWEQ_ERR_NULL;
    if (rows <= 0 || K <= 0 || (K % 8) != 0 || ld < K) return AWEQ_ERR_SHAPE;
    if ((ld % 8) != 0 || (reinterpret_cast<uintptr_t>(a) & 7u) || (reinterpret_cast<uintptr_t>(b) & 7u)) return AWEQ_ERR_ALIGN;
    return AWEQ_OK;
}
}  // namespace aweq

extern "C" size_t aweq_panel_bytes(int64_t rows, int64_t K)
{
    if (rows <= 0 || K <= 0) return 0;
    return (size_t)(aweq::panel_count(K) * rows * aweq::kPanel);
}

extern "C" int aweq_pack_panels_i8(const int8_t* src, int64_t rows, int64_t K, int64_t ld, int8_t* panels, void* stream)
{
    const int rc = aweq::check_panels(src, panels, rows, K, ld);
    if (rc != AWEQ_OK) return rc;
    const int64_t units = aweq::panel_count(K) * rows * 8;
    const int64_t blocks = aweq::cdiv(units, 256);
    if (blocks > 0x7fffffffll) return AWEQ_ERR_SHAPE;
    aweq::pack_panels_kernel<<<(unsigned)blocks, 256, 0, aweq::as_stream(stream)>>>(src, rows, K, ld, panels, units);
    return aweq::launch_status();
}

extern "C" int aweq_unpack_panels_i8(const int8_t* panels, int64_t rows, int64_t K, int8_t* dst, int64_t ld, void* stream)
{
    const int rc = aweq::check_panels(panels, dst, rows, K, ld);
    if (rc != AWEQ_OK) return rc;
    const int64_t units = rows * (K / 8);
    const int64_t blocks = aweq::cdiv(units, 256);
    if (blocks > 0x7fffffffll) return AWEQ_ERR_SHAPE;
    aweq::unpack_panels_kernel<<<(unsigned)blocks, 256, 0, aweq::as_stream(stream)>>>(panels, rows, K, dst, ld, units);
    return aweq::launch_status();
}
