// Host-only helpers of the C ABI: workspace sizes and error names.
#include "common.hpp"

namespace aweq {
size_t stats_ws_bytes_export(int64_t rows, int64_t K);
}

extern "C" size_t aweq_workspace_size(aweq_op op, int64_t rows, int64_t K, int64_t N)
{
    (void)N;
    if (rows <= 0 || K <= 0) return 0;
    switch (op) {
    case AWEQ_OP_CALIB_STATS: return aweq::stats_ws_bytes_export(rows, K);
    case AWEQ_OP_QUANT_WEIGHT: return 16;  // tensor-wide extremes for group = -1
    case AWEQ_OP_EQUALIZE:
    case AWEQ_OP_W8A8_GEMM:
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
