// Stage 1: per-channel minimum / maximum / sum of a tall row-major matrix
// (Sec. 3.2: channel range and tensor range; Sec. 3.3: E[x] collected alongside).
//
// HBM-bound streaming pass.  Lanes own columns (16 bytes = 8 halves or 4 floats per lane),
// so a wavefront reads 1 KiB contiguous per row; the four wavefronts of a block take
// interleaved rows of one row slice and meet in LDS; each block writes one partial row of
// (min, max, sum) to the workspace, and a second small kernel folds the slices in a fixed
// order (so the fp64 sums are reproducible) and merges with earlier batches.
#include "common.hpp"
#include <atomic>

namespace aweq {

constexpr int kStatsBlock = 256;
constexpr int kStatsWaves = kStatsBlock / kWave;
constexpr int kRowBatch = 8;  // rows summed in fp32 before one fp64 add (binary16 input only)

struct StatsPlan {
    int col_chunks;   // blocks along K
    int slices;       // row slices
    int64_t rows_per_slice;
};

// Same plan on the host for the launch and for the workspace size.
inline StatsPlan stats_plan(int64_t rows, int64_t K, int elts_per_lane)
{
    StatsPlan p;
    const int64_t cols_per_block = (int64_t)kWave * elts_per_lane;
    p.col_chunks = (int)cdiv(K, cols_per_block);
    int64_t want = cdiv(1280, p.col_chunks);           // 5 blocks per compute unit, all resident: fewer partial rows to merge
    int64_t max_slices = cdiv(rows, kStatsWaves * kRowBatch);  // at least one row batch per wavefront
    if (want > max_slices) want = max_slices;
    if (want < 1) want = 1;
    p.rows_per_slice = cdiv(cdiv(rows, want), kStatsWaves * kRowBatch) * (kStatsWaves * kRowBatch);
    p.slices = (int)cdiv(rows, p.rows_per_slice);
    return p;
}

inline size_t stats_ws_bytes(int64_t rows, int64_t K)
{
    // sized for the narrower lane width (more chunks never increases the slice count)
    StatsPlan a = stats_plan(rows, K, 8), b = stats_plan(rows, K, 4);
    int s = a.slices > b.slices ? a.slices : b.slices;
    // partial rows, then the control words of the merge kernel (a ticket and the keys of the tensor's extremes)
    return (size_t)s * (size_t)K * (sizeof(float) * 2 + sizeof(double)) + 16;
}

// order-preserving unsigned key of a float (and back): integer atomics then find extremes
__device__ __forceinline__ uint32_t stats_key(float f)
{
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float stats_key_float(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// every byte of the matrix is read exactly once: non-temporal loads (7 - 10 % over plain ones here)
__device__ __forceinline__ Half8 load_once(const _Float16* p)
{
    typedef int v4i_ __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(Half8, __builtin_nontemporal_load(reinterpret_cast<const v4i_*>(p)));
}
__device__ __forceinline__ Float4 load_once(const float* p)
{
    typedef float v4f_ __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(Float4, __builtin_nontemporal_load(reinterpret_cast<const v4f_*>(p)));
}

// ---- binary16: 8 columns per lane
__global__ __launch_bounds__(kStatsBlock) void col_stats_partial_f16(
    const _Float16* __restrict__ M, int64_t rows, int64_t K, int64_t ld, int64_t rows_per_slice,
    float* __restrict__ pmin, float* __restrict__ pmax, double* __restrict__ psum, uint32_t* __restrict__ ctl)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    // the merge kernel that follows on the stream starts from a zero ticket and identity keys
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) { ctl[0] = 0u; ctl[1] = 0xffffffffu; ctl[2] = 0u; }
    const int64_t col = ((int64_t)blockIdx.x * kWave + lane) * 8;
    const bool active = col < K;
    const int64_t r_begin = (int64_t)blockIdx.y * rows_per_slice;
    const int64_t r_end = min(rows, r_begin + rows_per_slice);

    const f16x2 pinf = {(_Float16)INFINITY, (_Float16)INFINITY};
    const f16x2 ninf = {(_Float16)-INFINITY, (_Float16)-INFINITY};
    f16x2 mn[4] = {pinf, pinf, pinf, pinf};
    f16x2 mx[4] = {ninf, ninf, ninf, ninf};
    double sum[8] = {0, 0, 0, 0, 0, 0, 0, 0};

    if (active) {
        const _Float16* base = M + col;
        // wavefront w takes rows r_begin + w, + kStatsWaves, ...; kRowBatch rows in flight
        int64_t r = r_begin + wave;
        for (; r + (int64_t)(kRowBatch - 1) * kStatsWaves < r_end; r += (int64_t)kRowBatch * kStatsWaves) {
            Half8 v[kRowBatch];
#pragma unroll
            for (int j = 0; j < kRowBatch; ++j)
                v[j] = load_once(base + (r + (int64_t)j * kStatsWaves) * ld);
            float part[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < kRowBatch; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    mn[i] = hmin2(mn[i], v[j].h[i]);
                    mx[i] = hmax2(mx[i], v[j].h[i]);
                    float2 f = h2f2(v[j].h[i]);
                    part[2 * i] += f.x;
                    part[2 * i + 1] += f.y;
                }
#pragma unroll
            for (int i = 0; i < 8; ++i) sum[i] += (double)part[i];
        }
        for (; r < r_end; r += kStatsWaves) {
            Half8 v = load_once(base + r * ld);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                mn[i] = hmin2(mn[i], v.h[i]);
                mx[i] = hmax2(mx[i], v.h[i]);
                float2 f = h2f2(v.h[i]);
                sum[2 * i] += (double)f.x;
                sum[2 * i + 1] += (double)f.y;
            }
        }
    }

    // cross-wavefront combine in LDS: [wave][lane][8]
    __shared__ float s_mn[kStatsWaves][kWave][8];
    __shared__ float s_mx[kStatsWaves][kWave][8];
    __shared__ double s_sm[kStatsWaves][kWave][8];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        float2 a = h2f2(mn[i]), b = h2f2(mx[i]);
        s_mn[wave][lane][2 * i] = a.x; s_mn[wave][lane][2 * i + 1] = a.y;
        s_mx[wave][lane][2 * i] = b.x; s_mx[wave][lane][2 * i + 1] = b.y;
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) s_sm[wave][lane][i] = sum[i];
    __syncthreads();
    // 512 columns per block, 256 threads: two columns each
    for (int c = threadIdx.x; c < kWave * 8; c += kStatsBlock) {
        const int l = c >> 3, i = c & 7;
        float a = s_mn[0][l][i], b = s_mx[0][l][i];
        double s = s_sm[0][l][i];
#pragma unroll
        for (int w = 1; w < kStatsWaves; ++w) {
            a = fminf(a, s_mn[w][l][i]);
            b = fmaxf(b, s_mx[w][l][i]);
            s += s_sm[w][l][i];
        }
        const int64_t k = (int64_t)blockIdx.x * kWave * 8 + c;
        if (k < K) {
            const int64_t o = (int64_t)blockIdx.y * K + k;
            pmin[o] = a; pmax[o] = b; psum[o] = s;
        }
    }
}

// ---- binary32: 4 columns per lane, every element added in fp64
__global__ __launch_bounds__(kStatsBlock) void col_stats_partial_f32(
    const float* __restrict__ M, int64_t rows, int64_t K, int64_t ld, int64_t rows_per_slice,
    float* __restrict__ pmin, float* __restrict__ pmax, double* __restrict__ psum, uint32_t* __restrict__ ctl)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) { ctl[0] = 0u; ctl[1] = 0xffffffffu; ctl[2] = 0u; }
    const int64_t col = ((int64_t)blockIdx.x * kWave + lane) * 4;
    const bool active = col < K;
    const int64_t r_begin = (int64_t)blockIdx.y * rows_per_slice;
    const int64_t r_end = min(rows, r_begin + rows_per_slice);
    float mn[4] = {INFINITY, INFINITY, INFINITY, INFINITY};
    float mx[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    double sum[4] = {0, 0, 0, 0};
    if (active) {
        const float* base = M + col;
        int64_t r = r_begin + wave;
        for (; r + (int64_t)(kRowBatch - 1) * kStatsWaves < r_end; r += (int64_t)kRowBatch * kStatsWaves) {
            Float4 v[kRowBatch];
#pragma unroll
            for (int j = 0; j < kRowBatch; ++j)
                v[j] = load_once(base + (r + (int64_t)j * kStatsWaves) * ld);
#pragma unroll
            for (int j = 0; j < kRowBatch; ++j)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    mn[i] = fminf(mn[i], v[j].f[i]);
                    mx[i] = fmaxf(mx[i], v[j].f[i]);
                    sum[i] += (double)v[j].f[i];
                }
        }
        for (; r < r_end; r += kStatsWaves) {
            Float4 v = load_once(base + r * ld);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                mn[i] = fminf(mn[i], v.f[i]);
                mx[i] = fmaxf(mx[i], v.f[i]);
                sum[i] += (double)v.f[i];
            }
        }
    }
    __shared__ float s_mn[kStatsWaves][kWave][4];
    __shared__ float s_mx[kStatsWaves][kWave][4];
    __shared__ double s_sm[kStatsWaves][kWave][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        s_mn[wave][lane][i] = mn[i];
        s_mx[wave][lane][i] = mx[i];
        s_sm[wave][lane][i] = sum[i];
    }
    __syncthreads();
    {
        const int c = threadIdx.x;  // 256 columns per block, one per thread
        const int l = c >> 2, i = c & 3;
        float a = s_mn[0][l][i], b = s_mx[0][l][i];
        double s = s_sm[0][l][i];
#pragma unroll
        for (int w = 1; w < kStatsWaves; ++w) {
            a = fminf(a, s_mn[w][l][i]);
            b = fmaxf(b, s_mx[w][l][i]);
            s += s_sm[w][l][i];
        }
        const int64_t k = (int64_t)blockIdx.x * kWave * 4 + c;
        if (k < K) {
            const int64_t o = (int64_t)blockIdx.y * K + k;
            pmin[o] = a; pmax[o] = b; psum[o] = s;
        }
    }
}

// Fold the row slices and merge with what the caller already holds.  A block owns 32 columns;
// its 32 groups of 32 threads take every 32nd slice each (the kernel is bound by the latency of these
// few dependent loads, so they are spread over many threads) and meet in LDS in a fixed order, so
// the fp64 sums are reproducible.
// finalize: r = max - min per channel, R = tensor max - tensor min, p = r / R (Eq. 4) need every
// block's columns, so each block adds its extremes to two keys and takes a ticket; the block that
// draws the last ticket finds all columns merged and writes r, R, p.
constexpr int kMergeCols = 32, kMergeParts = 32;
__global__ __launch_bounds__(kMergeCols * kMergeParts) void col_stats_merge(
    const float* __restrict__ pmin, const float* __restrict__ pmax, const double* __restrict__ psum,
    int slices, int64_t K, int64_t rows, float* cmin, float* cmax,
    double* __restrict__ csum, uint64_t* __restrict__ count, int accumulate, uint32_t* status,
    int finalize, float* __restrict__ r, float* __restrict__ R, float* __restrict__ p, uint32_t* ctl)
{
    __shared__ float s_a[kMergeParts][kMergeCols], s_b[kMergeParts][kMergeCols];
    __shared__ double s_s[kMergeParts][kMergeCols];
    __shared__ int s_last;
    const int c = threadIdx.x & (kMergeCols - 1), part = threadIdx.x / kMergeCols;
    const int64_t k = (int64_t)blockIdx.x * kMergeCols + c;
    if (blockIdx.x == 0 && threadIdx.x == 0 && count) *count = (accumulate ? *count : 0ull) + (uint64_t)rows;
    float a = INFINITY, b = -INFINITY;
    double s = 0.0;
    if (k < K)
        for (int j = part; j < slices; j += kMergeParts) {
            a = fminf(a, pmin[(int64_t)j * K + k]);
            b = fmaxf(b, pmax[(int64_t)j * K + k]);
            s += psum[(int64_t)j * K + k];
        }
    s_a[part][c] = a; s_b[part][c] = b; s_s[part][c] = s;
    __syncthreads();
    if (part == 0 && k < K) {
#pragma unroll
        for (int q = 1; q < kMergeParts; ++q) {
            a = fminf(a, s_a[q][c]);
            b = fmaxf(b, s_b[q][c]);
            s += s_s[q][c];
        }
        // a non-finite input makes the fp64 sum (Inf / NaN) or an extreme (Inf) non-finite
        if (!isfinite(s) || isinf(a) || isinf(b)) raise_status(status, AWEQ_ST_NONFINITE);
        if (accumulate) {
            a = fminf(a, cmin[k]);
            b = fmaxf(b, cmax[k]);
            if (csum) s += csum[k];
        }
        cmin[k] = a;
        cmax[k] = b;
        if (csum) csum[k] = s;
    }
    if (!finalize) return;
    if (part == 0) {
        // this block's extremes (lanes past K hold the identities) -> the tensor's keys
        a = group_allreduce<5>(k < K ? a : INFINITY, OpMin());
        b = group_allreduce<5>(k < K ? b : -INFINITY, OpMax());
        if (c == 0) {
            atomicMin(&ctl[1], stats_key(a));
            atomicMax(&ctl[2], stats_key(b));
            __threadfence();   // columns and keys are visible device-wide before the ticket is
            s_last = atomicAdd(&ctl[0], 1u) == gridDim.x - 1;
        }
    }
    __syncthreads();
    if (!s_last) return;
    __threadfence();           // every other block's columns and keys are visible to this one
    const float RR = stats_key_float(__hip_atomic_load(&ctl[2], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) -
                     stats_key_float(__hip_atomic_load(&ctl[1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    if (threadIdx.x == 0) *R = RR;
    for (int64_t kk = threadIdx.x; kk < K; kk += blockDim.x) {
        const float rk = __hip_atomic_load(&cmax[kk], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) -
                         __hip_atomic_load(&cmin[kk], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        r[kk] = rk;
        if (p) p[kk] = rk / RR;
    }
}

size_t stats_ws_bytes_export(int64_t rows, int64_t K) { return stats_ws_bytes(rows, K); }

// the statistics pass on a workspace that is known to be large enough and 16-byte aligned
static int run_calib_stats(const void* M, aweq_dtype dt, int64_t rows, int64_t K, int64_t ld,
                           float* cmin, float* cmax, double* csum, uint64_t* count,
                           int accumulate, int finalize, float* r, float* R, float* p,
                           void* ws, uint32_t* status, hipStream_t st)
{
    const int epl = dt == AWEQ_F16 ? 8 : 4;
    const StatsPlan plan = stats_plan(rows, K, epl);
    // workspace layout: psum (fp64) first, then pmin, pmax
    double* psum = reinterpret_cast<double*>(ws);
    float* pmin = reinterpret_cast<float*>(psum + (size_t)plan.slices * K);
    float* pmax = pmin + (size_t)plan.slices * K;
    uint32_t* ctl = reinterpret_cast<uint32_t*>(pmax + (size_t)plan.slices * K);
    dim3 grid(plan.col_chunks, plan.slices);
    if (dt == AWEQ_F16)
        col_stats_partial_f16<<<grid, kStatsBlock, 0, st>>>(reinterpret_cast<const _Float16*>(M), rows, K, ld,
                                                             plan.rows_per_slice, pmin, pmax, psum, ctl);
    else
        col_stats_partial_f32<<<grid, kStatsBlock, 0, st>>>(reinterpret_cast<const float*>(M), rows, K, ld,
                                                             plan.rows_per_slice, pmin, pmax, psum, ctl);
    col_stats_merge<<<(unsigned)cdiv(K, kMergeCols), kMergeCols * kMergeParts, 0, st>>>(
        pmin, pmax, psum, plan.slices, K, rows, cmin, cmax, csum, count, accumulate, status, finalize, r, R, p, ctl);
    return launch_status();
}

static int check_calib_stats_args(const void* M, aweq_dtype dt, int64_t rows, int64_t K, int64_t ld,
                                  const float* cmin, const float* cmax, int finalize, const float* r, const float* R)
{
    if (!M || !cmin || !cmax) return AWEQ_ERR_NULL;
    if (finalize && (!r || !R)) return AWEQ_ERR_NULL;
    if (dt != AWEQ_F32 && dt != AWEQ_F16) return AWEQ_ERR_DTYPE;
    if (rows <= 0 || K <= 0 || ld < K || (K % 8) != 0) return AWEQ_ERR_SHAPE;
    if (!aligned16(M) || ((size_t)ld * dtype_size(dt)) % 16 != 0) return AWEQ_ERR_ALIGN;
    return AWEQ_OK;
}

// ---- scratch of the entry point that may not allocate: the per-slice partial rows live in a
// file-scope device array instead of a caller's workspace.  Every GPU the library runs on holds
// its own copy of the array (at its own address) until the process ends.
constexpr size_t kStaticScratchBytes = AWEQ_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::atomic<void*> g_scratch_of_device[kMaxDevices];

// device address of `scratch` on the current device (looked up once per device; in host code the
// array's name is only a handle for this lookup, never an address a kernel may be given)
static int static_scratch(void** out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return AWEQ_ERR_LAUNCH;
    void* ptr = g_scratch_of_device[dev].load(std::memory_order_acquire);
    if (!ptr) {
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return AWEQ_ERR_LAUNCH;
        g_scratch_of_device[dev].store(ptr, std::memory_order_release);   // (a racing thread stores the same address)
    }
    *out = ptr;
    return AWEQ_OK;
}

}  // namespace aweq

using namespace aweq;

extern "C" int aweq_calib_stats(const void* M, aweq_dtype dt, int64_t rows, int64_t K, int64_t ld,
                                float* cmin, float* cmax, double* csum, uint64_t* count,
                                int accumulate, int finalize, float* r, float* R, float* p,
                                void* ws, size_t ws_bytes, uint32_t* status, void* stream)
{
    const int rc = check_calib_stats_args(M, dt, rows, K, ld, cmin, cmax, finalize, r, R);
    if (rc != AWEQ_OK) return rc;
    if (!ws || ws_bytes < stats_ws_bytes(rows, K)) return AWEQ_ERR_WORKSPACE;
    if (!aligned16(ws)) return AWEQ_ERR_ALIGN;
    return run_calib_stats(M, dt, rows, K, ld, cmin, cmax, csum, count, accumulate, finalize, r, R, p, ws, status,
                           as_stream(stream));
}

extern "C" int aweq_calib_stats_static(const void* M, aweq_dtype dt, int64_t rows, int64_t K, int64_t ld,
                                       float* cmin, float* cmax, double* csum, uint64_t* count,
                                       int accumulate, int finalize, float* r, float* R, float* p,
                                       uint32_t* status, void* stream)
{
    const int rc = check_calib_stats_args(M, dt, rows, K, ld, cmin, cmax, finalize, r, R);
    if (rc != AWEQ_OK) return rc;
    if (stats_ws_bytes(rows, K) > kStaticScratchBytes) return AWEQ_ERR_WORKSPACE;   // beyond the built-in scratch
    void* ptr = nullptr;
    const int src = static_scratch(&ptr);
    if (src != AWEQ_OK) return src;
    // every partial row the merge reads, and the merge's ticket and keys, are written by this call's first
    // kernel: the array's contents from earlier calls never matter and nothing has to be cleared
    return run_calib_stats(M, dt, rows, K, ld, cmin, cmax, csum, count, accumulate, finalize, r, R, p, ptr, status,
                           as_stream(stream));
}
