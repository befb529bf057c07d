// Stage 4b: W8A8 GEMM  acc[t,n] = sum_k xq[t,k] wq[n,k]  (int8 x int8 -> int32) on the
// gfx950 matrix cores, with the epilogues the calibration path needs: raw int32 output,
// de-quantised output, and the per-output-channel sum over tokens (int64) that feeds the
// bias correction of Sec. 3.3.
//
// MFMA-bound.  One workgroup (4 wavefronts, one per SIMD) owns a 256 x 256 tile of the
// output; each wavefront owns 128 x 128 of it as 4 x 4 v_mfma_i32_32x32x32_i8 tiles
// (256 accumulator registers per lane).  Both operands are K-contiguous, so a lane's MFMA
// operand is 16 consecutive bytes of one row; tiles of 256 rows x 64 bytes are staged in LDS
// with an XOR swizzle of the 16-byte chunks and double-buffered against the global loads.
// Workgroups are numbered so that the ones resident on one XCD (which share an L2) form a
// compact patch of the output.
#include "common.hpp"

namespace aweq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kGemmThreads = 256;
constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kChunksPerRow = BK / 16;                       // 16-byte chunks per tile row
constexpr int kTileBytes = BM * BK;                          // 16 KiB per operand tile
constexpr int kLoadsPerThread = BM * kChunksPerRow / kGemmThreads;  // 4
constexpr int kXcds = 8;

// chunk position of (row, chunk) inside a tile row: rows that share LDS banks get distinct
// positions both for 8 and for 16 consecutive rows read at one chunk index
__device__ __forceinline__ int swz(int row, int chunk)
{
    const int g = (((row >> 2) & 1) << 1) | (((row >> 1) ^ (row >> 3)) & 1);
    return chunk ^ g;
}

struct GemmArgs {
    const int8_t* A;   // xq [T x K]
    const int8_t* B;   // wq [N x K]
    int64_t T, N, K;
    int32_t* out_i32;
    void* out_deq;
    int out_f16;
    int64_t ldo;
    long long* colsum_acc;
    const float* act_step;
    const int32_t* act_zero;
    const float* step_w;
    const int32_t* zero_w;
    const int32_t* rowsum_x;
    const int32_t* rowsum_w;
    const float* bias;
    int tiles_m, tiles_n, patch_m, patch_n, patches_n, n_patches;
};

__global__ __launch_bounds__(kGemmThreads) void gemm_i8_kernel(GemmArgs g)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    // [buffer][A | B][kTileBytes]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // ---- workgroup -> output tile.  Consecutive workgroup ids go round-robin over the XCDs,
    // so id % 8 names the XCD; each XCD walks its own sequence of patch_m x patch_n patches.
    const int b = blockIdx.x;
    const int xcd = b % kXcds;
    const int seq = b / kXcds;
    const int per_patch = g.patch_m * g.patch_n;
    const int patch = (seq / per_patch) * kXcds + xcd;
    if (patch >= g.n_patches) return;
    const int within = seq % per_patch;
    const int pm = patch / g.patches_n, pn = patch % g.patches_n;
    const int tile_m = pm * g.patch_m + within % g.patch_m;
    const int tile_n = pn * g.patch_n + within / g.patch_m;
    if (tile_m >= g.tiles_m || tile_n >= g.tiles_n) return;
    const int64_t m0 = (int64_t)tile_m * BM, n0 = (int64_t)tile_n * BN;

    // ---- global -> register staging: thread owns chunk (tid % 4) of rows tid/4 + 64 i
    const int ld_chunk = tid & (kChunksPerRow - 1);
    const int ld_row = tid / kChunksPerRow;
    const int8_t* a_ptr[kLoadsPerThread];
    const int8_t* b_ptr[kLoadsPerThread];
    int lds_off[kLoadsPerThread];
#pragma unroll
    for (int i = 0; i < kLoadsPerThread; ++i) {
        const int row = ld_row + i * (kGemmThreads / kChunksPerRow);
        // rows past the edge re-read the last valid row; their results are never stored
        const int64_t ra = min(m0 + row, g.T - 1), rb = min(n0 + row, g.N - 1);
        a_ptr[i] = g.A + ra * g.K + ld_chunk * 16;
        b_ptr[i] = g.B + rb * g.K + ld_chunk * 16;
        lds_off[i] = row * BK + swz(row, ld_chunk) * 16;
    }
    v4i ra[kLoadsPerThread], rb[kLoadsPerThread];
    const int nk = (int)((g.K + BK - 1) / BK);

    auto load_global = [&](int kt) {
        const int64_t k = (int64_t)kt * BK;
        const bool ok = k + ld_chunk * 16 < g.K;  // K % 16 == 0: a chunk is all in or all out
#pragma unroll
        for (int i = 0; i < kLoadsPerThread; ++i) {
            ra[i] = ok ? *reinterpret_cast<const v4i*>(a_ptr[i] + k) : v4i{0, 0, 0, 0};
            rb[i] = ok ? *reinterpret_cast<const v4i*>(b_ptr[i] + k) : v4i{0, 0, 0, 0};
        }
    };
    auto store_lds = [&](int buf) {
        char* base = lds + buf * 2 * kTileBytes;
#pragma unroll
        for (int i = 0; i < kLoadsPerThread; ++i) {
            *reinterpret_cast<v4i*>(base + lds_off[i]) = ra[i];
            *reinterpret_cast<v4i*>(base + kTileBytes + lds_off[i]) = rb[i];
        }
    };

    v16i acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    // operand fragment addresses: lane reads row (lane % 32) of a 32-row sub-tile, 16-byte
    // chunk (lane / 32) + 2 kk of the tile row
    const int fr_row = lane & 31;
    const int fr_half = lane >> 5;

    load_global(0);
    store_lds(0);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) load_global(kt + 1);
        const char* a_base = lds + (kt & 1) * 2 * kTileBytes;
        const char* b_base = a_base + kTileBytes;
#pragma unroll
        for (int kk = 0; kk < BK / 32; ++kk) {
            v4i af[4], bf[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = wm * 128 + i * 32 + fr_row;
                af[i] = *reinterpret_cast<const v4i*>(a_base + row * BK + swz(row, kk * 2 + fr_half) * 16);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int row = wn * 128 + j * 32 + fr_row;
                bf[j] = *reinterpret_cast<const v4i*>(b_base + row * BK + swz(row, kk * 2 + fr_half) * 16);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_lds((kt + 1) & 1);
        __syncthreads();
    }

    // ---- epilogue.  Accumulator register v of lane l in sub-tile (i, j) is the element
    // row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32.
    const int64_t col_base = n0 + wn * 128 + (lane & 31);
    const int64_t row_base = m0 + wm * 128 + 4 * (lane >> 5);

    if (g.out_i32) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int64_t t = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
                if (t < g.T) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        const int64_t n = col_base + j * 32;
                        if (n < g.N) g.out_i32[t * g.ldo + n] = acc[i][j][v];
                    }
                }
            }
    }

    if (g.out_deq) {
        const int zx = *g.act_zero - 128;
        const double sx = (double)*g.act_step;
        const int Ki = (int)g.K;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t n = col_base + j * 32;
            if (n >= g.N) continue;
            const int zw = g.zero_w[n] - 128;
            const double scale = sx * (double)g.step_w[n];
            const double bs = g.bias ? (double)g.bias[n] : 0.0;
            // integer part in wrap-around 32-bit arithmetic: the final value fits (|.| <= 255^2 K)
            const unsigned cn = (unsigned)Ki * (unsigned)zx * (unsigned)zw - (unsigned)zx * (unsigned)g.rowsum_w[n];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int64_t t = row_base + i * 32 + 8 * (v >> 2) + (v & 3);
                    if (t >= g.T) continue;
                    const unsigned iv = (unsigned)acc[i][j][v] + cn - (unsigned)zw * (unsigned)g.rowsum_x[t];
                    const float y = (float)((double)(int)iv * scale + bs);
                    if (g.out_f16) reinterpret_cast<_Float16*>(g.out_deq)[t * g.ldo + n] = (_Float16)y;
                    else reinterpret_cast<float*>(g.out_deq)[t * g.ldo + n] = y;
                }
        }
    }

    if (g.colsum_acc) {
        // per-lane column partials over the wavefront's 128 rows; groups of four fit in int32
        __syncthreads();  // the k-loop's LDS tiles are dead: reuse for the cross-wavefront sum
        long long* red = reinterpret_cast<long long*>(lds);  // [BN]
        long long cs[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            long long s = 0;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int v4 = 0; v4 < 4; ++v4) {
                    int part = 0;
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int64_t t = row_base + i * 32 + 8 * v4 + v;
                        part += (t < g.T) ? acc[i][j][v4 * 4 + v] : 0;
                    }
                    s += part;
                }
            s += partner<5>(s);  // lanes l and l + 32 hold the same column
            cs[j] = s;
        }
        if (wm == 1 && lane < 32) {
#pragma unroll
            for (int j = 0; j < 4; ++j) red[wn * 128 + j * 32 + lane] = cs[j];
        }
        __syncthreads();
        if (wm == 0 && lane < 32) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t n = col_base + j * 32;
                if (n < g.N)
                    atomicAdd(reinterpret_cast<unsigned long long*>(&g.colsum_acc[n]),
                              (unsigned long long)(cs[j] + red[wn * 128 + j * 32 + lane]));
            }
        }
    }
}

__global__ void zero_fill_u32_gemm(uint32_t* p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// from quant_act.hip
int launch_quant_act(const void* X, aweq_dtype dt, int64_t T, int64_t K, int64_t ldx, const float* inv_s,
                     const float* act_step, const int32_t* act_zero, int8_t* xq, int32_t* rowsum_x,
                     int64_t* colsum_xq, uint32_t* status, hipStream_t st);
int check_quant_act_args(const void* X, aweq_dtype dt, int64_t T, int64_t K, int64_t ldx, const float* inv_s,
                         const float* act_step, const int32_t* act_zero, const int8_t* xq);

}  // namespace aweq

using namespace aweq;

extern "C" int aweq_w8a8_gemm(const void* X, aweq_dtype x_dt, int64_t T, int64_t K, int64_t ldx,
                              const float* inv_s, const float* act_step, const int32_t* act_zero,
                              int8_t* xq, int32_t* rowsum_x, int64_t* colsum_xq,
                              const int8_t* wq, int64_t N, const float* step_w, const int32_t* zero_w,
                              const int32_t* rowsum_w, const float* bias,
                              int32_t* out_i32, void* out_deq, aweq_dtype out_dt, int64_t ldo,
                              int64_t* colsum_acc, void* ws, size_t ws_bytes,
                              uint32_t* status, void* stream)
{
    (void)ws; (void)ws_bytes;
    if (!X || !wq) return AWEQ_ERR_NULL;
    if (x_dt != AWEQ_F32 && x_dt != AWEQ_F16 && x_dt != AWEQ_I8) return AWEQ_ERR_DTYPE;
    if (T <= 0 || N <= 0 || K <= 0 || (K % 16) != 0) return AWEQ_ERR_SHAPE;
    if (K > 32768) return AWEQ_ERR_SHAPE;  // keeps 128*128*K and 255*255*K inside int32
    const int8_t* a = nullptr;
    if (x_dt == AWEQ_I8) {
        if (ldx != K) return AWEQ_ERR_SHAPE;
        a = reinterpret_cast<const int8_t*>(X);
    } else {
        const int rc = check_quant_act_args(X, x_dt, T, K, ldx, inv_s, act_step, act_zero, xq);
        if (rc != AWEQ_OK) return rc;
        a = xq;
    }
    if (!aligned16(a) || !aligned16(wq)) return AWEQ_ERR_ALIGN;
    if (out_i32 || out_deq) {
        if (ldo < N) return AWEQ_ERR_SHAPE;
    }
    if (out_deq) {
        if (out_dt != AWEQ_F32 && out_dt != AWEQ_F16) return AWEQ_ERR_DTYPE;
        if (!act_step || !act_zero || !step_w || !zero_w || !rowsum_x || !rowsum_w) return AWEQ_ERR_NULL;
    }
    const int64_t tiles_m = cdiv(T, BM), tiles_n = cdiv(N, BN);
    if (tiles_m * tiles_n > (1ll << 30)) return AWEQ_ERR_SHAPE;

    hipStream_t st = as_stream(stream);
    if (x_dt != AWEQ_I8) {
        const int rc = launch_quant_act(X, x_dt, T, K, ldx, inv_s, act_step, act_zero, xq, rowsum_x, colsum_xq, status, st);
        if (rc != AWEQ_OK) return rc;
    }
    if (!out_i32 && !out_deq && !colsum_acc) return launch_status();

    GemmArgs g;
    g.A = a; g.B = wq; g.T = T; g.N = N; g.K = K;
    g.out_i32 = out_i32; g.out_deq = out_deq; g.out_f16 = out_dt == AWEQ_F16; g.ldo = ldo;
    g.colsum_acc = reinterpret_cast<long long*>(colsum_acc);
    g.act_step = act_step; g.act_zero = act_zero; g.step_w = step_w; g.zero_w = zero_w;
    g.rowsum_x = rowsum_x; g.rowsum_w = rowsum_w; g.bias = bias;
    g.tiles_m = (int)tiles_m; g.tiles_n = (int)tiles_n;
    // patch of output tiles an XCD works on at a time: 32 tiles (one per compute unit)
    g.patch_n = (int)(tiles_n < 4 ? tiles_n : 4);
    g.patch_m = 32 / g.patch_n;
    if (g.patch_m > tiles_m) g.patch_m = (int)tiles_m;
    g.patches_n = (int)cdiv(tiles_n, g.patch_n);
    const int64_t patches_m = cdiv(tiles_m, g.patch_m);
    g.n_patches = (int)(patches_m * g.patches_n);
    const int64_t rounds = cdiv(g.n_patches, kXcds);
    const int64_t blocks = rounds * kXcds * g.patch_m * g.patch_n;
    if (blocks > 0x7fffffffll) return AWEQ_ERR_SHAPE;

    if (colsum_acc) zero_fill_u32_gemm<<<(unsigned)cdiv(2 * N, 256), 256, 0, st>>>(reinterpret_cast<uint32_t*>(colsum_acc), 2 * N);
    const size_t lds_bytes = 2 * 2 * kTileBytes;  // 64 KiB
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(gemm_i8_kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds_bytes) != hipSuccess)
        return AWEQ_ERR_LAUNCH;
    gemm_i8_kernel<<<(unsigned)blocks, kGemmThreads, lds_bytes, st>>>(g);
    return launch_status();
}
