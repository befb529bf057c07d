// Stage 4b: W8A8 GEMM  acc[t,n] = sum_k xq[t,k] wq[n,k]  (int8 x int8 -> int32) on the
// gfx950 matrix cores, with the epilogues the calibration path needs: raw int32 output,
// de-quantised output, and the per-output-channel sum over tokens (int64) that feeds the
// bias correction of Sec. 3.3.
//
// Both operands arrive in the K-panel layout (64-byte panels of K, rows back to back inside a
// panel, zero fill past K): the 256 rows x 64 bytes an output tile needs of one panel are one
// contiguous 16 KiB block, every cache line is used whole, and any K % 8 == 0 works.
//
// MFMA-bound by design, load-round-trip-bound in practice, which fixes the structure.  Two kernels:
//  - gemm_i8_fast (N % 4 == 0, 16-byte aligned outputs): one workgroup of 8 wavefronts
//    (two per SIMD) owns a 256 x 256 output tile, each wavefront 128 (t) x 64 (n) of it as
//    4 x 2 v_mfma_i32_32x32x32_i8 tiles; a lane's MFMA operand is 16 consecutive bytes of one
//    row.  Half-stages of one panel (256 rows x 64 bytes per operand, 32 KiB) go through a ring
//    of four LDS slots filled by LDS-DMA loads (global_load_lds_dwordx4, no staging registers),
//    three half-stages ahead of the one being multiplied: the round trip of a load under
//    load (about 1.5 us when part of it misses the L2) is longer than the 0.5 - 1 us a stage of
//    MFMAs lasts, so a two-buffer scheme stalls on every stage whatever the issue order.
//    The slots are XOR swizzled by choosing which 16-byte chunk each lane fetches; loads, LDS
//    fragment reads for the next K-step and MFMAs are interleaved by hand.  The MFMA is
//    issued with the weight fragment as its first operand, so a lane ends up with four
//    consecutive n of one token: 16-byte output stores.
//  - gemm_i8_generic (any N, any alignment): 4 wavefronts, half-stages through registers;
//    slower, used for shapes the fast kernel does not take.
// Workgroups are numbered so that the ones resident on one XCD (which share an L2) form a
// compact patch of the output.
#include "common.hpp"
#include <type_traits>

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
    const int8_t* A;   // xq [T x K], K-panel layout
    const int8_t* B;   // wq [N x K], K-panel layout
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
    int w_per_tensor;  // step_w / zero_w hold one entry for the whole weight instead of one per output channel
    int tiles_m, tiles_n, patch_m, patch_n, patches_n, n_patches;
    int n_ids;  // workgroup ids that may name a tile (whole rounds of patches over the XCDs)
    // tiled kernel: the tile columns that do not fill a whole patch column form patches of their own shape
    int main_pn, n_main, tail_cols, tail_pm, per_patch, n_patches_fast;
    // fused epilogues on the de-quantised binary16 output y (the next layer's calibration input)
    int act;                    // 0: none, 1: ReLU before y is rounded
    uint32_t* ykeys;            // [2 N] order-preserving keys of the column minimum / maximum of y
    long long* yfix;            // [N] column sums of y in units of 2^-24 (exact: y is binary16)
    const float* next_inv_s;    // [N] the next layer's 1 / s, Step and Z: y is quantised with them
    const float* next_step;
    const int32_t* next_zero;
    int8_t* yq;                 // [T x N] codes of y, K-panel layout (panels of 64 output channels)
    int32_t* rowsum_y;          // [T]
    long long* colsum_yq;       // [N]
    uint32_t* status;
};

// order-preserving unsigned key of a float (and back): integer atomics then find extremes
__device__ __forceinline__ uint32_t ykey(float f)
{
    const uint32_t b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float ykey_float(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ __launch_bounds__(kGemmThreads) void gemm_i8_generic(GemmArgs g)
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
        a_ptr[i] = g.A + ra * kPanel + ld_chunk * 16;
        b_ptr[i] = g.B + rb * kPanel + ld_chunk * 16;
        lds_off[i] = row * BK + swz(row, ld_chunk) * 16;
    }
    v4i ra[kLoadsPerThread], rb[kLoadsPerThread];
    const int nk = (int)panel_count(g.K);
    const int64_t panelA = g.T * kPanel, panelB = g.N * kPanel;

    auto load_global = [&](int kt) {
        // the last panel is zero filled past K in both operands
#pragma unroll
        for (int i = 0; i < kLoadsPerThread; ++i) {
            ra[i] = *reinterpret_cast<const v4i*>(a_ptr[i] + kt * panelA);
            rb[i] = *reinterpret_cast<const v4i*>(b_ptr[i] + kt * panelB);
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
            const int64_t pi = g.w_per_tensor ? 0 : n;
            const int zw = g.zero_w[pi] - 128;
            if (zw < -128 || zw > 127 || zx < -128 || zx > 127) raise_status(g.status, AWEQ_ST_ZEROPOINT);
            const double scale = sx * (double)g.step_w[pi];
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


// ---------------------------------------------------------------------------- fast kernel
namespace fast {
constexpr int kThreads = 512;
constexpr int kHalf = BM * kPanel;   // 16 KiB per operand per slot
constexpr int kSlot = 2 * kHalf;     // 32 KiB: one panel of the A tile and of the B tile
constexpr int kSlots = 4;
constexpr int kLds = kSlots * kSlot + 32768;  // 128 KiB ring + 32 KiB: the epilogue's slabs use the last slot and the tail = 160 KiB

// chunk swizzle for 64-byte slot rows: the four rows r, r + 4, r + 8, r + 12 share LDS banks,
// so 16 consecutive rows read at one chunk index land on distinct banks
__device__ __forceinline__ int f4(int r) { return (r >> 2) & 3; }

// LDS-DMA load the compiler does not track (it would otherwise wait for every outstanding one
// before each LDS read): lane i's 16 bytes land at lds_addr + 16 i, lds_addr wave-uniform.
// The global address is a wave-uniform base (SGPR pair) plus a 32-bit per-lane offset.
__device__ __forceinline__ void dma16(const int8_t* sbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

#define SB() __builtin_amdgcn_sched_barrier(0)
#define MF(A_, B_, i, j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(B_[j], A_[i], acc[i][j], 0, 0, 0)

// workgroup id -> output tile (false: the id names no tile).  Ids go round-robin over the XCDs,
// so id % 8 names the XCD; each XCD walks its own sequence of patch_m x patch_n patches.
// The last tile columns, when they do not fill a patch column, are walked as patches of their own
// shape (tail_pm x tail_cols, as many tiles as fit 32): a ragged patch would leave part of the XCD's
// workgroups without a tile, they would run ahead to their next id and the XCD's workgroups would
// stop walking K together, which is what lets them share operand panels in the L2.
__host__ __device__ __forceinline__ bool tile_of(const GemmArgs& g, int vb, int& tile_m, int& tile_n)
{
    const int xcd = vb % kXcds, seq = vb / kXcds;
    const int patch = (seq / g.per_patch) * kXcds + xcd;
    if (patch >= g.n_patches_fast) return false;
    const int within = seq % g.per_patch;
    if (patch < g.n_main) {
        const int pm = patch / g.main_pn, pn = patch % g.main_pn;
        tile_m = pm * g.patch_m + within % g.patch_m;
        tile_n = pn * g.patch_n + within / g.patch_m;
        return tile_m < g.tiles_m && tile_n < g.tiles_n;
    }
    if (within >= g.tail_pm * g.tail_cols) return false;
    tile_m = (patch - g.n_main) * g.tail_pm + within % g.tail_pm;
    tile_n = g.main_pn * g.patch_n + within / g.tail_pm;
    return tile_m < g.tiles_m;
}

// DEQ: 0 none, 1 fp32, 2 fp16.  Persistent: the grid is one workgroup per compute unit
// (a multiple of 8), workgroup b takes the ids b, b + grid, b + 2 grid, ...; the first panels
// of its next tile are requested before the epilogue of the current one starts, so the loads
// fly while the results are stored.
// EPI (with DEQ == 2): bit 0 collects the column statistics of the binary16 output, bit 1 quantises
// it for the next layer; STORE = false keeps the output itself from being written.
template <bool I32, int DEQ, bool COLSUM, int EPI = 0, bool STORE = true>
__global__ __launch_bounds__(kThreads) void gemm_i8_fast(GemmArgs g)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int stride = gridDim.x;

    int vb = blockIdx.x, tile_m = 0, tile_n = 0;
    while (vb < g.n_ids && !tile_of(g, vb, tile_m, tile_n)) vb += stride;
    if (vb >= g.n_ids) return;

    const int64_t panelA = g.T * kPanel, panelB = g.N * kPanel;
    const int nh = (int)panel_count(g.K);
    const int pre = nh < 3 ? nh : 3;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const uint32_t wave_off = __builtin_amdgcn_readfirstlane(wave) * 2048;

    // fragment of K-step ks of a panel: lane reads row lane % 32 of a 32-row sub-tile, chunk
    // 2 ks + lane / 32 (sub-tiles start at multiples of 32 rows, so f4(row) = f4(lane % 32))
    const int fr_row = lane & 31, fr_half = lane >> 5;
    int offA[2], offB[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        offA[ks] = (wm * 128 + fr_row) * kPanel + ((ks * 2 + fr_half) ^ f4(fr_row)) * 16;
        offB[ks] = kHalf + (wn * 64 + fr_row) * kPanel + ((ks * 2 + fr_half) ^ f4(fr_row)) * 16;
    }

    // global -> LDS: wave w brings tile rows 32 w .. 32 w + 31 of both operands, 16 rows x 64 B
    // per instruction; lane i sits at row i / 4, chunk slot i % 4 and fetches chunk slot ^ f4(row)
    uint32_t oa[2], ob[2];  // byte offsets from the tile's first row inside a panel: < 16 KiB
    const int8_t* srcA;     // the tile's rows in the panel being fetched
    const int8_t* srcB;
    int64_t m0, n0;

#define DMA_A(q) dma16(srcA, oa[q], dst_slot + (q) * 1024)
#define DMA_B(q) dma16(srcB, ob[q], dst_slot + kHalf + (q) * 1024)
    // addresses of tile (tm, tn) and its first `pre` panels on their way into slots 0 ..
    auto start_tile = [&](int tm, int tn) {
        // (wave-uniform by construction; say so, the panel base addresses live in scalar registers)
        m0 = (int64_t)__builtin_amdgcn_readfirstlane(tm) * BM;
        n0 = (int64_t)__builtin_amdgcn_readfirstlane(tn) * BN;
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            const int row = wave * 32 + q * 16 + (lane >> 2);
            const int chunk = (lane & 3) ^ f4(row);
            // rows past the edge re-read the last valid row; their results are never stored
            const int64_t ra = min(m0 + row, g.T - 1) - m0, rb = min(n0 + row, g.N - 1) - n0;
            oa[q] = (uint32_t)(ra * kPanel + chunk * 16);
            ob[q] = (uint32_t)(rb * kPanel + chunk * 16);
        }
        srcA = g.A + m0 * kPanel;
        srcB = g.B + n0 * kPanel;
        for (int h = 0; h < pre; ++h) {
            const uint32_t dst_slot = lds0 + h * kSlot + wave_off;
            DMA_A(0); DMA_B(0); DMA_A(1); DMA_B(1);
            srcA += panelA; srcB += panelB;
        }
    };

    start_tile(tile_m, tile_n);
    if (pre >= 3) wait_vm<8>(); else if (pre == 2) wait_vm<4>(); else wait_vm<0>();

    // Vector memory operations of a wave complete in the order issued.  A tile that lies inside
    // the output issues at least kStores stores per wave after requesting the next tile's first
    // three panels, so "at most kStores operations pending" means those panels have landed
    // while the stores may still be on their way (relaxed: set for the tile that follows).
    static_assert(EPI == 0 || DEQ == 2, "the fused epilogues work on the binary16 output");
    // 4 sub-tile rows x 8 passes each, per kind of output; the atomics of the fused epilogues come
    // on top and are not counted: a lower bound is what the relaxed wait needs
    constexpr int kStoresAll = (I32 ? 32 : 0) + (DEQ != 0 && STORE ? 32 : 0) + ((EPI & 2) != 0 ? 32 : 0);
    constexpr int kStores = kStoresAll > 63 ? 63 : kStoresAll;
    bool relaxed = false;

    for (;;) {
        const int64_t cm0 = m0, cn0 = n0;   // the tile being multiplied
        v16i acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
        v4i a0[4], b0[2], a1[4], b1[2];

#define RDA(dst, ks, i) dst[i] = *reinterpret_cast<const v4i*>(st + offA[ks] + (i) * 32 * kPanel)
#define RDB(dst, ks, j) dst[j] = *reinterpret_cast<const v4i*>(st + offB[ks] + (j) * 32 * kPanel)
        __builtin_amdgcn_s_barrier();  // panel 0 has landed for every wave
        {
            const char* st = lds;
#pragma unroll
            for (int i = 0; i < 4; ++i) RDA(a0, 0, i);
            RDB(b0, 0, 0); RDB(b0, 0, 1);
        }

        // one panel (64 bytes of K) = two K-steps of 8 MFMAs per wave.  F0 / F1 are the two
        // fragment register sets; each K-step multiplies one and fetches the other.  ISSUE: panel
        // h + 3 is fetched into the slot panel h - 1 occupied (every wave finished reading it before
        // the barrier of panel h - 1).  WAITN: loads this wave may leave in flight when panel h + 1
        // has to be complete (4 per panel issued after it).
        auto half = [&](int h, auto issue_c, auto waitn_c, auto next_c) {
            constexpr bool ISSUE = decltype(issue_c)::value;
            constexpr int WAITN = decltype(waitn_c)::value;
            constexpr bool NEXT = decltype(next_c)::value;
            const char* st = lds + (h & 3) * kSlot;
            const uint32_t dst_slot = lds0 + ((h + 3) & 3) * kSlot + wave_off;
            SB();
            RDA(a1, 1, 0); RDB(b1, 1, 0); RDB(b1, 1, 1); MF(a0, b0, 0, 0);
            SB();
            if constexpr (ISSUE) DMA_A(0);
            RDA(a1, 1, 1); RDA(a1, 1, 2); MF(a0, b0, 0, 1);
            SB();
            if constexpr (ISSUE) DMA_B(0);
            RDA(a1, 1, 3); MF(a0, b0, 1, 0);
            SB();
            if constexpr (ISSUE) DMA_A(1);
            MF(a0, b0, 1, 1);
            SB();
            if constexpr (ISSUE) DMA_B(1);
            MF(a0, b0, 2, 0); MF(a0, b0, 2, 1); MF(a0, b0, 3, 0); MF(a0, b0, 3, 1);
            SB();
            if constexpr (ISSUE) { srcA += panelA; srcB += panelB; }
            if constexpr (NEXT) {
                // my loads of the next panel have landed, my reads of this one are done; after the
                // barrier that holds for every wave
                wait_vm<WAITN>();
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                SB();
                st = lds + ((h + 1) & 3) * kSlot;
                RDA(a0, 0, 0); RDB(b0, 0, 0); RDB(b0, 0, 1); MF(a1, b1, 0, 0);
                SB();
                RDA(a0, 0, 1); RDA(a0, 0, 2); MF(a1, b1, 0, 1);
                SB();
                RDA(a0, 0, 3); MF(a1, b1, 1, 0);
                SB();
                MF(a1, b1, 1, 1); MF(a1, b1, 2, 0); MF(a1, b1, 2, 1); MF(a1, b1, 3, 0); MF(a1, b1, 3, 1);
                SB();
            } else {
                MF(a1, b1, 0, 0); MF(a1, b1, 0, 1); MF(a1, b1, 1, 0); MF(a1, b1, 1, 1);
                MF(a1, b1, 2, 0); MF(a1, b1, 2, 1); MF(a1, b1, 3, 0); MF(a1, b1, 3, 1);
            }
        };
        using I0 = std::integral_constant<int, 0>;
        using I4 = std::integral_constant<int, 4>;
        using I8 = std::integral_constant<int, 8>;
        using I63 = std::integral_constant<int, 63>;
        int h = 0;
        if (relaxed) {
            // panels 1 and 2 landed together with panel 0: nothing to wait for, and a count of 8
            // here would wait for the previous tile's stores
            half(0, std::true_type{}, I63{}, std::true_type{});
            half(1, std::true_type{}, I63{}, std::true_type{});
            h = 2;
        }
        for (; h + 3 < nh; ++h) half(h, std::true_type{}, I8{}, std::true_type{});
        if (h + 2 < nh) { half(h, std::false_type{}, I4{}, std::true_type{}); ++h; }
        if (h + 1 < nh) { half(h, std::false_type{}, I0{}, std::true_type{}); ++h; }
        half(h, std::false_type{}, I0{}, std::false_type{});
#undef RDA
#undef RDB

        // ---- epilogue.  With the weight fragment as first MFMA operand, register v of lane l in
        // sub-tile (i, j) is token t = m0 + 128 wm + 32 i + l % 32 and output channel
        // n = n0 + 64 wn + 32 j + 8 (v / 4) + 4 (l / 32) + v % 4: four consecutive n per register quad.
        // Each wave turns its 32 (t) x 64 (n) slab of sub-tile row i around in a private 8 KiB LDS
        // region (rows of 256 bytes, 16-byte chunks XOR swizzled: conflict-free both ways) so that a
        // lane then holds 16 bytes of one output row and 16 lanes cover 256 contiguous bytes per store.
        // The slabs live in the last ring slot and behind the ring; the next tile's first three
        // panels are already on their way into the other slots.
        const int rd_r = lane >> 4, rd_c = lane & 15;
        const int64_t t_lane = cm0 + wm * 128 + rd_r;              // + 32 i + 4 p
        const int64_t n = cn0 + wn * 64 + rd_c * 4;                // this lane's four channels
        const bool n_ok = n < g.N;                                 // N % 4 == 0: all four or none

        // everything the epilogue reads from memory is requested before the next tile's panels,
        // so that waiting for it does not wait for them
        int rsx[2] = {0, 0};   // row sums of this wave's 128 tokens, two per lane: token 64 h + lane
        Float4 sw = {{0.f, 0.f, 0.f, 0.f}}, bs = {{0.f, 0.f, 0.f, 0.f}};
        int zwv[4] = {0, 0, 0, 0};          // Z'w = Z_w - 128 of this lane's channels
        unsigned cn[4] = {0, 0, 0, 0};      // K Z'x Z'w - Z'x rowsum_w, in wrap-around 32-bit arithmetic
        uint32_t est = 0;                   // status bits this lane raises for the tile
        int zx = 0;
        float sxf = 0.f;
        if constexpr (DEQ != 0) {
            zx = *g.act_zero - 128;
            sxf = *g.act_step;
            zx = __builtin_amdgcn_readfirstlane(zx);
            sxf = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(sxf)));
            // the integer part is formed in 32-bit arithmetic: exact while it fits, which zero points in
            // [0, 255] guarantee for K <= 32768; anything else is flagged
            if (zx < -128 || zx > 127) est |= AWEQ_ST_ZEROPOINT;
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const int64_t t = cm0 + wm * 128 + hh * 64 + lane;
                rsx[hh] = t < g.T ? g.rowsum_x[t] : 0;
            }
            if (n_ok) {
                v4i zw4;
                if (g.w_per_tensor) {
                    const float s0 = g.step_w[0];
                    const int z0 = g.zero_w[0];
                    sw = Float4{{s0, s0, s0, s0}};
                    zw4 = v4i{z0, z0, z0, z0};
                } else {
                    sw = *reinterpret_cast<const Float4*>(g.step_w + n);
                    zw4 = *reinterpret_cast<const v4i*>(g.zero_w + n);
                }
                const v4i rw4 = *reinterpret_cast<const v4i*>(g.rowsum_w + n);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    zwv[c] = zw4[c] - 128;
                    if (zw4[c] < 0 || zw4[c] > 255) est |= AWEQ_ST_ZEROPOINT;
                    cn[c] = (unsigned)g.K * (unsigned)zx * (unsigned)zwv[c] - (unsigned)zx * (unsigned)rw4[c];
                }
                if (g.bias) bs = *reinterpret_cast<const Float4*>(g.bias + n);
            }
            // pin the values in registers here: the compiler's wait for them then sits before the
            // panel requests below, which it cannot see, instead of behind them
            asm volatile("" : "+v"(rsx[0]));
            asm volatile("" : "+v"(rsx[1]));
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                asm volatile("" : "+v"(sw.f[c]));
                asm volatile("" : "+v"(bs.f[c]));
                asm volatile("" : "+v"(zwv[c]));
                asm volatile("" : "+v"(cn[c]));
            }
        }
        Float4 nis = {{1.f, 1.f, 1.f, 1.f}};   // the next layer's 1 / s for this lane's four channels
        float nstep = 1.0f, nrstep = 1.0f, nthr = 0.0f;
        int nzero = 0;
        bool nscreen = false;
        if constexpr ((EPI & 2) != 0) {
            if (n_ok) nis = *reinterpret_cast<const Float4*>(g.next_inv_s + n);
            const ActParams np_ = act_params(g.next_step, g.next_zero, true);
            nstep = np_.step; nzero = np_.zero; nrstep = np_.rstep; nthr = np_.thr;
            // the one-FMA quotient with its distance-to-tie test (see the activation quantizer): valid
            // for this lane if no binary16 value times its 1 / s can reach a quotient of 2^24
            nscreen = np_.screen;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                asm volatile("" : "+v"(nis.f[c]));
                nscreen = nscreen && 65600.0f * fabsf(nis.f[c]) * nrstep < 16777216.0f;
            }
            nstep = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(nstep)));
            nrstep = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(nrstep)));
            nthr = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(nthr)));
            nzero = __builtin_amdgcn_readfirstlane(nzero);
        }

        // next tile of this workgroup
        int nvb = vb + stride, ntm = 0, ntn = 0;
        while (nvb < g.n_ids && !tile_of(g, nvb, ntm, ntn)) nvb += stride;
        const bool more = nvb < g.n_ids;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();  // every wave is done reading the ring
        if (more) start_tile(ntm, ntn);

        // per-channel constants of the de-quantisation
        double scale[4] = {0, 0, 0, 0}, bsd[4] = {0, 0, 0, 0};
        if constexpr (DEQ != 0) {
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                scale[c] = (double)sxf * (double)sw.f[c];
                bsd[c] = (double)bs.f[c];
            }
        }
        char* slab = lds + 3 * kSlot + wave * 8192;
        const int wr_t = lane & 31;
        const int wr_sw = wr_t & 15, wr_half = lane >> 5;           // chunk (8 j + 2 q + l / 32) ^ (t & 15)
        // column sums of the accumulator itself (never of the corrected integer, which wraps for zero points far
        // outside [0, 255]: the sums the bias correction needs do not depend on zero points)
        long long csum[4] = {0, 0, 0, 0};
        int rows_in = 0;   // rows of this lane inside T (the fused code epilogue turns unsigned sums into signed ones)
        float ymn[4] = {INFINITY, INFINITY, INFINITY, INFINITY}, ymx[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
        double ysum[4] = {0.0, 0.0, 0.0, 0.0};   // exact: at most 128 binary16 values each
        float cqf[4] = {0.f, 0.f, 0.f, 0.f};     // column sums of the next layer's unsigned codes over this tile (exact: 32 rows)
        const bool yq_pad = (EPI & 2) != 0 && !n_ok && cn0 + wn * 64 < g.N;   // zero fill of the last panel
        int8_t* const yq_lane = (EPI & 2) != 0 ? g.yq + (((cn0 >> 6) + wn) * g.T) * kPanel + rd_c * 4 : nullptr;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    v4i o = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    *reinterpret_cast<v4i*>(slab + wr_t * 256 + (((8 * j + 2 * q + wr_half) ^ wr_sw) * 16)) = o;
                }
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int r = 4 * p + rd_r;
                const v4i o = *reinterpret_cast<const v4i*>(slab + r * 256 + ((rd_c ^ (r & 15)) * 16));
                const int64_t t = t_lane + i * 32 + 4 * p;
                unsigned rs = 0;
                int rsy = 0;   // this lane's share of the token's code sum for the next layer
                // row sum of token 32 i + 4 p + lane / 16 of the wave: held by lane (that % 64), half
                // i / 2 (fetched with every lane active: a switched-off source lane would read as 0)
                if constexpr (DEQ != 0) rs = (unsigned)__builtin_amdgcn_ds_bpermute((((i & 1) * 32 + 4 * p + rd_r) & 63) * 4, rsx[i >> 1]);
                if (t < g.T && n_ok) {
                    if constexpr (I32) __builtin_nontemporal_store(o, reinterpret_cast<v4i*>(g.out_i32 + t * g.ldo + n));
                    if constexpr (DEQ != 0) {
                        float y[4];
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            // |row sum| <= 128 K < 2^23 and |Z'w| < 2^23 for any zero point binary16 weights can
                            // produce: a 24-bit multiply (full rate); wider zero points take the 32-bit one
                            const int zr = (zwv[c] < (1 << 23) && zwv[c] > -(1 << 23)) ? __mul24(zwv[c], (int)rs) : zwv[c] * (int)rs;
                            const int iv = (int)((unsigned)o[c] + cn[c] - (unsigned)zr);
                            const double div = (double)iv;
                            // the binary32 output is the fp64 product and sum rounded once (two fp64 operations,
                            // like the definition); for binary16 one fused fp64 operation is far inside the rounding
                            // (the variant with both fused epilogues is out of registers: it widens the bias here)
                            const double bd = EPI == 3 ? (double)bs.f[c] : bsd[c];
                            if constexpr (DEQ == 1) y[c] = (float)(div * scale[c] + bd);
                            else y[c] = (float)__builtin_fma(div, scale[c], bd);
                        }
                        if constexpr ((EPI & 2) != 0) ++rows_in;
                        if constexpr (DEQ == 2) {
                            typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                            if constexpr (EPI != 0) {
                                if (g.act == 1) {
#pragma unroll
                                    for (int c = 0; c < 4; ++c) y[c] = fmaxf(y[c], 0.0f);
                                }
                            }
                            h4 oh = {(_Float16)y[0], (_Float16)y[1], (_Float16)y[2], (_Float16)y[3]};
                            if constexpr (STORE)
                                __builtin_nontemporal_store(oh, reinterpret_cast<h4*>(reinterpret_cast<_Float16*>(g.out_deq) + t * g.ldo + n));
                            if constexpr ((EPI & 1) != 0) {
#pragma unroll
                                for (int c = 0; c < 4; ++c) {
                                    const float yf = (float)oh[c];
                                    ymn[c] = fminf(ymn[c], yf);
                                    ymx[c] = fmaxf(ymx[c], yf);
                                    ysum[c] += (double)yf;
                                }
                            }
                            if constexpr ((EPI & 2) != 0) {
                                uint32_t w = 0;
                                const float zf = (float)nzero;
                                float cn_[4];
                                float dmax = 0.0f;
#pragma unroll
                                for (int c = 0; c < 4; ++c) {
                                    const float a = __builtin_fmaf((float)oh[c], nis.f[c], 0.0f);
                                    const float q = __builtin_fmaf(a, nrstep, zf);
                                    cn_[c] = rintf(q);
                                    dmax = fmaxf(dmax, fabsf(q - cn_[c]));
                                }
                                if (!nscreen || dmax > nthr) {
#pragma unroll
                                    for (int c = 0; c < 4; ++c)
                                        cn_[c] = (float)quant_div((float)oh[c] * nis.f[c], nstep, nzero, 255, est);
                                }
#pragma unroll
                                for (int c = 0; c < 4; ++c) {
                                    const float u = __builtin_amdgcn_fmed3f(cn_[c], 0.0f, 255.0f);
                                    cqf[c] += u;
                                    w = __builtin_amdgcn_cvt_pk_u8_f32(u, c, w);
                                }
                                w ^= 0x80808080u;   // u - 128 as a byte
                                rsy = __builtin_amdgcn_sdot4((int)w, 0x01010101, 0, false);
                                *reinterpret_cast<uint32_t*>(yq_lane + t * kPanel) = w;
                            }
                        } else {
                            typedef float f4 __attribute__((ext_vector_type(4)));
                            f4 of = {y[0], y[1], y[2], y[3]};
                            __builtin_nontemporal_store(of, reinterpret_cast<f4*>(reinterpret_cast<float*>(g.out_deq) + t * g.ldo + n));
                        }
                    }
                    if constexpr (COLSUM) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) csum[c] += o[c];
                    }
                } else if (yq_pad && t < g.T) {
                    *reinterpret_cast<uint32_t*>(yq_lane + t * kPanel) = 0u;
                }
                if constexpr ((EPI & 2) != 0) {
                    // the 16 lanes of one output row (every lane active here)
                    rsy = group_allreduce<4>(rsy, OpAdd());
                    if (rd_c == 0 && t < g.T && g.rowsum_y) atomicAdd(&g.rowsum_y[t], rsy);
                }
            }
        }
        if constexpr ((EPI & 1) != 0) {
            // lanes l, l ^ 16, l ^ 32 hold the same channels for different tokens
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                ymn[c] = fminf(ymn[c], partner<4>(ymn[c]));
                ymn[c] = fminf(ymn[c], partner<5>(ymn[c]));
                ymx[c] = fmaxf(ymx[c], partner<4>(ymx[c]));
                ymx[c] = fmaxf(ymx[c], partner<5>(ymx[c]));
                ysum[c] += partner<4>(ysum[c]);
                ysum[c] += partner<5>(ysum[c]);
            }
            if (lane < 16 && n_ok && ymn[0] <= ymx[0]) {   // (no token of this tile row was inside T: nothing to add)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    atomicMin(&g.ykeys[n + c], ykey(ymn[c]));
                    atomicMax(&g.ykeys[g.N + n + c], ykey(ymx[c]));
                    double f = ysum[c] * 16777216.0;   // an integer: binary16 values are multiples of 2^-24
                    if (!(fabs(f) < 9.0e18)) { f = 0.0; est |= AWEQ_ST_NONFINITE; }
                    atomicAdd(reinterpret_cast<unsigned long long*>(&g.yfix[n + c]), (unsigned long long)(long long)f);
                }
            }
        }
        if constexpr ((EPI & 2) != 0) {
            int cq[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                cq[c] = (int)cqf[c] - 128 * rows_in;
                cq[c] += partner<4>(cq[c]);
                cq[c] += partner<5>(cq[c]);
            }
            if (lane < 16 && n_ok && g.colsum_yq) {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    atomicAdd(reinterpret_cast<unsigned long long*>(&g.colsum_yq[n + c]), (unsigned long long)(long long)cq[c]);
            }
        }
        if constexpr (EPI != 0 || DEQ != 0) raise_status(g.status, est);
        if constexpr (COLSUM) {
            // lanes l, l ^ 16, l ^ 32 hold the same channels for different tokens
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                csum[c] += partner<4>(csum[c]);
                csum[c] += partner<5>(csum[c]);
            }
            if (lane < 16 && n_ok) {
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    atomicAdd(reinterpret_cast<unsigned long long*>(&g.colsum_acc[n + c]), (unsigned long long)csum[c]);
            }
        }
        if (!more) break;
        vb = nvb;
        // the panels requested before the epilogue have landed
        relaxed = kStores > 0 && nh >= 6 && cm0 + BM <= g.T && cn0 + BN <= g.N;
        if (relaxed) wait_vm<kStores>();
        else wait_vm<0>();
    }
#undef DMA_A
#undef DMA_B
}
#undef SB
#undef MF
}  // namespace fast

__global__ void zero_fill_u32_gemm(uint32_t* p, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// from quant_act.hip
int launch_quant_act(const void* X, aweq_dtype dt, int64_t T, int64_t K, int64_t ldx, const float* inv_s,
                     const float* act_step, const int32_t* act_zero, int8_t* xq, int32_t* rowsum_x,
                     int64_t* colsum_xq, void* ws, uint32_t* status, hipStream_t st);
int check_quant_act_ws(int64_t T, int64_t K, const int32_t* rowsum_x, const int64_t* colsum_xq, const void* ws, size_t ws_bytes);
int check_quant_act_args(const void* X, aweq_dtype dt, int64_t T, int64_t K, int64_t ldx, const float* inv_s,
                         const float* act_step, const int32_t* act_zero, const int8_t* xq, bool xq_optional);

}  // namespace aweq

using namespace aweq;

namespace aweq {

// tile / patch plan of a launch
static int plan_gemm(GemmArgs& g, int64_t T, int64_t N, int64_t K, int64_t& blocks)
{
    const int64_t tiles_m = cdiv(T, BM), tiles_n = cdiv(N, BN);
    if (tiles_m * tiles_n > (1ll << 30)) return AWEQ_ERR_SHAPE;
    g.tiles_m = (int)tiles_m; g.tiles_n = (int)tiles_n;
    // patch of output tiles an XCD works on at a time: 32 tiles (one per compute unit), 8 (t) x 4 (n);
    // 4 x 8 when the contraction is long against N: the activation panels, the operand that does not
    // fit the memory-side cache, are then fetched half as often (1-2 % here, 9 % in the binary16 GEMM)
    const int want_n = K >= 2 * N ? 8 : 4;
    g.patch_n = (int)(tiles_n < want_n ? tiles_n : want_n);
    g.patch_m = 32 / g.patch_n;
    if (g.patch_m > tiles_m) g.patch_m = (int)tiles_m;
    g.patches_n = (int)cdiv(tiles_n, g.patch_n);
    const int64_t patches_m = cdiv(tiles_m, g.patch_m);
    g.n_patches = (int)(patches_m * g.patches_n);
    const int64_t rounds = cdiv(g.n_patches, kXcds);
    blocks = rounds * kXcds * g.patch_m * g.patch_n;   // grid of the generic kernel
    if (blocks > 0x7fffffffll) return AWEQ_ERR_SHAPE;
    // the tiled kernel's walk: whole patch columns first, then the remaining tile columns as patches of their own
    g.per_patch = g.patch_m * g.patch_n;
    g.tail_cols = (int)(tiles_n % g.patch_n);
    g.main_pn = (int)(tiles_n / g.patch_n);
    g.tail_pm = g.tail_cols ? g.per_patch / g.tail_cols : 0;
    if (g.tail_cols && g.tail_pm > tiles_m) g.tail_pm = (int)tiles_m;
    g.n_main = (int)(patches_m * g.main_pn);
    g.n_patches_fast = g.n_main + (g.tail_cols ? (int)cdiv(tiles_m, g.tail_pm) : 0);
    g.n_ids = (int)(cdiv(g.n_patches_fast, kXcds) * kXcds * g.per_patch);   // <= blocks
    return AWEQ_OK;
}

// persistent launch of a fast-kernel instantiation: one workgroup per compute unit (a multiple of
// 8, so that id % 8 stays the XCD)
static int launch_fast(const void* fn, GemmArgs& g, hipStream_t st)
{
    const int64_t blocks = g.n_ids;
    int dev = 0, cus = 0;
    if (device_cus(dev, cus) != AWEQ_OK || raise_lds_limit(fn, dev, fast::kLds) != AWEQ_OK) return AWEQ_ERR_LAUNCH;
    void* args[] = {&g};
    int64_t grid = (cus / kXcds) * kXcds;
    if (grid < kXcds) grid = kXcds;
    if (grid > blocks) grid = blocks;
    if (hipLaunchKernel(fn, dim3((unsigned)grid), dim3(fast::kThreads), args, fast::kLds, st) != hipSuccess) return AWEQ_ERR_LAUNCH;
    return launch_status();
}

static void clear_fused(GemmArgs& g)
{
    g.w_per_tensor = 0;
    g.act = 0; g.ykeys = nullptr; g.yfix = nullptr; g.next_inv_s = nullptr; g.next_step = nullptr; g.next_zero = nullptr;
    g.yq = nullptr; g.rowsum_y = nullptr; g.colsum_yq = nullptr; g.status = nullptr;
}

// accumulators of the fused epilogues start from their identities (fill kernels: graph-capturable)
__global__ void fused_init(uint32_t* ykeys, long long* yfix, int64_t N, long long* colsum_yq, int32_t* rowsum_y, int64_t T)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N) {
        if (ykeys) { ykeys[i] = 0xffffffffu; ykeys[N + i] = 0u; yfix[i] = 0; }
        if (colsum_yq) colsum_yq[i] = 0;
    }
    if (rowsum_y && i < T) rowsum_y[i] = 0;
}

// keys / fixed-point sums -> the outputs aweq_calib_stats would give on the stored output
__global__ void fused_stats_finish(const uint32_t* ykeys, const long long* yfix, int64_t N, int64_t T, float* cmin, float* cmax,
                                   double* csum, uint64_t* count, int accumulate, uint32_t* status)
{
    const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (n == 0 && count) *count = (accumulate ? *count : 0) + (uint64_t)T;
    if (n >= N) return;
    float a = ykey_float(ykeys[n]), b = ykey_float(ykeys[N + n]);
    double s = (double)yfix[n] * 5.9604644775390625e-08;   // 2^-24
    if (isinf(a) || isinf(b)) raise_status(status, AWEQ_ST_NONFINITE);
    if (accumulate) {
        a = fminf(a, cmin[n]);
        b = fmaxf(b, cmax[n]);
        if (csum) s += csum[n];
    }
    cmin[n] = a;
    cmax[n] = b;
    if (csum) csum[n] = s;
}

}  // namespace aweq

using namespace aweq;

extern "C" int aweq_w8a8_gemm(const void* X, aweq_dtype x_dt, int64_t T, int64_t K, int64_t ldx,
                              const float* inv_s, const float* act_step, const int32_t* act_zero,
                              int8_t* xq, int32_t* rowsum_x, int64_t* colsum_xq,
                              const int8_t* wq, int64_t N, const float* step_w, const int32_t* zero_w, int w_group,
                              const int32_t* rowsum_w, const float* bias,
                              int32_t* out_i32, void* out_deq, aweq_dtype out_dt, int64_t ldo,
                              int64_t* colsum_acc, void* ws, size_t ws_bytes,
                              uint32_t* status, void* stream)
{
    if (!X || !wq) return AWEQ_ERR_NULL;
    if (w_group != 0 && w_group != -1) return AWEQ_ERR_GROUP;
    if (x_dt != AWEQ_F32 && x_dt != AWEQ_F16 && x_dt != AWEQ_I8) return AWEQ_ERR_DTYPE;
    if (T <= 0 || N <= 0 || K <= 0 || (K % 8) != 0) return AWEQ_ERR_SHAPE;
    if (K > 32768) return AWEQ_ERR_SHAPE;  // keeps 128*128*K and 255*255*K inside int32
    const int8_t* a = nullptr;
    if (x_dt == AWEQ_I8) {
        if (ldx != K) return AWEQ_ERR_SHAPE;
        a = reinterpret_cast<const int8_t*>(X);
    } else {
        int rc = check_quant_act_args(X, x_dt, T, K, ldx, inv_s, act_step, act_zero, xq, false);
        if (rc != AWEQ_OK) return rc;
        rc = check_quant_act_ws(T, K, rowsum_x, colsum_xq, ws, ws_bytes);
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
    hipStream_t st = as_stream(stream);
    if (x_dt != AWEQ_I8) {
        const int rc = launch_quant_act(X, x_dt, T, K, ldx, inv_s, act_step, act_zero, xq, rowsum_x, colsum_xq, ws, status, st);
        if (rc != AWEQ_OK) return rc;
    }
    if (!out_i32 && !out_deq && !colsum_acc) return launch_status();

    GemmArgs g;
    g.A = a; g.B = wq; g.T = T; g.N = N; g.K = K;
    g.out_i32 = out_i32; g.out_deq = out_deq; g.out_f16 = out_dt == AWEQ_F16; g.ldo = ldo;
    g.colsum_acc = reinterpret_cast<long long*>(colsum_acc);
    g.act_step = act_step; g.act_zero = act_zero; g.step_w = step_w; g.zero_w = zero_w;
    g.rowsum_x = rowsum_x; g.rowsum_w = rowsum_w; g.bias = bias;
    clear_fused(g);
    g.w_per_tensor = w_group == -1;
    g.status = status;
    int64_t blocks = 0;
    const int prc = plan_gemm(g, T, N, K, blocks);
    if (prc != AWEQ_OK) return prc;

    if (colsum_acc) zero_fill_u32_gemm<<<(unsigned)cdiv(2 * N, 256), 256, 0, st>>>(reinterpret_cast<uint32_t*>(colsum_acc), 2 * N);

    // the fast kernel stores 16-byte output quads
    bool fast_ok = (N % 4) == 0;
    if (out_i32 && (!aligned16(out_i32) || (ldo % 4) != 0)) fast_ok = false;
    if (out_deq && (!aligned16(out_deq) || (ldo % 4) != 0 || (w_group == 0 && (!aligned16(step_w) || !aligned16(zero_w))) ||
                    !aligned16(rowsum_w) || (bias && !aligned16(bias))))
        fast_ok = false;
    if (fast_ok) {
        const int deq = out_deq ? (out_dt == AWEQ_F16 ? 2 : 1) : 0;
        const void* fn = nullptr;
#define AWEQ_PICK(I, D, C) if ((out_i32 != nullptr) == I && deq == D && (colsum_acc != nullptr) == C) fn = reinterpret_cast<const void*>(fast::gemm_i8_fast<I, D, C>);
        AWEQ_PICK(true, 0, true) AWEQ_PICK(true, 0, false) AWEQ_PICK(false, 0, true)
        AWEQ_PICK(true, 1, true) AWEQ_PICK(true, 1, false) AWEQ_PICK(false, 1, true) AWEQ_PICK(false, 1, false)
        AWEQ_PICK(true, 2, true) AWEQ_PICK(true, 2, false) AWEQ_PICK(false, 2, true) AWEQ_PICK(false, 2, false)
#undef AWEQ_PICK
        return launch_fast(fn, g, st);
    }
    const size_t lds_bytes = 2 * 2 * kTileBytes;  // 64 KiB
    int dev = 0, cus = 0;
    if (device_cus(dev, cus) != AWEQ_OK || raise_lds_limit(reinterpret_cast<const void*>(gemm_i8_generic), dev, (int)lds_bytes) != AWEQ_OK)
        return AWEQ_ERR_LAUNCH;
    gemm_i8_generic<<<(unsigned)blocks, kGemmThreads, lds_bytes, st>>>(g);
    return launch_status();
}

extern "C" int aweq_w8a8_gemm_fused(const int8_t* xq, int64_t T, int64_t K, const int8_t* wq, int64_t N,
                                    const float* act_step, const int32_t* act_zero,
                                    const float* step_w, const int32_t* zero_w,
                                    const int32_t* rowsum_x, const int32_t* rowsum_w, const float* bias, int act,
                                    void* out_f16, int64_t ldo, int64_t* colsum_acc,
                                    float* ycmin, float* ycmax, double* ycsum, uint64_t* ycount, int accumulate,
                                    const float* next_inv_s, const float* next_step, const int32_t* next_zero,
                                    int8_t* yq, int32_t* rowsum_y, int64_t* colsum_yq,
                                    void* ws, size_t ws_bytes, uint32_t* status, void* stream)
{
    if (!xq || !wq || !act_step || !act_zero || !step_w || !zero_w || !rowsum_x || !rowsum_w || !colsum_acc) return AWEQ_ERR_NULL;
    const bool want_stats = ycmin != nullptr, want_quant = yq != nullptr;
    if (!want_stats && !want_quant) return AWEQ_ERR_NULL;
    if (want_stats && !ycmax) return AWEQ_ERR_NULL;
    if (want_quant && (!next_inv_s || !next_step || !next_zero)) return AWEQ_ERR_NULL;
    if (act != 0 && act != 1) return AWEQ_ERR_SHAPE;
    if (T <= 0 || N <= 0 || K <= 0 || (K % 8) != 0 || K > 32768 || (N % 4) != 0) return AWEQ_ERR_SHAPE;
    if (out_f16 && (ldo < N || (ldo % 4) != 0)) return AWEQ_ERR_SHAPE;
    if (!aligned16(xq) || !aligned16(wq) || !aligned16(step_w) || !aligned16(zero_w) || !aligned16(rowsum_w) ||
        (bias && !aligned16(bias)) || (out_f16 && !aligned16(out_f16)) || (want_quant && (!aligned16(next_inv_s) || !aligned16(yq))))
        return AWEQ_ERR_ALIGN;
    if (want_stats && (!ws || ws_bytes < (size_t)N * 16)) return AWEQ_ERR_WORKSPACE;
    if (want_stats && !aligned16(ws)) return AWEQ_ERR_ALIGN;

    GemmArgs g;
    g.A = xq; g.B = wq; g.T = T; g.N = N; g.K = K;
    g.out_i32 = nullptr; g.out_deq = out_f16; g.out_f16 = 1; g.ldo = ldo;
    g.colsum_acc = reinterpret_cast<long long*>(colsum_acc);
    g.act_step = act_step; g.act_zero = act_zero; g.step_w = step_w; g.zero_w = zero_w;
    g.rowsum_x = rowsum_x; g.rowsum_w = rowsum_w; g.bias = bias;
    clear_fused(g);
    g.act = act; g.status = status;
    if (want_stats) {
        g.yfix = reinterpret_cast<long long*>(ws);
        g.ykeys = reinterpret_cast<uint32_t*>(g.yfix + N);
    }
    if (want_quant) {
        g.next_inv_s = next_inv_s; g.next_step = next_step; g.next_zero = next_zero;
        g.yq = yq; g.rowsum_y = rowsum_y; g.colsum_yq = reinterpret_cast<long long*>(colsum_yq);
    }
    int64_t blocks = 0;
    const int prc = plan_gemm(g, T, N, K, blocks);
    if (prc != AWEQ_OK) return prc;

    hipStream_t st = as_stream(stream);
    zero_fill_u32_gemm<<<(unsigned)cdiv(2 * N, 256), 256, 0, st>>>(reinterpret_cast<uint32_t*>(colsum_acc), 2 * N);
    const int64_t init_n = (want_quant && rowsum_y && T > N) ? T : N;
    fused_init<<<(unsigned)cdiv(init_n, 256), 256, 0, st>>>(g.ykeys, g.yfix, N, want_quant ? g.colsum_yq : nullptr,
                                                            want_quant ? rowsum_y : nullptr, T);
    const int epi = (want_stats ? 1 : 0) | (want_quant ? 2 : 0);
    const bool store = out_f16 != nullptr;
    const void* fn = nullptr;
#define AWEQ_PICK(E, S) if (epi == E && store == S) fn = reinterpret_cast<const void*>(fast::gemm_i8_fast<false, 2, true, E, S>);
    AWEQ_PICK(1, true) AWEQ_PICK(1, false) AWEQ_PICK(2, true) AWEQ_PICK(2, false) AWEQ_PICK(3, true) AWEQ_PICK(3, false)
#undef AWEQ_PICK
    const int rc = launch_fast(fn, g, st);
    if (rc != AWEQ_OK) return rc;
    if (want_stats)
        fused_stats_finish<<<(unsigned)cdiv(N, 256), 256, 0, st>>>(g.ykeys, g.yfix, N, T, ycmin, ycmax, ycsum, ycount, accumulate, status);
    return launch_status();
}
