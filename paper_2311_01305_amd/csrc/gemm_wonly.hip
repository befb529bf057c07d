// Weight-only forward  y[t,n] = sum_k x_hat[t,k] w~[n,k] + b[n]  for the ultra-low-bit setting of
// Sec. 4.2 (INT4 / INT3 weights per group along K, FP16 activations): the weight codes are
// de-quantised (Eq. 1: w~ = Step (u - Z)) into binary16 and multiplied on the matrix cores
// (v_mfma_f32_32x32x16_f16, fp32 accumulation).
//
// Two kernels.  dequant_weight_h_kernel writes the binary16 weight [N x K] once per call into
// the caller's workspace: at calibration sizes (hundreds of thousands of tokens) that pass is
// noise, while de-quantising inside the GEMM costs every row tile of tokens the same VALU work
// again (measured: a third of the GEMM's time).  A lane widens two codes at a time into
// binary16 with the 1024 + u trick (the bit pattern 0x6400 | u is the binary16 number
// 1024 + u), subtracts 1024 + Z and multiplies by Step with packed binary16 arithmetic.  Step
// is rounded to binary16 first; for |u - Z| <= 2048 the packed product is the correctly
// rounded binary16 value of (u - Z) Step_h, the value the host-side definition fixes; zero
// points outside [-1024, 1024] take a binary32 path with the same result.
// gemm_f16_kernel: one workgroup of 8 wavefronts (two per SIMD) owns a 256 (t) x 256 (n) output
// tile, each wavefront 128 x 64 of it as 4 x 2 MFMA tiles.  A stage is 64 values of K = 128 bytes
// per row (whole cache lines of both row-major operands), brought in by LDS-DMA loads the
// compiler does not track.  The activation half of a stage goes through a ring of three
// 32 KiB slots (two stages ahead: it misses the L2 twice as often as the weight half and its
// round trip does not fit in one stage), the weight half through two slots; with the
// wavefront's loads retiring in issue order, "at most the 4 newest outstanding" at the end of a
// stage means everything the next stage reads has landed.  The MFMA is issued with the weight
// fragment first so that a lane ends with four consecutive n of one token.
#include "common.hpp"
#include <type_traits>

namespace aweq {
namespace wonly {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int kThreads = 512;
constexpr int BM = 256, BN = 256;
constexpr int BKH = 64;              // values of K per stage
constexpr int kRow = BKH * 2;        // bytes per tile row per stage
constexpr int kTile = BM * kRow;     // 32 KiB per operand
constexpr int kSlotsA = 3;
constexpr int kLdsB = kSlotsA * kTile;          // weight slots start behind the activation ring
constexpr int kLds = kSlotsA * kTile + 2 * kTile;  // 160 KiB
constexpr int kXcds = 8;

struct Args {
    const _Float16* X;     // x_hat [T x K], row-major
    int64_t ldx;
    const _Float16* W;     // de-quantised weight [N x K], row-major (the workspace)
    const float* bias;
    void* out;
    int64_t ldo;
    int64_t T, N, K;
    int tiles_m, tiles_n, patch_m, patch_n, n_patches;
    // the tile columns that do not fill a whole patch column form patches of their own shape
    int main_pn, n_main, tail_cols, tail_pm, per_patch;
    int n_ids;  // workgroup ids that may name a tile (whole rounds of patches over the XCDs)
};

// chunk swizzle for 128-byte tile rows: rows sharing LDS banks get distinct chunk positions
// both for 8 and for 16 consecutive rows read at one chunk index
__device__ __forceinline__ int g8(int r) { return (((r >> 1) & 3) << 1) | (((r >> 3) ^ r) & 1); }

// LDS-DMA load the compiler does not track: lane i's 16 bytes land at lds_addr + 16 i
__device__ __forceinline__ void dma16(const char* sbase, uint32_t voff, uint32_t lds_addr)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
}

__device__ __forceinline__ f16x2 as_h2(uint32_t u) { return __builtin_bit_cast(f16x2, u); }
__device__ __forceinline__ uint32_t as_u32(f16x2 h) { return __builtin_bit_cast(uint32_t, h); }

// 32 consecutive codes of one row (the lane's half of a stage row), as loaded
template <int BITS> struct RawCodes { uint32_t w[BITS == 4 ? 4 : 3]; };

// de-quantise the 8 codes k = 8 d .. 8 d + 7 of the lane's 32 into one 16-byte chunk (natural k order)
template <int BITS>
__device__ __forceinline__ v4i dequant8(const RawCodes<BITS>& rc, int d, float step_h, int z, bool fast)
{
    uint32_t o[4];
    if (fast) {
        const f16x2 zs = as_h2(0x64006400u) + f16x2{(_Float16)z, (_Float16)z};       // 1024 + Z, exact
        const f16x2 sp = {(_Float16)step_h, (_Float16)step_h};
        if constexpr (BITS == 4) {
            // (w >> 4 i) & 0x000f000f holds codes i and i + 4 of the dword in its two halves
            f16x2 h[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) h[i] = (as_h2(((rc.w[d] >> (4 * i)) & 0x000f000fu) | 0x64006400u) - zs) * sp;
            o[0] = __builtin_amdgcn_perm(as_u32(h[1]), as_u32(h[0]), 0x05040100u);  // k0 k1
            o[1] = __builtin_amdgcn_perm(as_u32(h[3]), as_u32(h[2]), 0x05040100u);  // k2 k3
            o[2] = __builtin_amdgcn_perm(as_u32(h[1]), as_u32(h[0]), 0x07060302u);  // k4 k5
            o[3] = __builtin_amdgcn_perm(as_u32(h[3]), as_u32(h[2]), 0x07060302u);  // k6 k7
        } else {
            // codes 2 j, 2 j + 1 are the 6 bits at bit 6 j of the 96-bit stream
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int j = 4 * d + q, bit = 6 * j, idx = bit >> 5, sh = bit & 31;
                const uint32_t lo = rc.w[idx], hi = idx + 1 < 3 ? rc.w[idx + 1] : 0u;
                const uint32_t f = __builtin_amdgcn_alignbit(hi, lo, sh);
                const uint32_t u2 = ((f & 0x38u) << 13) | ((f & 7u) | 0x64006400u);
                o[q] = as_u32((as_h2(u2) - zs) * sp);
            }
        }
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int c[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int k = 8 * d + 2 * q + e;
                if constexpr (BITS == 4) c[e] = (int)((rc.w[k >> 3] >> (4 * (k & 7))) & 15u);
                else {
                    const int bit = 3 * k, idx = bit >> 5, sh = bit & 31;
                    const uint32_t lo = rc.w[idx], hi = idx + 1 < 3 ? rc.w[idx + 1] : 0u;
                    c[e] = (int)(__builtin_amdgcn_alignbit(hi, lo, sh) & 7u);
                }
            }
            const f16x2 h = {(_Float16)((float)(c[0] - z) * step_h), (_Float16)((float)(c[1] - z) * step_h)};
            o[q] = as_u32(h);
        }
    }
    return v4i{(int)o[0], (int)o[1], (int)o[2], (int)o[3]};
}

// one thread per 32 consecutive codes of a row: 16 (INT4) or 12 (INT3) bytes in, 64 bytes out
template <int BITS>
__global__ __launch_bounds__(256) void dequant_weight_h_kernel(
    const uint8_t* __restrict__ codes, int64_t N, int64_t K, int group, const float* __restrict__ step,
    const int32_t* __restrict__ zero, _Float16* __restrict__ W)
{
    const int64_t per_row = K / 32;
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= N * per_row) return;
    const int64_t n = id / per_row, kk = id % per_row;
    const uint8_t* p = codes + n * (K * BITS / 8) + kk * (32 * BITS / 8);
    RawCodes<BITS> rc;
    if constexpr (BITS == 4) {
        const v4i w = *reinterpret_cast<const v4i*>(p);
        rc.w[0] = (uint32_t)w[0]; rc.w[1] = (uint32_t)w[1]; rc.w[2] = (uint32_t)w[2]; rc.w[3] = (uint32_t)w[3];
    } else {
        const uint32_t* p32 = reinterpret_cast<const uint32_t*>(p);
        rc.w[0] = p32[0]; rc.w[1] = p32[1]; rc.w[2] = p32[2];
    }
    const int64_t pi = group < 0 ? 0 : (group == 0 ? n : n * (K / group) + (kk * 32) / group);
    const float step_h = (float)(_Float16)step[pi];   // Step as binary16
    const int z = zero[pi];
    const bool fast = z >= -1024 && z <= 1024;
    v4i* dst = reinterpret_cast<v4i*>(W + n * K + kk * 32);
#pragma unroll
    for (int d = 0; d < 4; ++d) dst[d] = dequant8<BITS>(rc, d, step_h, z, fast);
}

#define SB() __builtin_amdgcn_sched_barrier(0)
#define MF(A_, B_, i, j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, B_[j]), __builtin_bit_cast(v8h, A_[i]), acc[i][j], 0, 0, 0)
template <int N>
__device__ __forceinline__ void wait_vm()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// workgroup id -> output tile (false: the id names no tile).  Ids go round-robin over the XCDs, so
// id % 8 names the XCD; each XCD walks its own sequence of patches of 32 tiles.  The tile columns that
// do not fill a whole patch column form patches of their own shape (tail_pm x tail_cols), so that an
// XCD's 32 workgroups always start a patch together and walk K together (a ragged patch would leave
// some of them without a tile).
__device__ __forceinline__ bool tile_of(const Args& g, int vb, int& tile_m, int& tile_n)
{
    const int xcd = vb % kXcds, seq = vb / kXcds;
    const int patch = (seq / g.per_patch) * kXcds + xcd;
    if (patch >= g.n_patches) return false;
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

// Persistent: the grid is one workgroup per compute unit (a multiple of 8), workgroup b takes the ids
// b, b + grid, b + 2 grid, ...; the first stages of its next tile are requested before the epilogue of
// the current one starts, so the loads fly while the results are stored.
template <bool OUT_F16>
__global__ __launch_bounds__(kThreads) void gemm_f16_kernel(Args g)
{
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 2, wn = wave & 3;
    const int stride = gridDim.x;

    int vb = blockIdx.x, tile_m = 0, tile_n = 0;
    while (vb < g.n_ids && !tile_of(g, vb, tile_m, tile_n)) vb += stride;
    if (vb >= g.n_ids) return;

    const int ns = (int)(g.K / BKH);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
    const uint32_t wave_off = __builtin_amdgcn_readfirstlane(wave) * 4096;

    // fragment of K-step qq (16 values = 32 bytes per row): lane reads row lane % 32 of a 32-row
    // sub-tile, chunk 2 qq + lane / 32
    const int fr_row = lane & 31, fr_half = lane >> 5;
    const int fsw = g8(fr_row);
    int offA[4], offB[4];
#pragma unroll
    for (int qq = 0; qq < 4; ++qq) {
        offA[qq] = (wm * 128 + fr_row) * kRow + ((qq * 2 + fr_half) ^ fsw) * 16;
        offB[qq] = kLdsB + (wn * 64 + fr_row) * kRow + ((qq * 2 + fr_half) ^ fsw) * 16;
    }

    // global -> LDS: wave w brings tile rows 32 w .. 32 w + 31 of both operands, 8 rows x 128 B per
    // instruction; lane i sits at row i / 8, chunk slot i % 8 and fetches chunk slot ^ g8(row)
    const char* baseA;   // the tile's first rows (wave-uniform: scalar registers)
    const char* baseB;
    uint32_t oa[4], ob[4];  // byte offsets from the tile's first row: < 256 * 2 ldx
    int64_t m0, n0;

#define RDA(dst, qq, i) dst[i] = *reinterpret_cast<const v4i*>(sa + offA[qq] + (i) * 32 * kRow)
#define RDB(dst, qq, j) dst[j] = *reinterpret_cast<const v4i*>(sb + offB[qq] + (j) * 32 * kRow)
#define DMA_A(q, s_) dma16(baseA + (int64_t)(s_) * kRow, oa[q], lds0 + ((s_) % kSlotsA) * kTile + wave_off + (q) * 1024)
#define DMA_B(q, s_) dma16(baseB + (int64_t)(s_) * kRow, ob[q], lds0 + kLdsB + ((s_) & 1) * kTile + wave_off + (q) * 1024)

    // addresses of tile (tm, tn); stage 0 of both operands and stage 1 of the activations on their way
    // (activation slots 0 and 1, weight slot 0)
    auto start_tile = [&](int tm, int tn) {
        m0 = (int64_t)__builtin_amdgcn_readfirstlane(tm) * BM;
        n0 = (int64_t)__builtin_amdgcn_readfirstlane(tn) * BN;
        baseA = reinterpret_cast<const char*>(g.X + m0 * g.ldx);
        baseB = reinterpret_cast<const char*>(g.W + n0 * g.K);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int row = wave * 32 + q * 8 + (lane >> 3);
            const int chunk = (lane & 7) ^ g8(row);
            // rows past the edge re-read the last valid row; their results are never stored
            const int64_t ra = min(m0 + row, g.T - 1) - m0, rb = min(n0 + row, g.N - 1) - n0;
            oa[q] = (uint32_t)(ra * g.ldx * 2 + chunk * 16);
            ob[q] = (uint32_t)(rb * g.K * 2 + chunk * 16);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) DMA_A(q, 0);
#pragma unroll
        for (int q = 0; q < 4; ++q) DMA_B(q, 0);
        if (ns > 1) {
#pragma unroll
            for (int q = 0; q < 4; ++q) DMA_A(q, 1);
        }
    };

    start_tile(tile_m, tile_n);
    if (ns > 1) wait_vm<4>(); else wait_vm<0>();

    // Vector memory operations of a wave complete in the order issued.  A tile that lies inside the
    // output issues 32 stores per wave after requesting the next tile's first stages, so "at most
    // 32 + 4 operations pending" means stage 0 has landed while the stores (and the 4 loads of the
    // activations' stage 1) may still be on their way.
    constexpr int kStores = 32;

    for (;;) {
        const int64_t cm0 = m0, cn0 = n0;   // the tile being multiplied
        v16f acc[4][2];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
        v4i a0[4], b0[2], a1[4], b1[2];

        __builtin_amdgcn_s_barrier();   // stage 0 has landed for every wave
        {
            const char* sa = lds;
            const char* sb = lds;
#pragma unroll
            for (int i = 0; i < 4; ++i) RDA(a0, 0, i);
            RDB(b0, 0, 0); RDB(b0, 0, 1);
        }

        // one stage (64 values of K) = four K-steps of 8 MFMAs per wave.  F0 / F1 are the two fragment
        // register sets; each K-step multiplies one and fetches the other.  NEXT: there is a stage
        // s + 1 (its weights are requested here); NEXT2: there is a stage s + 2 (its activations are).
        auto stage = [&](int s, auto next_c, auto next2_c) {
            constexpr bool NEXT = decltype(next_c)::value;
            constexpr bool NEXT2 = decltype(next2_c)::value;
            const char* sa = lds + (s % kSlotsA) * kTile;
            const char* sb = lds + (s & 1) * kTile;
            // K-step 0: multiply F0, fetch F1.  The slots of stage s - 1 are free (every wave passed that
            // stage's barrier): the weights of stage s + 1 and the activations of stage s + 2 go there
            SB();
            RDA(a1, 1, 0); RDB(b1, 1, 0); RDB(b1, 1, 1); MF(a0, b0, 0, 0);
            SB();
            if constexpr (NEXT) DMA_B(0, s + 1);
            RDA(a1, 1, 1); RDA(a1, 1, 2); MF(a0, b0, 0, 1);
            SB();
            if constexpr (NEXT) DMA_B(1, s + 1);
            RDA(a1, 1, 3); MF(a0, b0, 1, 0);
            SB();
            if constexpr (NEXT) DMA_B(2, s + 1);
            MF(a0, b0, 1, 1);
            SB();
            if constexpr (NEXT) DMA_B(3, s + 1);
            MF(a0, b0, 2, 0); MF(a0, b0, 2, 1); MF(a0, b0, 3, 0); MF(a0, b0, 3, 1);
            SB();
            // K-step 1: multiply F1, fetch F0
            RDA(a0, 2, 0); RDB(b0, 2, 0); RDB(b0, 2, 1); MF(a1, b1, 0, 0);
            SB();
            if constexpr (NEXT2) DMA_A(0, s + 2);
            RDA(a0, 2, 1); RDA(a0, 2, 2); MF(a1, b1, 0, 1);
            SB();
            if constexpr (NEXT2) DMA_A(1, s + 2);
            RDA(a0, 2, 3); MF(a1, b1, 1, 0);
            SB();
            if constexpr (NEXT2) DMA_A(2, s + 2);
            MF(a1, b1, 1, 1);
            SB();
            if constexpr (NEXT2) DMA_A(3, s + 2);
            MF(a1, b1, 2, 0); MF(a1, b1, 2, 1); MF(a1, b1, 3, 0); MF(a1, b1, 3, 1);
            SB();
            // K-step 2: multiply F0, fetch F1
            RDA(a1, 3, 0); RDB(b1, 3, 0); RDB(b1, 3, 1); MF(a0, b0, 0, 0);
            SB();
            RDA(a1, 3, 1); RDA(a1, 3, 2); MF(a0, b0, 0, 1);
            SB();
            RDA(a1, 3, 3); MF(a0, b0, 1, 0);
            SB();
            MF(a0, b0, 1, 1); MF(a0, b0, 2, 0); MF(a0, b0, 2, 1); MF(a0, b0, 3, 0); MF(a0, b0, 3, 1);
            SB();
            if constexpr (NEXT) {
                // stage s + 1 has landed for this wave (only the 4 newest loads, the activations of stage
                // s + 2, may still be out), its reads of stage s are done; after the barrier that holds
                // for every wave
                if constexpr (NEXT2) wait_vm<4>(); else wait_vm<0>();
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                SB();
                sa = lds + ((s + 1) % kSlotsA) * kTile;
                sb = lds + ((s + 1) & 1) * kTile;
                // K-step 3: multiply F1, fetch F0 = K-step 0 of the next stage
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
        int s = 0;
        for (; s + 2 < ns; ++s) stage(s, std::true_type{}, std::true_type{});
        if (s + 1 < ns) { stage(s, std::true_type{}, std::false_type{}); ++s; }
        stage(s, std::false_type{}, std::false_type{});

        // ---- epilogue.  With the weight fragment as first MFMA operand, register v of lane l in
        // sub-tile (i, j) is token t = m0 + 128 wm + 32 i + l % 32 and output channel
        // n = n0 + 64 wn + 32 j + 8 (v / 4) + 4 (l / 32) + v % 4.  Each wave turns its 32 (t) x 64 (n)
        // slab of sub-tile row i around in a private 8 KiB LDS region (256-byte rows, XOR-swizzled
        // 16-byte chunks) so that 16 lanes cover one output row of the slab per store.  The slabs live
        // in the third activation slot and the second weight slot: the next tile's first stages are
        // already on their way into the others.
        const int wr_t = lane & 31, wr_sw = wr_t & 15, wr_half = lane >> 5;
        const int rd_r = lane >> 4, rd_c = lane & 15;
        const int64_t n = cn0 + wn * 64 + rd_c * 4;      // this lane's four channels
        const bool n_ok = n < g.N;                       // N % 4 == 0: all four or none
        const int64_t t_lane = cm0 + wm * 128 + rd_r;    // + 32 i + 4 p
        // what the epilogue reads from memory is requested before the next tile's stages, so that
        // waiting for it does not wait for them (pinned: the compiler's wait then sits here)
        v4f bs = {0.f, 0.f, 0.f, 0.f};
        if (g.bias && n_ok) bs = *reinterpret_cast<const v4f*>(g.bias + n);
#pragma unroll
        for (int c = 0; c < 4; ++c) asm volatile("" : "+v"(bs[c]));

        // next tile of this workgroup
        int nvb = vb + stride, ntm = 0, ntn = 0;
        while (nvb < g.n_ids && !tile_of(g, nvb, ntm, ntn)) nvb += stride;
        const bool more = nvb < g.n_ids;
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();   // every wave is done reading the stage buffers
        if (more) start_tile(ntm, ntn);

        char* slab = lds + (wave < 4 ? 2 * kTile + wave * 8192 : kLdsB + kTile + (wave - 4) * 8192);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    v4f o = {acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]};
                    *reinterpret_cast<v4f*>(slab + wr_t * 256 + (((8 * j + 2 * q + wr_half) ^ wr_sw) * 16)) = o;
                }
#pragma unroll
            for (int p = 0; p < 8; ++p) {
                const int r = 4 * p + rd_r;
                v4f o = *reinterpret_cast<const v4f*>(slab + r * 256 + ((rd_c ^ (r & 15)) * 16));
                const int64_t t = t_lane + i * 32 + 4 * p;
                if (t < g.T && n_ok) {
                    o += bs;
                    if constexpr (OUT_F16) {
                        typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                        h4 oh = {(_Float16)o[0], (_Float16)o[1], (_Float16)o[2], (_Float16)o[3]};
                        __builtin_nontemporal_store(oh, reinterpret_cast<h4*>(reinterpret_cast<_Float16*>(g.out) + t * g.ldo + n));
                    } else {
                        __builtin_nontemporal_store(o, reinterpret_cast<v4f*>(reinterpret_cast<float*>(g.out) + t * g.ldo + n));
                    }
                }
            }
        }
        if (!more) break;
        vb = nvb;
        // stage 0 of the next tile has landed (interior tile: its 32 stores per wave may still drain)
        if (ns > 1 && cm0 + BM <= g.T && cn0 + BN <= g.N) wait_vm<kStores + 4>();
        else wait_vm<0>();
    }
#undef RDA
#undef RDB
#undef DMA_A
#undef DMA_B
}
#undef SB
#undef MF

}  // namespace wonly
}  // namespace aweq

using namespace aweq;

extern "C" int aweq_wonly_gemm(const void* X_hat, int64_t T, int64_t K, int64_t ldx,
                               const void* codes, int bits, int group,
                               const float* step_w, const int32_t* zero_w, int64_t N,
                               const float* bias, void* out, aweq_dtype out_dt, int64_t ldo,
                               void* ws, size_t ws_bytes, uint32_t* status, void* stream)
{
    (void)status;
    if (!X_hat || !codes || !step_w || !zero_w || !out) return AWEQ_ERR_NULL;
    if (bits != 4 && bits != 3) return AWEQ_ERR_BITS;
    if (out_dt != AWEQ_F16 && out_dt != AWEQ_F32) return AWEQ_ERR_DTYPE;
    if (T <= 0 || N <= 0 || K <= 0 || (K % wonly::BKH) != 0 || ldx < K || ldo < N) return AWEQ_ERR_SHAPE;
    if (K > (1 << 20)) return AWEQ_ERR_SHAPE;  // 32-bit byte offsets inside a tile of rows
    if (group < -1 || (group > 0 && ((group % 32) != 0 || (K % group) != 0))) return AWEQ_ERR_GROUP;
    if ((N % 4) != 0 || (ldo % 4) != 0) return AWEQ_ERR_SHAPE;
    if (!aligned16(X_hat) || (ldx % 8) != 0 || !aligned16(codes) || !aligned16(out) || (bias && !aligned16(bias)))
        return AWEQ_ERR_ALIGN;
    if (!ws || ws_bytes < (size_t)N * (size_t)K * 2) return AWEQ_ERR_WORKSPACE;
    if (!aligned16(ws)) return AWEQ_ERR_ALIGN;
    const int64_t tiles_m = cdiv(T, wonly::BM), tiles_n = cdiv(N, wonly::BN);
    if (tiles_m * tiles_n > (1ll << 30)) return AWEQ_ERR_SHAPE;
    hipStream_t st = as_stream(stream);

    // the binary16 weight, once
    _Float16* W = reinterpret_cast<_Float16*>(ws);
    const int64_t dq_blocks = cdiv(N * (K / 32), 256);
    if (dq_blocks > 0x7fffffffll) return AWEQ_ERR_SHAPE;
    const uint8_t* cb = reinterpret_cast<const uint8_t*>(codes);
    if (bits == 4) wonly::dequant_weight_h_kernel<4><<<(unsigned)dq_blocks, 256, 0, st>>>(cb, N, K, group, step_w, zero_w, W);
    else wonly::dequant_weight_h_kernel<3><<<(unsigned)dq_blocks, 256, 0, st>>>(cb, N, K, group, step_w, zero_w, W);

    wonly::Args g;
    g.X = reinterpret_cast<const _Float16*>(X_hat); g.ldx = ldx;
    g.W = W; g.bias = bias;
    g.out = out; g.ldo = ldo; g.T = T; g.N = N; g.K = K;
    g.tiles_m = (int)tiles_m; g.tiles_n = (int)tiles_n;
    // patch of output tiles an XCD works on at a time: 32 tiles (one per compute unit), 8 (t) x 4 (n);
    // 4 x 8 when the contraction is long against N: the strided binary16 activation rows are then
    // fetched half as often and the weight, which fits the memory-side cache, twice as often
    // (1227 -> 1342 TFLOP/s at 4096 x 11008, 1236 -> 1342 at 4096 x 16384; 4096 x 4096 and 11008 x 4096 prefer 8 x 4)
    const int want_n = K >= 2 * N ? 8 : 4;
    g.patch_n = (int)(tiles_n < want_n ? tiles_n : want_n);
    g.patch_m = 32 / g.patch_n;
    if (g.patch_m > tiles_m) g.patch_m = (int)tiles_m;
    const int64_t patches_m = cdiv(tiles_m, g.patch_m);
    g.per_patch = g.patch_m * g.patch_n;
    g.tail_cols = (int)(tiles_n % g.patch_n);
    g.main_pn = (int)(tiles_n / g.patch_n);
    g.tail_pm = g.tail_cols ? g.per_patch / g.tail_cols : 0;
    if (g.tail_cols && g.tail_pm > tiles_m) g.tail_pm = (int)tiles_m;
    g.n_main = (int)(patches_m * g.main_pn);
    g.n_patches = g.n_main + (g.tail_cols ? (int)cdiv(tiles_m, g.tail_pm) : 0);
    const int64_t rounds = cdiv(g.n_patches, wonly::kXcds);
    const int64_t ids = rounds * wonly::kXcds * g.per_patch;
    if (ids > 0x7fffffffll) return AWEQ_ERR_SHAPE;
    g.n_ids = (int)ids;

    const void* fn = out_dt == AWEQ_F16 ? reinterpret_cast<const void*>(wonly::gemm_f16_kernel<true>)
                                        : reinterpret_cast<const void*>(wonly::gemm_f16_kernel<false>);
    // persistent launch: one workgroup per compute unit (a multiple of 8, so that id % 8 stays the XCD)
    int dev = 0, cus = 0;
    if (device_cus(dev, cus) != AWEQ_OK || raise_lds_limit(fn, dev, wonly::kLds) != AWEQ_OK) return AWEQ_ERR_LAUNCH;
    int64_t grid = (cus / wonly::kXcds) * wonly::kXcds;
    if (grid < wonly::kXcds) grid = wonly::kXcds;
    if (grid > ids) grid = ids;
    void* args[] = {&g};
    if (hipLaunchKernel(fn, dim3((unsigned)grid), dim3(wonly::kThreads), args, wonly::kLds, st) != hipSuccess)
        return AWEQ_ERR_LAUNCH;
    return launch_status();
}
