// Stage 4a: static per-tensor int8 activation quantizer (Sec. 2, Eq. 1 with b = 8) applied
// to the equalised activation X_hat = X diag(s)^-1 (Sec. 3.1, Eq. 3) on the fly, with the
// per-token and per-channel code sums the GEMM epilogue and the bias correction need.
//
// HBM-bound (2 bytes in, 1 byte out per element for binary16) with a tight ALU budget, so
// the quotient x / Step is formed without the generic division sequence when that is
// provably the same: Step is one constant, y = RN(1 / Step) is computed once, and
//   q0 = RN(a y);  r = a - Step q (exact, FMA);  q = RN(q + r y)   applied twice
// gives the correctly rounded a / Step.  After the first correction q is within
// 1/2 + 2^-22 ulp of a / Step; a quotient of two binary32 numbers is at least
// 2^-25 / beta ulp away from a rounding boundary (beta = significand(Step) / 2^24 < 1),
// while the second correction's error is below (1/2 + 2^-22) beta 2^-24 ulp, which is
// smaller whenever beta <= 1 - 2^-20.  Steps with a significand above that, exponents
// outside [-60, 60], zero points beyond 2^23 and binary32 inputs take the true division.
//
// That sequence is still 6 of the 13 operations an element costs, and it only matters next to a
// rounding tie.  So the common case is screened: q' = RN(a y + Z) in one FMA, n' = rint(q').
// With Q = a / Step, the value the definition rounds is v = RN(Q) + Z, and
//   |q' - v| <= |Q| 2^-23 + ulp(q') / 2  <=  (257 + |Z|) 2^-23 + 2^-16   wherever n' is in [-1, 256],
// so if q' is farther than delta = (258 + |Z|) 2^-23 + 2^-15 from every half-integer, v lies in
// the same unit interval and rint(RN(Q)) + Z = n' (outside [-1, 256] the relative error 2^-22
// keeps both on the same side of the clamp).  Units of 8 values with an element inside delta
// (about 1.5e-4 of all elements for |Z| <= 255) are redone with the exact sequence.
#include "common.hpp"
#include <type_traits>

namespace aweq {

constexpr int kQaBlock = 256;
constexpr int kQaWaves = kQaBlock / kWave;
constexpr int kQaVpt = 2;                               // panels (units per thread per row) per wavefront
constexpr int kQaPanels = kQaWaves * kQaVpt;            // 8 panels = 512 columns per block
constexpr int kQaMaxRows = 512;                         // rows per block (LDS row-sum slots)
constexpr int kQaRowBatch = 4;                          // groups of 8 rows in flight per thread
constexpr int kQaRowsPerIter = 8 * kQaRowBatch;
constexpr unsigned kQaXcds = 8;                         // workgroup id % 8 names the XCD a workgroup runs on

// One unit (8 consecutive columns of one row): codes, packed store, column / row sums.
// FAST: the division-free quotient; the unsigned code is kept as an (integral) float, packed
// with v_cvt_pk_u8_f32 and turned into the stored signed code by flipping the top bit
// (u - 128 = u ^ 0x80 as a byte).  Column sums accumulate u in fp32 (exact: at most 512 rows
// of values <= 255 per block); the caller subtracts 128 per row afterwards.
// MODE 0: true division; 1: the exact division-free quotient; 2: screened (see the header).
template <int MODE>
__device__ __forceinline__ void act_unit(const float x[8], const float is[8], const ActParams& p, int8_t* dst,
                                         float csf[8], int csi[8], int& rs, float& big, uint32_t& st)
{
    uint32_t w[2] = {0u, 0u};
    if constexpr (MODE == 2) {
        const float zf = (float)p.zero;
        float n[8];
        float dmax = 0.0f;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            // x is a widened binary16 value: a = RN(x inv_s) as one mixed-precision FMA (+0 changes
            // nothing but the sign of a zero, which the quotient's rounding forgets)
            const float a = __builtin_fmaf(x[i], is[i], 0.0f);
            const float q = __builtin_fmaf(a, p.rstep, zf);
            n[i] = rintf(q);
            dmax = fmaxf(dmax, fabsf(q - n[i]));
        }
        if (dmax > p.thr) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const float a = x[i] * is[i];
                float q = a * p.rstep;
                float r = __builtin_fmaf(-p.step, q, a);
                q = __builtin_fmaf(r, p.rstep, q);
                r = __builtin_fmaf(-p.step, q, a);
                q = __builtin_fmaf(r, p.rstep, q);
                n[i] = rintf(q) + zf;   // |rint| < 2^24 here (checked per thread), |Z| <= 4096
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float u = __builtin_amdgcn_fmed3f(n[i], 0.0f, 255.0f);
            csf[i] += u;
            w[i >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(u, i & 3, w[i >> 2]);
        }
        w[0] ^= 0x80808080u;
        w[1] ^= 0x80808080u;
    } else if constexpr (MODE == 1) {
        const float zf = (float)p.zero;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float a = x[i] * is[i];
            float q = a * p.rstep;
            float r = __builtin_fmaf(-p.step, q, a);
            q = __builtin_fmaf(r, p.rstep, q);
            r = __builtin_fmaf(-p.step, q, a);
            q = __builtin_fmaf(r, p.rstep, q);
            const float n = rintf(q);
            big = fmaxf(big, fabsf(n));
            // |Z| < 2^23: n + Z is exact wherever it can land inside [0, 255]
            const float u = __builtin_amdgcn_fmed3f(n + zf, 0.0f, 255.0f);
            csf[i] += u;
            w[i >> 2] = __builtin_amdgcn_cvt_pk_u8_f32(u, i & 3, w[i >> 2]);
        }
        w[0] ^= 0x80808080u;
        w[1] ^= 0x80808080u;
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float a = x[i] * is[i];
            const int c = quant_div(a, p.step, p.zero, 255, st) - 128;
            csi[i] += c;
            w[i >> 2] |= (uint32_t)(c & 0xff) << (8 * (i & 3));
        }
    }
    rs = __builtin_amdgcn_sdot4((int)w[0], 0x01010101, rs, false);
    rs = __builtin_amdgcn_sdot4((int)w[1], 0x01010101, rs, false);
    typedef unsigned v2u_ __attribute__((ext_vector_type(2)));
    if (dst) __builtin_nontemporal_store(v2u_{w[0], w[1]}, reinterpret_cast<v2u_*>(dst));   // (sums only: no code buffer)
}

// 8 consecutive input values of one row as loaded (binary16: one 16-byte quad), converted to
// fp32 only when they are consumed so that the loads in flight stay cheap in registers
template <bool F16> struct RawUnit;
template <> struct RawUnit<true> {
    Half8 v;
    __device__ __forceinline__ void load(const void* X, int64_t elt)
    {
        typedef int v4i_ __attribute__((ext_vector_type(4)));
        const v4i_ r = __builtin_nontemporal_load(reinterpret_cast<const v4i_*>(reinterpret_cast<const _Float16*>(X) + elt));
        v = __builtin_bit_cast(Half8, r);
    }
    __device__ __forceinline__ void get(float x[8]) const
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float2 f = h2f2(v.h[i]);
            x[2 * i] = f.x;
            x[2 * i + 1] = f.y;
        }
    }
};
template <> struct RawUnit<false> {
    Float4 a, b;
    __device__ __forceinline__ void load(const void* X, int64_t elt)
    {
        const float* p = reinterpret_cast<const float*>(X) + elt;
        a = *reinterpret_cast<const Float4*>(p);
        b = *reinterpret_cast<const Float4*>(p + 4);
    }
    __device__ __forceinline__ void get(float x[8]) const
    {
#pragma unroll
        for (int i = 0; i < 4; ++i) { x[i] = a.f[i]; x[4 + i] = b.f[i]; }
    }
};

// One-dimensional grid over the (row slice, column chunk) pairs, column chunks of 8 panels varying fastest.
// Workgroup ids are dealt round-robin to the 8 XCDs, and the pass runs 12 - 23 % faster (K = 8192 / 4096;
// nothing to gain or lose at K = 22016) when each XCD works through a contiguous eighth of that sequence
// - a compact range of rows of X and of every output panel - instead of every eighth pair, so id b takes
// pair (b % 8) * ceil(pairs / 8) + b / 8.
// The codes go out in the K-panel layout the
// GEMM reads (64-byte panels, rows back to back), so a wavefront works on 8 rows x one panel
// per instruction: lane = 8 (row % 8) + unit; its load covers 8 whole 128-byte lines of
// binary16 input and its store 512 contiguous bytes of codes.  Each wavefront owns two
// panels, so a lane keeps the column sums of its 16 columns over the rows it visits.
template <bool F16>
__global__ __launch_bounds__(kQaBlock) void quant_act_kernel(
    const void* __restrict__ X, int64_t T, int64_t K, int64_t ldx, const float* __restrict__ inv_s,
    const float* __restrict__ act_step, const int32_t* __restrict__ act_zero, int8_t* __restrict__ xq,
    int32_t* __restrict__ rowsum_x, int32_t* __restrict__ colsum_part, int rows_per_block, int chunks,
    unsigned pairs, uint32_t* status)
{
    const unsigned pair = (blockIdx.x % kQaXcds) * (gridDim.x / kQaXcds) + blockIdx.x / kQaXcds;
    if (pair >= pairs) return;   // (the grid is rounded up to a multiple of 8)
    const int chunk = (int)(pair % (unsigned)chunks);
    const int64_t slice = pair / (unsigned)chunks;
    __shared__ int lds_rs[kQaMaxRows][kQaWaves];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int rsub = lane >> 3, c8 = lane & 7;
    const int64_t r0 = slice * rows_per_block;
    const int nrows = (int)min((int64_t)rows_per_block, T - r0);
    const int64_t np = panel_count(K);
    const ActParams p = act_params(act_step, act_zero, F16);

    const int64_t panel0 = (int64_t)chunk * kQaPanels + wave * kQaVpt;
    const int col0 = (int)(panel0 * kPanel) + c8 * 8;                      // K <= 2^31 - 1 columns
    int8_t* const dst0 = xq ? xq + (panel0 * T + r0) * kPanel + c8 * 8 : nullptr;   // this lane's 8 bytes of row r0, panel j = 0
    const int64_t dst_step = T * kPanel;                                   // to the next panel
    const char* const src0 = reinterpret_cast<const char*>(X) + (r0 * ldx + col0) * (F16 ? 2 : 4);
    bool valid[kQaVpt], pad[kQaVpt];
    float is[kQaVpt][8];
    bool fast_thread = p.fast;
    float is_max = 0.0f;
#pragma unroll
    for (int j = 0; j < kQaVpt; ++j) {
        valid[j] = col0 + j * kPanel < K;
        pad[j] = !valid[j] && panel0 + j < np;  // zero fill of the last panel
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            is[j][i] = valid[j] ? inv_s[col0 + j * kPanel + i] : 1.0f;
            // the exactness argument needs a y not to overflow: binary16 |x| < 2^16, Step >= 2^-60
            if (!(fabsf(is[j][i]) < 1.0e12f)) fast_thread = false;
            is_max = fmaxf(is_max, fabsf(is[j][i]));
        }
    }
    // the screened path does not track the largest quotient: it needs |x inv_s / Step| < 2^24
    // for every binary16 x up front (65504 max|inv_s| / Step with a margin for the roundings)
    const bool screen_thread = fast_thread && p.screen && 65600.0f * is_max * p.rstep < 16777216.0f;
    // one path for the whole block (the choice is uniform unless an inv_s is absurd)
    const bool fast = __syncthreads_and(fast_thread ? 1 : 0) != 0;
    const bool screen = __syncthreads_and(screen_thread ? 1 : 0) != 0;
    uint32_t st = 0;
    float big = 0.0f;
    float csf[kQaVpt][8];
    int csi[kQaVpt][8];
#pragma unroll
    for (int j = 0; j < kQaVpt; ++j)
#pragma unroll
        for (int i = 0; i < 8; ++i) { csf[j][i] = 0.0f; csi[j][i] = 0; }
    int my_rows = 0;

    auto rows_loop = [&](auto mode_c) {
        constexpr int MODE = decltype(mode_c)::value;
        for (int rb = 0; rb < nrows; rb += kQaRowsPerIter) {
            RawUnit<F16> raw[kQaRowBatch][kQaVpt];
#pragma unroll
            for (int b = 0; b < kQaRowBatch; ++b)
#pragma unroll
                for (int j = 0; j < kQaVpt; ++j) {
                    const int row = rb + 8 * b + rsub;
                    if (row < nrows && valid[j]) raw[b][j].load(src0, (int64_t)row * ldx + j * kPanel);
                }
#pragma unroll
            for (int b = 0; b < kQaRowBatch; ++b) {
                const int row = rb + 8 * b + rsub;
                const bool row_ok = row < nrows;
                int rs = 0;
                if (row_ok) {
                    ++my_rows;
#pragma unroll
                    for (int j = 0; j < kQaVpt; ++j) {
                        int8_t* d = dst0 ? dst0 + j * dst_step + row * kPanel : nullptr;
                        if (valid[j]) {
                            float x[8];
                            raw[b][j].get(x);
                            act_unit<MODE>(x, is[j], p, d, csf[j], csi[j], rs, big, st);
                        } else if (pad[j] && d) {
                            *reinterpret_cast<uint2*>(d) = make_uint2(0u, 0u);
                        }
                    }
                }
                rs = group_allreduce<3>(rs, OpAdd());  // the 8 lanes of one row
                if (row_ok && c8 == 0) lds_rs[row][wave] = rs;
            }
        }
    };
    if constexpr (F16) {
        if (screen) rows_loop(std::integral_constant<int, 2>{});
        else if (fast) rows_loop(std::integral_constant<int, 1>{});
        else rows_loop(std::integral_constant<int, 0>{});
    } else {
        rows_loop(std::integral_constant<int, 0>{});   // binary32 input: the true division
    }
    if (big >= 16777216.0f) st |= AWEQ_ST_BIGQUOT;
    raise_status(status, st);

    if (colsum_part) {
        // lanes l, l ^ 8, l ^ 16, l ^ 32 hold the same columns for different rows; this block's sums over
        // its row slice (at most 512 rows of codes in [-128, 127]) go to row `slice` of the partial buffer
        int32_t* const part = colsum_part + slice * K;
#pragma unroll
        for (int j = 0; j < kQaVpt; ++j) {
            int v[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                v[i] = fast ? ((int)csf[j][i] - 128 * my_rows) : csi[j][i];
                v[i] += xor8(v[i]);
                v[i] += partner<4>(v[i]);
                v[i] += partner<5>(v[i]);
            }
            if (lane < 8 && valid[j]) {
                typedef int v4i_ __attribute__((ext_vector_type(4)));
                v4i_* d = reinterpret_cast<v4i_*>(part + col0 + j * kPanel);
                d[0] = v4i_{v[0], v[1], v[2], v[3]};
                d[1] = v4i_{v[4], v[5], v[6], v[7]};
            }
        }
    }
    __syncthreads();
    // with several column chunks `rowsum_x` is the partial buffer [chunks][T], folded by the merge kernel
    if (rowsum_x)
        for (int i = threadIdx.x; i < nrows; i += kQaBlock) {
            int tot = 0;
#pragma unroll
            for (int w = 0; w < kQaWaves; ++w) tot += lds_rs[i][w];
            rowsum_x[(int64_t)chunk * T + r0 + i] = tot;
        }
}

// Fold the per-slice column sums (fixed order, 64-bit) and the per-chunk row sums.  Blocks
// [0, col_blocks) own 32 columns each: 32 groups of 32 threads take every 32nd slice (few dependent loads
// per thread: the kernel is bound by their latency) and meet in LDS; the remaining blocks own 1024 rows each.
constexpr int kQaMergeCols = 32, kQaMergeParts = 32;
__global__ __launch_bounds__(kQaMergeCols * kQaMergeParts) void quant_act_merge(
    const int32_t* __restrict__ colsum_part, int slices, int64_t K, long long* __restrict__ colsum_xq,
    const int32_t* __restrict__ rowsum_part, int chunks, int64_t T, int32_t* __restrict__ rowsum_x, int col_blocks)
{
    if ((int)blockIdx.x < col_blocks) {
        __shared__ long long s_s[kQaMergeParts][kQaMergeCols];
        const int c = threadIdx.x & (kQaMergeCols - 1), part = threadIdx.x / kQaMergeCols;
        const int64_t k = (int64_t)blockIdx.x * kQaMergeCols + c;
        long long s = 0;
        if (k < K)
            for (int j = part; j < slices; j += kQaMergeParts) s += colsum_part[(int64_t)j * K + k];
        s_s[part][c] = s;
        __syncthreads();
        if (part != 0 || k >= K) return;
#pragma unroll
        for (int q = 1; q < kQaMergeParts; ++q) s += s_s[q][c];
        colsum_xq[k] = s;
    } else {
        const int64_t t = ((int64_t)blockIdx.x - col_blocks) * (kQaMergeCols * kQaMergeParts) + threadIdx.x;
        if (t >= T) return;
        int tot = 0;
        for (int c = 0; c < chunks; ++c) tot += rowsum_part[(int64_t)c * T + t];
        rowsum_x[t] = tot;
    }
}

struct QaPlan {
    int chunks;      // column chunks of 8 panels
    int64_t slices;  // row slices
    int64_t rpb;     // rows per slice
};

static QaPlan qa_plan(int64_t T, int64_t K)
{
    QaPlan p;
    p.chunks = (int)cdiv(panel_count(K), kQaPanels);
    int64_t slices = cdiv(8192, p.chunks);
    int64_t rpb = cdiv(T, slices);
    rpb = cdiv(rpb, kQaRowsPerIter) * kQaRowsPerIter;
    if (rpb > kQaMaxRows) rpb = kQaMaxRows;
    p.rpb = rpb;
    p.slices = cdiv(T, rpb);
    return p;
}

// workspace: per-slice column sums [slices][K] int32, then (several column chunks only) per-chunk
// row sums [chunks][T] int32
size_t quant_act_ws_bytes(int64_t T, int64_t K)
{
    const QaPlan p = qa_plan(T, K);
    return (size_t)p.slices * (size_t)K * 4 + (p.chunks > 1 ? (size_t)p.chunks * (size_t)T * 4 : 0);
}

int launch_quant_act(const void* X, aweq_dtype dt, int64_t T, int64_t K, int64_t ldx, const float* inv_s,
                     const float* act_step, const int32_t* act_zero, int8_t* xq, int32_t* rowsum_x,
                     int64_t* colsum_xq, void* ws, uint32_t* status, hipStream_t st)
{
    const QaPlan p = qa_plan(T, K);
    if (p.slices * p.chunks > 0x7ffffff0ll) return AWEQ_ERR_SHAPE;
    const bool multi = p.chunks > 1;
    int32_t* const colsum_part = colsum_xq ? reinterpret_cast<int32_t*>(ws) : nullptr;
    int32_t* const rowsum_part = reinterpret_cast<int32_t*>(ws) + (size_t)p.slices * K;
    int32_t* const rs_out = !rowsum_x ? nullptr : (multi ? rowsum_part : rowsum_x);
    const unsigned pairs = (unsigned)(p.slices * p.chunks);
    const unsigned grid = (unsigned)(cdiv(pairs, kQaXcds) * kQaXcds);
    if (dt == AWEQ_F16)
        quant_act_kernel<true><<<grid, kQaBlock, 0, st>>>(X, T, K, ldx, inv_s, act_step, act_zero, xq, rs_out, colsum_part,
                                                          (int)p.rpb, p.chunks, pairs, status);
    else
        quant_act_kernel<false><<<grid, kQaBlock, 0, st>>>(X, T, K, ldx, inv_s, act_step, act_zero, xq, rs_out, colsum_part,
                                                           (int)p.rpb, p.chunks, pairs, status);
    const int col_blocks = colsum_xq ? (int)cdiv(K, kQaMergeCols) : 0;
    const int64_t row_blocks = (rowsum_x && multi) ? cdiv(T, kQaMergeCols * kQaMergeParts) : 0;
    if (col_blocks + row_blocks > 0)
        quant_act_merge<<<(unsigned)(col_blocks + row_blocks), kQaMergeCols * kQaMergeParts, 0, st>>>(
            colsum_part, (int)p.slices, K, reinterpret_cast<long long*>(colsum_xq), rowsum_part, p.chunks, T, rowsum_x, col_blocks);
    return launch_status();
}

int check_quant_act_args(const void* X, aweq_dtype dt, int64_t T, int64_t K, int64_t ldx, const float* inv_s,
                         const float* act_step, const int32_t* act_zero, const int8_t* xq, bool xq_optional)
{
    if (!X || !inv_s || !act_step || !act_zero || (!xq && !xq_optional)) return AWEQ_ERR_NULL;
    if (dt != AWEQ_F32 && dt != AWEQ_F16) return AWEQ_ERR_DTYPE;
    if (T <= 0 || K <= 0 || ldx < K || (K % 8) != 0) return AWEQ_ERR_SHAPE;
    if (!aligned16(X) || ((size_t)ldx * dtype_size(dt)) % 16 != 0 || !aligned16(xq)) return AWEQ_ERR_ALIGN;
    return AWEQ_OK;
}

// the sums need the workspace (rowsum_x only with several column chunks)
int check_quant_act_ws(int64_t T, int64_t K, const int32_t* rowsum_x, const int64_t* colsum_xq, const void* ws, size_t ws_bytes)
{
    const bool need = colsum_xq || (rowsum_x && qa_plan(T, K).chunks > 1);
    if (!need) return AWEQ_OK;
    if (!ws || ws_bytes < quant_act_ws_bytes(T, K)) return AWEQ_ERR_WORKSPACE;
    if (!aligned16(ws)) return AWEQ_ERR_ALIGN;
    return AWEQ_OK;
}

}  // namespace aweq

using namespace aweq;

extern "C" int aweq_quant_act(const void* X, aweq_dtype dt, int64_t T, int64_t K, int64_t ldx,
                              const float* inv_s, const float* act_step, const int32_t* act_zero,
                              int8_t* xq, int32_t* rowsum_x, int64_t* colsum_xq,
                              void* ws, size_t ws_bytes, uint32_t* status, void* stream)
{
    if (!xq && !rowsum_x && !colsum_xq) return AWEQ_ERR_NULL;   // nothing to produce
    int rc = check_quant_act_args(X, dt, T, K, ldx, inv_s, act_step, act_zero, xq, true);
    if (rc != AWEQ_OK) return rc;
    rc = check_quant_act_ws(T, K, rowsum_x, colsum_xq, ws, ws_bytes);
    if (rc != AWEQ_OK) return rc;
    return launch_quant_act(X, dt, T, K, ldx, inv_s, act_step, act_zero, xq, rowsum_x, colsum_xq, ws, status, as_stream(stream));
}
