// Dense route of a layer whose density is high (the density-adaptive layer that the paper plans in
// "Discussion and Conclusion" and Appendix C.3: dense computation where it is the faster one).
// One zero-filled dense copy of the weights, D[i * ld + j] = W(i, j) (row-major, ld = cols rounded up to
// 64, zero off the pattern and in the padding), serves three fp32 MFMA products:
//     Y  = act(W X + b)          dense_nn_kernel      A operand = rows of D, 16 bytes per lane along k
//     dX = (W^T dZ) * [mask > 0]  dense_tn_kernel      A operand = D read down its columns: the same copy,
//                                                      16 bytes per lane along the output rows
//     G  = dZ X^T                dense_nt_kernel      both operands 16 bytes per lane along the batch
// followed, for the last one, by dense_update_kernel, which picks the entries of G that lie on the
// pattern and applies the momentum step to values[] (the state stays sparse; the copy is derived).
//
// v_mfma_f32_16x16x4_f32: lane l supplies A(l % 16, l / 16) and B(l / 16, l % 16) of a 16 x 4 by 4 x 16
// step; register r of lane l holds C(4 * (l / 16) + r, l % 16).  A lane's four k slots need not be
// consecutive k as long as A and B agree, so one 16-byte load along k feeds four steps (slot q of
// step s: k = base + 4 q + s), and one 16-byte load along the output rows feeds four tiles (tile u
// holds the rows base + 4 r + u).  Small tiles (16 rows) on purpose: these products are a few hundred
// MFLOP, and only thousands of tiles fill 1024 matrix units.  Every sum has one fixed order.
#include "kernels.h"

namespace nerva {
namespace {

constexpr int kWave = 64;
constexpr int kDenseWaves = 4;
constexpr int kDenseBlock = kWave * kDenseWaves;
typedef float v4f __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int wave_id() { return __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6)); }
__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ v4f mfma(float a, float b, v4f c) { return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0); }

__device__ __forceinline__ void dense_epilogue(const DenseArgs &a, int row, int col, int m_rows, float y)
{
    if (row >= m_rows || col >= a.batch) return;
    if (a.bias) y += a.bias[row];
    if (a.relu) y = y > 0.f ? y : 0.f;
    if (a.YM) y = a.YM[static_cast<int64_t>(row) * a.ldym + col] > 0.f ? y : 0.f;
    a.Y[static_cast<int64_t>(row) * a.ldy + col] = y;
}

// Y (rows x batch) = act(D X + b).  Work-group: 16 rows x NB * 16 columns; its kNnWaves waves split K = cols
// into contiguous slices (multiples of 16) and meet in LDS, where wave w adds register (w % 4) of all slices in
// slice order for the tile columns t = w / 4, w / 4 + kNnWaves / 4, ...  The loads of kNnDepth chunks of 16 k are
// all issued before the first of their MFMA steps.  (kSplitWaves: the same split in the transposed product.)
constexpr int kSplitWaves = 16;
constexpr int kSplitBlock = kSplitWaves * kWave;
constexpr int kNnDepth = 2;

// VECX: the NB columns of a lane are consecutive (tile t holds the columns n0 + NB * r + t), so that one
// 8- or 16-byte load along the batch feeds the NB tiles; needs X 16-byte aligned with ldx a multiple of 4.
// A batch of kNnDepth chunks: its loads (nn_load) are issued while the MFMA steps of the batch before (nn_mfma)
// run -- the waves of a work-group start together and would otherwise all load, then all multiply.
template <int NB>
struct NnBatch {
    float4 w4[kNnDepth];
    float b[kNnDepth][4][NB];
};

template <int NB, bool VECX>
__device__ __forceinline__ void nn_load(const DenseArgs &a, const float *wrow, const int64_t (&xcol)[NB], int q, int c0, int n_chunks,
                                        NnBatch<NB> &B)
{
    const int K = a.cols;
#pragma unroll
    for (int d = 0; d < kNnDepth; ++d) {
        const int kb = (c0 + (d < n_chunks ? d : 0)) * 16;   // (chunks past the end repeat the first one and are not used)
        B.w4[d] = ld4(wrow + kb);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const int k = kb + q * 4 + s;
            const float *xr = a.X + static_cast<int64_t>(k < K ? k : 0) * a.ldx;
            if constexpr (VECX && NB == 4) {
                const float4 x = ld4(xr + xcol[0]);
                B.b[d][s][0] = x.x; B.b[d][s][1] = x.y; B.b[d][s][2] = x.z; B.b[d][s][3] = x.w;
            } else if constexpr (VECX && NB == 2) {
                const float2 x = *reinterpret_cast<const float2 *>(xr + xcol[0]);
                B.b[d][s][0] = x.x; B.b[d][s][1] = x.y;
            } else {
#pragma unroll
                for (int t = 0; t < NB; ++t) B.b[d][s][t] = xr[xcol[t]];
            }
        }
    }
}

// EXACT: rows and K are multiples of 16, so no operand has to be zeroed (columns beyond the batch repeat column 0
// and their results are never stored): the MFMA steps take the loaded registers as they are.
template <int NB, bool EXACT>
__device__ __forceinline__ void nn_mfma(int K, bool row_ok, const bool (&col_ok)[NB], int q, int c0, int n_chunks, const NnBatch<NB> &B,
                                        v4f (&acc)[NB])
{
#pragma unroll
    for (int d = 0; d < kNnDepth; ++d) {
        if (d >= n_chunks) break;  // wave-uniform
        const int kb = (c0 + d) * 16;
        const float wv4[4] = {B.w4[d].x, B.w4[d].y, B.w4[d].z, B.w4[d].w};
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const bool k_ok = kb + q * 4 + s < K;
#pragma unroll
            for (int t = 0; t < NB; ++t) {
                if constexpr (EXACT)
                    acc[t] = mfma(wv4[s], B.b[d][s][t], acc[t]);
                else
                    acc[t] = mfma(row_ok ? wv4[s] : 0.f, (k_ok && col_ok[t]) ? B.b[d][s][t] : 0.f, acc[t]);
            }
        }
    }
}

constexpr int kNnWaves = 8;   // measured on the 1024 x 3072 x 100 product: 21.3 / 18.6 / 20.6 us with 4 / 8 / 16 waves
constexpr int kNnBlock = kNnWaves * kWave;
template <int NB, bool VECX, bool EXACT>
__global__ __launch_bounds__(kNnBlock) void dense_nn_kernel(const DenseArgs a)
{
    __shared__ float part[kNnWaves][NB][4][kWave];
    const int lane = threadIdx.x & (kWave - 1), wv = wave_id();
    const int r = lane & 15, q = lane >> 4;
    // Work-group ids go round the 8 XCDs: the column tiles of one row tile get ids 8 apart, so that they run on one
    // XCD and the rows of the copy they all read come out of its L2 after the first of them has fetched them.
    const int n_col_tiles = (a.batch + 16 * NB - 1) / (16 * NB);
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int m_tile = (slot / n_col_tiles) * 8 + xcd;
    if (m_tile * 16 >= a.rows) return;  // (the grid is padded to whole rounds of the XCDs)
    const int i0 = m_tile * 16, n0 = (slot % n_col_tiles) * (16 * NB);
    const int K = a.cols;
    const int row = i0 + r;
    const bool row_ok = row < a.rows;
    const float *wrow = a.W + static_cast<int64_t>(row_ok ? row : 0) * a.ldw + q * 4;
    int64_t xcol[NB];
    bool col_ok[NB];
    int col[NB];
#pragma unroll
    for (int t = 0; t < NB; ++t) {
        col[t] = VECX ? n0 + NB * r + t : n0 + 16 * t + r;
        col_ok[t] = col[t] < a.batch;
        xcol[t] = col_ok[t] ? col[t] : 0;     // lanes beyond the batch re-read column 0 and contribute 0
    }
    if constexpr (VECX) xcol[0] = col_ok[0] ? col[0] : 0;  // (the access of NB columns starts inside the row when its first column does)
    const int k16 = (K + 15) / 16;                                   // chunks of 16 k (the copy's rows are padded with zeros)
    const int per = (k16 + kNnWaves - 1) / kNnWaves;
    const int c_begin = min(wv * per, k16), c_end = min(c_begin + per, k16);
    v4f acc[NB];
#pragma unroll
    for (int t = 0; t < NB; ++t) acc[t] = v4f{0.f, 0.f, 0.f, 0.f};
    NnBatch<NB> B0, B1;
    if (c_begin < c_end) nn_load<NB, VECX>(a, wrow, xcol, q, c_begin, min(kNnDepth, c_end - c_begin), B0);
    for (int c = c_begin; c < c_end; c += 2 * kNnDepth) {
        const int c1 = c + kNnDepth, c2 = c + 2 * kNnDepth;
        if (c1 < c_end) nn_load<NB, VECX>(a, wrow, xcol, q, c1, min(kNnDepth, c_end - c1), B1);
        nn_mfma<NB, EXACT>(K, row_ok, col_ok, q, c, min(kNnDepth, c_end - c), B0, acc);
        if (c2 < c_end) nn_load<NB, VECX>(a, wrow, xcol, q, c2, min(kNnDepth, c_end - c2), B0);
        if (c1 < c_end) nn_mfma<NB, EXACT>(K, row_ok, col_ok, q, c1, min(kNnDepth, c_end - c1), B1, acc);
    }
#pragma unroll
    for (int t = 0; t < NB; ++t)
#pragma unroll
        for (int g = 0; g < 4; ++g) part[wv][t][g][lane] = acc[t][g];
    __syncthreads();
    const int g = wv & 3;
    for (int t = wv >> 2; t < NB; t += kNnWaves / 4) {
        float y = 0.f;
#pragma unroll
        for (int w = 0; w < kNnWaves; ++w) y += part[w][t][g][lane];
        dense_epilogue(a, i0 + 4 * q + g, VECX ? n0 + NB * r + t : n0 + 16 * t + r, a.rows, y);
    }
}

// Y (cols x batch) = (D^T X) * [YM > 0].  Work-group: 64 output rows (four tiles fed by one 16-byte load along
// the row of D: tile u holds the output rows j0 + 4 r' + u) x NB * 16 columns; the waves split K = rows, kTnDepth
// steps of loads in flight.  Wave w adds tile (w / 4), register (w % 4) of all slices in slice order.
constexpr int kTnDepth = 8;

template <int NB>
__global__ __launch_bounds__(kSplitBlock) void dense_tn_kernel(const DenseArgs a)
{
    __shared__ float part[kSplitWaves][4][NB][4][kWave];
    const int lane = threadIdx.x & (kWave - 1), wv = wave_id();
    const int r = lane & 15, q = lane >> 4;
    const int j0 = blockIdx.x * 64, n0 = blockIdx.y * (16 * NB);
    const int K = a.rows;
    const float *wcol = a.W + j0 + r * 4;     // (ld is a multiple of 64: the access stays inside the row)
    int64_t xcol[NB];
    bool col_ok[NB];
#pragma unroll
    for (int t = 0; t < NB; ++t) {
        const int c = n0 + 16 * t + r;
        col_ok[t] = c < a.batch;
        xcol[t] = col_ok[t] ? c : 0;
    }
    const int k4 = (K + 3) / 4;                                     // steps of 4 k (one per slot)
    const int per = (k4 + kSplitWaves - 1) / kSplitWaves;
    const int c_begin = min(wv * per, k4), c_end = min(c_begin + per, k4);
    v4f acc[4][NB];
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int t = 0; t < NB; ++t) acc[u][t] = v4f{0.f, 0.f, 0.f, 0.f};
    for (int c = c_begin; c < c_end; c += kTnDepth) {
        const int n_steps = min(kTnDepth, c_end - c);
        float4 w4[kTnDepth];
        float b[kTnDepth][NB];
#pragma unroll
        for (int d = 0; d < kTnDepth; ++d) {
            const int i = (c + (d < n_steps ? d : 0)) * 4 + q;       // (steps past the end repeat the first one and are not used)
            const int64_t ii = i < K ? i : 0;
            w4[d] = ld4(wcol + ii * a.ldw);
#pragma unroll
            for (int t = 0; t < NB; ++t) b[d][t] = a.X[ii * a.ldx + xcol[t]];
        }
#pragma unroll
        for (int d = 0; d < kTnDepth; ++d) {
            if (d >= n_steps) break;  // wave-uniform
            const bool i_ok = (c + d) * 4 + q < K;
            const float wv4[4] = {w4[d].x, w4[d].y, w4[d].z, w4[d].w};
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int t = 0; t < NB; ++t) acc[u][t] = mfma(i_ok ? wv4[u] : 0.f, (i_ok && col_ok[t]) ? b[d][t] : 0.f, acc[u][t]);
        }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int t = 0; t < NB; ++t)
#pragma unroll
            for (int g = 0; g < 4; ++g) part[wv][u][t][g][lane] = acc[u][t][g];
    __syncthreads();
    const int u = wv >> 2, g = wv & 3;
#pragma unroll
    for (int t = 0; t < NB; ++t) {
        float y = 0.f;
#pragma unroll
        for (int w = 0; w < kSplitWaves; ++w) y += part[w][u][t][g][lane];
        dense_epilogue(a, j0 + 4 * (4 * q + g) + u, n0 + 16 * t + r, a.cols, y);
    }
}

// G (rows x ldg) = dZ X^T over the batch: G[i][j] = sum_c dZ[i, c] * X[j, c].  K = batch is short, so there
// is no split: a wave owns MB * 16 rows x NB * 16 columns of G.  Columns of the batch beyond `batch` inside a
// 16-byte access are dropped (padding may hold anything).
template <int MB, int NB>
__global__ __launch_bounds__(kDenseBlock) void dense_nt_kernel(const float *__restrict__ dZ, int64_t lddz, const float *__restrict__ X,
                                                              int64_t ldx, float *__restrict__ G, int64_t ldg, int rows, int cols, int batch)
{
    const int lane = threadIdx.x & (kWave - 1), wv = wave_id();
    const int r = lane & 15, q = lane >> 4;
    const int i0 = blockIdx.x * (16 * MB), j0 = (blockIdx.y * kDenseWaves + wv) * (16 * NB);
    if (j0 >= cols) return;  // wave-uniform
    const float *zr[MB], *xr[NB];
    bool z_ok[MB], x_ok[NB];
#pragma unroll
    for (int m = 0; m < MB; ++m) {
        const int i = i0 + 16 * m + r;
        z_ok[m] = i < rows;
        zr[m] = dZ + static_cast<int64_t>(z_ok[m] ? i : 0) * lddz;
    }
#pragma unroll
    for (int t = 0; t < NB; ++t) {
        const int j = j0 + 16 * t + r;
        x_ok[t] = j < cols;
        xr[t] = X + static_cast<int64_t>(x_ok[t] ? j : 0) * ldx;
    }
    auto masked = [&](const float *p, int c, bool ok) {
        // the access starts inside the row's allocation when c < batch (leading dimensions are multiples of 4)
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (ok && c < batch) {
            v = ld4(p + c);
            if (c + 1 >= batch) v.y = 0.f;
            if (c + 2 >= batch) v.z = 0.f;
            if (c + 3 >= batch) v.w = 0.f;
        }
        return v;
    };
    v4f acc[MB][NB];
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int t = 0; t < NB; ++t) acc[m][t] = v4f{0.f, 0.f, 0.f, 0.f};
    constexpr int kDepth = 4;  // chunks of 16 columns of the batch whose loads are in flight together
    for (int kb = 0; kb < batch; kb += 16 * kDepth) {
        float4 z4[kDepth][MB], x4[kDepth][NB];
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            const int c = kb + 16 * d + q * 4;
#pragma unroll
            for (int m = 0; m < MB; ++m) z4[d][m] = masked(zr[m], c, z_ok[m]);
#pragma unroll
            for (int t = 0; t < NB; ++t) x4[d][t] = masked(xr[t], c, x_ok[t]);
        }
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            if (kb + 16 * d >= batch) break;  // wave-uniform
#pragma unroll
            for (int m = 0; m < MB; ++m) {
                const float zv[4] = {z4[d][m].x, z4[d][m].y, z4[d][m].z, z4[d][m].w};
#pragma unroll
                for (int t = 0; t < NB; ++t) {
                    const float xv[4] = {x4[d][t].x, x4[d][t].y, x4[d][t].z, x4[d][t].w};
#pragma unroll
                    for (int s = 0; s < 4; ++s) acc[m][t] = mfma(zv[s], xv[s], acc[m][t]);
                }
            }
        }
    }
#pragma unroll
    for (int m = 0; m < MB; ++m)
#pragma unroll
        for (int t = 0; t < NB; ++t)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int i = i0 + 16 * m + 4 * q + g, j = j0 + 16 * t + r;
                if (i < rows && j < cols) G[static_cast<int64_t>(i) * ldg + j] = acc[m][t][g];
            }
}

__device__ __forceinline__ void momentum_step(float &w, float &v, float g, float lr, float mu, int nesterov)
{
    const float step = lr * g;
    v = fmaf(mu, v, -step);
    w = nesterov ? w + fmaf(mu, v, -step) : w + v;
}

// A work-group per row of W: the row's stored entries take their gradient from G, the momentum step is applied
// to values[] / velocity[], and the new weight goes to the mirror and to the dense copy; the row sum of dZ is
// the bias gradient (first wave).  Four strides of loads are in flight per thread.
__global__ __launch_bounds__(kDenseBlock) void dense_update_kernel(const DenseUpdateArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    constexpr int kU = 4;
    for (int64_t i = blockIdx.x; i < a.rows; i += gridDim.x) {
        const int32_t b = a.indptr[i], e = a.indptr[i + 1];
        const float *grow = a.G + i * a.ldg;
        float *drow = a.D + i * a.ldw;
        for (int32_t p0 = b + threadIdx.x; p0 < e; p0 += kU * kDenseBlock) {
            int32_t p[kU], j[kU], pt[kU];
            float w[kU], v[kU], g[kU];
            bool ok[kU];
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                p[u] = p0 + u * kDenseBlock;
                ok[u] = p[u] < e;
                if (!ok[u]) p[u] = p0;
                j[u] = a.indices[p[u]];
                w[u] = a.values[p[u]];
                v[u] = a.velocity[p[u]];
                pt[u] = a.values_t ? a.pos_t[p[u]] : 0;
            }
#pragma unroll
            for (int u = 0; u < kU; ++u) g[u] = grow[j[u]];
#pragma unroll
            for (int u = 0; u < kU; ++u) {
                if (!ok[u]) continue;
                momentum_step(w[u], v[u], g[u], a.lr, a.momentum, a.nesterov);
                a.values[p[u]] = w[u];
                a.velocity[p[u]] = v[u];
                if (a.values_t) a.values_t[pt[u]] = w[u];
                drow[j[u]] = w[u];
            }
        }
        if (a.bias && wave_id() == 0) {
            const float *zr = a.dZ + i * a.lddz;
            float s = 0.f;
            for (int c = lane; c < a.batch; c += kWave) s += zr[c];
#pragma unroll
            for (int m = 32; m >= 1; m >>= 1) s += __shfl_xor(s, m, kWave);   // every lane ends with the same bits
            if (lane == 0) {
                float w = a.bias[i], v = a.bias_velocity[i];
                momentum_step(w, v, s, a.lr, a.momentum, a.nesterov);
                a.bias[i] = w;
                a.bias_velocity[i] = v;
            }
        }
    }
}

// One wave per row of the CSR matrix: scatters the row's values into the dense copy.
__global__ __launch_bounds__(kDenseBlock) void dense_refresh_kernel(const int32_t *__restrict__ indptr, const int32_t *__restrict__ indices,
                                                                   const float *__restrict__ values, int rows, float *D, int64_t ld)
{
    const int lane = threadIdx.x & (kWave - 1);
    for (int i = blockIdx.x * kDenseWaves + wave_id(); i < rows; i += gridDim.x * kDenseWaves)
        for (int p = indptr[i] + lane; p < indptr[i + 1]; p += kWave) D[static_cast<int64_t>(i) * ld + indices[p]] = values[p];
}

inline int blocks_for_rows(int64_t rows)
{
    int64_t b = (rows + kDenseWaves - 1) / kDenseWaves;
    if (b < 1) b = 1;
    if (b > 8192) b = 8192;
    return static_cast<int>(b);
}

}  // namespace

// Columns of the batch per work-group: as many as still leave the chip's 256 compute units a work-group each.
static int dense_nb(int64_t m_tiles, int batch)
{
    for (int nb = 4; nb > 1; nb >>= 1)
        if (m_tiles * ((batch + 16 * nb - 1) / (16 * nb)) >= 256) return nb;
    return 1;
}

hipError_t launch_dense_product(const DenseArgs &a, hipStream_t s)
{
    if (a.rows <= 0 || a.cols <= 0 || a.batch <= 0) return hipSuccess;
    if (!a.trans) {
        const int64_t mt = (a.rows + 15) / 16;
        const int nb = dense_nb(mt, a.batch);
        const dim3 grid(static_cast<unsigned>((mt + 7) / 8 * 8 * ((a.batch + 16 * nb - 1) / (16 * nb))));
        const bool vec = a.ldx % 4 == 0 && (reinterpret_cast<uintptr_t>(a.X) & 15u) == 0;
        const bool exact = a.rows % 16 == 0 && a.cols % 16 == 0;
        if (nb == 4 && vec && exact) hipLaunchKernelGGL((dense_nn_kernel<4, true, true>), grid, dim3(kNnBlock), 0, s, a);
        else if (nb == 4 && vec) hipLaunchKernelGGL((dense_nn_kernel<4, true, false>), grid, dim3(kNnBlock), 0, s, a);
        else if (nb == 4) hipLaunchKernelGGL((dense_nn_kernel<4, false, false>), grid, dim3(kNnBlock), 0, s, a);
        else if (nb == 2 && vec && exact) hipLaunchKernelGGL((dense_nn_kernel<2, true, true>), grid, dim3(kNnBlock), 0, s, a);
        else if (nb == 2 && vec) hipLaunchKernelGGL((dense_nn_kernel<2, true, false>), grid, dim3(kNnBlock), 0, s, a);
        else if (nb == 2) hipLaunchKernelGGL((dense_nn_kernel<2, false, false>), grid, dim3(kNnBlock), 0, s, a);
        else if (exact) hipLaunchKernelGGL((dense_nn_kernel<1, false, true>), grid, dim3(kNnBlock), 0, s, a);
        else hipLaunchKernelGGL((dense_nn_kernel<1, false, false>), grid, dim3(kNnBlock), 0, s, a);
    } else {
        // (one tile column per work-group: the 16 slices of 4 x 4 registers already take 64 KiB of LDS)
        const dim3 grid(static_cast<unsigned>((a.cols + 63) / 64), (a.batch + 15) / 16);
        hipLaunchKernelGGL(dense_tn_kernel<1>, grid, dim3(kSplitBlock), 0, s, a);
    }
    return hipGetLastError();
}

hipError_t launch_dense_sddmm_update(const DenseUpdateArgs &a, const float *X, int64_t ldx, hipStream_t s)
{
    if (a.rows <= 0 || a.cols <= 0 || a.batch <= 0) return hipSuccess;
    constexpr int MB = 2, NB = 2;
    const dim3 grid((a.rows + 16 * MB - 1) / (16 * MB), (a.cols + kDenseWaves * 16 * NB - 1) / (kDenseWaves * 16 * NB));
    hipLaunchKernelGGL((dense_nt_kernel<MB, NB>), grid, dim3(kDenseBlock), 0, s, a.dZ, a.lddz, X, ldx, a.G, a.ldg, a.rows, a.cols, a.batch);
    hipLaunchKernelGGL(dense_update_kernel, dim3(a.rows < 16384 ? a.rows : 16384), dim3(kDenseBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_dense_refresh(const int32_t *indptr, const int32_t *indices, const float *values, int32_t rows, float *D, int64_t ld,
                                hipStream_t s)
{
    if (rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(dense_refresh_kernel, dim3(blocks_for_rows(rows)), dim3(kDenseBlock), 0, s, indptr, indices, values, rows, D, ld);
    return hipGetLastError();
}

}  // namespace nerva
