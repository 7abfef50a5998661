// Device side of binding a pattern to a layer (sparse_linear_create / sparse_linear_rebind): everything
// whose cost grows with the number of stored entries runs here, on the caller's device arrays --
// the check that the pattern is canonical CSR, the CSC mirror with the two position maps, and the
// segment bounds of the staged product.  What depends on the row lengths only (the row partitions)
// is planned on the host from a copy of the row pointers.
//
// The mirror is the stable counting sort of the stored entries by column.  The rows are cut into T
// tiles of consecutive rows with about nnz / T entries each, one wave per tile:
//   1. every tile counts its entries per column                      cnt[t][j]
//   2. per column, an exclusive scan over the tiles turns the counts into the tile's first slot
//      inside the column, and gives the column's length
//   3. an exclusive scan over the columns gives indptr_t
//   4. every tile walks its rows in order; a row's entries (distinct columns) take the next free
//      slot of their columns, cnt[t][j]++.  Rows are walked one after the other by one wave and
//      the counter is an L2 atomic whose result the wave waits for, so inside a column the slots
//      are handed out in row order: the result is the canonical CSR of W^T, bit for bit the same
//      on every run.
#include "kernels.h"

#include <climits>

namespace nerva {
namespace {

constexpr int kWave = 64;
constexpr int kSetupBlock = 256;

__global__ void status_init_kernel(int32_t *status)
{
    if (threadIdx.x == 0) {
        status[0] = 0;
        status[1] = INT_MAX;  // first row whose row pointers are wrong
        status[2] = INT_MAX;  // first stored entry whose column index is wrong
        status[3] = 0;
    }
}

__global__ __launch_bounds__(kSetupBlock) void validate_indptr_kernel(int32_t rows, int32_t nnz, const int32_t *__restrict__ indptr,
                                                                      int32_t *status)
{
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kSetupBlock + threadIdx.x;  // 0 .. rows
    if (i > rows) return;
    const int32_t v = indptr[i];
    int flags = 0;
    if (i == 0 && v != 0) flags |= kCsrBadFirst;
    if (v < 0 || v > nnz) flags |= kCsrBeyondNnz;
    if (i < rows && indptr[i + 1] < v) flags |= kCsrDecreasing;
    if (i == rows && v != nnz) flags |= kCsrBadLast;
    if (flags) {
        atomicOr(&status[0], flags);
        atomicMin(&status[1], static_cast<int32_t>(i));
    }
}

// A wave per row.  A row whose bounds are not inside [0, nnz] is left alone (the other kernel
// reports it): nothing is read outside indices[0 .. nnz).
__global__ __launch_bounds__(kSetupBlock) void validate_indices_kernel(int32_t rows, int32_t cols, int32_t nnz,
                                                                       const int32_t *__restrict__ indptr,
                                                                       const int32_t *__restrict__ indices, int32_t *status)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t n_waves = static_cast<int64_t>(gridDim.x) * (kSetupBlock / kWave);
    for (int64_t row = static_cast<int64_t>(blockIdx.x) * (kSetupBlock / kWave) + (threadIdx.x >> 6); row < rows; row += n_waves) {
        const int32_t b = indptr[row], e = indptr[row + 1];
        if (b < 0 || e > nnz || e < b) continue;
        for (int32_t p = b + lane; p < e; p += kWave) {
            const int32_t j = indices[p];
            int flags = 0;
            if (j < 0 || j >= cols)
                flags = kCsrColumnRange;
            else if (p > b && indices[p - 1] >= j)
                flags = kCsrNotAscending;
            if (flags) {
                atomicOr(&status[0], flags);
                atomicMin(&status[2], p);
            }
        }
    }
}

// First row of tile t: the first row i with indptr[i] * T >= t * nnz (a row belongs to the tile
// its first entry falls into; empty rows go along with their neighbours).
__device__ __forceinline__ int32_t tile_first_row(const int32_t *indptr, int32_t rows, int64_t nnz, int32_t T, int32_t t)
{
    const int64_t target = static_cast<int64_t>(t) * nnz;
    int32_t lo = 0, hi = rows;
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo) / 2;
        if (static_cast<int64_t>(indptr[mid]) * T >= target)
            hi = mid;
        else
            lo = mid + 1;
    }
    return lo;
}

__global__ __launch_bounds__(kSetupBlock) void mirror_count_kernel(int32_t rows, int32_t cols, int32_t nnz,
                                                                   const int32_t *__restrict__ indptr,
                                                                   const int32_t *__restrict__ indices, int32_t *cnt, int32_t T)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int32_t t = __builtin_amdgcn_readfirstlane(static_cast<int32_t>(blockIdx.x * (kSetupBlock / kWave) + (threadIdx.x >> 6)));
    if (t >= T) return;
    const int32_t r0 = tile_first_row(indptr, rows, nnz, T, t), r1 = tile_first_row(indptr, rows, nnz, T, t + 1);
    int32_t *c = cnt + static_cast<int64_t>(t) * cols;
    // the entries of consecutive rows are consecutive: no need to know the rows here
    for (int32_t p = indptr[r0] + lane; p < indptr[r1]; p += kWave) atomicAdd(&c[indices[p]], 1);
}

// Per column: counts of the tiles -> each tile's first slot inside the column; the column's length.
__global__ __launch_bounds__(kSetupBlock) void mirror_tile_scan_kernel(int32_t cols, int32_t T, int32_t *cnt, int32_t *col_count)
{
    const int64_t j = static_cast<int64_t>(blockIdx.x) * kSetupBlock + threadIdx.x;
    if (j >= cols) return;
    int32_t run = 0;
    int32_t t = 0;
    for (; t + 8 <= T; t += 8) {
        int32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = cnt[static_cast<int64_t>(t + u) * cols + j];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            cnt[static_cast<int64_t>(t + u) * cols + j] = run;
            run += v[u];
        }
    }
    for (; t < T; ++t) {
        const int32_t v = cnt[static_cast<int64_t>(t) * cols + j];
        cnt[static_cast<int64_t>(t) * cols + j] = run;
        run += v;
    }
    col_count[j] = run;
}

// out[0 .. n] = exclusive prefix sums of in[0 .. n), one work-group walking the array in chunks.
constexpr int kScanBlock = 1024;
__global__ __launch_bounds__(kScanBlock) void exclusive_scan_kernel(const int32_t *__restrict__ in, int32_t *__restrict__ out, int32_t n)
{
    __shared__ int32_t wave_total[kScanBlock / kWave];
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    int32_t carry = 0;
    for (int32_t base = 0; base < n; base += kScanBlock) {
        const int32_t i = base + threadIdx.x;
        const int32_t v = i < n ? in[i] : 0;
        int32_t x = v;
#pragma unroll
        for (int d = 1; d < kWave; d <<= 1) {
            const int32_t y = __shfl_up(x, d, kWave);
            if (lane >= d) x += y;
        }
        if (lane == kWave - 1) wave_total[wv] = x;
        __syncthreads();
        int32_t before = 0, total = 0;
#pragma unroll
        for (int w = 0; w < kScanBlock / kWave; ++w) {
            const int32_t s = wave_total[w];
            before += w < wv ? s : 0;
            total += s;
        }
        if (i < n) out[i] = carry + before + x - v;
        carry += total;
        __syncthreads();
    }
    if (threadIdx.x == 0) out[n] = carry;
}

__global__ __launch_bounds__(kSetupBlock) void mirror_scatter_kernel(int32_t rows, int32_t cols, int32_t nnz,
                                                                     const int32_t *__restrict__ indptr,
                                                                     const int32_t *__restrict__ indices,
                                                                     const int32_t *__restrict__ indptr_t, int32_t *cnt, int32_t T,
                                                                     int32_t *__restrict__ indices_t, int32_t *__restrict__ perm,
                                                                     int32_t *__restrict__ pos_t)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int32_t t = __builtin_amdgcn_readfirstlane(static_cast<int32_t>(blockIdx.x * (kSetupBlock / kWave) + (threadIdx.x >> 6)));
    if (t >= T) return;
    const int32_t r0 = tile_first_row(indptr, rows, nnz, T, t), r1 = tile_first_row(indptr, rows, nnz, T, t + 1);
    int32_t *c = cnt + static_cast<int64_t>(t) * cols;
    for (int32_t row = r0; row < r1; ++row) {
        const int32_t b = indptr[row], e = indptr[row + 1];
        for (int32_t p = b + lane; p < e; p += kWave) {
            const int32_t j = indices[p];
            // Columns are distinct inside a row, so the lanes of one instruction never meet; the
            // ordering (acquire + release at work-group scope) makes the wave wait for the result
            // before it issues the next row's, which may name the same column.
            const int32_t slot = __hip_atomic_fetch_add(&c[j], 1, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_WORKGROUP);
            const int32_t q = indptr_t[j] + slot;
            indices_t[q] = row;
            perm[q] = p;
            pos_t[p] = q;
        }
    }
}

// Segment bounds of the staged product: per slot of every range and per column block b, the position
// of the slot's first stored entry with column >= b * kStageRows (b = n_cb: one past the row's last
// entry; unused slots: 0 throughout).
__global__ __launch_bounds__(kSetupBlock) void staged_ends_kernel(const int32_t *__restrict__ indptr,
                                                                  const int32_t *__restrict__ indices,
                                                                  const int32_t *__restrict__ slot_rows, int32_t *__restrict__ ends,
                                                                  int32_t ranges, int32_t n_cb)
{
    const int64_t idx = static_cast<int64_t>(blockIdx.x) * kSetupBlock + threadIdx.x;
    const int64_t total = static_cast<int64_t>(ranges) * (n_cb + 1) * kStageRangeRows;
    if (idx >= total) return;
    const int32_t slot = static_cast<int32_t>(idx % kStageRangeRows);
    const int32_t b = static_cast<int32_t>((idx / kStageRangeRows) % (n_cb + 1));
    const int64_t q = idx / (static_cast<int64_t>(kStageRangeRows) * (n_cb + 1));
    int32_t r = slot_rows[q * kStageRangeRows + slot];
    if (r < 0) {
        ends[idx] = 0;
        return;
    }
    r &= ~kStageQuad;
    int32_t lo = indptr[r], hi = indptr[r + 1];
    const int64_t target = static_cast<int64_t>(b) * kStageRows;
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo) / 2;
        if (indices[mid] >= target)
            hi = mid;
        else
            lo = mid + 1;
    }
    ends[idx] = lo;
}

}  // namespace

hipError_t launch_validate_csr(int32_t rows, int32_t cols, int32_t nnz, const int32_t *indptr, const int32_t *indices,
                               int32_t *status, hipStream_t s)
{
    hipLaunchKernelGGL(status_init_kernel, dim3(1), dim3(kWave), 0, s, status);
    const int64_t n = static_cast<int64_t>(rows) + 1;
    hipLaunchKernelGGL(validate_indptr_kernel, dim3(static_cast<unsigned>((n + kSetupBlock - 1) / kSetupBlock)), dim3(kSetupBlock), 0, s,
                       rows, nnz, indptr, status);
    if (nnz > 0) {
        int64_t groups = (static_cast<int64_t>(rows) + kSetupBlock / kWave - 1) / (kSetupBlock / kWave);
        if (groups > 256 * 64) groups = 256 * 64;  // grid-stride beyond that
        hipLaunchKernelGGL(validate_indices_kernel, dim3(static_cast<unsigned>(groups)), dim3(kSetupBlock), 0, s, rows, cols, nnz, indptr,
                           indices, status);
    }
    return hipGetLastError();
}

int32_t mirror_tiles(int32_t rows, int32_t cols, int32_t nnz)
{
    // a tile's wave makes about (rows + nnz / 64) / T dependent round trips; its counters take T * cols ints
    int64_t T = (static_cast<int64_t>(rows) + nnz / kWave) / 64;
    if (T > 1024) T = 1024;
    const int64_t by_memory = (32ll << 20) / (cols > 0 ? cols : 1);  // at most 128 MiB of counters
    if (T > by_memory) T = by_memory;
    if (T < 1) T = 1;
    return static_cast<int32_t>(T);
}

size_t mirror_work_ints(int32_t cols, int32_t T) { return static_cast<size_t>(T) * cols + cols; }

hipError_t launch_build_mirror(int32_t rows, int32_t cols, int32_t nnz, const int32_t *indptr, const int32_t *indices,
                               int32_t *indptr_t, int32_t *indices_t, int32_t *perm, int32_t *pos_t, int32_t *work, int32_t T,
                               hipStream_t s)
{
    int32_t *cnt = work, *col_count = work + static_cast<size_t>(T) * cols;
    hipError_t e = hipMemsetAsync(cnt, 0, static_cast<size_t>(T) * cols * sizeof(int32_t), s);  // (set-up call: never captured in a graph)
    if (e != hipSuccess) return e;
    const unsigned tile_groups = static_cast<unsigned>((T + kSetupBlock / kWave - 1) / (kSetupBlock / kWave));
    const unsigned col_groups = static_cast<unsigned>((static_cast<int64_t>(cols) + kSetupBlock - 1) / kSetupBlock);
    if (nnz > 0) hipLaunchKernelGGL(mirror_count_kernel, dim3(tile_groups), dim3(kSetupBlock), 0, s, rows, cols, nnz, indptr, indices, cnt, T);
    hipLaunchKernelGGL(mirror_tile_scan_kernel, dim3(col_groups), dim3(kSetupBlock), 0, s, cols, T, cnt, col_count);
    hipLaunchKernelGGL(exclusive_scan_kernel, dim3(1), dim3(kScanBlock), 0, s, col_count, indptr_t, cols);
    if (nnz > 0)
        hipLaunchKernelGGL(mirror_scatter_kernel, dim3(tile_groups), dim3(kSetupBlock), 0, s, rows, cols, nnz, indptr, indices, indptr_t, cnt,
                           T, indices_t, perm, pos_t);
    return hipGetLastError();
}

hipError_t launch_staged_ends(const int32_t *indptr, const int32_t *indices, const int32_t *slot_rows, int32_t *ends, int32_t ranges,
                              int32_t n_cb, hipStream_t s)
{
    const int64_t total = static_cast<int64_t>(ranges) * (n_cb + 1) * kStageRangeRows;
    if (total <= 0) return hipSuccess;
    hipLaunchKernelGGL(staged_ends_kernel, dim3(static_cast<unsigned>((total + kSetupBlock - 1) / kSetupBlock)), dim3(kSetupBlock), 0, s,
                       indptr, indices, slot_rows, ends, ranges, n_cb);
    return hipGetLastError();
}

}  // namespace nerva
