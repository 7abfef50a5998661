// gfx950 kernels of the truly sparse MLP training step.
//
// Mapping shared by the sparse kernels: lanes of a 64-wide wavefront run along the batch
// dimension, so every gather of a dense row is one contiguous, coalesced read (one example
// per column, batch contiguous).  Where a gather fills the whole wave (wide batches) row
// pointers, column indices and weights are wave-uniform and travel through the scalar path;
// for narrow batches and column tiles several stored entries share one gather instruction, their
// indices loaded one per lane and handed round with ds_bpermute.  Rows are handed to work-groups
// by a static partition (RowBlocks) that gives long rows several waves, each with a contiguous
// share of the row's stored entries; partial sums of one row meet in LDS and are added in a
// fixed order.  There are no float atomics: every output element is produced by one lane in one
// order, so results are bit-reproducible from run to run.  (The exceptions to "along the batch":
// spmv_kernel and head_kernel, whose lanes run across a row's entries, and the opt-in dense
// route, an MFMA product.)
#include "kernels.h"

#include <utility>

namespace nerva {
namespace {

constexpr int kWave = 64;
constexpr int kBlock = kWave * kWavesPerBlock;
constexpr int kEwBlock = 256;  // work-group of the element-wise kernels

__device__ __forceinline__ int wave_in_block()
{
    return __builtin_amdgcn_readfirstlane(static_cast<int>(threadIdx.x >> 6));
}

__device__ __forceinline__ float4 keep_where_positive(float4 x, float4 m)
{
    x.x = m.x > 0.f ? x.x : 0.f;
    x.y = m.y > 0.f ? x.y : 0.f;
    x.z = m.z > 0.f ? x.z : 0.f;
    x.w = m.w > 0.f ? x.w : 0.f;
    return x;
}
__device__ __forceinline__ float keep_where_positive(float x, float m) { return m > 0.f ? x : 0.f; }

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }

// Data-parallel-primitive move: lane l receives x from the lane that CTRL names; lanes in rows
// not selected by ROW_MASK receive 0.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ float dpp(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, ROW_MASK, 0xF, false));
}

// Sum over each row of 16 lanes, all 64 lanes active; every lane of a row gets the same bits.
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp<0xB1>(x);   // quad_perm [1,0,3,2]
    x += dpp<0x4E>(x);   // quad_perm [2,3,0,1]
    x += dpp<0x141>(x);  // row_half_mirror
    x += dpp<0x140>(x);  // row_mirror
    return x;
}

// Sum over groups of G lanes (8: per half row; 16: per row; 64: whole wave, returned wave-uniform).
template <int G>
__device__ __forceinline__ float group_sum(float x)
{
    static_assert(G == 8 || G == 16 || G == 32 || G == 64, "group sizes with a reduction");
    if constexpr (G == 8) {
        x += dpp<0xB1>(x);   // quad_perm [1,0,3,2]
        x += dpp<0x4E>(x);   // quad_perm [2,3,0,1]
        x += dpp<0x141>(x);  // row_half_mirror
        return x;
    }
    x = row16_sum(x);
    if constexpr (G == 32) x += __shfl_xor(x, 16, kWave);  // the other row of the pair (through the LDS crossbar)
    if constexpr (G == 64) {
        x += dpp<0x142, 0xA>(x);  // row_bcast15 into rows 1 and 3
        x += dpp<0x143, 0xC>(x);  // row_bcast31 into rows 2 and 3
        x = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
    }
    return x;
}

// The momentum step of one element; the same expression in the fused and the stand-alone path.
// nesterov: the weight moves by the look-ahead mu*v_new - lr*g instead of v_new.
__device__ __forceinline__ void momentum_step(float &w, float &v, float g, float lr, float mu, int nesterov)
{
    const float step = lr * g;
    v = fmaf(mu, v, -step);
    w = nesterov ? w + fmaf(mu, v, -step) : w + v;
}

// Which row, and which contiguous run [s0, s1) of its stored entries, the calling wave serves.
struct WaveTask {
    int row;     // -1: nothing to do
    int part;    // index of this wave among the waves that share the row inside this work-group
    int lg;      // log2(waves that share the row in this work-group); uniform over the work-group
    int s0, s1;  // the wave's stored entries
    bool huge;   // the work-group holds one share of a huge row: its result is a partial sum
    bool lead;   // first wave of the row's first share (owner of per-row by-products)
};
// One 16-byte scalar load per wave: the partition table is spelled out per wave when the
// pattern is bound, so nothing about the row has to be looked up before its entries are fetched.
__device__ __forceinline__ WaveTask wave_task(const RowBlocks &b, int block)
{
    const int4 d = b.waves[block * kWavesPerBlock + wave_in_block()];
    WaveTask t;
    t.row = d.x;
    t.s0 = d.y;
    t.s1 = d.z;
    t.part = d.w & 15;
    t.lg = (d.w >> 4) & 15;
    t.lead = (d.w >> 8) & 1;
    t.huge = (d.w >> 9) & 1;
    return t;
}

// Address of row j of a dense matrix whose rows are ld_bytes apart, kept in scalar registers:
// the readfirstlane fences stop the compiler from folding the per-lane column offset into a
// 64-bit vector multiply-add, so the gather uses the scalar-base + 32-bit lane offset form.
typedef const __attribute__((address_space(1))) char *gmem_ptr;  // global (device) memory
__device__ __forceinline__ gmem_ptr row_base(const void *base, int j, uint32_t ld_bytes)
{
    const uint64_t addr = reinterpret_cast<uint64_t>(base) + static_cast<uint64_t>(static_cast<uint32_t>(j)) * ld_bytes;
    const uint32_t lo = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(addr));
    const uint32_t hi = __builtin_amdgcn_readfirstlane(static_cast<uint32_t>(addr >> 32));
    return reinterpret_cast<gmem_ptr>((static_cast<uint64_t>(hi) << 32) | lo);
}
__device__ __forceinline__ gmem_ptr as_gmem(const void *p) { return reinterpret_cast<gmem_ptr>(reinterpret_cast<uint64_t>(p)); }
typedef float v4f __attribute__((ext_vector_type(4)));
template <typename V>
__device__ __forceinline__ V gload(gmem_ptr row, uint32_t byte_offset);
template <>
__device__ __forceinline__ float4 gload<float4>(gmem_ptr row, uint32_t byte_offset)
{
    const v4f r = *reinterpret_cast<const __attribute__((address_space(1))) v4f *>(row + byte_offset);
    return make_float4(r.x, r.y, r.z, r.w);
}
template <>
__device__ __forceinline__ float gload<float>(gmem_ptr row, uint32_t byte_offset)
{
    return *reinterpret_cast<const __attribute__((address_space(1))) float *>(row + byte_offset);
}

template <int VEC> struct Pack;
template <> struct Pack<4> { using type = float4; };
template <> struct Pack<1> { using type = float; };

__device__ __forceinline__ void fma_into(float (&acc)[4], float w, float4 x)
{
    acc[0] = fmaf(w, x.x, acc[0]);
    acc[1] = fmaf(w, x.y, acc[1]);
    acc[2] = fmaf(w, x.z, acc[2]);
    acc[3] = fmaf(w, x.w, acc[3]);
}
__device__ __forceinline__ void fma_into(float (&acc)[1], float w, float x) { acc[0] = fmaf(w, x, acc[0]); }

// U consecutive stored entries starting at p: all index/weight fetches, then all gathers, then
// the FMAs, so that U*NV reads are in flight per wave.
template <int VEC, int NV, bool XMASK, int U>
__device__ __forceinline__ void spmm_step(const SpmmArgs &a, int p, uint32_t ldxb, uint32_t ldmb,
                                          const uint32_t (&off)[NV], float (&acc)[NV][VEC])
{
    using V = typename Pack<VEC>::type;
    int j[U];
    float w[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        j[u] = a.indices[p + u];
        w[u] = a.values[p + u];
    }
    V x[U][NV];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const gmem_ptr xr = row_base(a.X, j[u], ldxb);
#pragma unroll
        for (int t = 0; t < NV; ++t) x[u][t] = gload<V>(xr, off[t]);
        if constexpr (XMASK) {
            const gmem_ptr mr = row_base(a.XM, j[u], ldmb);
#pragma unroll
            for (int t = 0; t < NV; ++t) x[u][t] = keep_where_positive(x[u][t], gload<V>(mr, off[t]));
        }
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int t = 0; t < NV; ++t) fma_into(acc[t], w[u], x[u][t]);
}

// ---------------------------------------------------------------------------------------
// SpMM.  VEC = floats per lane access (4: 16-byte accesses, needs leading dimensions that are
// multiples of 4 and 16-byte aligned bases; 1: anything).  A wave covers 64*VEC*NV columns;
// blockIdx.y walks over column tiles.
// ---------------------------------------------------------------------------------------
template <int VEC, int NV, bool XMASK>
__device__ __forceinline__ void spmm_body(const SpmmArgs &a, const int block, const int col_tile)
{
    constexpr int U = NV >= 4 ? 2 : (NV == 2 ? 4 : 8);
    __shared__ float red[kWavesPerBlock][NV][VEC][kWave];

    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const WaveTask task = wave_task(a.blocks, block);
    const int col_base = col_tile * (kWave * VEC * NV);

    // Lanes whose columns lie beyond the batch re-read the tile's first columns and are never stored.
    // A 4-wide access that starts below `batch` stays inside the row: ld is a multiple of 4 and >= batch.
    int col[NV];
    bool on[NV];
    uint32_t off[NV];
    float acc[NV][VEC];
#pragma unroll
    for (int t = 0; t < NV; ++t) {
        col[t] = col_base + (t * kWave + lane) * VEC;
        on[t] = col[t] < a.batch;
        off[t] = static_cast<uint32_t>(on[t] ? col[t] : col_base) * 4u;
#pragma unroll
        for (int k = 0; k < VEC; ++k) acc[t][k] = 0.f;
    }

    if (task.row >= 0) {
        const uint32_t ldxb = static_cast<uint32_t>(a.ldx) * 4u;
        const uint32_t ldmb = XMASK ? static_cast<uint32_t>(a.ldxm) * 4u : 0u;
        int p = task.s0;
        const int pe = task.s1;
        // only entries of this wave's share are gathered: the gather stream is what the kernel pays for
        for (; p + U <= pe; p += U) spmm_step<VEC, NV, XMASK, U>(a, p, ldxb, ldmb, off, acc);
        if constexpr (U >= 8)
            if (p + 4 <= pe) { spmm_step<VEC, NV, XMASK, 4>(a, p, ldxb, ldmb, off, acc); p += 4; }
        if constexpr (U >= 4)
            if (p + 2 <= pe) { spmm_step<VEC, NV, XMASK, 2>(a, p, ldxb, ldmb, off, acc); p += 2; }
        if (p < pe) spmm_step<VEC, NV, XMASK, 1>(a, p, ldxb, ldmb, off, acc);
    }

    if (task.lg > 0) {  // uniform over the work-group
        if (task.part != 0) {
#pragma unroll
            for (int t = 0; t < NV; ++t)
#pragma unroll
                for (int k = 0; k < VEC; ++k) red[wv][t][k][lane] = acc[t][k];
        }
        __syncthreads();
        if (task.part == 0) {
            for (int s = 1; s < (1 << task.lg); ++s)
#pragma unroll
                for (int t = 0; t < NV; ++t)
#pragma unroll
                    for (int k = 0; k < VEC; ++k) acc[t][k] += red[wv + s][t][k][lane];
        }
    }
    if (task.row < 0 || task.part != 0) return;

    if (task.huge) {
        // one share of a huge row: the raw partial sum goes to this work-group's scratch row
        float *sr = a.scratch + static_cast<int64_t>(block) * a.scratch_ld;
#pragma unroll
        for (int t = 0; t < NV; ++t)
#pragma unroll
            for (int k = 0; k < VEC; ++k)
                if (col[t] + k < a.batch) sr[col[t] + k] = acc[t][k];
        return;
    }

    const float b = a.bias ? a.bias[task.row] : 0.f;
    float *yr = a.Y + static_cast<int64_t>(task.row) * a.ldy;
    const float *ym = a.YM ? a.YM + static_cast<int64_t>(task.row) * a.ldym : nullptr;
#pragma unroll
    for (int t = 0; t < NV; ++t) {
        if (!on[t]) continue;
        float y[VEC];
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            y[k] = acc[t][k] + b;
            if (a.relu) y[k] = y[k] > 0.f ? y[k] : 0.f;
        }
        if constexpr (VEC == 4) {
            if (col[t] + 4 <= a.batch) {
                float4 o = make_float4(y[0], y[1], y[2], y[3]);
                if (ym) o = keep_where_positive(o, ld4(ym + col[t]));
                st4(yr + col[t], o);
            } else {
                for (int k = 0; k < 4; ++k)
                    if (col[t] + k < a.batch) {
                        float o = y[k];
                        if (ym) o = keep_where_positive(o, ym[col[t] + k]);
                        yr[col[t] + k] = o;
                    }
            }
        } else {
            float o = y[0];
            if (ym) o = keep_where_positive(o, ym[col[t]]);
            yr[col[t]] = o;
        }
    }
}

// One pass of U gather instructions of the grouped SpMM: every index move, then every gather,
// then the FMAs.  Straight-line on purpose: with no branch between the gathers the compiler
// counts outstanding loads exactly (vmcnt U-1 ... 0) and all U stay in flight; a branch inside
// makes it wait for every earlier load before each later one.
// src: byte address (lane * 4) of the lane that holds this group's entry of the pass's first
// step; consecutive steps lie STEP_BYTES further on.
template <int U, int STEP_BYTES, bool XMASK>
__device__ __forceinline__ void grouped_pass(gmem_ptr Xg, gmem_ptr Mg, int src, int my_ro, int my_mo, float my_w,
                                             uint32_t off, float (&acc)[4])
{
    uint32_t ro[U], mo[U];
    float w[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        ro[u] = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(src + u * STEP_BYTES, my_ro));
        w[u] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src + u * STEP_BYTES, __builtin_bit_cast(int, my_w)));
        if constexpr (XMASK) mo[u] = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(src + u * STEP_BYTES, my_mo));
    }
    float4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) x[u] = gload<float4>(Xg, ro[u] + off);
    if constexpr (XMASK) {
#pragma unroll
        for (int u = 0; u < U; ++u) x[u] = keep_where_positive(x[u], gload<float4>(Mg, mo[u] + off));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
        acc[0] = fmaf(w[u], x[u].x, acc[0]);
        acc[1] = fmaf(w[u], x[u].y, acc[1]);
        acc[2] = fmaf(w[u], x[u].z, acc[2]);
        acc[3] = fmaf(w[u], x[u].w, acc[3]);
    }
}

// SpMM for batches of at most GS*4 columns, GS in {8, 16, 32}: a gather instruction costs the
// memory pipeline the same whether 25 or 64 lanes take part, so each group of GS lanes works on
// its own stored entry and one instruction fetches 64/GS rows of the dense operand.  Entries of
// the wave's share are dealt to the groups round-robin; the groups' partial sums meet in LDS
// together with those of the other waves of the row and are added in (wave, group) order.
// Row offsets are 32-bit byte offsets from the operand's base: the operand (and its mask) must
// span less than 4 GiB, which the launcher checks.
template <int GS, bool XMASK>
__device__ __forceinline__ void spmm_body_grouped(const SpmmArgs &a, const int block, const int col0 = 0)
{
    constexpr int NE = kWave / GS;   // entries per gather instruction
    constexpr int SB = NE * 4;       // lane-address distance between consecutive steps
    __shared__ float red[kWavesPerBlock][4][kWave];

    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const int grp = lane / GS;
    const int lig = lane % GS;
    const WaveTask task = wave_task(a.blocks, block);
    const int col = col0 + lig * 4;
    const bool on = col < a.batch;
    const uint32_t off = static_cast<uint32_t>(on ? col : col0) * 4u;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};

    if (task.row >= 0) {
        const uint32_t ldxb = static_cast<uint32_t>(a.ldx) * 4u;
        const uint32_t ldmb = XMASK ? static_cast<uint32_t>(a.ldxm) * 4u : 0u;
        const gmem_ptr Xg = as_gmem(a.X);
        const gmem_ptr Mg = as_gmem(a.XM);
        for (int pc = task.s0; pc < task.s1; pc += kWave) {
            const int n = min(kWave, task.s1 - pc);
            // Entry pc+l of the chunk sits in lane l; step u hands entry u*NE+grp to group grp.
            // Lanes past the chunk's end repeat its first entry with weight 0: a gather of theirs
            // reads a row this output row reads anyway, and adds nothing.
            const int q = lane < n ? lane : 0;
            const int my_j = a.indices[pc + q];
            float my_w = a.values[pc + q];
            my_w = lane < n ? my_w : 0.f;
            const int my_ro = static_cast<int>(static_cast<uint32_t>(my_j) * ldxb);
            const int my_mo = XMASK ? static_cast<int>(static_cast<uint32_t>(my_j) * ldmb) : 0;
            const int steps = (n + NE - 1) / NE;
            int src = grp * 4;
            int u0 = 0;
            for (; u0 + 8 <= steps; u0 += 8, src += 8 * SB)
                grouped_pass<8, SB, XMASK>(Xg, Mg, src, my_ro, my_mo, my_w, off, acc);
            if (u0 + 4 <= steps) {
                grouped_pass<4, SB, XMASK>(Xg, Mg, src, my_ro, my_mo, my_w, off, acc);
                u0 += 4; src += 4 * SB;
            }
            if (u0 + 2 <= steps) {
                grouped_pass<2, SB, XMASK>(Xg, Mg, src, my_ro, my_mo, my_w, off, acc);
                u0 += 2; src += 2 * SB;
            }
            if (u0 < steps) grouped_pass<1, SB, XMASK>(Xg, Mg, src, my_ro, my_mo, my_w, off, acc);
        }
    }

    // every wave leaves its 64 lanes' partial sums in LDS; the row's first wave adds them up
#pragma unroll
    for (int k = 0; k < 4; ++k) red[wv][k][lane] = acc[k];
    __syncthreads();
    if (task.row < 0 || task.part != 0 || grp != 0) return;
#pragma unroll
    for (int k = 0; k < 4; ++k) acc[k] = 0.f;
    for (int s = 0; s < (1 << task.lg); ++s)
#pragma unroll
        for (int g = 0; g < NE; ++g)
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[k] += red[wv + s][k][g * GS + lig];
    if (!on) return;

    if (task.huge) {
        float *sr = a.scratch + static_cast<int64_t>(block) * a.scratch_ld;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (col + k < a.batch) sr[col + k] = acc[k];
        return;
    }
    const float b = a.bias ? a.bias[task.row] : 0.f;
    float *yr = a.Y + static_cast<int64_t>(task.row) * a.ldy;
    const float *ym = a.YM ? a.YM + static_cast<int64_t>(task.row) * a.ldym : nullptr;
    float y[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        y[k] = acc[k] + b;
        if (a.relu) y[k] = y[k] > 0.f ? y[k] : 0.f;
    }
    if (col + 4 <= a.batch) {
        float4 o = make_float4(y[0], y[1], y[2], y[3]);
        if (ym) o = keep_where_positive(o, ld4(ym + col));
        st4(yr + col, o);
    } else {
        for (int k = 0; k < 4; ++k)
            if (col + k < a.batch) {
                float o = y[k];
                if (ym) o = keep_where_positive(o, ym[col + k]);
                yr[col + k] = o;
            }
    }
}

// Packed SpMM for short rows: each group of GS lanes owns one row, so a gather instruction
// fetches one entry of each of 64/GS rows and no sum across groups or waves is needed.  The rows
// come from RowBlocks::short_rows, longest first, so the rows of a set have nearly the same
// length; a group whose row is exhausted repeats that row's first entry with weight 0.  A wave
// can serve kPackSets sets one after the other, fetching the next set's rows and indices one
// step ahead; measured, one set per wave is best (more, shorter work-groups balance better than
// the saved start-up is worth).
template <int GS, bool XMASK>
__device__ __forceinline__ void spmm_body_packed(const SpmmArgs &a, const int block, const int col0, const int n_pack_blocks)
{
    constexpr int NE = kWave / GS;
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const int grp = lane / GS;
    const int lig = lane % GS;
    const int col = col0 + lig * 4;
    const bool on = col < a.batch;
    const uint32_t off = static_cast<uint32_t>(on ? col : col0) * 4u;
    const uint32_t ldxb = static_cast<uint32_t>(a.ldx) * 4u;
    const uint32_t ldmb = XMASK ? static_cast<uint32_t>(a.ldxm) * 4u : 0u;
    const gmem_ptr Xg = as_gmem(a.X);
    const gmem_ptr Mg = as_gmem(a.XM);
    const int n_sets = (a.blocks.n_short + NE - 1) / NE;
    const int src0 = grp * GS * 4;  // byte address of the group's first lane
    // The sets are sorted by length, so they are dealt to the waves round-robin: wave k of the
    // launch's n_waves takes sets k, k + n_waves, k + 2 n_waves, ... and every wave gets its share
    // of long and of short rows (consecutive sets per wave left the first work-groups 1.4x the work
    // of the average on rows of 40..85 entries, and a launch is one round of work-groups).
    const int n_waves = n_pack_blocks * kWavesPerBlock;
    const int first_set = block * kWavesPerBlock + wv;
    if (first_set >= n_sets) return;  // wave-uniform
    const int last_set = first_set + ((n_sets - 1 - first_set) / n_waves) * n_waves;  // <= first_set + (kPackSets - 1) * n_waves

    // Entry base+lig of the group's row: column index and weight (0 past the row's end, where the
    // row's first entry is repeated; an empty row reads entry 0 of the matrix and is zeroed below).
    auto fetch = [&](int s0, int len, int base, int &j, float &w) {
        const int e = base + lig;
        const bool ok = e < len;
        const int p = len > 0 ? s0 + (ok ? e : 0) : 0;
        j = a.indices[p];
        w = a.values[p];
        w = ok ? w : 0.f;
    };

    // One step ahead: while a chunk of GS entries per row is gathered, the indices and weights of
    // the next chunk (or of the next set's first chunk) and the next set's rows are on their way.
    int4 d = a.blocks.short_rows[first_set * NE + grp];  // the table is padded to whole sets
    int cur_j;
    float cur_w;
    fetch(d.y, d.z, 0, cur_j, cur_w);
    for (int set = first_set; set <= last_set; set += n_waves) {
        const int row = d.x, s0 = d.y, len = d.z;
        const int maxlen = __builtin_amdgcn_readfirstlane(len);  // group 0 holds the set's longest row
        const int4 dn = a.blocks.short_rows[min(set + n_waves, last_set) * NE + grp];
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        int base = 0;
        do {
            const bool more = base + GS < maxlen;  // wave-uniform
            int next_j;
            float next_w;
            fetch(more ? s0 : dn.y, more ? len : dn.z, more ? base + GS : 0, next_j, next_w);
            const int my_ro = static_cast<int>(static_cast<uint32_t>(cur_j) * ldxb);
            const int my_mo = XMASK ? static_cast<int>(static_cast<uint32_t>(cur_j) * ldmb) : 0;
            const float my_w = cur_w;
            const int steps = min(GS, maxlen - base);  // 0 for a set of empty rows
            int src = src0;
            int u0 = 0;
            for (; u0 + 8 <= steps; u0 += 8, src += 32) grouped_pass<8, 4, XMASK>(Xg, Mg, src, my_ro, my_mo, my_w, off, acc);
            if (u0 + 4 <= steps) {
                grouped_pass<4, 4, XMASK>(Xg, Mg, src, my_ro, my_mo, my_w, off, acc);
                u0 += 4; src += 16;
            }
            if (u0 + 2 <= steps) {
                grouped_pass<2, 4, XMASK>(Xg, Mg, src, my_ro, my_mo, my_w, off, acc);
                u0 += 2; src += 8;
            }
            if (u0 < steps) grouped_pass<1, 4, XMASK>(Xg, Mg, src, my_ro, my_mo, my_w, off, acc);
            cur_j = next_j;
            cur_w = next_w;
            base += GS;
        } while (base < maxlen);
        d = dn;
        if (row < 0 || !on) continue;
        const float b = a.bias ? a.bias[row] : 0.f;
        float *yr = a.Y + static_cast<int64_t>(row) * a.ldy;
        const float *ym = a.YM ? a.YM + static_cast<int64_t>(row) * a.ldym : nullptr;
        float y[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            y[k] = (len > 0 ? acc[k] : 0.f) + b;  // an empty row gathered (with weight 0) from entry 0 of the matrix
            if (a.relu) y[k] = y[k] > 0.f ? y[k] : 0.f;
        }
        if (col + 4 <= a.batch) {
            float4 o = make_float4(y[0], y[1], y[2], y[3]);
            if (ym) o = keep_where_positive(o, ld4(ym + col));
            st4(yr + col, o);
        } else {
            for (int k = 0; k < 4; ++k)
                if (col + k < a.batch) {
                    float o = y[k];
                    if (ym) o = keep_where_positive(o, ym[col + k]);
                    yr[col + k] = o;
                }
        }
    }
}

// Short rows through the packed body, the remaining rows through the grouped body, in one grid,
// for every column tile; work-group ids are decoded XCD-first as in spmm_tiled_kernel.
template <int GS, bool XMASK>
__global__ __launch_bounds__(kBlock) void spmm_packed_kernel(const SpmmArgs a, const int n_tiles, const int spread,
                                                             const int n_pack_blocks)
{
    const int nrb = n_pack_blocks + a.blocks.n_long_blocks;
    int tile, rb;
    if (spread) {
        const int xcd = blockIdx.x & 7, k = blockIdx.x >> 3;
        tile = (k / nrb) * 8 + xcd;
        rb = k % nrb;
    } else {
        tile = blockIdx.x / nrb;
        rb = blockIdx.x % nrb;
    }
    if (tile >= n_tiles) return;
    if (rb < n_pack_blocks) {
        spmm_body_packed<GS, XMASK>(a, rb, tile * GS * 4, n_pack_blocks);
    } else {
        SpmmArgs al = a;
        al.blocks.waves = a.blocks.long_waves;
        spmm_body_grouped<GS, XMASK>(al, rb - n_pack_blocks, tile * GS * 4);
    }
}

template <int GS, bool XMASK>
__global__ __launch_bounds__(kBlock) void spmm_grouped_kernel(const SpmmArgs a)
{
    spmm_body_grouped<GS, XMASK>(a, blockIdx.x);
}

// Column-tiled launch for dense operands that do not fit an L2: the batch is cut into tiles of
// GS*4 columns, narrow enough that one tile of the whole operand (x_rows x GS*4 floats) stays
// resident in a 4 MiB L2 while every stored entry gathers from it.  Work-groups are dealt to the
// 8 XCDs round-robin by their id, so the id is decoded XCD-first: with 8 or more tiles each XCD
// owns every 8th tile (each tile is fetched from HBM by one L2 only) and sweeps the row partition
// once per tile; with fewer tiles every XCD walks all tiles in the same order.
template <int GS, bool XMASK>
__global__ __launch_bounds__(kBlock) void spmm_tiled_kernel(const SpmmArgs a, const int n_tiles, const int spread)
{
    const int nrb = a.blocks.n_blocks;
    int tile, rb;
    if (spread) {
        const int xcd = blockIdx.x & 7, k = blockIdx.x >> 3;
        tile = (k / nrb) * 8 + xcd;
        rb = k % nrb;
    } else {
        tile = blockIdx.x / nrb;
        rb = blockIdx.x % nrb;
    }
    if (tile >= n_tiles) return;
    spmm_body_grouped<GS, XMASK>(a, rb, tile * GS * 4);
}

template <int VEC, int NV, bool XMASK>
__global__ __launch_bounds__(kBlock) void spmm_kernel(const SpmmArgs a)
{
    spmm_body<VEC, NV, XMASK>(a, blockIdx.x, blockIdx.y);
}

// SpMM for batches of at most 4 columns (inference on one or a few examples): there is no batch
// dimension to spread lanes over, so lanes run across the stored entries of the wave's share
// instead -- coalesced index/weight reads, a 4-byte gather per entry and column, a DPP sum over
// the wave, and the usual ordered LDS combine of the row's shares.  Any leading dimension.
template <int NB>
__global__ __launch_bounds__(kBlock) void spmv_kernel(const SpmmArgs a)
{
    __shared__ float red[kWavesPerBlock][NB];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const WaveTask task = wave_task(a.blocks, blockIdx.x);
    float acc[NB];
#pragma unroll
    for (int c = 0; c < NB; ++c) acc[c] = 0.f;
    if (task.row >= 0) {
        for (int p = task.s0 + lane; p < task.s1; p += kWave) {
            const int64_t j = a.indices[p];
            const float w = a.values[p];
            const float *xr = a.X + j * a.ldx;
            const float *mr = a.XM ? a.XM + j * a.ldxm : nullptr;
#pragma unroll
            for (int c = 0; c < NB; ++c)
                if (c < a.batch) {
                    float x = xr[c];
                    if (mr) x = keep_where_positive(x, mr[c]);
                    acc[c] = fmaf(w, x, acc[c]);
                }
        }
    }
#pragma unroll
    for (int c = 0; c < NB; ++c) acc[c] = group_sum<kWave>(acc[c]);  // all lanes of every wave take part
    if (task.lg > 0) {
        if (lane == 0)
#pragma unroll
            for (int c = 0; c < NB; ++c) red[wv][c] = acc[c];
        __syncthreads();
        if (task.part == 0)
            for (int s = 1; s < (1 << task.lg); ++s)
#pragma unroll
                for (int c = 0; c < NB; ++c) acc[c] += red[wv + s][c];
    }
    if (task.row < 0 || task.part != 0 || lane >= a.batch || lane >= NB) return;
    float y = acc[0];
#pragma unroll
    for (int c = 1; c < NB; ++c) y = lane == c ? acc[c] : y;
    if (task.huge) {
        a.scratch[static_cast<int64_t>(blockIdx.x) * a.scratch_ld + lane] = y;
        return;
    }
    y += a.bias ? a.bias[task.row] : 0.f;
    if (a.relu) y = y > 0.f ? y : 0.f;
    if (a.YM) y = keep_where_positive(y, a.YM[static_cast<int64_t>(task.row) * a.ldym + lane]);
    a.Y[static_cast<int64_t>(task.row) * a.ldy + lane] = y;
}

// Product with a FULL matrix of few rows (every entry stored, rows <= kFullMaxRows): values[] is
// the row-major dense matrix, so instead of gathering the operand once per row the kernel streams
// it once for all rows.  A work-group of 4 waves owns kFullSlice consecutive operand rows and 256
// batch columns (4 per lane); wave w walks the slice's operand rows w*32 .. w*32+31, eight 16-byte
// loads in flight, weights through uniform loads, one accumulator per matrix row; the waves'
// accumulators meet in LDS and are added in wave order.  The slice's partial result goes to
// full_scratch; full_rows_finish_kernel adds the slices in order and applies the epilogue.
constexpr int kFullWaves = 4;  // 4 waves x 16 rows x 1 KiB of LDS at most: 64 KiB
__global__ __launch_bounds__(kFullWaves * kWave) void full_rows_kernel(const SpmmArgs a)
{
    extern __shared__ float4 full_red[];  // [kFullWaves][rows][kWave]
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const int K = a.x_rows;
    const int slice = blockIdx.x;
    const int col = (blockIdx.y * kWave + lane) * 4;
    const bool on = col < a.batch;
    const int64_t xoff = on ? col : 0;
    constexpr int KW = kFullSlice / kFullWaves;  // operand rows per wave: all requested before the first use
    static_assert(KW <= 64 && (KW & (KW - 1)) == 0, "one weight per lane");
    const int k_begin = slice * kFullSlice + wv * KW;
    float4 acc[kFullMaxRows];
    float4 x[KW];
#pragma unroll
    for (int u = 0; u < KW; ++u) {
        const int64_t k = k_begin + u < K ? k_begin + u : K - 1;  // rows past the end are re-read and get weight 0
        x[u] = ld4(a.X + k * a.ldx + xoff);
    }
    // lane u (and u + 32) holds row r's weight of operand row k_begin + u
    float wrow[kFullMaxRows];
    const int kl = k_begin + (lane & (KW - 1));
#pragma unroll
    for (int r = 0; r < kFullMaxRows; ++r)
        wrow[r] = (r < a.rows && kl < K) ? a.values[static_cast<int64_t>(r) * K + kl] : 0.f;
#pragma unroll
    for (int r = 0; r < kFullMaxRows; ++r) {
        acc[r] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (r < a.rows) {  // uniform
#pragma unroll
            for (int u = 0; u < KW; ++u) {
                const float w = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, wrow[r]), u));
                acc[r].x = fmaf(w, x[u].x, acc[r].x);
                acc[r].y = fmaf(w, x[u].y, acc[r].y);
                acc[r].z = fmaf(w, x[u].z, acc[r].z);
                acc[r].w = fmaf(w, x[u].w, acc[r].w);
            }
        }
    }
#pragma unroll
    for (int r = 0; r < kFullMaxRows; ++r)
        if (r < a.rows) full_red[(wv * a.rows + r) * kWave + lane] = acc[r];
    __syncthreads();
    if (!on) return;
    for (int r = wv; r < a.rows; r += kFullWaves) {
        float4 y = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int w = 0; w < kFullWaves; ++w) {
            const float4 p = full_red[(w * a.rows + r) * kWave + lane];
            y.x += p.x; y.y += p.y; y.z += p.z; y.w += p.w;
        }
        st4(a.full_scratch + (static_cast<int64_t>(slice) * a.rows + r) * a.full_scratch_ld + col, y);
    }
}

__global__ __launch_bounds__(kEwBlock) void full_rows_finish_kernel(const SpmmArgs a, const int n_slices)
{
    const int r = blockIdx.x;
    const int c = blockIdx.y * kEwBlock + threadIdx.x;
    if (c >= a.batch) return;
    const float *p = a.full_scratch + static_cast<int64_t>(r) * a.full_scratch_ld + c;
    const int64_t step = static_cast<int64_t>(a.rows) * a.full_scratch_ld;
    float y = 0.f;
    int q = 0;
    for (; q + 8 <= n_slices; q += 8) {  // eight loads in flight, added in slice order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = p[(q + u) * step];
#pragma unroll
        for (int u = 0; u < 8; ++u) y += v[u];
    }
    for (; q < n_slices; ++q) y += p[q * step];
    y += a.bias ? a.bias[r] : 0.f;
    if (a.relu) y = y > 0.f ? y : 0.f;
    if (a.YM) y = keep_where_positive(y, a.YM[static_cast<int64_t>(r) * a.ldym + c]);
    a.Y[static_cast<int64_t>(r) * a.ldy + c] = y;
}

// The same finish pass for an output layer, with the softmax cross-entropy on top: wave r of a work-group adds the
// slices of row r for 64 columns, the rows meet in LDS, and every wave then forms its own row of the loss gradient
// (each lane repeats the column's maximum and sum over the <= 16 rows, in the order of softmax_ce_kernel, so the
// gradient has the same bits); wave 0 also stores the column's loss.
__global__ __launch_bounds__(kBlock) void full_rows_finish_softmax_kernel(const SpmmArgs a, const int n_slices)
{
    __shared__ float zs[kWavesPerBlock][kWave];
    static_assert(kFullMaxRows <= kWavesPerBlock, "one wave per row");
    const int lane = threadIdx.x & (kWave - 1);
    const int r = wave_in_block();
    const int c = blockIdx.x * kWave + lane;
    const bool on = r < a.rows && c < a.batch;
    float y = 0.f;
    if (on) {
        const float *p = a.full_scratch + static_cast<int64_t>(r) * a.full_scratch_ld + c;
        const int64_t step = static_cast<int64_t>(a.rows) * a.full_scratch_ld;
        int q = 0;
        for (; q + 8 <= n_slices; q += 8) {  // eight loads in flight, added in slice order
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = p[(q + u) * step];
#pragma unroll
            for (int u = 0; u < 8; ++u) y += v[u];
        }
        for (; q < n_slices; ++q) y += p[q * step];
        y += a.bias ? a.bias[r] : 0.f;
        a.Y[static_cast<int64_t>(r) * a.ldy + c] = y;
    }
    zs[r][lane] = y;
    __syncthreads();
    if (!on) return;
    const int t = a.ce_labels[c];
    float z[kFullMaxRows];
#pragma unroll
    for (int i = 0; i < kFullMaxRows; ++i) z[i] = i < a.rows ? zs[i][lane] : -INFINITY;
    float m = z[0];
#pragma unroll
    for (int i = 1; i < kFullMaxRows; ++i) m = fmaxf(m, z[i]);
    float sum = 0.f, zt = 0.f;
#pragma unroll
    for (int i = 0; i < kFullMaxRows; ++i) {
        if (i < a.rows) sum += expf(z[i] - m);
        zt = i == t ? z[i] : zt;
    }
    const float lse = m + logf(sum);
    a.ce_dZ[static_cast<int64_t>(r) * a.ce_lddz + c] = (expf(y - lse) - (r == t ? 1.f : 0.f)) * (1.0f / static_cast<float>(a.batch));
    if (r == 0) a.ce_loss_cols[c] = lse - zt;
}

// ---- staged product ----------------------------------------------------------------------
// For wide batches and matrices with many entries per operand row the gathers are served from
// LDS instead of the L2, and the results stay in registers until they are complete.  A
// work-group of 16 waves owns a range of at most kStageRangeRows rows and kStageCols columns of
// the batch; a row of 16 lanes owns up to kStageJ of those rows, a float4 of the batch per lane
// and row.  The work-group walks the column blocks of the matrix in order: it copies the
// block's kStageRows operand rows (128 KiB) into LDS, then every lane row serves, out of that
// copy, the segment (row, block) of each of its rows.  A segment's (column, weight) pairs are
// loaded one per lane, a block ahead, and reach the other lanes of the row through DPP row
// broadcasts, so the only LDS traffic is the gather itself.  Bias, ReLU and the output mask are
// applied when the rows are stored, once, after the last block.  A row marked kStageQuad is
// shared by the four lane rows of a wave, a quarter of each segment each, and their four results
// are added in a fixed order before the store.  Every output element is summed in one order.
// With a partial plan (RowBlocks::staged_partial) the kernel serves the long rows only and a
// second launch, the packed kernel, the others.
constexpr int kStageWaves = kWavesPerBlock;
// LDS byte offset of a zero-filled row behind the staged block: where a lane with no entry of its own
// gathers from, so that it multiplies its weight 0 with 0 and not with an operand row that the
// output row does not reference (which may hold Inf or NaN).
constexpr int kStageZeroRow = kStageRows * kStageCols * 4;
constexpr int kStageRounds = 2;  // rounds in which a block is copied into LDS (8 / kStageRounds float4 per thread and round)
static_assert(kStageRangeRows == kStageWaves * 4 * kStageJ && kStageJ <= 16, "a lane row owns kStageJ rows of the range");

template <int... I, typename F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, I...>, F &&f)
{
    (f(std::integral_constant<int, I>{}), ...);
}

// lane i of every row of 16 lanes receives the value of the row's lane I
template <int I>
__device__ __forceinline__ int row_lane(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x150 + I, 0xF, 0xF, true); }
// lane i of every row of 16 lanes receives the value of the row's lane (i + K) % 16
template <int K>
__device__ __forceinline__ int row_rotate_down(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x120 + (16 - K), 0xF, 0xF, true); }

template <int I>
__device__ __forceinline__ void staged_step(const char *lds, int off, float w, float4 &acc)
{
    const int o = row_lane<I>(off);
    const float wi = __builtin_bit_cast(float, row_lane<I>(__builtin_bit_cast(int, w)));
    const float4 x = *reinterpret_cast<const float4 *>(lds + o);
    acc.x = fmaf(wi, x.x, acc.x);
    acc.y = fmaf(wi, x.y, acc.y);
    acc.z = fmaf(wi, x.z, acc.z);
    acc.w = fmaf(wi, x.w, acc.w);
}
// the first N entries of every lane row, in entry order; afterwards entry N sits in lane 0
template <int N>
__device__ __forceinline__ void staged_pass(const char *lds, int &off, float &w, float4 &acc)
{
    staged_step<0>(lds, off, w, acc);
    if constexpr (N > 1) staged_step<1>(lds, off, w, acc);
    if constexpr (N > 2) { staged_step<2>(lds, off, w, acc); staged_step<3>(lds, off, w, acc); }
    if constexpr (N > 4) {
        staged_step<4>(lds, off, w, acc); staged_step<5>(lds, off, w, acc);
        staged_step<6>(lds, off, w, acc); staged_step<7>(lds, off, w, acc);
    }
    if constexpr (N > 8) {
        staged_step<8>(lds, off, w, acc); staged_step<9>(lds, off, w, acc);
        staged_step<10>(lds, off, w, acc); staged_step<11>(lds, off, w, acc);
        staged_step<12>(lds, off, w, acc); staged_step<13>(lds, off, w, acc);
        staged_step<14>(lds, off, w, acc); staged_step<15>(lds, off, w, acc);
    }
    if constexpr (N < 16) {
        off = row_rotate_down<N>(off);
        w = __builtin_bit_cast(float, row_rotate_down<N>(__builtin_bit_cast(int, w)));
    }
}

// One segment per lane row: entries [p0, p0 + len) of one of the lane row's rows, the first 16
// of them already in (off, w) as LDS byte offset and weight; adds the products to acc.
__device__ __forceinline__ void staged_segment(const SpmmArgs &a, const char *lds, int cb0, int lig, int p0, int len,
                                               int off, float w, float4 &acc)
{
    // the longest of the four segments sets the number of steps; shorter ones ride along with weight 0
    const int l01 = max(__builtin_amdgcn_readlane(len, 0), __builtin_amdgcn_readlane(len, 16));
    const int l23 = max(__builtin_amdgcn_readlane(len, 32), __builtin_amdgcn_readlane(len, 48));
    const int longest = max(l01, l23);
    auto passes = [&](int n) {
        if (n >= 16) {
            staged_pass<16>(lds, off, w, acc);
        } else {
            if (n & 8) staged_pass<8>(lds, off, w, acc);
            if (n & 4) staged_pass<4>(lds, off, w, acc);
            if (n & 2) staged_pass<2>(lds, off, w, acc);
            if (n & 1) staged_pass<1>(lds, off, w, acc);
        }
    };
    if (longest <= 16) {
        // no load in this path, hence no wait: whatever the kernel has in flight stays in flight
        passes(longest);
        return;
    }
    // long segments: kStageDepth chunks of 16 entries are served while the next kStageDepth travel
    constexpr int kStageDepth = 2;
    int o[kStageDepth], o2[kStageDepth];
    float ww[kStageDepth], w2[kStageDepth];
    auto load_chunk = [&](int first, int &oo, float &wo) {
        oo = kStageZeroRow;
        wo = 0.f;
        if (first < longest) {  // uniform
            const int e = first + lig;
            if (e < len) {
                oo = (a.indices[p0 + e] - cb0) * (kStageCols * 4);
                wo = a.values[p0 + e];
            }
        }
    };
    o[0] = off;
    ww[0] = w;
#pragma unroll
    for (int k = 1; k < kStageDepth; ++k) load_chunk(16 * k, o[k], ww[k]);
    for (int c = 0; c < longest; c += 16 * kStageDepth) {
#pragma unroll
        for (int k = 0; k < kStageDepth; ++k) load_chunk(c + 16 * (kStageDepth + k), o2[k], w2[k]);
#pragma unroll
        for (int k = 0; k < kStageDepth; ++k) {
            const int n = longest - c - 16 * k;
            if (n > 0) {
                off = o[k];
                w = ww[k];
                passes(n);
            }
        }
#pragma unroll
        for (int k = 0; k < kStageDepth; ++k) {
            o[k] = o2[k];
            ww[k] = w2[k];
        }
    }
}

// Work-group barrier that orders LDS accesses only: global loads issued before it stay in flight
// across it (the staged kernel has no global data that one wave writes and another reads).
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Work-groups of one column tile stage the same operand rows: where there are eight tiles or
// more, each of eight tiles gets an XCD (consecutive work-groups go to consecutive XCDs) and its
// L2 to itself; left-over tiles are dealt out plainly.
__device__ __forceinline__ void staged_ids(int n_ranges, int n_tiles, int &range, int &tile)
{
    const int aligned = (n_tiles >> 3) * 8 * n_ranges;
    if (static_cast<int>(blockIdx.x) < aligned) {
        const int slot = blockIdx.x >> 3;
        range = slot % n_ranges;
        tile = (slot / n_ranges) * 8 + (blockIdx.x & 7);
    } else {
        const int rest = blockIdx.x - aligned, left = n_tiles & 7;
        tile = (n_tiles >> 3) * 8 + rest % left;
        range = rest / left;
    }
}

template <bool XMASK>
__global__ __launch_bounds__(kStageWaves * kWave) void spmm_staged_kernel(const SpmmArgs a, const int n_tiles)
{
    __shared__ float4 stage[kStageRows * kStageCols / 4 + kStageCols / 4];  // the block, then one row of zeros
    const int n_ranges = a.blocks.staged_ranges;
    int range, tile;
    staged_ids(n_ranges, n_tiles, range, tile);
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const int lrow = lane >> 4, lig = lane & 15;
    const int col = tile * kStageCols + lig * 4;
    const bool col_on = col < a.batch;
    const char *lds = reinterpret_cast<const char *>(stage) + lig * 16;
    if (threadIdx.x < kStageCols / 4) stage[kStageRows * kStageCols / 4 + threadIdx.x] = make_float4(0.f, 0.f, 0.f, 0.f);  // (visible after the first barrier)
    const int n_cb = a.blocks.staged_cblocks;
    // The lane row's J-th row sits in slot (J * 16 + wave) * 4 + lrow of the range; lane J of the
    // lane row keeps that slot's row id and, block after block, its segment bounds.
    const int my_slot = ((lig & (kStageJ - 1)) * kStageWaves + wv) * 4 + lrow;
    const int my_row = a.blocks.staged_rows[range * kStageRangeRows + my_slot];
    const int n_j = a.blocks.staged_groups[range];  // rows of the range / 64, rounded up
    const int32_t *ends = a.blocks.staged_ends + static_cast<int64_t>(range) * (n_cb + 1) * kStageRangeRows + my_slot;
    constexpr auto all_j = std::make_integer_sequence<int, kStageJ>{};
    float4 acc[kStageJ];
    static_for(all_j, [&](auto jc) { acc[decltype(jc)::value] = make_float4(0.f, 0.f, 0.f, 0.f); });
    // first 16 entries of the segments of column block blk; e_lo, e_hi: the lane's bounds blk and blk + 1
    // the lane row's J-th segment in a block whose bounds lane J holds in e_lo, e_hi: the slot's
    // entries, or this lane row's quarter of them where the four lane rows share a long row
    auto segment = [&](auto jc, int e_lo, int e_hi, int &p0, int &len) {
        constexpr int j = decltype(jc)::value;
        p0 = row_lane<j>(e_lo);
        len = row_lane<j>(e_hi) - p0;
        if (row_lane<j>(my_row) & kStageQuad) {
            const int from = (len * lrow) >> 2;
            p0 += from;
            len = ((len * (lrow + 1)) >> 2) - from;
        }
    };
    auto first_chunks = [&](int blk, int e_lo, int e_hi, int (&off)[kStageJ], float (&w)[kStageJ]) {
        static_for(all_j, [&](auto jc) {
            constexpr int j = decltype(jc)::value;
            off[j] = kStageZeroRow;
            w[j] = 0.f;
            if (j < n_j) {
                int p0, len;
                segment(jc, e_lo, e_hi, p0, len);
                if (lig < len) {
                    off[j] = (a.indices[p0 + lig] - blk * kStageRows) * (kStageCols * 4);
                    w[j] = a.values[p0 + lig];
                }
            }
        });
    };
    int e0 = ends[0], e1 = ends[kStageRangeRows];
    int e2 = n_cb >= 2 ? ends[2 * kStageRangeRows] : e1;
    int off_cur[kStageJ];
    float w_cur[kStageJ];
    first_chunks(0, e0, e1, off_cur, w_cur);
    for (int b = 0; b < n_cb; ++b) {
        const int cb0 = b * kStageRows;
        lds_barrier();  // the previous block's gathers are done
#pragma unroll
        for (int h = 0; h < kStageRounds; ++h) {
            constexpr int kHalf = kStageRows / (64 * kStageRounds);
            float4 v[kHalf];
#pragma unroll
            for (int i = 0; i < kHalf; ++i) {
                const int k = cb0 + (h * kHalf + i) * 64 + static_cast<int>(threadIdx.x >> 4);
                v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k < a.x_rows && col_on) {
                    v[i] = ld4(a.X + static_cast<int64_t>(k) * a.ldx + col);
                    if constexpr (XMASK) v[i] = keep_where_positive(v[i], ld4(a.XM + static_cast<int64_t>(k) * a.ldxm + col));
                }
            }
#pragma unroll
            for (int i = 0; i < kHalf; ++i) stage[((h * kHalf + i) * 64 + (threadIdx.x >> 4)) * 16 + lig] = v[i];
        }
        // the next block's first chunks travel while this block is served
        int off_next[kStageJ];
        float w_next[kStageJ];
        int e3 = e2;
        if (b + 1 < n_cb) {
            first_chunks(b + 1, e1, e2, off_next, w_next);
            if (b + 3 <= n_cb) e3 = ends[(b + 3) * kStageRangeRows];
        } else {
            static_for(all_j, [&](auto jc) { off_next[decltype(jc)::value] = kStageZeroRow; w_next[decltype(jc)::value] = 0.f; });
        }
        lds_barrier();
        static_for(all_j, [&](auto jc) {
            constexpr int j = decltype(jc)::value;
            if (j < n_j) {
                int p0, len;
                segment(jc, e0, e1, p0, len);
                staged_segment(a, lds, cb0, lig, p0, len, off_cur[j], w_cur[j], acc[j]);
            }
        });
        static_for(all_j, [&](auto jc) { off_cur[decltype(jc)::value] = off_next[decltype(jc)::value]; w_cur[decltype(jc)::value] = w_next[decltype(jc)::value]; });
        e0 = e1;
        e1 = e2;
        e2 = e3;
    }
    static_for(all_j, [&](auto jc) {
        constexpr int j = decltype(jc)::value;
        const int slot_row = row_lane<j>(my_row);
        const bool quad = slot_row >= 0 && (slot_row & kStageQuad);
        const int row = slot_row < 0 ? -1 : (slot_row & ~kStageQuad);
        if (j < n_j && __builtin_amdgcn_readfirstlane(quad)) {
            // the four lane rows hold a quarter of the row's sum each: (0 + 1) + (2 + 3), in every lane row
            acc[j].x += __shfl_xor(acc[j].x, 16); acc[j].y += __shfl_xor(acc[j].y, 16);
            acc[j].z += __shfl_xor(acc[j].z, 16); acc[j].w += __shfl_xor(acc[j].w, 16);
            acc[j].x += __shfl_xor(acc[j].x, 32); acc[j].y += __shfl_xor(acc[j].y, 32);
            acc[j].z += __shfl_xor(acc[j].z, 32); acc[j].w += __shfl_xor(acc[j].w, 32);
        }
        if (j < n_j && row >= 0 && col_on && (!quad || lrow == 0)) {
            const float bb = a.bias ? a.bias[row] : 0.f;
            float4 r = make_float4(acc[j].x + bb, acc[j].y + bb, acc[j].z + bb, acc[j].w + bb);
            if (a.relu) r = make_float4(r.x > 0.f ? r.x : 0.f, r.y > 0.f ? r.y : 0.f, r.z > 0.f ? r.z : 0.f, r.w > 0.f ? r.w : 0.f);
            if (a.YM) r = keep_where_positive(r, ld4(a.YM + static_cast<int64_t>(row) * a.ldym + col));
            st4(a.Y + static_cast<int64_t>(row) * a.ldy + col, r);
        }
    });
}

// Second pass for huge rows: adds the partial rows of a row's work-groups in share order, then
// bias, ReLU and the optional output mask.  One thread per column.
__global__ __launch_bounds__(256) void spmm_finish_kernel(const SpmmArgs a)
{
    const int4 h = a.blocks.huge_rows[blockIdx.x];
    const int c = blockIdx.y * 256 + threadIdx.x;
    if (c >= a.batch) return;
    const float *sr = a.scratch + static_cast<int64_t>(h.y) * a.scratch_ld + c;
    float y = 0.f;
    int q = 0;
    for (; q + 8 <= h.z; q += 8) {  // eight loads in flight, added in share order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = sr[static_cast<int64_t>(q + u) * a.scratch_ld];
#pragma unroll
        for (int u = 0; u < 8; ++u) y += v[u];
    }
    for (; q < h.z; ++q) y += sr[static_cast<int64_t>(q) * a.scratch_ld];
    y += a.bias ? a.bias[h.x] : 0.f;
    if (a.relu) y = y > 0.f ? y : 0.f;
    if (a.YM) y = keep_where_positive(y, a.YM[static_cast<int64_t>(h.x) * a.ldym + c]);
    a.Y[static_cast<int64_t>(h.x) * a.ldy + c] = y;
}

// ---------------------------------------------------------------------------------------
// SDDMM.  The row of dZ stays in registers; the wave is cut into 64/G groups of G lanes, each
// group computing the dot product of one stored entry at a time (lanes along the batch, 4
// columns per lane and tile, NV tiles: G*4*NV >= batch), reduced inside the group with DPP
// moves.  Results of up to 64 consecutive entries are collected one per lane, so the store of
// g -- or the fused momentum step on values/velocity -- is a coalesced access.
// EXACT4: batch is a multiple of 4 (no column tail inside a 4-wide access).
// Lanes whose columns lie beyond the batch hold dZ = 0 and re-read columns 0..3 of the row.
// ---------------------------------------------------------------------------------------
// By-product carried by an SDDMM launch: the mean of the per-column losses the head kernel left.
__device__ __forceinline__ void mean_loss_task(const SddmmArgs &a, int block)
{
    if (!a.loss_cols || block != 0 || wave_in_block() != 0) return;  // wave-uniform
    const int lane = threadIdx.x & (kWave - 1);
    float s = 0.f;
    for (int c = lane; c < a.loss_n; c += kWave) s += a.loss_cols[c];
    s = group_sum<kWave>(s);
    if (lane == 0) *a.loss_out = s / static_cast<float>(a.loss_n);
}

// One pass of the SDDMM over U stored entries per group: every index move, then every gather,
// then the dot products and their reductions.  Straight-line, so that all U*NV gathers stay in
// flight (see grouped_pass).  Group `grp` works on slot it*NG+grp of the chunk in iteration it;
// that slot's row offset sits in lane grp*G+it, and its result is kept by the lane with lig == it.
template <int G, int NV, bool EXACT4, int U>
__device__ __forceinline__ void sddmm_pass(gmem_ptr Xg, int it0, int my_ro, const uint32_t (&off)[NV],
                                           const float4 (&dz)[NV], int batch, float &res)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int lig = lane % G;
    uint32_t ro[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        if constexpr (G == kWave)
            ro[u] = static_cast<uint32_t>(__builtin_amdgcn_readlane(my_ro, it0 + u));
        else
            ro[u] = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(((lane / G) * G + it0 + u) * 4, my_ro));
    }
    float4 x[U][NV];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int t = 0; t < NV; ++t) x[u][t] = gload<float4>(Xg, ro[u] + off[t]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        float part = 0.f;
#pragma unroll
        for (int t = 0; t < NV; ++t) {
            if constexpr (!EXACT4) {
                // padding columns inside the access may hold anything, also NaN: drop them
                const int c = (t * G + lig) * 4;
                if (c + 1 >= batch) x[u][t].y = 0.f;
                if (c + 2 >= batch) x[u][t].z = 0.f;
                if (c + 3 >= batch) x[u][t].w = 0.f;
                if (c >= batch) x[u][t].x = 0.f;
            }
            part = fmaf(dz[t].x, x[u][t].x, part);
            part = fmaf(dz[t].y, x[u][t].y, part);
            part = fmaf(dz[t].z, x[u][t].z, part);
            part = fmaf(dz[t].w, x[u][t].w, part);
        }
        part = group_sum<G>(part);
        if (lig == it0 + u) res = part;
    }
}

template <int G, int NV, bool EXACT4>
__device__ __forceinline__ void sddmm_body(const SddmmArgs &a, const int block)
{
    constexpr int NG = kWave / G;
    constexpr int UI = NV >= 4 ? 2 : (NV == 2 ? 4 : 8);   // 32 registers of gathered data: two 16-wave work-groups fit a compute unit
    const int lane = threadIdx.x & (kWave - 1);
    mean_loss_task(a, block);
    const WaveTask task = wave_task(a.blocks, block);
    if (task.row < 0) return;
    const int row = task.row;
    const int grp = lane / G;
    const int lig = lane % G;

    float4 dz[NV];
    uint32_t off[NV];
    {
        const float *zr = a.dZ + static_cast<int64_t>(row) * a.lddz;
        const float *zm = a.ZM ? a.ZM + static_cast<int64_t>(row) * a.ldzm : nullptr;
#pragma unroll
        for (int t = 0; t < NV; ++t) {
            const int c = (t * G + lig) * 4;
            dz[t] = make_float4(0.f, 0.f, 0.f, 0.f);
            off[t] = 0u;
            if (c < a.batch) {
                off[t] = static_cast<uint32_t>(c) * 4u;
                dz[t] = ld4(zr + c);
                if (zm) dz[t] = keep_where_positive(dz[t], ld4(zm + c));
                if constexpr (!EXACT4) {
                    if (c + 1 >= a.batch) dz[t].y = 0.f;
                    if (c + 2 >= a.batch) dz[t].z = 0.f;
                    if (c + 3 >= a.batch) dz[t].w = 0.f;
                }
            }
        }
    }

    if (task.lead && (a.db || (a.fused && a.bias))) {
        float s = 0.f;
#pragma unroll
        for (int t = 0; t < NV; ++t) s += (dz[t].x + dz[t].y) + (dz[t].z + dz[t].w);
        s = group_sum<G>(s);
        if (lane == 0) {
            if (a.db) a.db[row] = s;
            if (a.fused && a.bias) {
                float w = a.bias[row], v = a.bias_velocity[row];
                momentum_step(w, v, s, a.lr, a.momentum, a.nesterov);
                a.bias[row] = w;
                a.bias_velocity[row] = v;
            }
        }
    }
    if (a.skip_products) return;

    const int s0 = task.s0;
    const int s1 = task.s1;
    const uint32_t ldxb = static_cast<uint32_t>(a.ldx) * 4u;
    const gmem_ptr Xg = as_gmem(a.X);
    const int q_mine = lig * NG + grp;  // slot of this lane inside a chunk of 64 entries

    for (int pc = s0; pc < s1; pc += kWave) {
        const int n = min(kWave, s1 - pc);
        const bool mine = q_mine < n;
        // lanes whose slot lies past the chunk's end work on its first entry and store nothing
        const int p = pc + (mine ? q_mine : 0);
        const int my_j = a.indices[p];
        // operands of the fused update travel together with the column index
        float w_old = 0.f, v_old = 0.f;
        int mirror_pos = 0;
        if (a.fused) {
            w_old = a.values[p];
            v_old = a.velocity[p];
            if (a.values_t) mirror_pos = a.pos_t[p];
        }
        const int my_ro = static_cast<int>(static_cast<uint32_t>(my_j) * ldxb);
        const int iters = (n + NG - 1) / NG;
        float res = 0.f;
        int it = 0;
        for (; it + UI <= iters; it += UI) sddmm_pass<G, NV, EXACT4, UI>(Xg, it, my_ro, off, dz, a.batch, res);
        if constexpr (UI >= 8)
            if (it + 4 <= iters) { sddmm_pass<G, NV, EXACT4, 4>(Xg, it, my_ro, off, dz, a.batch, res); it += 4; }
        if constexpr (UI >= 4)
            if (it + 2 <= iters) { sddmm_pass<G, NV, EXACT4, 2>(Xg, it, my_ro, off, dz, a.batch, res); it += 2; }
        if (it < iters) sddmm_pass<G, NV, EXACT4, 1>(Xg, it, my_ro, off, dz, a.batch, res);
        if (mine) {
            if (a.g) a.g[p] = res;
            if (a.fused) {
                momentum_step(w_old, v_old, res, a.lr, a.momentum, a.nesterov);
                a.values[p] = w_old;
                a.velocity[p] = v_old;
                if (a.values_t) a.values_t[mirror_pos] = w_old;
                if (a.dense) a.dense[static_cast<int64_t>(row) * a.dense_ld + my_j] = w_old;
            }
        }
    }
}

template <int G, int NV, bool EXACT4>
__global__ __launch_bounds__(kBlock) void sddmm_kernel(const SddmmArgs a)
{
    sddmm_body<G, NV, EXACT4>(a, blockIdx.x);
}

// Column-tiled SDDMM for operands X that no L2 holds: tile t covers columns [t*W, t*W + W), W =
// G*4*NV; a work-group computes the partial products of its rows over one tile, as sddmm_body on
// the sub-matrices that start at the tile's first column, and stores them (and the partial row
// sums of dZ) in the tile's slice of the partial buffer.  Work-group ids are decoded XCD-first as
// in spmm_tiled_kernel, so an operand tile stays in one L2 while every entry gathers from it.
template <int G, int NV, bool EXACT4>
__global__ __launch_bounds__(kBlock) void sddmm_tiled_kernel(const SddmmArgs a, const int n_tiles, const int spread)
{
    const int nrb = a.blocks.n_blocks;
    int tile, rb;
    if (spread) {
        const int xcd = blockIdx.x & 7, k = blockIdx.x >> 3;
        tile = (k / nrb) * 8 + xcd;
        rb = k % nrb;
    } else {
        tile = blockIdx.x / nrb;
        rb = blockIdx.x % nrb;
    }
    if (tile >= n_tiles) return;
    const int col0 = tile * (G * 4 * NV);
    SddmmArgs t = a;
    t.dZ = a.dZ + col0;
    t.X = a.X + col0;
    if (a.ZM) t.ZM = a.ZM + col0;
    t.batch = min(G * 4 * NV, a.batch - col0);
    t.fused = 0;
    t.g = a.partial + static_cast<int64_t>(tile) * a.partial_stride;
    t.db = t.g + a.partial_db_at;
    if (tile != 0) t.loss_cols = nullptr;
    sddmm_body<G, NV, EXACT4>(t, rb);
}

// ---- staged SDDMM --------------------------------------------------------------------------
// The SDDMM on the staged product's plan: same ranges, tiles, column blocks and LDS copy of the
// operand; a lane row keeps the tile's 64 columns of dZ of its 8 rows in registers instead of
// results.  An entry's product is a dot product over the lane row: each lane multiplies its four
// columns, and 16 entries at a time are summed across the 16 lanes by a transposing butterfly
// (45 instructions per 16 entries instead of 6 per entry), after which lane i holds entry i's sum
// and the lane row stores 16 consecutive partial products.  Partial products and partial row
// sums of dZ go to the tile's slice of the partial buffer; sddmm_finish_kernel adds the tiles.

// d[i] is this lane's share of value i; returns, in lane i of every row of 16 lanes, the sum of
// the 16 lanes' d[i].  Fixed pairing: lane l with l^8, l^7, l^2, l^1 in turn.
__device__ __forceinline__ float row16_transpose_sum(const float (&d)[16], int lig)
{
    // every lane has a partner in these four moves: no lane keeps the old value
    auto from = [](auto ctrl, float x) {
        return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value, 0xF, 0xF, true));
    };
    using ror8 = std::integral_constant<int, 0x128>;         // row_ror:8
    using half_mirror = std::integral_constant<int, 0x141>;  // row_half_mirror
    using xor2 = std::integral_constant<int, 0x4E>;          // quad_perm [2,3,0,1]
    using xor1 = std::integral_constant<int, 0xB1>;          // quad_perm [1,0,3,2]
    const bool b3 = lig & 8, b2 = lig & 4, b1 = lig & 2, b0 = lig & 1;
    float e[8], f[4], g[2];
#pragma unroll
    for (int k = 0; k < 8; ++k) e[k] = (b3 ? d[k + 8] : d[k]) + from(ror8{}, b3 ? d[k] : d[k + 8]);
#pragma unroll
    for (int k = 0; k < 4; ++k) f[k] = (b2 ? e[k + 4] : e[k]) + from(half_mirror{}, b2 ? e[k] : e[k + 4]);
#pragma unroll
    for (int k = 0; k < 2; ++k) g[k] = (b1 ? f[k + 2] : f[k]) + from(xor2{}, b1 ? f[k] : f[k + 2]);
    return (b0 ? g[1] : g[0]) + from(xor1{}, b0 ? g[0] : g[1]);
}

template <int I>
__device__ __forceinline__ float staged_dot(const char *lds, int off, const float4 &z)
{
    const float4 x = *reinterpret_cast<const float4 *>(lds + row_lane<I>(off));
    return fmaf(x.w, z.w, fmaf(x.z, z.z, fmaf(x.y, z.y, x.x * z.x)));
}

// Up to 16 entries of every lane row (n: the most any of the four has left, uniform): products of
// the entries whose LDS byte offsets the lanes hold in off, stored by lane i for entry first + i.
__device__ __forceinline__ void sddmm_staged_chunk(const char *lds, int off, const float4 &z, int n, int lig,
                                                   int first, int end, float *gp)
{
    float d[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) d[i] = 0.f;
    d[0] = staged_dot<0>(lds, off, z); d[1] = staged_dot<1>(lds, off, z);
    d[2] = staged_dot<2>(lds, off, z); d[3] = staged_dot<3>(lds, off, z);
    if (n > 4) {
        d[4] = staged_dot<4>(lds, off, z); d[5] = staged_dot<5>(lds, off, z);
        d[6] = staged_dot<6>(lds, off, z); d[7] = staged_dot<7>(lds, off, z);
    }
    if (n > 8) {
        d[8] = staged_dot<8>(lds, off, z); d[9] = staged_dot<9>(lds, off, z);
        d[10] = staged_dot<10>(lds, off, z); d[11] = staged_dot<11>(lds, off, z);
    }
    if (n > 12) {
        d[12] = staged_dot<12>(lds, off, z); d[13] = staged_dot<13>(lds, off, z);
        d[14] = staged_dot<14>(lds, off, z); d[15] = staged_dot<15>(lds, off, z);
    }
    const float sum = row16_transpose_sum(d, lig);
    if (first + lig < end) gp[first + lig] = sum;
}

__device__ __forceinline__ void sddmm_staged_segment(const SddmmArgs &a, const char *lds, int cb0, int lig, int p0, int len,
                                                     int off, const float4 &z, float *gp)
{
    const int l01 = max(__builtin_amdgcn_readlane(len, 0), __builtin_amdgcn_readlane(len, 16));
    const int l23 = max(__builtin_amdgcn_readlane(len, 32), __builtin_amdgcn_readlane(len, 48));
    const int longest = max(l01, l23);
    if (longest <= 16) {
        if (longest > 0) sddmm_staged_chunk(lds, off, z, longest, lig, p0, p0 + len, gp);
        return;
    }
    constexpr int kDepth = 2;  // chunks of 16 entries served while the next kDepth travel
    int o[kDepth], o2[kDepth];
    auto load_chunk = [&](int first, int &oo) {
        oo = 0;
        if (first < longest && first + lig < len) oo = (a.indices[p0 + first + lig] - cb0) * (kStageCols * 4);
    };
    o[0] = off;
#pragma unroll
    for (int k = 1; k < kDepth; ++k) load_chunk(16 * k, o[k]);
    for (int c = 0; c < longest; c += 16 * kDepth) {
#pragma unroll
        for (int k = 0; k < kDepth; ++k) load_chunk(c + 16 * (kDepth + k), o2[k]);
#pragma unroll
        for (int k = 0; k < kDepth; ++k) {
            const int n = longest - c - 16 * k;
            if (n > 0) sddmm_staged_chunk(lds, o[k], z, n, lig, p0 + c + 16 * k, p0 + len, gp);
        }
#pragma unroll
        for (int k = 0; k < kDepth; ++k) o[k] = o2[k];
    }
}

__global__ __launch_bounds__(kStageWaves * kWave) void sddmm_staged_kernel(const SddmmArgs a, const int n_tiles)
{
    __shared__ float4 stage[kStageRows * kStageCols / 4];
    const int n_ranges = a.blocks.staged_ranges;
    int range, tile;
    staged_ids(n_ranges, n_tiles, range, tile);
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const int lrow = lane >> 4, lig = lane & 15;
    const int col = tile * kStageCols + lig * 4;
    const bool col_on = col < a.batch;
    const char *lds = reinterpret_cast<const char *>(stage) + lig * 16;
    const int n_cb = a.blocks.staged_cblocks;
    const int my_slot = ((lig & (kStageJ - 1)) * kStageWaves + wv) * 4 + lrow;
    const int my_row = a.blocks.staged_rows[range * kStageRangeRows + my_slot];
    const int n_j = a.blocks.staged_groups[range];
    const int32_t *ends = a.blocks.staged_ends + static_cast<int64_t>(range) * (n_cb + 1) * kStageRangeRows + my_slot;
    float *gp = a.partial + static_cast<int64_t>(tile) * a.partial_stride;
    constexpr auto all_j = std::make_integer_sequence<int, kStageJ>{};
    // the tile's columns of dZ for the lane row's rows, and their sums (the tile's share of db)
    float4 z[kStageJ];
    static_for(all_j, [&](auto jc) {
        constexpr int j = decltype(jc)::value;
        z[j] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (j < n_j) {
            const int slot_row = row_lane<j>(my_row);
            const int row = slot_row < 0 ? -1 : (slot_row & ~kStageQuad);
            if (row >= 0 && col_on) {
                z[j] = ld4(a.dZ + static_cast<int64_t>(row) * a.lddz + col);
                if (a.ZM) z[j] = keep_where_positive(z[j], ld4(a.ZM + static_cast<int64_t>(row) * a.ldzm + col));
            }
            const float sum = row16_sum((z[j].x + z[j].y) + (z[j].z + z[j].w));
            // (the four lane rows of a split row hold the same dZ: the first one reports it)
            if (row >= 0 && lig == 0 && (!(slot_row & kStageQuad) || lrow == 0)) gp[a.partial_db_at + row] = sum;
        }
    });
    auto segment = [&](auto jc, int e_lo, int e_hi, int &p0, int &len) {  // as in spmm_staged_kernel
        constexpr int j = decltype(jc)::value;
        p0 = row_lane<j>(e_lo);
        len = row_lane<j>(e_hi) - p0;
        if (row_lane<j>(my_row) & kStageQuad) {
            const int from = (len * lrow) >> 2;
            p0 += from;
            len = ((len * (lrow + 1)) >> 2) - from;
        }
    };
    auto first_chunks = [&](int blk, int e_lo, int e_hi, int (&off)[kStageJ]) {
        static_for(all_j, [&](auto jc) {
            constexpr int j = decltype(jc)::value;
            off[j] = 0;
            if (j < n_j) {
                int p0, len;
                segment(jc, e_lo, e_hi, p0, len);
                if (lig < len) off[j] = (a.indices[p0 + lig] - blk * kStageRows) * (kStageCols * 4);
            }
        });
    };
    int e0 = ends[0], e1 = ends[kStageRangeRows];
    int e2 = n_cb >= 2 ? ends[2 * kStageRangeRows] : e1;
    int off_cur[kStageJ];
    first_chunks(0, e0, e1, off_cur);
    for (int b = 0; b < n_cb; ++b) {
        const int cb0 = b * kStageRows;
        lds_barrier();  // the previous block's gathers are done
#pragma unroll
        for (int h = 0; h < kStageRounds; ++h) {
            constexpr int kHalf = kStageRows / (64 * kStageRounds);
            float4 v[kHalf];
#pragma unroll
            for (int i = 0; i < kHalf; ++i) {
                const int k = cb0 + (h * kHalf + i) * 64 + static_cast<int>(threadIdx.x >> 4);
                v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (k < a.x_rows && col_on) v[i] = ld4(a.X + static_cast<int64_t>(k) * a.ldx + col);
            }
#pragma unroll
            for (int i = 0; i < kHalf; ++i) stage[((h * kHalf + i) * 64 + (threadIdx.x >> 4)) * 16 + lig] = v[i];
        }
        int off_next[kStageJ];
        int e3 = e2;
        if (b + 1 < n_cb) {
            first_chunks(b + 1, e1, e2, off_next);
            if (b + 3 <= n_cb) e3 = ends[(b + 3) * kStageRangeRows];
        } else {
            static_for(all_j, [&](auto jc) { off_next[decltype(jc)::value] = 0; });
        }
        lds_barrier();
        static_for(all_j, [&](auto jc) {
            constexpr int j = decltype(jc)::value;
            if (j < n_j) {
                int p0, len;
                segment(jc, e0, e1, p0, len);
                sddmm_staged_segment(a, lds, cb0, lig, p0, len, off_cur[j], z[j], gp);
            }
        });
        static_for(all_j, [&](auto jc) { off_cur[decltype(jc)::value] = off_next[decltype(jc)::value]; });
        e0 = e1;
        e1 = e2;
        e2 = e3;
    }
}

// SDDMM of a full matrix of few rows (every entry stored, rows <= kFullMaxRows): dZ, a few rows,
// is copied into LDS once per work-group and X is streamed once, a wave per row of X: the lane
// multiplies its columns of the X row with the same columns of every dZ row, the row's `rows`
// products are summed over the wave by the transposing butterfly, and lane i stores (or applies the
// momentum step to) entry (i, row of X).  The first work-group also sums the rows of dZ for db.
// WITH_T: the layer's transposed product in the same pass -- row j of W^T is column j of the full matrix,
// the very entries this wave updates, and its result is masked by the row of X the wave holds:
//     dX[j, :] = (sum_i W(i, j) dZ[i, :]) * [X[j, :] > 0],  i ascending, the weights of the step's start
// (read before the update; no other wave touches column j).  X is read once for both.
template <bool WITH_T>
__global__ __launch_bounds__(kBlock) void full_sddmm_kernel(const SddmmArgs a, const int n_chunks, float *__restrict__ dX, const int lddx)
{
    extern __shared__ float4 dz_s[];  // [rows][n_chunks][kWave]
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const int R = a.rows, K = a.x_rows;
    for (int idx = threadIdx.x; idx < R * n_chunks * kWave; idx += kBlock) {
        const int i = idx / (n_chunks * kWave), c4 = idx % (n_chunks * kWave);
        float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c4 * 4 < a.batch) {
            v = ld4(a.dZ + static_cast<int64_t>(i) * a.lddz + c4 * 4);
            if (a.ZM) v = keep_where_positive(v, ld4(a.ZM + static_cast<int64_t>(i) * a.ldzm + c4 * 4));
        }
        dz_s[idx] = v;
    }
    __syncthreads();
    mean_loss_task(a, blockIdx.x);
    if (blockIdx.x == 0 && wv < R && (a.db || (a.fused && a.bias))) {
        float sum = 0.f;
        for (int ch = 0; ch < n_chunks; ++ch) {
            const float4 z = dz_s[(wv * n_chunks + ch) * kWave + lane];
            sum += (z.x + z.y) + (z.z + z.w);
        }
        sum = group_sum<kWave>(sum);
        if (lane == 0) {
            if (a.db) a.db[wv] = sum;
            if (a.fused && a.bias) {
                float w = a.bias[wv], v = a.bias_velocity[wv];
                momentum_step(w, v, sum, a.lr, a.momentum, a.nesterov);
                a.bias[wv] = w;
                a.bias_velocity[wv] = v;
            }
        }
    }
    for (int j = blockIdx.x * kWavesPerBlock + wv; j < K; j += gridDim.x * kWavesPerBlock) {
        float d[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) d[i] = 0.f;
        const float *xr = a.X + static_cast<int64_t>(j) * a.ldx;
        float w_own = 0.f;  // lane i: W(i, j)
        float below = 0.f;  // the lane's share of the row sum of dX[j, :]
        if constexpr (WITH_T)
            if (lane < R) w_own = a.values[static_cast<int64_t>(lane) * K + j];
        for (int ch = 0; ch < n_chunks; ++ch) {
            const int col = (ch * kWave + lane) * 4;
            const float4 x = col < a.batch ? ld4(xr + col) : make_float4(0.f, 0.f, 0.f, 0.f);
            float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
            for (int i = 0; i < kFullMaxRows; ++i) {
                if (i < R) {  // uniform
                    const float4 z = dz_s[(i * n_chunks + ch) * kWave + lane];
                    d[i] = fmaf(x.w, z.w, fmaf(x.z, z.z, fmaf(x.y, z.y, fmaf(x.x, z.x, d[i]))));
                    if constexpr (WITH_T) {
                        const float wi = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, w_own), i));
                        t.x = fmaf(wi, z.x, t.x);
                        t.y = fmaf(wi, z.y, t.y);
                        t.z = fmaf(wi, z.z, t.z);
                        t.w = fmaf(wi, z.w, t.w);
                    }
                }
            }
            if constexpr (WITH_T) {
                const float4 o = keep_where_positive(t, x);  // (columns beyond the batch: x = 0, so o = 0)
                if (col < a.batch) st4(dX + static_cast<int64_t>(j) * lddx + col, o);  // (batch % 4 == 0)
                below += (o.x + o.y) + (o.z + o.w);
            }
        }
        if constexpr (WITH_T) {
            if (a.below_bias) {  // uniform
                below = group_sum<kWave>(below);
                if (lane == 0) {
                    float w = a.below_bias[j], v = a.below_bias_velocity[j];
                    momentum_step(w, v, below, a.lr, a.momentum, a.nesterov);
                    a.below_bias[j] = w;
                    a.below_bias_velocity[j] = v;
                }
            }
        }
        // lane i of each row of 16 lanes gets that row's sum of product i; then the four rows: (0 + 1) + (2 + 3)
        float g = row16_transpose_sum(d, lane & 15);
        g += __shfl_xor(g, 16);
        g += __shfl_xor(g, 32);
        if (lane < R) {
            const int64_t p = static_cast<int64_t>(lane) * K + j;
            if (a.g) a.g[p] = g;
            if (a.fused) {
                float w = WITH_T ? w_own : a.values[p], v = a.velocity[p];
                momentum_step(w, v, g, a.lr, a.momentum, a.nesterov);
                a.values[p] = w;
                a.velocity[p] = v;
                if (a.values_t) a.values_t[a.pos_t[p]] = w;
            }
        }
    }
}

// Second pass of the tiled SDDMM: adds the tiles' partial products in tile order, then stores the
// gradient or applies the fused momentum step (and the mirror scatter); the same for the biases.
__global__ __launch_bounds__(kEwBlock) void sddmm_finish_kernel(const SddmmArgs a, const int n_tiles)
{
    const int64_t stride = static_cast<int64_t>(blockDim.x) * gridDim.x;
    for (int64_t p = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; p < a.nnz; p += stride) {
        float g = 0.f;
        int t = 0;
        for (; t + 8 <= n_tiles; t += 8) {  // eight loads in flight, added in tile order
            float v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = a.partial[static_cast<int64_t>(t + u) * a.partial_stride + p];
#pragma unroll
            for (int u = 0; u < 8; ++u) g += v[u];
        }
        for (; t < n_tiles; ++t) g += a.partial[static_cast<int64_t>(t) * a.partial_stride + p];
        if (a.g) a.g[p] = g;
        if (a.fused) {
            float w = a.values[p], v = a.velocity[p];
            momentum_step(w, v, g, a.lr, a.momentum, a.nesterov);
            a.values[p] = w;
            a.velocity[p] = v;
            if (a.values_t) a.values_t[a.pos_t[p]] = w;
        }
    }
    if (!(a.db || (a.fused && a.bias))) return;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < a.rows; i += stride) {
        float s = 0.f;
        for (int t = 0; t < n_tiles; ++t) s += a.partial[static_cast<int64_t>(t) * a.partial_stride + a.partial_db_at + i];
        if (a.db) a.db[i] = s;
        if (a.fused && a.bias) {
            float w = a.bias[i], v = a.bias_velocity[i];
            momentum_step(w, v, s, a.lr, a.momentum, a.nesterov);
            a.bias[i] = w;
            a.bias_velocity[i] = v;
        }
    }
}

// ---- backward pass of a hidden layer in one gather stream --------------------------------------
// The transposed product dX = W^T dZ and the SDDMM g = (dZ X^T) on W's pattern gather the same
// rows: taken in the mirror's order (row j of W^T, its entries i ascending), stored entry (i, j)
// needs dZ[i, :] for both.  One kernel walks the mirror like spmm_body_packed (one mirror row per
// group of GS lanes, inside column tiles), gathers dZ[i, tile] once and uses it twice:
//     acc[j, tile]        += values_t[q] * dZ[i, tile]
//     partial[tile][q]     = <dZ[i, tile], X[j, tile]>        (X[j, tile] is held by the lane group)
// and stores dX[j, tile] = acc * [X[j, tile] > 0] (the ReLU derivative of the layer below, whose
// output X is).  The per-tile partial products, in mirror order, are added in tile order by
// backward_finish_kernel, which applies the momentum step through perm (mirror -> CSR position)
// and also forms the bias gradient (row sums of dZ).  Every mirror row must be short (packed).
constexpr int kBwdWaves = 4;  // waves per work-group: no sums across waves, and smaller groups schedule finer (measured on the wide MLP:
                              // 134 / 138 / 142 us with 4 / 8 / 16 waves; gather depth 4 instead of 8 and a register cap of 64 change nothing)

template <int U, int GS>
__device__ __forceinline__ void bwd_pass(gmem_ptr Zg, int src, int my_ro, float my_w, uint32_t off, const float4 &ax, int it0, int lig,
                                         float (&acc)[4], float &res)
{
    uint32_t ro[U];
    float w[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        ro[u] = static_cast<uint32_t>(__builtin_amdgcn_ds_bpermute(src + u * 4, my_ro));
        w[u] = __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute(src + u * 4, __builtin_bit_cast(int, my_w)));
    }
    float4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) x[u] = gload<float4>(Zg, ro[u] + off);
#pragma unroll
    for (int u = 0; u < U; ++u) {
        acc[0] = fmaf(w[u], x[u].x, acc[0]);
        acc[1] = fmaf(w[u], x[u].y, acc[1]);
        acc[2] = fmaf(w[u], x[u].z, acc[2]);
        acc[3] = fmaf(w[u], x[u].w, acc[3]);
        float part = fmaf(ax.w, x[u].w, fmaf(ax.z, x[u].z, fmaf(ax.y, x[u].y, ax.x * x[u].x)));
        part = group_sum<GS>(part);
        res = lig == it0 + u ? part : res;
    }
}

template <int GS>
__global__ __launch_bounds__(kBwdWaves * kWave) void backward_fused_kernel(const BackwardArgs a, const int n_tiles, const int spread,
                                                                          const int n_pack_blocks)
{
    int tile, rb;
    if (spread) {
        const int xcd = blockIdx.x & 7, k = blockIdx.x >> 3;
        tile = (k / n_pack_blocks) * 8 + xcd;
        rb = k % n_pack_blocks;
    } else {
        tile = blockIdx.x / n_pack_blocks;
        rb = blockIdx.x % n_pack_blocks;
    }
    if (tile >= n_tiles) return;
    constexpr int NE = kWave / GS;
    const int col0 = tile * GS * 4;
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const int grp = lane / GS;
    const int lig = lane % GS;
    const int col = col0 + lig * 4;
    const bool on = col < a.batch;  // (batch is a multiple of 4: a lane's four columns are all in or all out)
    const uint32_t off = static_cast<uint32_t>(on ? col : col0) * 4u;
    const uint32_t ldzb = static_cast<uint32_t>(a.lddz) * 4u;
    const gmem_ptr Zg = as_gmem(a.dZ);
    const int n_sets = (a.blocks.n_short + NE - 1) / NE;
    const int src0 = grp * GS * 4;
    const int n_waves = n_pack_blocks * kBwdWaves;
    const int first_set = rb * kBwdWaves + wv;
    if (first_set >= n_sets) return;  // wave-uniform
    float *gp = a.partial + static_cast<int64_t>(tile) * a.partial_stride;

    auto fetch = [&](int s0, int len, int base, int &j, float &w) {  // as in spmm_body_packed
        const int e = base + lig;
        const bool ok = e < len;
        const int p = len > 0 ? s0 + (ok ? e : 0) : 0;
        j = a.indices[p];
        w = a.values[p];
        w = ok ? w : 0.f;
    };

    for (int set = first_set; set < n_sets; set += n_waves) {
        const int4 d = a.blocks.short_rows[set * NE + grp];  // the table is padded to whole sets
        const int row = d.x, s0 = d.y, len = d.z;
        const int maxlen = __builtin_amdgcn_readfirstlane(len);  // group 0 holds the set's longest row
        // the group's row of X: the second operand of its entries' products, and the mask of its result;
        // lanes beyond the batch hold zeros, so that the columns they re-read add nothing to a product
        float4 ax = make_float4(0.f, 0.f, 0.f, 0.f);
        if (row >= 0 && on) ax = ld4(a.X + static_cast<int64_t>(row) * a.ldx + col);
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
        int cur_j;
        float cur_w;
        fetch(s0, len, 0, cur_j, cur_w);
        for (int base = 0; base < maxlen; base += GS) {
            int next_j = 0;
            float next_w = 0.f;
            if (base + GS < maxlen) fetch(s0, len, base + GS, next_j, next_w);  // wave-uniform: one chunk ahead
            const int my_ro = static_cast<int>(static_cast<uint32_t>(cur_j) * ldzb);
            const int steps = min(GS, maxlen - base);
            float res = 0.f;
            int src = src0;
            int u0 = 0;
            for (; u0 + 8 <= steps; u0 += 8, src += 32) bwd_pass<8, GS>(Zg, src, my_ro, cur_w, off, ax, u0, lig, acc, res);
            if (u0 + 4 <= steps) {
                bwd_pass<4, GS>(Zg, src, my_ro, cur_w, off, ax, u0, lig, acc, res);
                u0 += 4; src += 16;
            }
            if (u0 + 2 <= steps) {
                bwd_pass<2, GS>(Zg, src, my_ro, cur_w, off, ax, u0, lig, acc, res);
                u0 += 2; src += 8;
            }
            if (u0 < steps) bwd_pass<1, GS>(Zg, src, my_ro, cur_w, off, ax, u0, lig, acc, res);
            if (row >= 0 && base + lig < len) gp[s0 + base + lig] = res;  // GS consecutive entries of the row: one coalesced store
            cur_j = next_j;
            cur_w = next_w;
        }
        if (row < 0 || !on) continue;
        float4 y = len > 0 ? make_float4(acc[0], acc[1], acc[2], acc[3]) : make_float4(0.f, 0.f, 0.f, 0.f);
        if (a.mask) y = keep_where_positive(y, ax);
        st4(a.dX + static_cast<int64_t>(row) * a.lddx + col, y);
    }
}

// Second pass: work-groups [0, n_entry_blocks) add the tiles' partial products of mirror entry q in tile
// order and apply the momentum step to the entry's CSR position perm[q] (or store the gradient there);
// the remaining work-groups, a wave per row of W, sum the rows of dZ for the bias gradient.
__global__ __launch_bounds__(kEwBlock) void backward_finish_kernel(const BackwardArgs a, const int n_tiles, const int n_entry_blocks)
{
    if (static_cast<int>(blockIdx.x) < n_entry_blocks) {
        const int64_t stride = static_cast<int64_t>(kEwBlock) * n_entry_blocks;
        for (int64_t q = static_cast<int64_t>(blockIdx.x) * kEwBlock + threadIdx.x; q < a.nnz; q += stride) {
            float g = 0.f;
            int t = 0;
            for (; t + 8 <= n_tiles; t += 8) {  // eight loads in flight, added in tile order
                float v[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v[u] = a.partial[static_cast<int64_t>(t + u) * a.partial_stride + q];
#pragma unroll
                for (int u = 0; u < 8; ++u) g += v[u];
            }
            for (; t < n_tiles; ++t) g += a.partial[static_cast<int64_t>(t) * a.partial_stride + q];
            const int p = a.perm[q];
            if (a.g) a.g[p] = g;
            if (a.fused) {
                float w = a.w[p], v = a.velocity[p];
                momentum_step(w, v, g, a.lr, a.momentum, a.nesterov);
                a.w[p] = w;
                a.velocity[p] = v;
                a.w_t[q] = w;
            }
        }
        return;
    }
    if (!(a.db || (a.fused && a.bias))) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t n_waves = static_cast<int64_t>(gridDim.x - n_entry_blocks) * (kEwBlock / kWave);
    for (int64_t i = static_cast<int64_t>(blockIdx.x - n_entry_blocks) * (kEwBlock / kWave) + (threadIdx.x >> 6); i < a.x_rows; i += n_waves) {
        const float *zr = a.dZ + i * a.lddz;
        float s = 0.f;
        for (int c = lane * 4; c < a.batch; c += kWave * 4) {
            const float4 z = ld4(zr + c);
            s += (z.x + z.y) + (z.z + z.w);
        }
        s = group_sum<kWave>(s);
        if (lane == 0) {
            if (a.db) a.db[i] = s;
            if (a.fused && a.bias) {
                float w = a.bias[i], v = a.bias_velocity[i];
                momentum_step(w, v, s, a.lr, a.momentum, a.nesterov);
                a.bias[i] = w;
                a.bias_velocity[i] = v;
            }
        }
    }
}

// Two independent launches of a training step in one grid: work-groups [0, na) run the first,
// the rest the second.  Saves a launch (and its drain) on the step's critical path.
template <int GS_S, int NV_S, int G, int NV_D, bool EXACT4>
__global__ __launch_bounds__(kBlock) void spmm_sddmm_pair_kernel(const SpmmArgs a, const SddmmArgs b, const int na)
{
    if (static_cast<int>(blockIdx.x) < na) {
        if constexpr (GS_S < kWave)
            spmm_body_grouped<GS_S, false>(a, blockIdx.x);
        else
            spmm_body<4, NV_S, false>(a, blockIdx.x, 0);
    } else {
        sddmm_body<G, NV_D, EXACT4>(b, blockIdx.x - na);
    }
}
template <int G, int NV_D, bool EXACT4>
__global__ __launch_bounds__(kBlock) void sddmm_pair_kernel(const SddmmArgs a, const SddmmArgs b, const int na)
{
    if (static_cast<int>(blockIdx.x) < na)
        sddmm_body<G, NV_D, EXACT4>(a, blockIdx.x);
    else
        sddmm_body<G, NV_D, EXACT4>(b, blockIdx.x - na);
}

// Any batch size, any leading dimension, any alignment: one column per lane and pass, both
// operands re-read per stored entry.  The slow path behind sddmm_kernel.
__global__ __launch_bounds__(kBlock) void sddmm_generic(const SddmmArgs a)
{
    const int lane = threadIdx.x & (kWave - 1);
    mean_loss_task(a, blockIdx.x);
    const WaveTask task = wave_task(a.blocks, blockIdx.x);
    if (task.row < 0) return;
    const int row = task.row;
    const float *zr = a.dZ + static_cast<int64_t>(row) * a.lddz;
    const float *zm = a.ZM ? a.ZM + static_cast<int64_t>(row) * a.ldzm : nullptr;

    if (task.lead && (a.db || (a.fused && a.bias))) {
        float s = 0.f;
        for (int c = lane; c < a.batch; c += kWave) {
            float z = zr[c];
            if (zm) z = keep_where_positive(z, zm[c]);
            s += z;
        }
        s = group_sum<kWave>(s);
        if (lane == 0) {
            if (a.db) a.db[row] = s;
            if (a.fused && a.bias) {
                float w = a.bias[row], v = a.bias_velocity[row];
                momentum_step(w, v, s, a.lr, a.momentum, a.nesterov);
                a.bias[row] = w;
                a.bias_velocity[row] = v;
            }
        }
    }
    if (a.skip_products) return;

    const int s0 = task.s0;
    const int s1 = task.s1;
    for (int p = s0; p < s1; ++p) {
        const float *xr = a.X + static_cast<int64_t>(a.indices[p]) * a.ldx;
        float part = 0.f;
        for (int c = lane; c < a.batch; c += kWave) {
            float z = zr[c];
            if (zm) z = keep_where_positive(z, zm[c]);
            part = fmaf(z, xr[c], part);
        }
        part = group_sum<kWave>(part);
        if (lane == 0) {
            if (a.g) a.g[p] = part;
            if (a.fused) {
                float w = a.values[p], v = a.velocity[p];
                momentum_step(w, v, part, a.lr, a.momentum, a.nesterov);
                a.values[p] = w;
                a.velocity[p] = v;
                if (a.values_t) a.values_t[a.pos_t[p]] = w;
                if (a.dense) a.dense[static_cast<int64_t>(row) * a.dense_ld + a.indices[p]] = w;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------
// Element-wise kernels
// ---------------------------------------------------------------------------------------

__global__ __launch_bounds__(kEwBlock) void momentum_kernel(float *__restrict__ w, float *__restrict__ v,
                                                            const float *__restrict__ g, int64_t n,
                                                            float lr, float mu, int nesterov, int vec4)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (vec4) {
        const int64_t n4 = n >> 2;
        for (int64_t k = i; k < n4; k += stride) {
            float4 ww = ld4(w + 4 * k), vv = ld4(v + 4 * k);
            const float4 gg = ld4(g + 4 * k);
            momentum_step(ww.x, vv.x, gg.x, lr, mu, nesterov);
            momentum_step(ww.y, vv.y, gg.y, lr, mu, nesterov);
            momentum_step(ww.z, vv.z, gg.z, lr, mu, nesterov);
            momentum_step(ww.w, vv.w, gg.w, lr, mu, nesterov);
            st4(v + 4 * k, vv);
            st4(w + 4 * k, ww);
        }
        i += n4 << 2;  // tail: elements 4*n4 .. n-1, one per thread of the first work-group
        if (i < n) {
            float ww = w[i], vv = v[i];
            momentum_step(ww, vv, g[i], lr, mu, nesterov);
            v[i] = vv;
            w[i] = ww;
        }
    } else {
        for (; i < n; i += stride) {
            float ww = w[i], vv = v[i];
            momentum_step(ww, vv, g[i], lr, mu, nesterov);
            v[i] = vv;
            w[i] = ww;
        }
    }
}

__global__ __launch_bounds__(kEwBlock) void gather_kernel(float *__restrict__ dst, const float *__restrict__ src,
                                                          const int32_t *__restrict__ perm, int64_t n)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n; i += stride)
        dst[i] = src[perm[i]];
}

__global__ __launch_bounds__(kEwBlock) void copy_kernel(float *__restrict__ dst, const float *__restrict__ src,
                                                        int64_t n, int vec4)
{
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (vec4) {
        const int64_t n4 = n >> 2;
        for (int64_t k = i; k < n4; k += stride) st4(dst + 4 * k, ld4(src + 4 * k));
        i += n4 << 2;
        if (i < n) dst[i] = src[i];
    } else {
        for (; i < n; i += stride) dst[i] = src[i];
    }
}

// Softmax cross-entropy, one column (example) per thread, a single work-group so that the
// mean over the batch is summed in one fixed order (wave sums by DPP, then the wave leaders'
// values in wave order).  The logits matrix is classes x batch: small next to the layers that
// feed it.  CMAX > 0: classes <= CMAX and a column's logits are read once into registers.
constexpr int kSoftmaxBlock = 1024;
template <int CMAX>
__global__ __launch_bounds__(kSoftmaxBlock) void softmax_ce_kernel(const float *Z, int64_t ldz,
                                                                   const int32_t *__restrict__ labels,
                                                                   int classes, int batch, float *dZ,
                                                                   int64_t lddz, float *loss_out)
{
    __shared__ float wave_loss[kSoftmaxBlock / kWave];
    const float inv_b = 1.0f / static_cast<float>(batch);
    float loss = 0.f;
    for (int c = threadIdx.x; c < batch; c += blockDim.x) {
        const int t = labels[c];
        if constexpr (CMAX > 0) {
            float z[CMAX];
#pragma unroll
            for (int i = 0; i < CMAX; ++i) z[i] = i < classes ? Z[static_cast<int64_t>(i) * ldz + c] : -INFINITY;
            float m = z[0];
#pragma unroll
            for (int i = 1; i < CMAX; ++i) m = fmaxf(m, z[i]);
            float s = 0.f, zt = 0.f;
#pragma unroll
            for (int i = 0; i < CMAX; ++i) {
                if (i < classes) s += expf(z[i] - m);
                zt = i == t ? z[i] : zt;
            }
            const float lse = m + logf(s);
            loss += lse - zt;
#pragma unroll
            for (int i = 0; i < CMAX; ++i)
                if (i < classes) dZ[static_cast<int64_t>(i) * lddz + c] = (expf(z[i] - lse) - (i == t ? 1.f : 0.f)) * inv_b;
        } else {
            float m = -INFINITY;
            for (int i = 0; i < classes; ++i) m = fmaxf(m, Z[static_cast<int64_t>(i) * ldz + c]);
            float s = 0.f;
            for (int i = 0; i < classes; ++i) s += expf(Z[static_cast<int64_t>(i) * ldz + c] - m);
            const float lse = m + logf(s);
            loss += lse - Z[static_cast<int64_t>(t) * ldz + c];
            for (int i = 0; i < classes; ++i) {
                const float p = expf(Z[static_cast<int64_t>(i) * ldz + c] - lse);
                dZ[static_cast<int64_t>(i) * lddz + c] = (p - (i == t ? 1.f : 0.f)) * inv_b;
            }
        }
    }
    loss = group_sum<kWave>(loss);  // every lane of every wave arrives here
    if ((threadIdx.x & (kWave - 1)) == 0) wave_loss[threadIdx.x >> 6] = loss;
    __syncthreads();
    if (threadIdx.x == 0 && loss_out) {
        float total = 0.f;
        for (int w = 0; w < static_cast<int>(blockDim.x >> 6); ++w) total += wave_loss[w];
        *loss_out = total * inv_b;
    }
}

// Output-layer head (see HeadArgs).  Forward: wave w takes rows w, w+16, ..., lanes run across
// the row's stored entries, DPP sum.  Softmax-CE: one wave per column, one class per lane.
// Transposed product: one thread per row of W^T, dZ read from LDS.  Each column's loss goes to
// loss_cols; their mean is taken by a later launch of the step (SddmmArgs::loss_cols).
constexpr int kHeadCols = 4;
__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) x = fmaxf(x, __shfl_xor(x, m, kWave));
    return x;
}
__global__ __launch_bounds__(kBlock) void head_kernel(const HeadArgs a)
{
    __shared__ float z[kHeadMaxRows][kHeadCols];
    const int lane = threadIdx.x & (kWave - 1);
    const int wv = wave_in_block();
    const int c0 = blockIdx.x * kHeadCols;
    const int nc = min(kHeadCols, a.batch - c0);
    const bool vec = nc == kHeadCols && a.ldx % 4 == 0 && (reinterpret_cast<uintptr_t>(a.X) & 15u) == 0;

    // Operands of the last phase are requested first: their latency passes behind the forward product.
    const int j0 = threadIdx.x;
    int q0 = 0, q1 = 0;
    float mask[kHeadCols] = {0.f, 0.f, 0.f, 0.f};
    if (j0 < a.cols) {
        q0 = a.indptr_t[j0];
        q1 = a.indptr_t[j0 + 1];
        const float *mr = a.X + static_cast<int64_t>(j0) * a.ldx + c0;
        if (vec) {
            const float4 m = ld4(mr);
            mask[0] = m.x; mask[1] = m.y; mask[2] = m.z; mask[3] = m.w;
        } else {
#pragma unroll
            for (int c = 0; c < kHeadCols; ++c)
                if (c < nc) mask[c] = mr[c];
        }
    }
    const int label = wv < nc ? a.labels[c0 + wv] : 0;

    for (int i = wv; i < a.rows; i += kWavesPerBlock) {
        float acc[kHeadCols] = {0.f, 0.f, 0.f, 0.f};
        for (int p = a.indptr[i] + lane; p < a.indptr[i + 1]; p += kWave) {
            const float w = a.values[p];
            const float *xr = a.X + static_cast<int64_t>(a.indices[p]) * a.ldx + c0;
            if (vec) {
                const float4 x = ld4(xr);
                acc[0] = fmaf(w, x.x, acc[0]);
                acc[1] = fmaf(w, x.y, acc[1]);
                acc[2] = fmaf(w, x.z, acc[2]);
                acc[3] = fmaf(w, x.w, acc[3]);
            } else {
#pragma unroll
                for (int c = 0; c < kHeadCols; ++c)
                    if (c < nc) acc[c] = fmaf(w, xr[c], acc[c]);
            }
        }
#pragma unroll
        for (int c = 0; c < kHeadCols; ++c) acc[c] = group_sum<kWave>(acc[c]);
        if (lane == 0) {
            const float b = a.bias ? a.bias[i] : 0.f;
#pragma unroll
            for (int c = 0; c < kHeadCols; ++c) z[i][c] = acc[c] + b;
        }
    }
    __syncthreads();

    // softmax cross-entropy of column c0+wv by wave wv: one class per lane (rows <= 32)
    if (wv < nc) {
        const bool live = lane < a.rows;
        const float zi = live ? z[lane][wv] : -INFINITY;
        const float m = wave_max(zi);
        const float lse = m + logf(group_sum<kWave>(live ? expf(zi - m) : 0.f));
        const float zt = group_sum<kWave>(lane == label ? zi : 0.f);  // one non-zero term: exact
        const float d = (expf(zi - lse) - (lane == label ? 1.f : 0.f)) / static_cast<float>(a.batch);
        if (live) {
            a.Z[static_cast<int64_t>(lane) * a.ldz + c0 + wv] = zi;
            a.dZ[static_cast<int64_t>(lane) * a.lddz + c0 + wv] = d;
            z[lane][wv] = d;
        }
        if (lane == 0) a.loss_cols[c0 + wv] = lse - zt;
    }
    __syncthreads();

    for (int j = j0; j < a.cols; j += kBlock) {
        if (j != j0) {
            q0 = a.indptr_t[j];
            q1 = a.indptr_t[j + 1];
            const float *mr = a.X + static_cast<int64_t>(j) * a.ldx + c0;
#pragma unroll
            for (int c = 0; c < kHeadCols; ++c)
                if (c < nc) mask[c] = mr[c];
        }
        float acc[kHeadCols] = {0.f, 0.f, 0.f, 0.f};
        for (int q = q0; q < q1; ++q) {
            const float w = a.values_t[q];
            const int i = a.indices_t[q];
#pragma unroll
            for (int c = 0; c < kHeadCols; ++c) acc[c] = fmaf(w, z[i][c], acc[c]);
        }
        float *dr = a.dX + static_cast<int64_t>(j) * a.lddx + c0;
        if (vec && a.lddx % 4 == 0 && (reinterpret_cast<uintptr_t>(a.dX) & 15u) == 0) {
            st4(dr, make_float4(keep_where_positive(acc[0], mask[0]), keep_where_positive(acc[1], mask[1]),
                                keep_where_positive(acc[2], mask[2]), keep_where_positive(acc[3], mask[3])));
        } else {
#pragma unroll
            for (int c = 0; c < kHeadCols; ++c)
                if (c < nc) dr[c] = keep_where_positive(acc[c], mask[c]);
        }
    }
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int elementwise_blocks(int64_t work_items)
{
    int64_t b = (work_items + kEwBlock - 1) / kEwBlock;
    if (b < 1) b = 1;
    if (b > 256 * 32) b = 256 * 32;  // 256 compute units; grid-stride beyond that
    return static_cast<int>(b);
}

template <int VEC, int NV>
hipError_t spmm_go(const SpmmArgs &a, hipStream_t s)
{
    const int tile = kWave * VEC * NV;
    dim3 grid(a.blocks.n_blocks, (a.batch + tile - 1) / tile);
    if (a.XM)
        hipLaunchKernelGGL((spmm_kernel<VEC, NV, true>), grid, dim3(kBlock), 0, s, a);
    else
        hipLaunchKernelGGL((spmm_kernel<VEC, NV, false>), grid, dim3(kBlock), 0, s, a);
    if (a.blocks.n_huge_rows > 0)
        hipLaunchKernelGGL(spmm_finish_kernel, dim3(a.blocks.n_huge_rows, (a.batch + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

template <int GS>
hipError_t spmm_grouped_go(const SpmmArgs &a, hipStream_t s)
{
    dim3 grid(a.blocks.n_blocks);
    if (a.XM)
        hipLaunchKernelGGL((spmm_grouped_kernel<GS, true>), grid, dim3(kBlock), 0, s, a);
    else
        hipLaunchKernelGGL((spmm_grouped_kernel<GS, false>), grid, dim3(kBlock), 0, s, a);
    if (a.blocks.n_huge_rows > 0)
        hipLaunchKernelGGL(spmm_finish_kernel, dim3(a.blocks.n_huge_rows, (a.batch + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

// The gathered operand (and its mask) should stay in one 4 MiB L2 while it is being gathered
// from: if the whole operand is too large for that, the batch is walked in column tiles of
// 4 * (return value) columns.  0: no tiling.
int spmm_tile_group(const SpmmArgs &a)
{
    if (static_cast<int64_t>(a.blocks.n_blocks) * ((a.batch + 31) / 32 + 8) >= (1ll << 31)) return 0;
    return tile_columns(a.x_rows, a.batch, a.nnz, a.rows, a.blocks.hot_share, a.XM != nullptr) / 4;
}

template <int GS>
hipError_t spmm_tiled_go(const SpmmArgs &a, hipStream_t s)
{
    const int n_tiles = (a.batch + GS * 4 - 1) / (GS * 4);
    const int spread = n_tiles >= 8;
    const int64_t ids = spread ? static_cast<int64_t>((n_tiles + 7) / 8) * 8 * a.blocks.n_blocks
                               : static_cast<int64_t>(n_tiles) * a.blocks.n_blocks;
    dim3 grid(static_cast<unsigned>(ids));
    if (a.XM)
        hipLaunchKernelGGL((spmm_tiled_kernel<GS, true>), grid, dim3(kBlock), 0, s, a, n_tiles, spread);
    else
        hipLaunchKernelGGL((spmm_tiled_kernel<GS, false>), grid, dim3(kBlock), 0, s, a, n_tiles, spread);
    if (a.blocks.n_huge_rows > 0)
        hipLaunchKernelGGL(spmm_finish_kernel, dim3(a.blocks.n_huge_rows, (a.batch + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

constexpr int64_t kMaxGridIds = (1ll << 31) - 1;

// Work-groups of the packed launch for lane groups of gs lanes: those that serve the short rows, and
// the launch's grid size (tiles rounded up to whole rounds of the 8 XCDs when the ids are decoded
// XCD-first).  One place, so that the launch and the checks that the grid fits agree.
struct PackedGrid {
    int n_tiles, spread, n_pack_blocks;
    int64_t ids;
};
PackedGrid packed_grid(const SpmmArgs &a, int gs, bool with_long_rows)
{
    PackedGrid g;
    const int ne = kWave / gs;
    g.n_tiles = (a.batch + gs * 4 - 1) / (gs * 4);
    g.spread = g.n_tiles >= 8;
    const int64_t n_sets = (static_cast<int64_t>(a.blocks.n_short) + ne - 1) / ne;
    g.n_pack_blocks = static_cast<int>((n_sets + kWavesPerBlock * kPackSets - 1) / (kWavesPerBlock * kPackSets));
    const int64_t nrb = static_cast<int64_t>(g.n_pack_blocks) + (with_long_rows ? a.blocks.n_long_blocks : 0);
    g.ids = (g.spread ? static_cast<int64_t>((g.n_tiles + 7) / 8) * 8 : g.n_tiles) * nrb;
    return g;
}
template <int GS>
hipError_t spmm_packed_go(const SpmmArgs &a, hipStream_t s)
{
    const PackedGrid pg = packed_grid(a, GS, true);
    const int n_tiles = pg.n_tiles, spread = pg.spread, n_pack_blocks = pg.n_pack_blocks;
    if (pg.ids > kMaxGridIds) return hipErrorInvalidConfiguration;  // (callers check before choosing this path)
    dim3 grid(static_cast<unsigned>(pg.ids));
    if (a.XM)
        hipLaunchKernelGGL((spmm_packed_kernel<GS, true>), grid, dim3(kBlock), 0, s, a, n_tiles, spread, n_pack_blocks);
    else
        hipLaunchKernelGGL((spmm_packed_kernel<GS, false>), grid, dim3(kBlock), 0, s, a, n_tiles, spread, n_pack_blocks);
    if (a.blocks.n_huge_rows > 0)
        hipLaunchKernelGGL(spmm_finish_kernel, dim3(a.blocks.n_huge_rows, (a.batch + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

template <int G, int NV>
hipError_t sddmm_go(const SddmmArgs &a, hipStream_t s)
{
    dim3 grid(a.blocks.n_blocks);
    if (a.batch % 4 == 0)
        hipLaunchKernelGGL((sddmm_kernel<G, NV, true>), grid, dim3(kBlock), 0, s, a);
    else
        hipLaunchKernelGGL((sddmm_kernel<G, NV, false>), grid, dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

// The grouped kernels address the gathered operand with 32-bit byte offsets from its base.
inline bool spans_below_4gib(int64_t rows, int64_t ld) { return rows * ld * 4 < (1ll << 32); }

bool spmm_vec_ok(const SpmmArgs &a);

// The staged product pays where a work-group finds several stored entries per operand row it
// copies into LDS, fills its column tiles, and has enough siblings to occupy the chip; where the
// segments are long (the gathers then dominate everything else) or the operand is beyond any
// L2 and evenly used (the gathers of the other kernels then go to memory); and where no single lane row's share,
// served at about one entry per 60 ns, outlasts the rest of the matrix, which
// the chip's 256 LDS serve at about one entry and tile per 3.3 ns each.
bool staged_pays(const RowBlocks &blocks, int32_t x_rows, int32_t batch, int32_t long_segment)
{
    if (!blocks.staged_rows || batch < kStageMinBatch || batch % 4 != 0) return false;
    // (an operand of a few rows is in cache wherever it is gathered from: config 4's 8192 x 10 mirror, 21 against 28 us)
    if (x_rows < kStageRows / 2 && !blocks.staged_preferred) return false;
    const int64_t rows = blocks.staged_row_count, nnz = blocks.staged_nnz;  // what the plan covers
    const int64_t n_tiles = (batch + kStageCols - 1) / kStageCols;
    if (!blocks.staged_preferred && static_cast<int64_t>(batch) * 5 < n_tiles * kStageCols * 4) return false;  // a fifth or more of the tiles' columns idle
    const int64_t groups = n_tiles * blocks.staged_ranges;
    if (groups >= (1ll << 31)) return false;
    if (blocks.staged_preferred) return true;
    // (three quarters of the compute units busy at least; half where the plan covers a matrix's long rows only,
    // whose alternative is gathering from memory: 580 long rows of the 0.3 % power-law matrix make 144 work-groups)
    if (groups < (blocks.staged_partial ? kStageTargetGroups / 2 : kStageTargetGroups * 3 / 4)) return false;
    if (static_cast<double>(nnz) < static_cast<double>(kStageMinReuse) * blocks.staged_ranges * x_rows) return false;
    if (static_cast<int64_t>(blocks.staged_longest_share) * 4096 > nnz * n_tiles) return false;
    // An operand beyond the L2s, evenly used, on rows of similar length: shorter segments already pay, because the other
    // kernels' gathers partly go to memory there (a few hot operand rows that take most gathers would stay cached on
    // the other paths; on a power-law matrix most (row, block) pairs hold one entry or none and cost a visit all the
    // same).  Measured on 16384^2 uniform matrices at batch 1024 against the column-tiled kernels, product / SDDMM:
    // 0.7 % (3.6 entries per segment) 648 / 851 us staged against 429 / 595; 1 % (5.1) 692 / 1012 against 662 / 836;
    // 2 % (10.2) 880 / 1259 against 1341 / 1642.
    const bool big_operand = static_cast<int64_t>(x_rows) * batch * 4 >= kStageBigOperand && blocks.hot_share < 0.5f &&
                             static_cast<int64_t>(blocks.staged_longest_row) * rows <= 4 * nnz;
    const int64_t segment = big_operand ? std::min(long_segment, kStageSegmentBigOperand) : long_segment;
    return nnz >= segment * rows * blocks.staged_cblocks;
}

int spmm_tile_group(const SpmmArgs &a);
bool spmm_offsets_ok(const SpmmArgs &a);
constexpr int64_t kSplitMinOperand = 48ll << 20;  // operand bytes from which long rows go into column tiles of their own: beyond the eight L2s

// Lanes per row (4 columns each) of the column tiles in which the LONG rows of a matrix run while its short rows run
// untiled: for an operand that the L2s together cannot hold, gathered about evenly, on a matrix whose long rows
// (beyond kPackMaxLen entries; they have a partition of their own) hold most of the stored entries.  0: no split.
int spmm_split_group(const SpmmArgs &a)
{
    if (a.blocks.n_long_blocks <= 0 || a.blocks.n_rest_blocks <= 0 || a.batch < 128) return 0;
    if (static_cast<int64_t>(a.x_rows) * a.batch * 4 < kSplitMinOperand || a.blocks.hot_share >= 0.5f) return 0;
    if (static_cast<int64_t>(a.blocks.long_nnz) * 2 < a.nnz) return 0;
    const int64_t budget = (a.XM ? 5 : 10) * (1 << 18), row_bytes = static_cast<int64_t>(a.x_rows) * 4;
    // 64-column tiles as long as a tile of the operand fits an L2 at all (measured on a 16384-row operand at 1024
    // columns: 137 us with 64-column tiles, 150 with 128, 174 with 32 -- a pass over the long rows per tile
    // costs more than the misses of a tile that fills the L2 -- and 173 us unsplit)
    int g = 0;
    if (row_bytes * 128 <= budget) g = 32;
    else if (row_bytes * 64 <= (a.XM ? (2ll << 20) : (4ll << 20))) g = 16;
    else if (row_bytes * 32 <= budget) g = 8;
    if (g == 0) return 0;
    const int64_t n_tiles = (a.batch + g * 4 - 1) / (g * 4);
    if ((n_tiles + 8) * a.blocks.n_long_blocks > kMaxGridIds) return 0;
    return g;
}

bool spmm_staged_ok(const SpmmArgs &a)
{
    if (!spmm_vec_ok(a) || !staged_pays(a.blocks, a.x_rows, a.batch, kStageLongSegment)) return false;
    return !a.blocks.staged_partial || a.blocks.n_rest_blocks > 0;  // (the rows the plan leaves out need a partition of their own)
}

// whether the rows a partial plan leaves out take the packed kernel, which runs inside column tiles only
bool staged_rest_packed(const SpmmArgs &a, int tg)
{
    return a.blocks.n_short > 0 && tg != 0 && spmm_offsets_ok(a) && packed_grid(a, tg, false).ids <= kMaxGridIds;
}

bool sddmm_vec_ok(const SddmmArgs &a);

// a full matrix of few rows whose dZ fits in 64 KiB of LDS
bool sddmm_full_ok(const SddmmArgs &a)
{
    if (a.rows > kFullMaxRows || a.x_rows < 256 || static_cast<int64_t>(a.nnz) != static_cast<int64_t>(a.rows) * a.x_rows) return false;
    if (a.batch < 64 || a.batch % 4 != 0 || a.skip_products || a.dense || a.loss_cols || !sddmm_vec_ok(a)) return false;
    return static_cast<int64_t>(a.rows) * ((a.batch + 255) / 256) <= 64;
}

// the staged SDDMM needs room for one slice of partial products per 64-column tile
bool sddmm_staged_ok(const SddmmArgs &a)
{
    if (!a.partial || a.skip_products || a.dense || a.loss_cols || !sddmm_vec_ok(a)) return false;
    if ((a.batch + kStageCols - 1) / kStageCols > a.partial_tiles) return false;
    return staged_pays(a.blocks, a.x_rows, a.batch, kStageLongSegmentSddmm) && (!a.blocks.staged_partial || a.blocks.n_rest_blocks > 0);
}

bool spmm_offsets_ok(const SpmmArgs &a)
{
    return spans_below_4gib(a.x_rows, a.ldx) && (!a.XM || spans_below_4gib(a.x_rows, a.ldxm));
}

template <int G, int NV>
hipError_t sddmm_tiled_go(const SddmmArgs &a, hipStream_t s)
{
    const int W = G * 4 * NV;
    const int n_tiles = (a.batch + W - 1) / W;
    const int spread = n_tiles >= 8;
    const int64_t ids = (spread ? static_cast<int64_t>((n_tiles + 7) / 8) * 8 : n_tiles) * a.blocks.n_blocks;
    dim3 grid(static_cast<unsigned>(ids));
    if (a.batch % 4 == 0)
        hipLaunchKernelGGL((sddmm_tiled_kernel<G, NV, true>), grid, dim3(kBlock), 0, s, a, n_tiles, spread);
    else
        hipLaunchKernelGGL((sddmm_tiled_kernel<G, NV, false>), grid, dim3(kBlock), 0, s, a, n_tiles, spread);
    const int64_t work = a.nnz > a.rows ? a.nnz : a.rows;
    hipLaunchKernelGGL(sddmm_finish_kernel, dim3(elementwise_blocks(work)), dim3(kEwBlock), 0, s, a, n_tiles);
    return hipGetLastError();
}

bool spmm_vec_ok(const SpmmArgs &a)
{
    bool vec = a.ldx % 4 == 0 && a.ldy % 4 == 0 && aligned16(a.X) && aligned16(a.Y);
    if (a.XM) vec = vec && a.ldxm % 4 == 0 && aligned16(a.XM);
    if (a.YM) vec = vec && a.ldym % 4 == 0 && aligned16(a.YM);
    return vec;
}

bool sddmm_vec_ok(const SddmmArgs &a)
{
    bool vec = a.lddz % 4 == 0 && aligned16(a.dZ);
    if (!a.skip_products) vec = vec && a.ldx % 4 == 0 && aligned16(a.X) && spans_below_4gib(a.x_rows, a.ldx);
    if (a.ZM) vec = vec && a.ldzm % 4 == 0 && aligned16(a.ZM);
    return vec;
}

template <int GS_S, int NV_S, int G, int NV_D>
hipError_t pair_go(const SpmmArgs &a, const SddmmArgs &b, hipStream_t s)
{
    const int na = a.blocks.n_blocks;
    dim3 grid(na + b.blocks.n_blocks);
    if (a.batch % 4 == 0)
        hipLaunchKernelGGL((spmm_sddmm_pair_kernel<GS_S, NV_S, G, NV_D, true>), grid, dim3(kBlock), 0, s, a, b, na);
    else
        hipLaunchKernelGGL((spmm_sddmm_pair_kernel<GS_S, NV_S, G, NV_D, false>), grid, dim3(kBlock), 0, s, a, b, na);
    if (a.blocks.n_huge_rows > 0)
        hipLaunchKernelGGL(spmm_finish_kernel, dim3(a.blocks.n_huge_rows, (a.batch + 255) / 256), dim3(256), 0, s, a);
    return hipGetLastError();
}

template <int G, int NV_D>
hipError_t sddmm_pair_go(const SddmmArgs &a, const SddmmArgs &b, hipStream_t s)
{
    const int na = a.blocks.n_blocks;
    dim3 grid(na + b.blocks.n_blocks);
    if (a.batch % 4 == 0)
        hipLaunchKernelGGL((sddmm_pair_kernel<G, NV_D, true>), grid, dim3(kBlock), 0, s, a, b, na);
    else
        hipLaunchKernelGGL((sddmm_pair_kernel<G, NV_D, false>), grid, dim3(kBlock), 0, s, a, b, na);
    return hipGetLastError();
}

}  // namespace

int sddmm_tile_columns(const SddmmArgs &a);

int tile_columns(int32_t x_rows, int32_t batch, int64_t nnz, int32_t rows, float hot_share, bool masked, bool for_sddmm)
{
    const int64_t budget = (masked ? 5 : 10) * (1 << 18);  // 2.5 MiB (half of it with a mask operand)
    const int64_t row_bytes = static_cast<int64_t>(x_rows) * 4;
    if (x_rows <= 0 || row_bytes * batch <= budget) return 0;
    // A matrix of few rows is in flight as a whole: its rows gather the same operand rows at about
    // the same time, which serves them from cache without tiling (measured on a dense 10 x 8192 layer).
    if (rows <= 256) return 0;
    // (the SDDMM, whose second operand is a row per matrix row and not a gather, still gains from 128-column
    // tiles when they fill a whole L2: config 4's 8192-row operand, 120 -> 113 us, where the product loses 7 %)
    if (row_bytes * 128 <= (for_sddmm ? (4ll << 20) : budget) && batch > 128) return 128;
    if (row_bytes * 64 <= budget && batch > 64) return 64;
    if (batch <= 32) return 0;
    // Short rows on an operand whose 64-column tile (4 MiB for 16384 rows) no longer fits beside the rest in an L2: wide tiles
    // still pay at wide batches, because they cut the set of operand rows in flight by 8 to 16 and what misses the L2
    // then hits the infinity cache.  Measured on 16384^2 matrices at batch 1024 (512): uniform rows at 0.1 / 0.3 %,
    // products 165 -> 83 and 458 -> 197 us with 64 columns (109 / 282 with 128), SDDMM 156 -> 111 and 442 -> 271 with
    // 128; power-law rows at 0.1 %, forward 142 -> 110 (85 -> 60), SDDMM 165 -> 134 (80 -> 69; 147 with 64 columns).
    // Where a few operand rows take most gathers (the transposed product of the power-law matrix) 64 columns lose
    // (57 -> 63, 554 -> 597 us at 0.1 / 1 %) and 128 do not (58, 475).
    // (Beside the staged long rows of the power-law matrix at 1 % the short rows then run in 64- instead of 32-column
    // tiles: forward 495 -> 450 us.)
    // (The same holds with tiles twice that size: 32768^2 at batch 1024, uniform rows at 0.1 / 0.5 %, products 629 -> 478
    // and 2577 -> 1814 us; 12288^2: 94 -> 49 and 395 -> 163.)
    if (batch >= 512 && row_bytes * 64 <= (8ll << 20)) return for_sddmm || hot_share >= 0.5f ? 128 : 64;
    // Narrower batches (128 .. 511) on such an operand: 64-column tiles from about 128 entries per row on, unless a few
    // operand rows take most gathers.  16384^2 at 1 %, batch 128 / 256: uniform rows, products 105 -> 90 and 252 -> 173 us
    // (32-column tiles: 136, 250), SDDMM 108 -> 97 and 225 -> 181; power-law rows, forward 96 -> 81 and 210 -> 154,
    // SDDMM 93 -> 89 and 204 -> 164, transposed (hot rows) 83 -> 100 and 131 -> 171: left untiled.  At 16 entries per
    // row tiles lose at these batches (power-law 0.1 %, batch 128: forward 24 -> 36 us).
    if (batch >= 128 && row_bytes * 64 <= (4ll << 20) && row_bytes * batch >= (8ll << 20) && hot_share < 0.5f &&
        nnz >= static_cast<int64_t>(rows) * 128)
        return 64;
    // Narrower tiles, for operands larger still: they multiply the per-wave set-up (one pass
    // over the row partition per tile) by 32 or more.  Measured on 16384^2 matrices at batch 1024 against untiled
    // launches: they pay from about 128 entries per row on (1 % density: 1.48 -> 1.18 ms, 10 %: 1.4x) unless a few
    // operand rows take most of the gathers (the transposed product of a power-law matrix: 0.58 -> 1.08 ms); at 16
    // entries per row they lose, and so they do on an 8 MiB operand (batch 128), half of which an L2 holds anyway.
    if (nnz >= static_cast<int64_t>(rows) * 1024) return 32;
    if (nnz >= static_cast<int64_t>(rows) * 128 && hot_share < 0.5f && row_bytes * batch >= (16ll << 20)) return 32;
    return 0;
}

bool can_pair(const SpmmArgs &a, const SddmmArgs &b)
{
    return a.batch == b.batch && a.batch > 4 && a.batch <= 1024 && !a.XM && a.rows > 0 && b.rows > 0 &&
           a.blocks.n_blocks > 0 && b.blocks.n_blocks > 0 && spmm_vec_ok(a) && spmm_offsets_ok(a) &&
           sddmm_vec_ok(b) && spmm_tile_group(a) == 0 && !spmm_staged_ok(a) && sddmm_tile_columns(b) == 0 &&
           !sddmm_staged_ok(b) && !sddmm_full_ok(b);
}

bool can_pair(const SddmmArgs &a, const SddmmArgs &b)
{
    return a.batch == b.batch && a.batch > 0 && a.batch <= 1024 && a.rows > 0 && b.rows > 0 &&
           a.blocks.n_blocks > 0 && b.blocks.n_blocks > 0 && sddmm_vec_ok(a) && sddmm_vec_ok(b) &&
           sddmm_tile_columns(a) == 0 && sddmm_tile_columns(b) == 0 && !sddmm_staged_ok(a) && !sddmm_staged_ok(b) &&
           !sddmm_full_ok(a) && !sddmm_full_ok(b);
}

hipError_t launch_pair(const SpmmArgs &a, const SddmmArgs &b, hipStream_t s)
{
    if (a.batch <= 64) return pair_go<16, 1, 16, 1>(a, b, s);
    if (a.batch <= 128) return pair_go<32, 1, 16, 2>(a, b, s);
    if (a.batch <= 256) return pair_go<64, 1, 16, 4>(a, b, s);
    if (a.batch <= 512) return pair_go<64, 2, 64, 2>(a, b, s);
    return pair_go<64, 4, 64, 4>(a, b, s);
}

hipError_t launch_pair(const SddmmArgs &a, const SddmmArgs &b, hipStream_t s)
{
    if (a.batch <= 64) return sddmm_pair_go<16, 1>(a, b, s);
    if (a.batch <= 128) return sddmm_pair_go<16, 2>(a, b, s);
    if (a.batch <= 256) return sddmm_pair_go<16, 4>(a, b, s);
    if (a.batch <= 512) return sddmm_pair_go<64, 2>(a, b, s);
    return sddmm_pair_go<64, 4>(a, b, s);
}

// The transposed product t and the SDDMM g of one layer can share their gathers when t would run the
// packed kernel inside column tiles on a mirror all of whose rows are short, its result mask is the
// SDDMM's second operand (the output of the layer below), and the layer's partial buffer has a slice
// per tile for the products in mirror order.
// Lanes per mirror row of the fused backward pass: the transposed product's own tiles, widened to 128 columns
// while a tile of dZ still fills no more than an L2 -- half as many tiles halve the partial products that go
// out and come back (wide MLP, 8192 x 8192 layer: 128.6 -> 122.6 us; the product alone loses 7 % with them).
static int backward_tile_group(const SpmmArgs &t)
{
    const int tg = spmm_tile_group(t);
    if (tg == 16 && t.batch > 128 && static_cast<int64_t>(t.x_rows) * 4 * 128 <= (4ll << 20)) return 32;
    return tg;
}

bool backward_fused_ok(const SpmmArgs &t, const SddmmArgs &g)
{
    if (t.batch != g.batch || t.batch % 4 != 0 || t.XM || !t.YM || t.YM != g.X || t.ldym != g.ldx || t.X != g.dZ || t.ldx != g.lddz) return false;
    if (t.rows != g.x_rows || t.x_rows != g.rows || t.nnz != g.nnz || t.nnz <= 0) return false;
    if (g.ZM || g.skip_products || g.dense || g.loss_cols || !g.partial || !g.perm) return false;
    if (!spmm_vec_ok(t) || !spmm_offsets_ok(t) || !sddmm_vec_ok(g) || spmm_staged_ok(t)) return false;
    if (t.blocks.n_short != t.rows || t.blocks.n_long_blocks != 0) return false;  // every mirror row packed
    const int tg = backward_tile_group(t);
    if (tg != 16 && tg != 32) return false;  // (32-column tiles are only chosen for rows too long to be packed)
    const int n_tiles = (t.batch + tg * 4 - 1) / (tg * 4);
    if (n_tiles > g.partial_tiles || g.partial_stride < t.nnz) return false;
    const int64_t sets = (static_cast<int64_t>(t.blocks.n_short) + kWave / tg - 1) / (kWave / tg);
    return ((n_tiles + 7) / 8) * 8 * ((sets + kBwdWaves - 1) / kBwdWaves) <= kMaxGridIds;
}

// The same sharing for a full matrix of few rows (a saturated output layer): its SDDMM streams the layer's
// input once, a wave per input row, and that row is also the mask of the transposed product's result row.
bool full_backward_ok(const SpmmArgs &t, const SddmmArgs &g)
{
    SddmmArgs plain = g;
    plain.loss_cols = nullptr;  // (this launch can carry the mean of the losses, the plain one is not asked to)
    if (!sddmm_full_ok(plain) || !g.fused || g.ZM || !g.values || !g.velocity) return false;
    if (t.batch != g.batch || t.XM || t.bias || t.relu || !t.YM || t.YM != g.X || t.ldym != g.ldx || t.X != g.dZ || t.ldx != g.lddz) return false;
    if (t.rows != g.x_rows || t.x_rows != g.rows || t.nnz != g.nnz || !t.Y) return false;
    return t.ldy % 4 == 0 && (reinterpret_cast<uintptr_t>(t.Y) & 15u) == 0;
}

hipError_t launch_full_backward(const SpmmArgs &t, const SddmmArgs &g, hipStream_t s)
{
    const int n_chunks = (g.batch + 255) / 256;
    const int groups = (g.x_rows + kWavesPerBlock - 1) / kWavesPerBlock;
    hipLaunchKernelGGL(full_sddmm_kernel<true>, dim3(groups < 1024 ? groups : 1024), dim3(kBlock),
                       static_cast<size_t>(g.rows) * n_chunks * kWave * sizeof(float4), s, g, n_chunks, t.Y, static_cast<int>(t.ldy));
    return hipGetLastError();
}

hipError_t launch_backward_fused(const SpmmArgs &t, const SddmmArgs &g, hipStream_t s)
{
    BackwardArgs a{};
    a.blocks = t.blocks; a.indices = t.indices; a.values = t.values;
    a.dZ = t.X; a.lddz = t.ldx; a.X = g.X; a.ldx = g.ldx; a.dX = t.Y; a.lddx = t.ldy; a.mask = 1;
    a.rows = t.rows; a.x_rows = t.x_rows; a.batch = t.batch; a.nnz = t.nnz;
    a.partial = g.partial; a.partial_stride = g.partial_stride; a.perm = g.perm;
    a.g = g.g; a.db = g.db; a.fused = g.fused; a.nesterov = g.nesterov; a.lr = g.lr; a.momentum = g.momentum;
    a.w = g.values; a.velocity = g.velocity; a.w_t = g.values_t; a.bias = g.bias; a.bias_velocity = g.bias_velocity;
    const int tg = backward_tile_group(t);
    const int n_tiles = (t.batch + tg * 4 - 1) / (tg * 4);
    const int spread = n_tiles >= 8;
    const int64_t sets = (static_cast<int64_t>(t.blocks.n_short) + kWave / tg - 1) / (kWave / tg);
    const int n_pack_blocks = static_cast<int>((sets + kBwdWaves - 1) / kBwdWaves);
    const int64_t ids = static_cast<int64_t>(spread ? (n_tiles + 7) / 8 * 8 : n_tiles) * n_pack_blocks;
    if (tg == 32)
        hipLaunchKernelGGL(backward_fused_kernel<32>, dim3(static_cast<unsigned>(ids)), dim3(kBwdWaves * kWave), 0, s, a, n_tiles, spread, n_pack_blocks);
    else
        hipLaunchKernelGGL(backward_fused_kernel<16>, dim3(static_cast<unsigned>(ids)), dim3(kBwdWaves * kWave), 0, s, a, n_tiles, spread, n_pack_blocks);
    const int n_entry_blocks = elementwise_blocks(t.nnz);
    const int64_t row_blocks = (static_cast<int64_t>(a.x_rows) + kEwBlock / kWave - 1) / (kEwBlock / kWave);
    const int n_row_blocks = (a.db || (a.fused && a.bias)) ? static_cast<int>(row_blocks < 2048 ? row_blocks : 2048) : 0;
    hipLaunchKernelGGL(backward_finish_kernel, dim3(n_entry_blocks + n_row_blocks), dim3(kEwBlock), 0, s, a, n_tiles, n_entry_blocks);
    return hipGetLastError();
}

// whether launch_spmm serves `a` by streaming (full matrix of few rows), where the softmax epilogue can ride along
static bool spmm_full_rows_ok(const SpmmArgs &a)
{
    return a.batch > 4 && a.full_scratch && !a.XM && a.batch >= 64 && a.rows <= kFullMaxRows && spmm_vec_ok(a) && a.full_scratch_ld % 4 == 0;
}
bool spmm_softmax_epilogue_ok(const SpmmArgs &a)
{
    return a.rows > 0 && a.blocks.n_blocks > 0 && spmm_full_rows_ok(a) && !a.relu && !a.YM && a.ce_labels && a.ce_dZ && a.ce_loss_cols;
}

hipError_t launch_spmm(const SpmmArgs &a, hipStream_t s)
{
    if (a.rows <= 0 || a.batch <= 0 || a.blocks.n_blocks <= 0) return hipSuccess;
    if (a.batch <= 4) {
        if (a.batch == 1)
            hipLaunchKernelGGL(spmv_kernel<1>, dim3(a.blocks.n_blocks), dim3(kBlock), 0, s, a);
        else
            hipLaunchKernelGGL(spmv_kernel<4>, dim3(a.blocks.n_blocks), dim3(kBlock), 0, s, a);
        if (a.blocks.n_huge_rows > 0)
            hipLaunchKernelGGL(spmm_finish_kernel, dim3(a.blocks.n_huge_rows, 1), dim3(256), 0, s, a);
        return hipGetLastError();
    }
    if (spmm_full_rows_ok(a)) {
        const int n_slices = (a.x_rows + kFullSlice - 1) / kFullSlice;
        hipLaunchKernelGGL(full_rows_kernel, dim3(n_slices, (a.batch + 255) / 256), dim3(kFullWaves * kWave),
                           static_cast<size_t>(kFullWaves) * a.rows * kWave * sizeof(float4), s, a);
        if (a.ce_labels)
            hipLaunchKernelGGL(full_rows_finish_softmax_kernel, dim3((a.batch + kWave - 1) / kWave), dim3(kBlock), 0, s, a, n_slices);
        else
            hipLaunchKernelGGL(full_rows_finish_kernel, dim3(a.rows, (a.batch + kEwBlock - 1) / kEwBlock), dim3(kEwBlock), 0, s, a, n_slices);
        return hipGetLastError();
    }
    if (spmm_staged_ok(a)) {
        const int n_tiles = (a.batch + kStageCols - 1) / kStageCols;
        const dim3 grid(n_tiles * a.blocks.staged_ranges), block(kStageWaves * kWave);
        if (a.XM)
            hipLaunchKernelGGL(spmm_staged_kernel<true>, grid, block, 0, s, a, n_tiles);
        else
            hipLaunchKernelGGL(spmm_staged_kernel<false>, grid, block, 0, s, a, n_tiles);
        if (a.blocks.staged_partial) {
            // the short rows: packed where that path runs (inside column tiles), and nothing else in that grid;
            // otherwise whatever kernel the batch asks for, on the short rows' own partition
            SpmmArgs rest = a;
            rest.blocks.n_huge_rows = 0;
            const int tg = spmm_tile_group(a);
            if (staged_rest_packed(a, tg)) {
                rest.blocks.n_long_blocks = 0;
                switch (tg) {
                    case 32: return spmm_packed_go<32>(rest, s);
                    case 16: return spmm_packed_go<16>(rest, s);
                    default: return spmm_packed_go<8>(rest, s);
                }
            }
            rest.blocks.staged_rows = nullptr;
            rest.blocks.n_short = 0;
            rest.blocks.waves = a.blocks.rest_waves;
            rest.blocks.n_blocks = a.blocks.n_rest_blocks;
            return launch_spmm(rest, s);
        }
        return hipGetLastError();
    }
    if (spmm_vec_ok(a)) {
        if (spmm_offsets_ok(a)) {
            const int tg = spmm_tile_group(a);
            const int sg = tg == 0 ? spmm_split_group(a) : 0;
            if (sg != 0) {
                // Long rows inside column tiles (their gathers are most of the traffic and then hit in the L2s),
                // short rows outside (a pass over them per tile would cost more than their gathers): two launches.
                SpmmArgs longs = a, rest = a;
                longs.blocks.waves = a.blocks.long_waves;
                longs.blocks.n_blocks = a.blocks.n_long_blocks;
                longs.blocks.n_short = 0;
                rest.blocks.waves = a.blocks.rest_waves;
                rest.blocks.n_blocks = a.blocks.n_rest_blocks;
                rest.blocks.n_huge_rows = 0;
                rest.blocks.n_short = 0;
                rest.blocks.n_long_blocks = 0;   // (nothing left to split off)
                rest.blocks.staged_rows = nullptr;
                const hipError_t e = launch_spmm(rest, s);
                if (e != hipSuccess) return e;
                switch (sg) {
                    case 32: return spmm_tiled_go<32>(longs, s);
                    case 16: return spmm_tiled_go<16>(longs, s);
                    default: return spmm_tiled_go<8>(longs, s);
                }
            }
            if (a.blocks.n_short > 0 && tg != 0 && packed_grid(a, tg, true).ids <= kMaxGridIds) {
                switch (tg) {
                    case 32: return spmm_packed_go<32>(a, s);
                    case 16: return spmm_packed_go<16>(a, s);
                    default: return spmm_packed_go<8>(a, s);
                }
            }
            switch (tg) {
                case 32: return spmm_tiled_go<32>(a, s);
                case 16: return spmm_tiled_go<16>(a, s);
                case 8: return spmm_tiled_go<8>(a, s);
                default: break;
            }
            if (a.batch <= 64) return spmm_grouped_go<16>(a, s);
            if (a.batch <= 128) return spmm_grouped_go<32>(a, s);
        }
        if (a.batch <= 256) return spmm_go<4, 1>(a, s);
        if (a.batch <= 512) return spmm_go<4, 2>(a, s);
        return spmm_go<4, 4>(a, s);
    }
    if (a.batch <= 64) return spmm_go<1, 1>(a, s);
    if (a.batch <= 128) return spmm_go<1, 2>(a, s);
    return spmm_go<1, 4>(a, s);
}

// Columns per tile of the column-tiled SDDMM, 0: one pass over the whole batch.
int sddmm_tile_columns(const SddmmArgs &a)
{
    if (!a.partial || a.skip_products || a.dense || !sddmm_vec_ok(a)) return 0;  // (the finish pass does not know an entry's row)
    // the operand rows an entry gathers are named by its column index: the matrix's own partition
    // carries the share of the most referenced ones
    const int w = tile_columns(a.x_rows, a.batch, a.nnz, a.rows, a.blocks.hot_share, false, true);
    if (w == 0) return 0;
    const int n_tiles = (a.batch + w - 1) / w;
    if (n_tiles > a.partial_tiles) return 0;
    if (static_cast<int64_t>(a.blocks.n_blocks) * (n_tiles + 8) >= (1ll << 31)) return 0;
    return w;
}

hipError_t launch_sddmm(const SddmmArgs &a, hipStream_t s)
{
    if (a.rows <= 0 || a.batch <= 0 || a.blocks.n_blocks <= 0) return hipSuccess;
    if (sddmm_full_ok(a)) {
        const int n_chunks = (a.batch + 255) / 256;
        const int groups = (a.x_rows + kWavesPerBlock - 1) / kWavesPerBlock;  // one row of X per wave, up to two rounds of work-groups
        hipLaunchKernelGGL(full_sddmm_kernel<false>, dim3(groups < 1024 ? groups : 1024), dim3(kBlock),
                           static_cast<size_t>(a.rows) * n_chunks * kWave * sizeof(float4), s, a, n_chunks, static_cast<float *>(nullptr), 0);
        return hipGetLastError();
    }
    if (sddmm_staged_ok(a)) {
        const int n_tiles = (a.batch + kStageCols - 1) / kStageCols;
        hipLaunchKernelGGL(sddmm_staged_kernel, dim3(n_tiles * a.blocks.staged_ranges), dim3(kStageWaves * kWave), 0, s, a, n_tiles);
        if (a.blocks.staged_partial) {
            // the rows the plan leaves out: the column-tiled SDDMM on their own partition, same tiles, same partial buffer
            SddmmArgs rest = a;
            rest.blocks.waves = a.blocks.rest_waves;
            rest.blocks.n_blocks = a.blocks.n_rest_blocks;
            const int spread = n_tiles >= 8;
            const int64_t ids = (spread ? static_cast<int64_t>((n_tiles + 7) / 8) * 8 : n_tiles) * rest.blocks.n_blocks;
            hipLaunchKernelGGL((sddmm_tiled_kernel<16, 1, true>), dim3(static_cast<unsigned>(ids)), dim3(kBlock), 0, s, rest, n_tiles, spread);
        }
        const int64_t work = a.nnz > a.rows ? a.nnz : a.rows;
        hipLaunchKernelGGL(sddmm_finish_kernel, dim3(elementwise_blocks(work)), dim3(kEwBlock), 0, s, a, n_tiles);
        return hipGetLastError();
    }
    switch (sddmm_tile_columns(a)) {
        case 128: return sddmm_tiled_go<16, 2>(a, s);
        case 64: return sddmm_tiled_go<16, 1>(a, s);
        case 32: return sddmm_tiled_go<8, 1>(a, s);
        default: break;
    }
    if (sddmm_vec_ok(a) && a.batch <= 1024) {
        if (a.batch <= 64) return sddmm_go<16, 1>(a, s);
        if (a.batch <= 128) return sddmm_go<16, 2>(a, s);
        if (a.batch <= 256) return sddmm_go<16, 4>(a, s);
        if (a.batch <= 512) return sddmm_go<64, 2>(a, s);
        return sddmm_go<64, 4>(a, s);
    }
    hipLaunchKernelGGL(sddmm_generic, dim3(a.blocks.n_blocks), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_momentum(float *w, float *v, const float *g, int64_t n, float lr, float mu, int nesterov,
                           hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int vec4 = aligned16(w) && aligned16(v) && aligned16(g);
    hipLaunchKernelGGL(momentum_kernel, dim3(elementwise_blocks(vec4 ? (n + 3) / 4 : n)), dim3(kEwBlock), 0, s,
                       w, v, g, n, lr, mu, nesterov, vec4);
    return hipGetLastError();
}

hipError_t launch_gather(float *values_t, const float *values, const int32_t *perm, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(gather_kernel, dim3(elementwise_blocks(n)), dim3(kEwBlock), 0, s, values_t, values, perm, n);
    return hipGetLastError();
}

hipError_t launch_softmax_ce(const float *Z, int64_t ldz, const int32_t *labels, int32_t classes, int32_t batch,
                             float *dZ, int64_t lddz, float *loss, hipStream_t s)
{
    int threads = (batch + kWave - 1) / kWave * kWave;
    if (threads > kSoftmaxBlock) threads = kSoftmaxBlock;
    if (classes <= 16)
        hipLaunchKernelGGL(softmax_ce_kernel<16>, dim3(1), dim3(threads), 0, s, Z, ldz, labels, classes, batch, dZ,
                           lddz, loss);
    else
        hipLaunchKernelGGL(softmax_ce_kernel<0>, dim3(1), dim3(threads), 0, s, Z, ldz, labels, classes, batch, dZ,
                           lddz, loss);
    return hipGetLastError();
}

// One work-group re-reads the whole layer for its 4 columns: only for layers of a few thousand entries.
bool head_ok(int32_t rows, int32_t cols, int32_t nnz)
{
    return rows > 0 && rows <= kHeadMaxRows && cols > 0 && nnz <= 8192;
}

hipError_t launch_head(const HeadArgs &a, hipStream_t s)
{
    hipLaunchKernelGGL(head_kernel, dim3((a.batch + kHeadCols - 1) / kHeadCols), dim3(kBlock), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_copy(float *dst, const float *src, int64_t n, hipStream_t s)
{
    if (n <= 0) return hipSuccess;
    const int vec4 = aligned16(dst) && aligned16(src);
    hipLaunchKernelGGL(copy_kernel, dim3(elementwise_blocks(vec4 ? (n + 3) / 4 : n)), dim3(kEwBlock), 0, s, dst, src,
                       n, vec4);
    return hipGetLastError();
}

}  // namespace nerva
