// LDS gather rate of the staged product's inner loop, alone.  A work-group copies 512 operand rows x
// 64 columns (128 KiB) into LDS; its 16 waves then gather rows from the copy by index, 16 lanes per
// row and a float4 per lane, four rows side by side per wave, with the (index, weight) pairs loaded
// one per lane and handed to the other lanes of a row by DPP row broadcast (row_newbcast).  NSTEP of
// the 16 entries a chunk holds are served; with few steps per chunk the loop is bound by the chunk
// loads instead of the LDS.  Prints microseconds and bytes gathered per second, and checks the sums
// of sampled waves against the host.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <utility>
#define CHECK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); exit(1);} } while (0)
typedef float v4f __attribute__((ext_vector_type(4)));
constexpr int CB = 512, TW = 64;

template <int I> __device__ __forceinline__ int bcast_i(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x150 + I, 0xf, 0xf, false); }

template <int I> __device__ __forceinline__ void step(const char *lds, int my_off, float my_w, int lig16, v4f &acc)
{
    const int off = bcast_i<I>(my_off);
    const float w = __builtin_bit_cast(float, bcast_i<I>(__builtin_bit_cast(int, my_w)));
    const v4f x = *reinterpret_cast<const v4f *>(lds + off + lig16);
    acc.x = fmaf(w, x.x, acc.x); acc.y = fmaf(w, x.y, acc.y); acc.z = fmaf(w, x.z, acc.z); acc.w = fmaf(w, x.w, acc.w);
}
template <int... I> __device__ __forceinline__ void steps(const char *lds, int my_off, float my_w, int lig16, v4f &acc, std::integer_sequence<int, I...>)
{
    (step<I>(lds, my_off, my_w, lig16, acc), ...);
}

template <int NSTEP>
__global__ __launch_bounds__(1024) void k(const float *X, const int *idx, const float *wts, int chunks, float *out)
{
    __shared__ v4f tile[CB * TW / 4];
    const int lane = threadIdx.x & 63;
    const int wv = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < CB * TW / 4; i += 1024) tile[i] = reinterpret_cast<const v4f *>(X)[i];
    __syncthreads();
    const int wave = blockIdx.x * 16 + wv;
    const int *my = idx + (size_t)wave * chunks * 64;
    const float *mw = wts + (size_t)wave * chunks * 64;
    const int slot = (lane & 15) * 4 + (lane >> 4);  // entry of the chunk this lane holds
    const int lig16 = (lane & 15) * 16;
    v4f acc = {0, 0, 0, 0};
    const char *lds = reinterpret_cast<const char *>(tile);
    int j = my[slot]; float w = mw[slot];
    for (int c = 0; c < chunks; ++c) {
        const int cn = c + 1 < chunks ? c + 1 : c;
        const int jn = my[cn * 64 + slot]; const float wn = mw[cn * 64 + slot];
        steps(lds, j * (TW * 4), w, lig16, acc, std::make_integer_sequence<int, NSTEP>{});
        j = jn; w = wn;
    }
    // rows of 16 lanes hold partial sums over their entries: add the four rows
    float4 r;
    r.x = acc.x + __shfl_xor(acc.x, 16) ; r.y = acc.y + __shfl_xor(acc.y, 16); r.z = acc.z + __shfl_xor(acc.z, 16); r.w = acc.w + __shfl_xor(acc.w, 16);
    r.x += __shfl_xor(r.x, 32); r.y += __shfl_xor(r.y, 32); r.z += __shfl_xor(r.z, 32); r.w += __shfl_xor(r.w, 32);
    if (lane < 16) reinterpret_cast<float4 *>(out)[(size_t)wave * 16 + lane] = r;
}

template <int NSTEP> void run(int blocks, int chunks, bool verify)
{
    const int waves = blocks * 16;
    std::vector<float> X(CB * TW); for (size_t i = 0; i < X.size(); ++i) X[i] = (float)((i * 2654435761u >> 8) & 1023) / 512.f - 1.f;
    std::vector<int> idx((size_t)waves * chunks * 64); std::vector<float> w(idx.size());
    uint32_t s = 12345;
    for (size_t i = 0; i < idx.size(); ++i) { s = s * 1664525u + 1013904223u; idx[i] = (s >> 10) % CB; w[i] = (float)((s >> 20) & 255) / 256.f; }
    float *dX, *dw, *dout; int *didx;
    CHECK(hipMalloc(&dX, X.size() * 4)); CHECK(hipMalloc(&dw, w.size() * 4)); CHECK(hipMalloc(&didx, idx.size() * 4)); CHECK(hipMalloc(&dout, (size_t)waves * 64 * 4));
    CHECK(hipMemcpy(dX, X.data(), X.size() * 4, hipMemcpyHostToDevice)); CHECK(hipMemcpy(dw, w.data(), w.size() * 4, hipMemcpyHostToDevice)); CHECK(hipMemcpy(didx, idx.data(), idx.size() * 4, hipMemcpyHostToDevice));
    hipEvent_t e0, e1; CHECK(hipEventCreate(&e0)); CHECK(hipEventCreate(&e1));
    auto launch = [&] { hipLaunchKernelGGL(k<NSTEP>, dim3(blocks), dim3(1024), 0, 0, dX, didx, dw, chunks, dout); };
    launch(); launch(); CHECK(hipDeviceSynchronize());
    CHECK(hipEventRecord(e0)); launch(); CHECK(hipEventRecord(e1)); CHECK(hipEventSynchronize(e1));
    float ms = 0; CHECK(hipEventElapsedTime(&ms, e0, e1));
    const double bytes = (double)waves * chunks * NSTEP * 4 * TW * 4;
    printf("NSTEP %2d blocks %d chunks %d: %.1f us, %.1f TB/s gathered from LDS\n", NSTEP, blocks, chunks, ms * 1e3, bytes / (ms * 1e-3) / 1e12);
    if (verify) {
        std::vector<float> out((size_t)waves * 64); CHECK(hipMemcpy(out.data(), dout, out.size() * 4, hipMemcpyDeviceToHost));
        double worst = 0;
        for (int wvi = 0; wvi < waves; wvi += 97) {
            std::vector<double> ref(TW, 0.0);
            for (int c = 0; c < chunks; ++c) for (int e = 0; e < NSTEP * 4; ++e) {
                const size_t p = ((size_t)wvi * chunks + c) * 64 + e;
                for (int t = 0; t < TW; ++t) ref[t] += (double)w[p] * X[(size_t)idx[p] * TW + t];
            }
            for (int t = 0; t < TW; ++t) { const double d = fabs(ref[t] - out[(size_t)wvi * 64 + t]) / (fabs(ref[t]) + 1.0); if (d > worst) worst = d; }
        }
        printf("   worst relative difference to the host sum: %.2e\n", worst);
    }
    CHECK(hipFree(dX)); CHECK(hipFree(dw)); CHECK(hipFree(didx)); CHECK(hipFree(dout));
}

int main()
{
    run<16>(256, 64, true);
    run<16>(256, 256, false);
    run<16>(512, 128, false);
    run<4>(256, 256, true);
    run<2>(256, 256, false);
    run<1>(256, 256, false);
    return 0;
}
