// Stand-alone measurement of what bounds the sparse kernels on one GPU: the rate at which a
// compute unit can gather rows of a cache-resident dense matrix (the inner operation of SpMM
// and SDDMM), as a function of how many lanes of a 16-byte-per-lane load take part, next to a
// plain streaming read and to the same gather out of LDS.  Prints one line per case.
//
//   hipcc --offload-arch=gfx950 -O3 microbench_gather.hip -o microbench_gather && ./microbench_gather
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <vector>

#define CHECK(x)                                                                   \
    do {                                                                           \
        hipError_t e_ = (x);                                                       \
        if (e_ != hipSuccess) {                                                    \
            printf("HIP error %s at line %d\n", hipGetErrorString(e_), __LINE__); \
            exit(1);                                                               \
        }                                                                          \
    } while (0)

constexpr int kRows = 3072, kLd = 128;  // 1.5 MiB: resident in every L2

// every wave reads `per_wave` rows named by idx[], U loads in flight, `lanes` lanes x 16 B each
template <int U>
__global__ __launch_bounds__(1024) void gather_l2(const float *__restrict__ X, const int *__restrict__ idx, int per_wave,
                                                  int lanes, float *out)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>((blockIdx.x * blockDim.x + threadIdx.x) >> 6));
    const int *my = idx + static_cast<size_t>(wave) * per_wave;
    float4 acc = make_float4(0, 0, 0, 0);
    if (lane < lanes) {
        const int off = lane * 4;
        for (int p = 0; p + U <= per_wave; p += U) {
            int j[U];
#pragma unroll
            for (int u = 0; u < U; ++u) j[u] = my[p + u];
            float4 x[U];
#pragma unroll
            for (int u = 0; u < U; ++u) x[u] = *reinterpret_cast<const float4 *>(X + static_cast<size_t>(j[u]) * kLd + off);
#pragma unroll
            for (int u = 0; u < U; ++u) { acc.x += x[u].x; acc.y += x[u].y; acc.z += x[u].z; acc.w += x[u].w; }
        }
    }
    if (acc.x == 12345.f) out[wave] = acc.x + acc.y + acc.z + acc.w;
}

// every work-group streams `reps` contiguous panels of panel_floats floats
__global__ __launch_bounds__(1024) void stream_l2(const float *__restrict__ X, size_t total_floats, int panel_floats,
                                                  float *out, int reps)
{
    float4 acc = make_float4(0, 0, 0, 0);
    for (int r = 0; r < reps; ++r) {
        const size_t base = (static_cast<size_t>(blockIdx.x + r * 7) * panel_floats) % total_floats;
        for (int i = threadIdx.x * 4; i < panel_floats; i += 1024 * 4) {
            const float4 a = *reinterpret_cast<const float4 *>(X + base + i);
            acc.x += a.x; acc.y += a.y; acc.z += a.z; acc.w += a.w;
        }
    }
    if (acc.x == 12345.f) out[blockIdx.x] = acc.x + acc.y;
}

// the same gather out of a 256-row panel held in LDS (128 KiB), VEC floats per lane
template <int VEC>
__global__ __launch_bounds__(1024) void gather_lds(const int *__restrict__ idx, int per_wave, int lanes, float *out)
{
    extern __shared__ float lds[];
    for (int i = threadIdx.x; i < 256 * kLd; i += 1024) lds[i] = static_cast<float>(i);
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(static_cast<int>((blockIdx.x * blockDim.x + threadIdx.x) >> 6));
    const int *my = idx + static_cast<size_t>(wave) * per_wave;
    float acc = 0;
    if (lane < lanes) {
        const int off = lane * VEC;
        for (int p = 0; p + 8 <= per_wave; p += 8) {
            int j[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) j[u] = my[p + u] & 255;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                if constexpr (VEC == 4) { const float4 x = *reinterpret_cast<const float4 *>(lds + j[u] * kLd + off); acc += x.x + x.y + x.z + x.w; }
                else if constexpr (VEC == 2) { const float2 x = *reinterpret_cast<const float2 *>(lds + j[u] * kLd + off); acc += x.x + x.y; }
                else acc += lds[j[u] * kLd + off];
            }
        }
    }
    if (acc == 12345.f) out[wave] = acc;
}

template <typename F>
float time_us(F launch)
{
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    launch();  // warm-up
    CHECK(hipEventRecord(e0));
    launch();
    CHECK(hipEventRecord(e1));
    CHECK(hipEventSynchronize(e1));
    float ms = 0;
    CHECK(hipEventElapsedTime(&ms, e0, e1));
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return ms * 1e3f;
}

int main()
{
    float *X, *out;
    CHECK(hipMalloc(&X, static_cast<size_t>(kRows) * kLd * 4));
    CHECK(hipMemset(X, 0, static_cast<size_t>(kRows) * kLd * 4));
    CHECK(hipMalloc(&out, 1 << 22));
    const int blocks = 2048, per_wave = 256, waves = blocks * 16;
    std::vector<int> h(static_cast<size_t>(waves) * per_wave);
    srand(1);
    for (auto &v : h) v = rand() % kRows;
    int *idx;
    CHECK(hipMalloc(&idx, h.size() * 4));
    CHECK(hipMemcpy(idx, h.data(), h.size() * 4, hipMemcpyHostToDevice));
    const double gathers = static_cast<double>(waves) * per_wave;
    for (int lanes : {16, 25, 32, 48, 64}) {
        const float us = time_us([&] { hipLaunchKernelGGL(gather_l2<8>, dim3(blocks), dim3(1024), 0, 0, X, idx, per_wave, lanes, out); });
        printf("L2 gather, %2d lanes x 16 B per row read: %8.1f us  %6.2f TB/s useful  %6.2f G row reads/s\n", lanes, us,
               gathers * lanes * 16 / us / 1e6, gathers / us / 1e3);
    }
    for (int vec : {1, 2, 4}) {
        const int lanes = 64;
        float us;
        if (vec == 4) us = time_us([&] { hipLaunchKernelGGL(gather_lds<4>, dim3(blocks), dim3(1024), 131072, 0, idx, per_wave, lanes, out); });
        else if (vec == 2) us = time_us([&] { hipLaunchKernelGGL(gather_lds<2>, dim3(blocks), dim3(1024), 131072, 0, idx, per_wave, lanes, out); });
        else us = time_us([&] { hipLaunchKernelGGL(gather_lds<1>, dim3(blocks), dim3(1024), 131072, 0, idx, per_wave, lanes, out); });
        printf("LDS gather, 64 lanes x %2d B per row read:  %8.1f us  %6.2f TB/s useful\n", vec * 4, us, gathers * lanes * vec * 4 / us / 1e6);
    }
    for (int reps : {1, 4, 16}) {
        const int panel = 128 * 256;  // 128 KiB
        const float us = time_us([&] { hipLaunchKernelGGL(stream_l2, dim3(1024), dim3(1024), 0, 0, X, static_cast<size_t>(kRows) * kLd - panel, panel, out, reps); });
        printf("L2 stream, 1024 work-groups x %2d panels of 128 KiB: %8.1f us  %6.2f TB/s\n", reps, us, 1024.0 * panel * 4 * reps / us / 1e6);
    }
    return 0;
}
