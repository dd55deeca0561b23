// Memory-system ceilings of the GPU for the access patterns of the feature kernels, measured with kernels
// that do nothing else: streaming read, streaming copy, and reads of whole feature rows picked at random
// from matrices of different sizes (one that the L2s partly hold, one the size of a gathered mini-batch
// matrix, one the size of a feature table).  The figures bound what the gather and the mean aggregation can
// reach on this machine whatever their code looks like; they are printed as a markdown table.
//
//   zg_ceilings [row_floats=600] [row_reads=102000]
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CK(x)                                                                          \
    do {                                                                               \
        hipError_t e_ = (x);                                                           \
        if (e_ != hipSuccess) {                                                        \
            std::fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_));               \
            std::exit(1);                                                              \
        }                                                                              \
    } while (0)

typedef float v4f __attribute__((ext_vector_type(4)));

// every lane reads four 16-byte pieces a round, 1 KB apart per wave; the impossible comparison keeps the loads alive
__global__ __launch_bounds__(256) void k_stream_read(const v4f *__restrict__ p, size_t n4, float *sink)
{
    v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
    const size_t stride = (size_t)gridDim.x * 1024;
    for (size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x; i + 768 < n4; i += stride) acc += p[i] + p[i + 256] + p[i + 512] + p[i + 768];
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[0] = 1.0f;
}

__global__ __launch_bounds__(256) void k_stream_copy(const v4f *__restrict__ p, v4f *__restrict__ q, size_t n4)
{
    const size_t stride = (size_t)gridDim.x * 1024;
    for (size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x; i + 768 < n4; i += stride) {
        const v4f a = p[i], b = p[i + 256], c = p[i + 512], d = p[i + 768];
        q[i] = a;
        q[i + 256] = b;
        q[i + 512] = c;
        q[i + 768] = d;
    }
}

// a workgroup reads `per_group` whole rows (ids[group * per_group ...]) as one flat run of 16-byte pieces
__global__ __launch_bounds__(256) void k_random_rows(const v4f *__restrict__ X, const int *__restrict__ ids, int reads, int row4,
                                                     int per_group, float *sink)
{
    v4f acc = {0.0f, 0.0f, 0.0f, 0.0f};
    const int first = blockIdx.x * per_group;
    const int total = per_group * row4;
    for (int e = threadIdx.x; e < total; e += 1024) {
        v4f v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ee = e + u * 256;
            v[u] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
            if (ee < total) {
                const int r = ee / row4, c = ee - r * row4;
                if (first + r < reads) v[u] = X[(size_t)ids[first + r] * row4 + c];
            }
        }
        acc += v[0] + v[1] + v[2] + v[3];
    }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[0] = 1.0f;
}

template <typename F> static double best_us(hipStream_t st, F launch)
{
    hipEvent_t a, b;
    CK(hipEventCreate(&a));
    CK(hipEventCreate(&b));
    launch();
    CK(hipStreamSynchronize(st));
    double best = 1e30;
    for (int t = 0; t < 3; ++t) {
        CK(hipEventRecord(a, st));
        for (int i = 0; i < 20; ++i) launch();
        CK(hipEventRecord(b, st));
        CK(hipEventSynchronize(b));
        float ms = 0.0f;
        CK(hipEventElapsedTime(&ms, a, b));
        if (ms * 50.0 < best) best = ms * 50.0; // ms / 20 launches, in us
    }
    CK(hipEventDestroy(a));
    CK(hipEventDestroy(b));
    return best;
}

int main(int argc, char **argv)
{
    const int row_floats = argc > 1 ? std::atoi(argv[1]) : 600;
    const int reads = argc > 2 ? std::atoi(argv[2]) : 102000;
    if (row_floats < 4 || row_floats % 4 || row_floats > 32768 || reads < 1 || reads > (1 << 24)) {
        std::fprintf(stderr, "row_floats must be a multiple of 4 in 4..32768, row_reads in 1..2^24\n");
        return 2;
    }
    const int row4 = row_floats / 4;
    hipStream_t st;
    CK(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
    float *sink;
    CK(hipMalloc(&sink, 256));
    const size_t big = (size_t)1 << 30;
    v4f *A, *B;
    CK(hipMalloc(&A, big));
    CK(hipMalloc(&B, big));
    CK(hipMemset(A, 1, big));
    CK(hipMemset(B, 0, big));
    std::printf("| pattern | bytes moved | us | TB/s |\n|---|---|---|---|\n");
    const size_t sizes[3] = {(size_t)92 << 20, (size_t)600 << 20, big};
    for (size_t bytes : sizes) {
        const size_t n4 = bytes / 16;
        double us = best_us(st, [&] { hipLaunchKernelGGL(k_stream_read, dim3(8192), dim3(256), 0, st, A, n4, sink); });
        std::printf("| streaming read, %zu MiB buffer | %.0f MB | %.1f | %.2f |\n", bytes >> 20, bytes / 1e6, us, bytes / us / 1e6);
        us = best_us(st, [&] { hipLaunchKernelGGL(k_stream_copy, dim3(8192), dim3(256), 0, st, A, B, n4); });
        std::printf("| streaming copy, %zu MiB buffer | %.0f MB read + as many written | %.1f | %.2f |\n", bytes >> 20, bytes / 1e6, us,
                    2.0 * bytes / us / 1e6);
        std::fflush(stdout);
    }
    const size_t row_bytes = (size_t)row_floats * 4;
    const int sets[3] = {(int)(((size_t)16 << 20) / row_bytes), (int)(((size_t)92 << 20) / row_bytes), (int)(((size_t)600 << 20) / row_bytes)};
    std::vector<int> ids((size_t)reads);
    int *d_ids;
    CK(hipMalloc(&d_ids, (size_t)reads * 4));
    for (int rows_in_set : sets) {
        if ((size_t)rows_in_set * row_bytes > big || rows_in_set < 1) continue;
        uint64_t s = 88172645463325252ull; // xorshift64
        for (int i = 0; i < reads; ++i) {
            s ^= s << 13;
            s ^= s >> 7;
            s ^= s << 17;
            ids[(size_t)i] = (int)(s % (uint64_t)rows_in_set);
        }
        CK(hipMemcpy(d_ids, ids.data(), (size_t)reads * 4, hipMemcpyHostToDevice));
        const int per_group = 8;
        const int grid = (reads + per_group - 1) / per_group;
        const double us = best_us(st, [&] { hipLaunchKernelGGL(k_random_rows, dim3(grid), dim3(256), 0, st, A, d_ids, reads, row4, per_group, sink); });
        const double bytes = (double)reads * (double)row_bytes;
        std::printf("| %d random rows of %zu B out of %d (%.0f MB) | %.0f MB | %.1f | %.2f |\n", reads, row_bytes, rows_in_set,
                    rows_in_set * (double)row_bytes / 1e6, bytes / 1e6, us, bytes / us / 1e6);
        std::fflush(stdout);
    }
    return 0;
}
