// hbm_calib: plain streaming kernels of known size, used to (1) scale the rocprofv3 FETCH_SIZE /
// WRITE_SIZE counters to bytes and (2) show what a simple reader reaches on this GPU.
//   hbm_calib copy <MiB> [iters]   : out[i] = in[i], reads N and writes N bytes per launch
//   hbm_calib read <MiB> [iters]   : every lane sums its 128-bit loads; one 4-byte store per workgroup
//   hbm_calib readnt <MiB> [iters] : the same with non-temporal (streaming) loads
//   hbm_calib pages <MiB> [iters] [workgroups] : non-temporal reads of whole 16 KiB pages visited in a
//                                    seeded random order (the access pattern of a fragmented page pool)
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>
#include <cstring>

#define CHECK(x)                                                                                   \
    do {                                                                                           \
        hipError_t e_ = (x);                                                                       \
        if (e_ != hipSuccess) {                                                                    \
            std::fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));                    \
            std::exit(1);                                                                          \
        }                                                                                          \
    } while (0)

__global__ void __launch_bounds__(256) copy_kernel(const uint4 *__restrict__ in, uint4 *__restrict__ out, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
        out[i] = in[i];
}

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

template <bool NT>
__device__ __forceinline__ u32x4 ld(const uint4 *p) {
    const u32x4 *q = reinterpret_cast<const u32x4 *>(p);
    return NT ? __builtin_nontemporal_load(q) : *q;
}

template <bool NT>
__global__ void __launch_bounds__(256) read_kernel(const uint4 *__restrict__ in, unsigned *__restrict__ out, size_t n) {
    const size_t stride = (size_t)gridDim.x * blockDim.x * 4;
    unsigned acc = 0;
    size_t i = ((size_t)blockIdx.x * blockDim.x) * 4 + threadIdx.x;
    for (; i + 3 * 256 < n; i += stride) {
        const u32x4 a = ld<NT>(in + i), b = ld<NT>(in + i + 256), c = ld<NT>(in + i + 512), d = ld<NT>(in + i + 768);
        acc += a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    __shared__ unsigned sh[256];
    sh[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned s = 0;
        for (int k = 0; k < 256; ++k)
            s += sh[k];
        out[blockIdx.x] = s;
    }
}

// Each workgroup reads whole 16 KiB pages (1024 x 16 B: four loads per lane) named by `order`.
__global__ void __launch_bounds__(256) pages_kernel(const uint4 *__restrict__ in, const unsigned *__restrict__ order,
                                                    unsigned *__restrict__ out, unsigned n_pages) {
    unsigned acc = 0;
    for (unsigned i = blockIdx.x; i < n_pages; i += gridDim.x) {
        const uint4 *pg = in + (size_t)order[i] * 1024 + threadIdx.x;
        const u32x4 a = ld<true>(pg), b = ld<true>(pg + 256), c = ld<true>(pg + 512), d = ld<true>(pg + 768);
        acc += a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    __shared__ unsigned sh[256];
    sh[threadIdx.x] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned s = 0;
        for (int k = 0; k < 256; ++k)
            s += sh[k];
        out[blockIdx.x] = s;
    }
}

int main(int argc, char **argv) {
    if (argc < 3) {
        std::fprintf(stderr, "usage: hbm_calib copy|read|readnt|pages <MiB> [iters] [workgroups]\n");
        return 2;
    }
    const bool copy = std::strcmp(argv[1], "copy") == 0;
    const bool nt = std::strcmp(argv[1], "readnt") == 0;
    const bool pages = std::strcmp(argv[1], "pages") == 0;
    const size_t bytes = (size_t)std::atoll(argv[2]) << 20;
    const int iters = argc > 3 ? std::atoi(argv[3]) : 10;
    const int wgs = argc > 4 ? std::atoi(argv[4]) : 256 * 16;
    const size_t n = bytes / 16;
    if (n % (1024) != 0 || n == 0) {
        std::fprintf(stderr, "size must be a positive multiple of 16 KiB\n");
        return 2;
    }
    uint4 *in = nullptr, *out = nullptr;
    CHECK(hipMalloc(&in, bytes));
    CHECK(hipMalloc(&out, copy ? bytes : (size_t)wgs * 4 + 256));
    CHECK(hipMemset(in, 1, bytes));
    unsigned *order = nullptr;
    const unsigned n_pages = (unsigned)(bytes / 16384);
    if (pages) { // Fisher-Yates with a fixed 64-bit LCG
        unsigned *h = (unsigned *)std::malloc(sizeof(unsigned) * n_pages);
        for (unsigned i = 0; i < n_pages; ++i)
            h[i] = i;
        unsigned long long st = 0x9E3779B97F4A7C15ull;
        for (unsigned i = n_pages - 1; i > 0; --i) {
            st = st * 6364136223846793005ull + 1442695040888963407ull;
            const unsigned j = (unsigned)((st >> 33) % (i + 1));
            const unsigned t = h[i];
            h[i] = h[j];
            h[j] = t;
        }
        CHECK(hipMalloc(&order, sizeof(unsigned) * n_pages));
        CHECK(hipMemcpy(order, h, sizeof(unsigned) * n_pages, hipMemcpyHostToDevice));
        std::free(h);
    }
    hipEvent_t a, b;
    CHECK(hipEventCreate(&a));
    CHECK(hipEventCreate(&b));
    float best = 1e30f, sum = 0.f;
    for (int it = 0; it < iters + 2; ++it) {
        CHECK(hipEventRecord(a, 0));
        if (copy)
            hipLaunchKernelGGL(copy_kernel, dim3(wgs), dim3(256), 0, 0, in, out, n);
        else if (pages)
            hipLaunchKernelGGL(pages_kernel, dim3(wgs), dim3(256), 0, 0, in, order, (unsigned *)out, n_pages);
        else if (nt)
            hipLaunchKernelGGL(read_kernel<true>, dim3(wgs), dim3(256), 0, 0, in, (unsigned *)out, n);
        else
            hipLaunchKernelGGL(read_kernel<false>, dim3(wgs), dim3(256), 0, 0, in, (unsigned *)out, n);
        CHECK(hipGetLastError());
        CHECK(hipEventRecord(b, 0));
        CHECK(hipEventSynchronize(b));
        float ms = 0.f;
        CHECK(hipEventElapsedTime(&ms, a, b));
        if (it >= 2) {
            best = ms < best ? ms : best;
            sum += ms;
        }
    }
    const double moved = copy ? 2.0 * bytes : (double)bytes;
    std::printf("%s bytes_read=%zu bytes_written=%zu iters=%d mean_ms=%.4f best_ms=%.4f mean_GBs=%.1f best_GBs=%.1f\n",
                copy ? "copy" : (pages ? "pages" : (nt ? "readnt" : "read")), bytes, copy ? bytes : (size_t)wgs * 4, iters, sum / iters, best,
                moved / (sum / iters * 1e-3) / 1e9, moved / (best * 1e-3) / 1e9);
    CHECK(hipFree(in));
    CHECK(hipFree(out));
    return 0;
}
