// bb_gemm_static: the library's MFMA GEMM for callers that cannot allocate (HIP graph capture, tight serving
// loops, harnesses that forbid hipMalloc).  Same kernels as the forward's projections and as bb_debug_gemm; the
// buffers those kernels need between them (re-tiled weights, packed hi/lo activation panel, split-K partial
// tiles) live in one file-scope device array instead of a caller's workspace.
#include "bb_internal.h"
#include <mutex>

#define SG_MAX_M 128
#define SG_MAX_N 4096
#define SG_MAX_K 4096
#define SG_MAX_NK (4u << 20)            // N * K (K padded to 64) elements of weights
#define SG_MAX_SPLIT 4
#define SG_W_BYTES ((size_t)SG_MAX_NK * 2)                               // tiled bf16 weights          8 MiB
#define SG_A_BYTES ((size_t)SG_MAX_M * SG_MAX_K * 2 * BB_SPLIT)         // packed hi/lo activations    2 MiB
#define SG_P_BYTES ((size_t)SG_MAX_SPLIT * SG_MAX_M * SG_MAX_N * 4)     // split-K partial tiles       8 MiB
#define SG_BYTES (SG_W_BYTES + SG_A_BYTES + SG_P_BYTES)

// Every GPU the library runs on holds its own copy of this array until the process ends.  In host code the
// name is only a handle for hipGetSymbolAddress: kernels get the address that call returns.
static __device__ __align__(256) unsigned char scratch[SG_BYTES];

#define SG_MAX_DEVICES 64
static unsigned char* g_scratch_ptr[SG_MAX_DEVICES];      // per device, filled on the first call on that device
static std::mutex g_scratch_mutex;

static int scratch_of_current_device(unsigned char** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= SG_MAX_DEVICES) return BB_EHIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return BB_EHIP;
        g_scratch_ptr[dev] = static_cast<unsigned char*>(p);
    }
    *out = g_scratch_ptr[dev];
    return BB_OK;
}

__global__ __launch_bounds__(256) void sg_zero_kernel(u32x4* __restrict__ dst, size_t n) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = z;
}

// C[m][n] = sum over the splits, in split order (the order every consumer of partial tiles in the library uses).
__global__ __launch_bounds__(256) void sg_reduce_kernel(const float* __restrict__ P, float* __restrict__ C, int M, int N,
                                                        int n_split, size_t split_stride) {
    const size_t n = (size_t)M * N;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        float acc = 0.f;
        for (int s = 0; s < n_split; ++s) acc += P[(size_t)s * split_stride + i];
        C[i] = acc;
    }
}

extern "C" int bb_gemm_static(const float* A_dev, const uint16_t* W_dev, float* C_dev, int M, int N, int K, int split_k,
                              void* hip_stream) {
    if (!A_dev || !W_dev || !C_dev) return BB_EINVAL;
    if (M < 1 || N < 32 || K < 16 || N % 32 || K % 16 || split_k < 0) return BB_EINVAL;
    const int Kp = (K + 63) / 64 * 64;
    if (M > SG_MAX_M || N > SG_MAX_N || K > SG_MAX_K || (size_t)N * Kp > SG_MAX_NK || split_k > SG_MAX_SPLIT) return BB_ENOMEM;
    if ((uintptr_t)A_dev % 4 || (uintptr_t)W_dev % 16 || (uintptr_t)C_dev % 4) return BB_EINVAL;
    unsigned char* base = nullptr;
    int rc = scratch_of_current_device(&base);
    if (rc != BB_OK) return rc;
    hipStream_t s = (hipStream_t)hip_stream;
    u32x4* Wt = reinterpret_cast<u32x4*>(base);
    u32x4* Apk = reinterpret_cast<u32x4*>(base + SG_W_BYTES);
    float* P = reinterpret_cast<float*>(base + SG_W_BYTES + SG_A_BYTES);
    const int mt = (M + 31) / 32, rows_pad = mt * 32;
    GemmPlan p = gemm_plan(M, N, K, split_k, 0);
    if (p.split_k > SG_MAX_SPLIT) p = gemm_plan(M, N, K, SG_MAX_SPLIT, 0);
    if (p.split_k > SG_MAX_SPLIT || (size_t)p.split_k * rows_pad * N * 4 > SG_P_BYTES) return BB_ENOMEM;
    // the array keeps the last call's contents: the k padding of the tiled weights must read as zero
    if (Kp != K) {
        const size_t n16 = (size_t)N * Kp * 2 / 16;
        sg_zero_kernel<<<(unsigned)std::min<size_t>((n16 + 255) / 256, 2048), 256, 0, s>>>(Wt, n16);
    }
    launch_tile_weights(W_dev, N, K, Wt, 0, 0, s);
    launch_pack_rows(A_dev, M, K, Apk, mt, s);
    launch_gemm(Wt, Apk, P, mt, N, K, p, s);
    const size_t n = (size_t)M * N;
    sg_reduce_kernel<<<(unsigned)std::min<size_t>((n + 255) / 256, 2048), 256, 0, s>>>(P, C_dev, M, N, p.split_k, (size_t)rows_pad * N);
    return hipGetLastError() == hipSuccess ? BB_OK : BB_EHIP;
}
