// bf16 MFMA GEMM for the projection, FFN and LM-head contractions:
//     C[m][n] = sum_k A[m][k] * W[n][k]          (fp32 accumulate)
// A is the activation panel (branch rows folded into m), held as two bf16 terms hi + lo per
// element so the product keeps ~16 significant bits of the activation; W are the bf16
// weights.  The kernel computes C^T tiles: the weight fragment is the MFMA A-operand
// (32 weight rows x 16 k) and the activation fragment the B-operand (16 k x 32 rows), so a
// wave streams its weight rows from HBM exactly once, in 1 KiB fragments that were laid out
// in lane order when the weights were loaded, while the (small) activation panel is staged
// through LDS and shared by the four waves of a workgroup.  With few activation rows the k range
// is split over several workgroups to occupy every CU; each writes its partial tile and the
// consumer kernel (residual + norm, SwiGLU, bias + RoPE + cache write) sums them in split order.
#include "bb_internal.h"

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define KC 4        // k-steps (of 16) per LDS chunk
#define MT 4        // m-tiles (of 32 rows) per workgroup
#define CHUNK_U4 (KC * MT * BB_SPLIT * 64)      // u32x4 per staged chunk (2048 = 32 KiB)

static __device__ __forceinline__ bf16x8 as_bf16x8(const u32x4& v) {
    return *reinterpret_cast<const bf16x8*>(&v);
}

template <int NT>
static __device__ __forceinline__ void load_w(u32x4 (&w)[KC][NT], const u32x4* __restrict__ Wt, const int (&nt)[NT],
                                              int ksteps, int ks0, int lane) {
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int k = 0; k < KC; ++k) {
            int ks = ks0 + k < ksteps ? ks0 + k : ksteps - 1;      // clamped; the product is skipped later
            w[k][t] = __builtin_nontemporal_load(&Wt[((size_t)nt[t] * ksteps + ks) * 64 + lane]);
        }
}

static __device__ __forceinline__ void load_a(u32x4 (&a)[CHUNK_U4 / 256], const u32x4* __restrict__ Apk, int mt_total,
                                              int mt0, int mt_cnt, int ksteps, int ks0) {
#pragma unroll
    for (int i = 0; i < CHUNK_U4 / 256; ++i) {
        int idx = i * 256 + threadIdx.x;
        int k = idx / (MT * BB_SPLIT * 64), rem = idx % (MT * BB_SPLIT * 64);
        int mt = rem / (BB_SPLIT * 64), tl = rem % (BB_SPLIT * 64);
        u32x4 v = u32x4{0u, 0u, 0u, 0u};
        if (mt < mt_cnt && ks0 + k < ksteps)
            v = Apk[((size_t)(ks0 + k) * mt_total + mt0 + mt) * (BB_SPLIT * 64) + tl];
        a[i] = v;
    }
}

template <int NT>
static __device__ __forceinline__ void compute_chunk(f32x16 (&acc)[NT][MT], const u32x4 (&w)[KC][NT], const u32x4* lds,
                                                     int mt_cnt, int kvalid, int lane) {
#pragma unroll
    for (int k = 0; k < KC; ++k) {
        if (k < kvalid) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if (mt < mt_cnt) {
#pragma unroll
                    for (int term = 0; term < BB_SPLIT; ++term) {
                        u32x4 b = lds[((k * MT + mt) * BB_SPLIT + term) * 64 + lane];
#pragma unroll
                        for (int t = 0; t < NT; ++t)
                            acc[t][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(w[k][t]), as_bf16x8(b),
                                                                                acc[t][mt], 0, 0, 0);
                    }
                }
            }
        }
    }
}

// P[split][m][n] (fp32, leading dimension ldp) = this workgroup's share of the k range.
template <int NT>
__global__ __launch_bounds__(256) void gemm_kernel(const u32x4* __restrict__ Wt, const u32x4* __restrict__ Apk,
                                                   float* __restrict__ P, size_t split_stride, int ldp, int mt_total,
                                                   int n_tiles, int ksteps, int chunks_per_split) {
    __shared__ u32x4 lds[2][CHUNK_U4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int mt0 = blockIdx.y * MT;
    const int mt_cnt = min(MT, mt_total - mt0);
    const int total_chunks = (ksteps + KC - 1) / KC;
    const int c0 = blockIdx.z * chunks_per_split;
    const int c1 = min(c0 + chunks_per_split, total_chunks);
    int nt[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int x = (blockIdx.x * 4 + wave) * NT + t;
        nt[t] = x < n_tiles ? x : n_tiles - 1;          // clamped loads; stores are guarded
    }
    f32x16 acc[NT][MT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][mt][r] = 0.f;

    u32x4 w0[KC][NT], w1[KC][NT], a[CHUNK_U4 / 256];
    if (c0 < c1) {
        load_a(a, Apk, mt_total, mt0, mt_cnt, ksteps, c0 * KC);
        load_w<NT>(w0, Wt, nt, ksteps, c0 * KC, lane);
#pragma unroll
        for (int i = 0; i < CHUNK_U4 / 256; ++i) lds[0][i * 256 + threadIdx.x] = a[i];
    }
    __syncthreads();
    for (int c = c0; c < c1; c += 2) {
        // even chunk: data in lds[0] / w0, prefetch into lds[1] / w1
        bool more = c + 1 < c1;
        if (more) {
            load_a(a, Apk, mt_total, mt0, mt_cnt, ksteps, (c + 1) * KC);
            load_w<NT>(w1, Wt, nt, ksteps, (c + 1) * KC, lane);
        }
        compute_chunk<NT>(acc, w0, lds[0], mt_cnt, min(KC, ksteps - c * KC), lane);
        if (more) {
#pragma unroll
            for (int i = 0; i < CHUNK_U4 / 256; ++i) lds[1][i * 256 + threadIdx.x] = a[i];
        }
        __syncthreads();
        if (!more) break;
        // odd chunk: data in lds[1] / w1, prefetch into lds[0] / w0
        more = c + 2 < c1;
        if (more) {
            load_a(a, Apk, mt_total, mt0, mt_cnt, ksteps, (c + 2) * KC);
            load_w<NT>(w0, Wt, nt, ksteps, (c + 2) * KC, lane);
        }
        compute_chunk<NT>(acc, w1, lds[1], mt_cnt, min(KC, ksteps - (c + 1) * KC), lane);
        if (more) {
#pragma unroll
            for (int i = 0; i < CHUNK_U4 / 256; ++i) lds[0][i * 256 + threadIdx.x] = a[i];
        }
        __syncthreads();
    }
    // C^T accumulator layout of the 32x32 MFMA: register r of lane l holds
    //   weight row n = 8*(r/4) + 4*(l/32) + r%4 of the tile, activation row m = l%32.
    float* Ps = P + (size_t)blockIdx.z * split_stride;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int x = (blockIdx.x * 4 + wave) * NT + t;
        if (x >= n_tiles) continue;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            if (mt >= mt_cnt) continue;
            size_t m = (size_t)(mt0 + mt) * 32 + (lane & 31);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                int n = x * 32 + 8 * q + 4 * (lane >> 5);
                float4 v = make_float4(acc[t][mt][4 * q], acc[t][mt][4 * q + 1], acc[t][mt][4 * q + 2], acc[t][mt][4 * q + 3]);
                *reinterpret_cast<float4*>(&Ps[m * ldp + n]) = v;
            }
        }
    }
}

// nt: weight tiles of 32 rows per wave (workgroup tile = 128 * nt columns); forced values <= 0 = choose.
GemmPlan gemm_plan(int m_rows, int N, int K, int forced_split, int forced_nt) {
    const int n_tiles = N / 32, mt_total = (m_rows + 31) / 32, ksteps = K / 16;
    const int m_groups = (mt_total + MT - 1) / MT, total_chunks = (ksteps + KC - 1) / KC;
    GemmPlan p;
    p.nt = forced_nt > 0 ? forced_nt : (n_tiles >= 8 ? 2 : 1);
    if (forced_nt <= 0 && m_groups == 1 && N <= 8192) p.nt = 1;     // few columns: narrower tiles, fewer splits
    if (p.nt == 2 && n_tiles < 8) p.nt = 1;
    const int n_groups = (n_tiles + 4 * p.nt - 1) / (4 * p.nt), base = n_groups * m_groups;
    int split = forced_split > 0 ? forced_split : (base >= 192 ? 1 : (256 + base - 1) / base);
    if (split > BB_MAX_SPLITK) split = BB_MAX_SPLITK;
    if (split > total_chunks / 4) split = total_chunks / 4;
    if (split < 1) split = 1;
    p.chunks_per_split = (total_chunks + split - 1) / split;
    p.split_k = (total_chunks + p.chunks_per_split - 1) / p.chunks_per_split;
    return p;
}

void launch_gemm(const u32x4* Wt, const u32x4* Apk, float* P, int mt_total, int N, int K, GemmPlan plan, hipStream_t s) {
    const int n_tiles = N / 32, ksteps = K / 16, m_groups = (mt_total + MT - 1) / MT;
    const size_t split_stride = (size_t)mt_total * 32 * N;
    if (plan.nt == 2) {
        dim3 grid((n_tiles + 7) / 8, m_groups, plan.split_k);
        gemm_kernel<2><<<grid, 256, 0, s>>>(Wt, Apk, P, split_stride, N, mt_total, n_tiles, ksteps, plan.chunks_per_split);
    } else {
        dim3 grid((n_tiles + 3) / 4, m_groups, plan.split_k);
        gemm_kernel<1><<<grid, 256, 0, s>>>(Wt, Apk, P, split_stride, N, mt_total, n_tiles, ksteps, plan.chunks_per_split);
    }
}

// ---- weight re-tiling (load time) and activation packing ------------------------------------------
// interleave != 0: source row r goes to fused row (r / 64) * 128 + r % 64 + row0 (gate rows with
// row0 = 0, up rows with row0 = 64), so a GEMM tile of 128 or 256 columns holds both halves of its features.
__global__ void tile_weights_kernel(const u32x4* __restrict__ src, int rows, int k8s, u32x4* __restrict__ dst, int row0,
                                    int interleave) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)rows * k8s) return;
    int r = (int)(i / k8s), k8 = (int)(i % k8s);
    int n = interleave ? (r / 64) * 128 + r % 64 + row0 : row0 + r;
    dst[tileW_u4(n, k8, k8s / 2)] = src[i];
}

void launch_tile_weights(const uint16_t* src, int rows, int K, u32x4* dst, int dst_row0, int interleave, hipStream_t s) {
    size_t n = (size_t)rows * (K / 8);
    tile_weights_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(reinterpret_cast<const u32x4*>(src), rows, K / 8, dst, dst_row0, interleave);
}

// fp32 row-major [M][K] -> packed hi/lo fragments; rows >= M inside the last tile are zero.
__global__ void pack_rows_kernel(const float* __restrict__ A, int M, int K, u32x4* __restrict__ Apk, int mt_total) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    int k8s = K / 8;
    if (i >= (size_t)mt_total * 32 * k8s) return;
    int m = (int)(i / k8s), k8 = (int)(i % k8s);
    uint16_t hi[8], lo[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float x = m < M ? A[(size_t)m * K + k8 * 8 + j] : 0.f;
        hi[j] = f32_to_bf16_rne(x);
        lo[j] = f32_to_bf16_rne(x - bf16_to_f32(hi[j]));
    }
    Apk[packA_u4(m, k8, mt_total, 0)] = *reinterpret_cast<u32x4*>(hi);
    Apk[packA_u4(m, k8, mt_total, 1)] = *reinterpret_cast<u32x4*>(lo);
}

void launch_pack_rows(const float* A, int M, int K, u32x4* Apk, int mt_total, hipStream_t s) {
    size_t n = (size_t)mt_total * 32 * (K / 8);
    pack_rows_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(A, M, K, Apk, mt_total);
}
