// bf16 MFMA GEMM for the projection, FFN and LM-head contractions:
//     C[m][n] = sum_k A[m][k] * W[n][k]          (fp32 accumulate)
// A is the activation panel (branch rows folded into m), held as two bf16 terms hi + lo per
// element so the product keeps ~16 significant bits of the activation; W are the bf16
// weights.  The kernel computes C^T tiles: the weight fragment is the MFMA A-operand
// (32 weight rows x 16 k) and the activation fragment the B-operand (16 k x 32 rows), so a
// wave streams its weight rows from HBM exactly once, in 1 KiB fragments that were laid out
// in lane order when the weights were loaded, while the (small) activation panel is staged
// through LDS and shared by the four waves of a workgroup.  The split-K reduction and the
// consumer's elementwise work (residual add, SwiGLU, bias + RoPE + cache write) run in the
// epilogue of the same kernel.
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

// ---- epilogues ---------------------------------------------------------------------------------
// Every workgroup writes its fp32 tile (its share of the k range) to P[split][m][n].  When the k
// range is split over several workgroups the last one to arrive (agent-scope counter, no
// waiting) sums the tile's partial results in split order - so the sum does not depend on which
// workgroup finishes last - and applies the epilogue; with a single split the workgroup
// finalises its own tile.  EPI_NONE: P itself is the result (single split only).
static __device__ __forceinline__ float tile_sum(const EpiArgs& E, size_t off) {
    float v = 0.f;
    for (int s = 0; s < E.n_split; ++s) v += E.P[s * E.split_stride + off];
    return v;
}
static __device__ __forceinline__ float4 tile_sum4(const EpiArgs& E, size_t off) {
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < E.n_split; ++s) {
        const float4 p = *reinterpret_cast<const float4*>(&E.P[s * E.split_stride + off]);
        v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    }
    return v;
}
static __device__ __forceinline__ void put2(half_t* hi_p, half_t* lo_p, float y) {
    const half_t hi = (half_t)y;
    *hi_p = hi;
    *lo_p = (half_t)(y - (float)hi);
}

template <int EPI>
static __device__ void finalize_tile(const Dev& D, const EpiArgs& E, int m0, int rows, int n0, int cols, float* lds) {
    const int t = threadIdx.x;
    const int m_valid = min(rows, *E.m_count - m0);         // rows beyond the packed count carry nothing
    if (m_valid <= 0) return;
    if (EPI == EPI_RESID) {
        const int c4 = cols >> 2;
        for (int it = t; it < m_valid * c4; it += 256) {
            const int m = m0 + it / c4, n = n0 + (it % c4) * 4;
            const float4 v = tile_sum4(E, (size_t)m * E.ldp + n);
            float4* hp = reinterpret_cast<float4*>(&E.h[(size_t)m * E.ldh + n]);
            float4 hv = *hp;
            hv.x += v.x; hv.y += v.y; hv.z += v.z; hv.w += v.w;
            *hp = hv;
        }
    } else if (EPI == EPI_SWIGLU) {
        // the fused gate/up matrix interleaves 128 gate rows with the 128 up rows of the same features
        const int f0 = (n0 >> 8) * 128;
        for (int it = t; it < m_valid * 16; it += 256) {
            const int m = m0 + it / 16, f8 = it % 16, f = f0 + f8 * 8;
            if (f >= E.f) continue;
            const size_t off = (size_t)m * E.ldp + n0 + f8 * 8;
            const float4 g0 = tile_sum4(E, off), g1 = tile_sum4(E, off + 4);
            const float4 u0 = tile_sum4(E, off + 128), u1 = tile_sum4(E, off + 132);
            const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
            const float u[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
            uint16_t hi[8], lo[8];
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const float y = g[q] / (1.0f + expf(-g[q])) * u[q];
                hi[q] = f32_to_bf16_rne(y);
                lo[q] = f32_to_bf16_rne(y - bf16_to_f32(hi[q]));
            }
            E.Apk[packA_u4(m, f >> 3, E.mt_total, 0)] = *reinterpret_cast<u32x4*>(hi);
            E.Apk[packA_u4(m, f >> 3, E.mt_total, 1)] = *reinterpret_cast<u32x4*>(lo);
        }
    } else if (EPI == EPI_QKV) {
        const int hd = D.hd, half = hd >> 1, nq = D.hq * hd, nk = D.hkv * hd;
        const size_t phys_rows = (size_t)D.max_req * D.phys_per_req;
        // q and k columns: rotate pairs (j, j + hd/2) by the row's position
        const int heads = cols / hd;
        for (int it = t; it < m_valid * heads * half; it += 256) {
            const int j = it % half, hh = (it / half) % heads, m = m0 + it / (half * heads);
            const int c0 = n0 + hh * hd;                // first column of this head
            if (c0 >= nq + nk) continue;                // a v head: handled below
            const size_t off = (size_t)m * E.ldp + c0 + j;
            float x1 = tile_sum(E, off), x2 = tile_sum(E, off + half);
            if (E.bias) { x1 += E.bias[c0 + j]; x2 += E.bias[c0 + j + half]; }
            const int pos = D.row_pos[m];
            const float c = D.rope_cos[(size_t)pos * half + j], sn = D.rope_sin[(size_t)pos * half + j];
            const float y1 = x1 * c - x2 * sn, y2 = x2 * c + x1 * sn;
            half_t* dst = c0 < nq ? E.Q + ((size_t)m * D.hq + c0 / hd) * 2 * hd
                                  : D.Kc + ((((size_t)E.layer * phys_rows + D.row_phys[m]) * D.lpad + pos) * D.hkv + (c0 - nq) / hd) * 2 * hd;
            put2(dst + j, dst + hd + j, y1);
            put2(dst + j + half, dst + hd + j + half, y2);
        }
        // v columns: transpose through LDS so the stores run along the token axis
        for (int cc = 0; cc < cols; cc += 64) {
            const int c0 = n0 + cc;
            if (c0 < nq + nk) continue;
            __syncthreads();
            for (int it = t; it < m_valid * 64; it += 256) {
                const int m = it / 64, c = it % 64;
                float v = tile_sum(E, (size_t)(m0 + m) * E.ldp + c0 + c);
                if (E.bias) v += E.bias[c0 + c];
                lds[c * 129 + m] = v;
            }
            __syncthreads();
            for (int it = t; it < m_valid * 64; it += 256) {
                const int c = it / m_valid, m = it % m_valid;
                const int e = c0 + c - nq - nk, head = e / hd, dd = e % hd;
                half_t* base = D.Vt + (((size_t)E.layer * phys_rows + D.row_phys[m0 + m]) * D.hkv + head) * 2 * hd * (size_t)D.lpad;
                const int pos = D.row_pos[m0 + m];
                put2(base + (size_t)dd * D.lpad + pos, base + (size_t)(hd + dd) * D.lpad + pos, lds[c * 129 + m]);
            }
        }
    }
}

template <int NT, int EPI>
__global__ __launch_bounds__(256) void gemm_kernel(Dev D, EpiArgs E, const u32x4* __restrict__ Wt,
                                                   const u32x4* __restrict__ Apk, int mt_total, int n_tiles, int ksteps,
                                                   int chunks_per_split) {
    __shared__ u32x4 lds[2][CHUNK_U4];
    __shared__ int s_last;
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
    float* Ps = E.P + (size_t)blockIdx.z * E.split_stride;
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
                *reinterpret_cast<float4*>(&Ps[m * E.ldp + n]) = v;
            }
        }
    }
    if (EPI == EPI_NONE) return;
    if (E.n_split > 1) {
        __threadfence();                                // publish this workgroup's partial tile
        __syncthreads();
        if (threadIdx.x == 0) {
            int* ctr = &E.counters[blockIdx.y * gridDim.x + blockIdx.x];
            const int old = atomicAdd(ctr, 1);
            s_last = old == E.n_split - 1;
            if (s_last) *ctr = 0;                        // ready for the next launch
        }
        __syncthreads();
        if (!s_last) return;
        __threadfence();                                // see the other workgroups' partial tiles
    } else {
        __syncthreads();
    }
    const int n0 = blockIdx.x * 128 * NT;
    finalize_tile<EPI>(D, E, mt0 * 32, mt_cnt * 32, n0, min(128 * NT, n_tiles * 32 - n0), reinterpret_cast<float*>(&lds[0][0]));
}

GemmPlan gemm_plan(int m_rows, int N, int K, int forced_split) {
    int n_tiles = N / 32, mt_total = (m_rows + 31) / 32, ksteps = K / 16;
    int nt = n_tiles >= 8 ? 2 : 1;
    int n_groups = (n_tiles + 4 * nt - 1) / (4 * nt), m_groups = (mt_total + MT - 1) / MT;
    int total_chunks = (ksteps + KC - 1) / KC;
    int base = n_groups * m_groups;
    int split = forced_split > 0 ? forced_split : (base >= 192 ? 1 : (256 + base - 1) / base);
    if (split > BB_MAX_SPLITK) split = BB_MAX_SPLITK;
    if (split > total_chunks / 4) split = total_chunks / 4;
    if (split < 1) split = 1;
    GemmPlan p;
    p.chunks_per_split = (total_chunks + split - 1) / split;
    p.split_k = (total_chunks + p.chunks_per_split - 1) / p.chunks_per_split;
    return p;
}

template <int EPI>
static void launch_gemm_t(const Dev& D, EpiArgs E, const u32x4* Wt, const u32x4* Apk, int mt_total, int N, int K,
                          GemmPlan plan, hipStream_t s) {
    int n_tiles = N / 32, ksteps = K / 16;
    int m_groups = (mt_total + MT - 1) / MT;
    E.n_split = plan.split_k;
    if (n_tiles >= 8) {
        dim3 grid((n_tiles + 7) / 8, m_groups, plan.split_k);
        gemm_kernel<2, EPI><<<grid, 256, 0, s>>>(D, E, Wt, Apk, mt_total, n_tiles, ksteps, plan.chunks_per_split);
    } else {
        dim3 grid((n_tiles + 3) / 4, m_groups, plan.split_k);
        gemm_kernel<1, EPI><<<grid, 256, 0, s>>>(D, E, Wt, Apk, mt_total, n_tiles, ksteps, plan.chunks_per_split);
    }
}

void launch_gemm(const Dev& D, int epi, const EpiArgs& E, const u32x4* Wt, const u32x4* Apk, int mt_total, int N, int K,
                 GemmPlan plan, hipStream_t s) {
    switch (epi) {
        case EPI_NONE: launch_gemm_t<EPI_NONE>(D, E, Wt, Apk, mt_total, N, K, plan, s); break;
        case EPI_RESID: launch_gemm_t<EPI_RESID>(D, E, Wt, Apk, mt_total, N, K, plan, s); break;
        case EPI_SWIGLU: launch_gemm_t<EPI_SWIGLU>(D, E, Wt, Apk, mt_total, N, K, plan, s); break;
        default: launch_gemm_t<EPI_QKV>(D, E, Wt, Apk, mt_total, N, K, plan, s); break;
    }
}

// ---- weight re-tiling (load time) and activation packing ------------------------------------------
// interleave != 0: source row r goes to fused row (r / 128) * 256 + r % 128 + row0 (gate rows with
// row0 = 0, up rows with row0 = 128), so a 256-column GEMM tile holds both halves of 128 features.
__global__ void tile_weights_kernel(const u32x4* __restrict__ src, int rows, int k8s, u32x4* __restrict__ dst, int row0,
                                    int interleave) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)rows * k8s) return;
    int r = (int)(i / k8s), k8 = (int)(i % k8s);
    int n = interleave ? (r / 128) * 256 + r % 128 + row0 : row0 + r;
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
