// Memory-bound glue kernels of the forward: embedding gather, RMSNorm (+ residual add of the
// previous GEMM's split-K partial sums) with packing into MFMA fragments, RoPE + KV-cache
// write, SwiGLU, and the online-softmax vocabulary reduction.
#include "bb_internal.h"

static __device__ __forceinline__ float wg_sum(float v, float* sh) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += sh[w];
    return t;
}

static __device__ __forceinline__ void store_split(u32x4* Apk, int m, int k8, int mt_total, const float (&y)[8]) {
    uint16_t hi[8], lo[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        hi[j] = f32_to_bf16_rne(y[j]);
        lo[j] = f32_to_bf16_rne(y[j] - bf16_to_f32(hi[j]));
    }
    Apk[packA_u4(m, k8, mt_total, 0)] = *reinterpret_cast<u32x4*>(hi);
    Apk[packA_u4(m, k8, mt_total, 1)] = *reinterpret_cast<u32x4*>(lo);
}

static __device__ __forceinline__ void zero_packed_row(u32x4* Apk, int m, int k8s, int mt_total) {
    u32x4 z = {0u, 0u, 0u, 0u};
    for (int k8 = threadIdx.x; k8 < k8s; k8 += blockDim.x) {
        Apk[packA_u4(m, k8, mt_total, 0)] = z;
        Apk[packA_u4(m, k8, mt_total, 1)] = z;
    }
}

// h0 = E[x]: one workgroup per packed row.
__global__ void embed_kernel(Dev D, const uint16_t* __restrict__ emb, float* __restrict__ h) {
    int row = blockIdx.x;
    float* dst = h + (size_t)row * D.d;
    if (row >= D.counts[0]) {
        for (int k = threadIdx.x; k < D.d; k += blockDim.x) dst[k] = 0.f;
        return;
    }
    const uint16_t* src = emb + (size_t)D.row_tok[row] * D.d;
    for (int k = threadIdx.x; k < D.d; k += blockDim.x) dst[k] = bf16_to_f32(src[k]);
}

void launch_embed(const Dev& D, const uint16_t* emb, float* h, int rows_cap, hipStream_t s) {
    embed_kernel<<<rows_cap, 256, 0, s>>>(D, emb, h);
}

// One workgroup per destination row j of the packed panel.  Source row r = j, or the j-th
// masked row when gather != 0 (LM-head panel).  h[r] += sum_s partial[s][r] first (the residual
// add of the preceding O / down projection), then y = h / sqrt(mean(h^2) + eps) * gain.
// In gather mode y is also stored as the branch's probability-map entry for that position
// (P_k(i, v) = exp(y . W_v - lse) is evaluated on demand by the merge), for every branch of
// the request when bcast != 0 (initial forward: all rows are identical).
__global__ __launch_bounds__(256) void rmsnorm_pack_kernel(Dev D, float* __restrict__ h, const float* __restrict__ partial,
                                                           int n_partial, size_t partial_stride,
                                                           const float* __restrict__ gain, u32x4* __restrict__ Apk,
                                                           int mt_total, int gather, int bcast) {
    __shared__ float sh[4];
    const int j = blockIdx.x, d = D.d, k8s = d >> 3;
    const int count = gather ? D.counts[1] : D.counts[0];
    if (j >= count) { zero_packed_row(Apk, j, k8s, mt_total); return; }
    const int r = gather ? D.lm_row[j] : j;
    float* hr = h + (size_t)r * d;
    float ss = 0.f;
    for (int k4 = threadIdx.x; k4 < (d >> 2); k4 += blockDim.x) {
        float4 v = reinterpret_cast<float4*>(hr)[k4];
        for (int s = 0; s < n_partial; ++s) {
            float4 p = reinterpret_cast<const float4*>(partial + s * partial_stride + (size_t)r * d)[k4];
            v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
        }
        if (n_partial) reinterpret_cast<float4*>(hr)[k4] = v;
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    ss = wg_sum(ss, sh);            // also orders the writes to hr before the reads below
    const float inv = 1.0f / sqrtf(ss / (float)d + D.rms_eps);
    int gbr = 0, nb = 1; size_t mrow = 0;
    if (gather) {
        gbr = D.row_gbr[r];
        const int slot = gbr / D.max_br;
        const int gi = D.row_pos[r] - D.hdr[slot].L_p;
        if (bcast) { gbr = slot * D.max_br; nb = D.hdr[slot].N; }
        mrow = (size_t)gbr * D.gmax + gi;
    }
    for (int k8 = threadIdx.x; k8 < k8s; k8 += blockDim.x) {
        float y[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) y[q] = hr[k8 * 8 + q] * inv * gain[k8 * 8 + q];
        store_split(Apk, j, k8, mt_total, y);
        if (gather)
            for (int b = 0; b < nb; ++b) {
                float* dst = D.map_hf + (mrow + (size_t)b * D.gmax) * d + k8 * 8;
#pragma unroll
                for (int q = 0; q < 8; ++q) dst[q] = y[q];
            }
    }
}

void launch_rmsnorm_pack(const Dev& D, float* h, const float* partial, int n_partial, size_t partial_stride,
                         const float* gain, u32x4* Apk, int rows_cap, int mt_total, int gather, int bcast,
                         hipStream_t s) {
    (void)rows_cap;
    rmsnorm_pack_kernel<<<mt_total * 32, 256, 0, s>>>(D, h, partial, n_partial, partial_stride, gain, Apk, mt_total, gather, bcast);
}

// q,k,v = sum of split-K partials (+ bias); rotate q and k by the row's absolute position
// (pairs (j, j + hd/2), angle pos * base^(-2j/hd), from a host-computed table); write q for
// the attention kernel, k into the row's cache page and v into the transposed cache, each as
// two fp16 terms hi + lo.
__global__ __launch_bounds__(256) void rope_kv_kernel(Dev D, const float* __restrict__ qkv, int n_partial,
                                                      size_t partial_stride, const float* __restrict__ bias,
                                                      half_t* __restrict__ Q, int layer) {
    const int row = blockIdx.x;
    if (row >= D.counts[0]) return;
    const int hd = D.hd, half = hd >> 1, pos = D.row_pos[row], phys = D.row_phys[row];
    const size_t phys_rows = (size_t)D.max_req * D.phys_per_req;
    const float* src = qkv + (size_t)row * D.nqkv;
    const float* cs = D.rope_cos + (size_t)pos * half;
    const float* sn = D.rope_sin + (size_t)pos * half;
    auto val = [&](int c) {
        float v = bias ? bias[c] : 0.f;
        for (int s = 0; s < n_partial; ++s) v += src[s * partial_stride + c];
        return v;
    };
    const int nq = D.hq * half, nk = D.hkv * half;
    auto put = [](half_t* hi_p, half_t* lo_p, float y) {
        const half_t hi = (half_t)y;
        *hi_p = hi;
        *lo_p = (half_t)(y - (float)hi);
    };
    for (int idx = threadIdx.x; idx < nq + nk; idx += blockDim.x) {
        const bool isq = idx < nq;
        const int e = isq ? idx : idx - nq;
        const int head = e / half, j = e % half;
        const int c0 = (isq ? 0 : D.hq * hd) + head * hd + j;
        const float x1 = val(c0), x2 = val(c0 + half), c = cs[j], s = sn[j];
        const float y1 = x1 * c - x2 * s, y2 = x2 * c + x1 * s;
        // both layouts: [.. head][term][hd]
        half_t* dst = isq ? Q + ((size_t)row * D.hq + head) * 2 * hd
                          : D.Kc + ((((size_t)layer * phys_rows + phys) * D.lpad + pos) * D.hkv + head) * 2 * hd;
        put(dst + j, dst + hd + j, y1);
        put(dst + j + half, dst + hd + j + half, y2);
    }
    const int voff = (D.hq + D.hkv) * hd;
    for (int e = threadIdx.x; e < D.hkv * hd; e += blockDim.x) {
        const int head = e / hd, dd = e % hd;
        half_t* base = D.Vt + (((size_t)layer * phys_rows + phys) * D.hkv + head) * 2 * hd * (size_t)D.lpad;
        put(base + (size_t)dd * D.lpad + pos, base + (size_t)(hd + dd) * D.lpad + pos, val(voff + e));
    }
}

void launch_rope_kv(const Dev& D, const float* qkv, int n_partial, size_t partial_stride, const float* bias,
                    half_t* Q, int layer, int rows_cap, hipStream_t s) {
    rope_kv_kernel<<<rows_cap, 256, 0, s>>>(D, qkv, n_partial, partial_stride, bias, Q, layer);
}

// act = SiLU(gate) * up, gate = columns [0, F), up = columns [F, 2F) of the fused projection.
__global__ void swiglu_pack_kernel(Dev D, const float* __restrict__ gu, int n_partial, size_t partial_stride,
                                   u32x4* __restrict__ Apk, int mt_total) {
    const int j = blockIdx.x, f = D.f, k8s = f >> 3;
    if (j >= D.counts[0]) { zero_packed_row(Apk, j, k8s, mt_total); return; }
    const float* src = gu + (size_t)j * 2 * f;
    for (int k8 = threadIdx.x; k8 < k8s; k8 += blockDim.x) {
        float y[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            float g = 0.f, u = 0.f;
            for (int s = 0; s < n_partial; ++s) {
                g += src[s * partial_stride + k8 * 8 + q];
                u += src[s * partial_stride + f + k8 * 8 + q];
            }
            y[q] = g / (1.0f + expf(-g)) * u;
        }
        store_split(Apk, j, k8, mt_total, y);
    }
}

void launch_swiglu_pack(const Dev& D, const float* gu, int n_partial, size_t partial_stride, u32x4* Apk,
                        int rows_cap, int mt_total, hipStream_t s) {
    (void)rows_cap;
    swiglu_pack_kernel<<<mt_total * 32, 256, 0, s>>>(D, gu, n_partial, partial_stride, Apk, mt_total);
}

// Top-1 confidence c = max_v softmax(l)_v = 1 / sum_v exp(l_v - max) and its token, in one
// pass over the row with a running (max, rescaled sum, index); the mask token is skipped and
// ties go to the lowest token id.  Probabilities are never written out.
struct MSI { float m, s; int i; };
static __device__ __forceinline__ MSI msi_merge(MSI a, MSI b) {
    MSI r;
    const bool a_wins = a.m > b.m || (a.m == b.m && a.i < b.i);
    r.m = a_wins ? a.m : b.m;
    r.i = a_wins ? a.i : b.i;
    const float ea = a.m == -INFINITY ? 0.f : expf(a.m - r.m), eb = b.m == -INFINITY ? 0.f : expf(b.m - r.m);
    r.s = a.s * ea + b.s * eb;
    return r;
}

__global__ __launch_bounds__(256) void vocab_reduce_kernel(Dev D, const float* __restrict__ logits, int bcast) {
    __shared__ MSI sh[4];
    const int j = blockIdx.x;
    if (j >= D.counts[1]) return;
    const float4* row = reinterpret_cast<const float4*>(logits + (size_t)j * D.vocab);
    MSI a = {-INFINITY, 0.f, 0x7fffffff};
    for (int v4 = threadIdx.x; v4 < (D.vocab >> 2); v4 += blockDim.x) {
        const float4 x4 = row[v4];
        const float xs[4] = {x4.x, x4.y, x4.z, x4.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int v = v4 * 4 + q;
            const float x = xs[q];
            if (v == D.mask_id) continue;
            if (x > a.m) { a.s = a.s * expf(a.m - x) + 1.f; a.m = x; a.i = v; }
            else a.s += expf(x - a.m);
        }
    }
    for (int o = 32; o > 0; o >>= 1) {
        MSI b = {__shfl_xor(a.m, o, 64), __shfl_xor(a.s, o, 64), __shfl_xor(a.i, o, 64)};
        a = msi_merge(a, b);
    }
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = a;
    __syncthreads();
    if (threadIdx.x == 0) {
        MSI t = sh[0];
        for (int w = 1; w < 4; ++w) t = msi_merge(t, sh[w]);
        const float conf = 1.0f / t.s, lse = t.m + logf(t.s);
        D.out_pred[j] = t.i; D.out_conf[j] = conf; D.out_lse[j] = lse;
        const int r = D.lm_row[j];
        int gbr = D.row_gbr[r], nb = 1;
        const int slot = gbr / D.max_br;
        const int gi = D.row_pos[r] - D.hdr[slot].L_p;
        if (bcast) { gbr = slot * D.max_br; nb = D.hdr[slot].N; }
        for (int b = 0; b < nb; ++b) {
            const size_t m = (size_t)(gbr + b) * D.gmax + gi;
            D.map_pred[m] = t.i; D.map_conf[m] = conf; D.map_lse[m] = lse;
        }
    }
}

void launch_vocab_reduce(const Dev& D, const float* logits, int lm_cap, int bcast, hipStream_t s) {
    vocab_reduce_kernel<<<lm_cap, 256, 0, s>>>(D, logits, bcast);
}
