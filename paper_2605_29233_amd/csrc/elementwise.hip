// Memory-bound glue kernels of the forward: embedding gather, RMSNorm with packing into MFMA
// fragments, and the online-softmax vocabulary reduction.  (Residual adds, SwiGLU, RoPE and
// the cache write live in the GEMM epilogues.)
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
// masked row when gather != 0 (LM-head panel).  y = h / sqrt(mean(h^2) + eps) * gain.
// In gather mode y is also stored as the branch's probability-map entry for that position
// (P_k(i, v) = exp(y . W_v - lse) is evaluated on demand by the merge), for every branch of
// the request when bcast != 0 (initial forward: all rows are identical).
__global__ __launch_bounds__(256) void rmsnorm_pack_kernel(Dev D, const float* __restrict__ h, const float* __restrict__ gain,
                                                           u32x4* __restrict__ Apk, int mt_total, int gather, int bcast) {
    __shared__ float sh[4];
    const int j = blockIdx.x, d = D.d, k8s = d >> 3;
    const int count = gather ? D.counts[1] : D.counts[0];
    if (j >= count) { zero_packed_row(Apk, j, k8s, mt_total); return; }
    const int r = gather ? D.lm_row[j] : j;
    const float* hr = h + (size_t)r * d;
    float ss = 0.f;
    for (int k4 = threadIdx.x; k4 < (d >> 2); k4 += blockDim.x) {
        const float4 v = reinterpret_cast<const float4*>(hr)[k4];
        ss += v.x * v.x + v.y * v.y + v.z * v.z + v.w * v.w;
    }
    ss = wg_sum(ss, sh);
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

void launch_rmsnorm_pack(const Dev& D, const float* h, const float* gain, u32x4* Apk, int mt_total, int gather, int bcast,
                         hipStream_t s) {
    rmsnorm_pack_kernel<<<mt_total * 32, 256, 0, s>>>(D, h, gain, Apk, mt_total, gather, bcast);
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
