// Memory-bound glue kernels of the forward: embedding gather, the consumers of the GEMMs'
// split-K partial results (residual add + RMSNorm + packing into MFMA fragments, bias + RoPE +
// KV-cache write, SwiGLU), and the second half of the vocabulary reduction.
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

static __device__ __forceinline__ void zero_packed_row(u32x4* Apk, int m, int k8s, int mt_total, int wide) {
    for (int k8 = threadIdx.x; k8 < k8s; k8 += blockDim.x) zero_panel8(Apk, m, k8, mt_total, wide);
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

// Sum of split-K partial results in split order, for N offsets at once: the loads of a batch (4 splits x N
// offsets) are all issued before the first add, so a thread pays the memory latency once per batch and not
// once per offset.
template <int N>
static __device__ __forceinline__ void part_sum4n(const float* __restrict__ P, int n_split, size_t stride, const size_t (&off)[N],
                                                  float4 (&out)[N]) {
#pragma unroll
    for (int i = 0; i < N; ++i) out[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s = 0; s < n_split; s += 4) {
        float4 p[4][N];
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < N; ++i)
                p[u][i] = s + u < n_split ? *reinterpret_cast<const float4*>(&P[(s + u) * stride + off[i]]) : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int i = 0; i < N; ++i) { out[i].x += p[u][i].x; out[i].y += p[u][i].y; out[i].z += p[u][i].z; out[i].w += p[u][i].w; }
    }
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
                                                           int mt_total, int gather, int bcast, int wide) {
    __shared__ float sh[4];
    const int j = blockIdx.x, d = D.d, k8s = d >> 3;
    const int count = gather ? D.counts[1] : D.counts[0];
    if (j >= count) { zero_packed_row(Apk, j, k8s, mt_total, wide); return; }
    const int r = gather ? D.lm_row[j] : j;
    float* hr = h + (size_t)r * d;
    // the row stays in registers between the two passes: thread t owns the 8-column groups t, t + 256, ...
    constexpr int MAXG = 4;             // d <= 8192
    float v[MAXG][8];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < MAXG; ++i) {
        const int k8 = threadIdx.x + 256 * i;
        if (k8 < k8s) {
            const float4 a = reinterpret_cast<const float4*>(hr)[2 * k8], b = reinterpret_cast<const float4*>(hr)[2 * k8 + 1];
            float4 p[2] = {make_float4(0.f, 0.f, 0.f, 0.f), make_float4(0.f, 0.f, 0.f, 0.f)};
            if (n_partial) {
                const size_t off[2] = {(size_t)r * d + k8 * 8, (size_t)r * d + k8 * 8 + 4};
                part_sum4n<2>(partial, n_partial, partial_stride, off, p);
            }
            v[i][0] = a.x + p[0].x; v[i][1] = a.y + p[0].y; v[i][2] = a.z + p[0].z; v[i][3] = a.w + p[0].w;
            v[i][4] = b.x + p[1].x; v[i][5] = b.y + p[1].y; v[i][6] = b.z + p[1].z; v[i][7] = b.w + p[1].w;
            if (n_partial) {
                reinterpret_cast<float4*>(hr)[2 * k8] = make_float4(v[i][0], v[i][1], v[i][2], v[i][3]);
                reinterpret_cast<float4*>(hr)[2 * k8 + 1] = make_float4(v[i][4], v[i][5], v[i][6], v[i][7]);
            }
#pragma unroll
            for (int q = 0; q < 8; ++q) ss += v[i][q] * v[i][q];
        }
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
#pragma unroll
    for (int i = 0; i < MAXG; ++i) {
        const int k8 = threadIdx.x + 256 * i;
        if (k8 >= k8s) break;
        const float4 g0 = reinterpret_cast<const float4*>(gain)[2 * k8], g1 = reinterpret_cast<const float4*>(gain)[2 * k8 + 1];
        const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        float y[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) y[q] = v[i][q] * inv * gg[q];
        store_panel8(Apk, j, k8, mt_total, y, wide);
        if (gather)
            for (int b = 0; b < nb; ++b) {
                float* dst = D.map_hf + (mrow + (size_t)b * D.gmax) * d + k8 * 8;
                reinterpret_cast<float4*>(dst)[0] = make_float4(y[0], y[1], y[2], y[3]);
                reinterpret_cast<float4*>(dst)[1] = make_float4(y[4], y[5], y[6], y[7]);
            }
    }
}

// The same for many rows (full-sequence passes), eight consecutive rows per workgroup: the eight rows' pieces
// of one 8-column group are adjacent in the packed panel, so a thread stores 128 contiguous bytes per term
// instead of eight workgroups storing 16 bytes each.  d <= 4096 (two column groups per thread).
__global__ __launch_bounds__(256) void rmsnorm_pack8_kernel(Dev D, float* __restrict__ h, const float* __restrict__ partial,
                                                            int n_partial, size_t partial_stride,
                                                            const float* __restrict__ gain, u32x4* __restrict__ Apk, int mt_total,
                                                            int wide) {
    constexpr int R = 8, G = 2;
    __shared__ float sh[4][R];
    const int j0 = blockIdx.x * R, d = D.d, k8s = d >> 3, count = D.counts[0], t = threadIdx.x;
    float v[R][G][8], ss[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        ss[r] = 0.f;
        const int j = j0 + r;
        float* hr = h + (size_t)j * d;
#pragma unroll
        for (int i = 0; i < G; ++i) {
            const int k8 = t + 256 * i;
#pragma unroll
            for (int q = 0; q < 8; ++q) v[r][i][q] = 0.f;
            if (j < count && k8 < k8s) {
                const float4 a = reinterpret_cast<const float4*>(hr)[2 * k8], b = reinterpret_cast<const float4*>(hr)[2 * k8 + 1];
                float4 p[2] = {make_float4(0.f, 0.f, 0.f, 0.f), make_float4(0.f, 0.f, 0.f, 0.f)};
                if (n_partial) {
                    const size_t off[2] = {(size_t)j * d + k8 * 8, (size_t)j * d + k8 * 8 + 4};
                    part_sum4n<2>(partial, n_partial, partial_stride, off, p);
                }
                v[r][i][0] = a.x + p[0].x; v[r][i][1] = a.y + p[0].y; v[r][i][2] = a.z + p[0].z; v[r][i][3] = a.w + p[0].w;
                v[r][i][4] = b.x + p[1].x; v[r][i][5] = b.y + p[1].y; v[r][i][6] = b.z + p[1].z; v[r][i][7] = b.w + p[1].w;
                if (n_partial) {
                    reinterpret_cast<float4*>(hr)[2 * k8] = make_float4(v[r][i][0], v[r][i][1], v[r][i][2], v[r][i][3]);
                    reinterpret_cast<float4*>(hr)[2 * k8 + 1] = make_float4(v[r][i][4], v[r][i][5], v[r][i][6], v[r][i][7]);
                }
#pragma unroll
                for (int q = 0; q < 8; ++q) ss[r] += v[r][i][q] * v[r][i][q];
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        for (int o = 32; o > 0; o >>= 1) ss[r] += __shfl_xor(ss[r], o, 64);
        if ((t & 63) == 0) sh[t >> 6][r] = ss[r];
    }
    __syncthreads();
    float inv[R];
#pragma unroll
    for (int r = 0; r < R; ++r) inv[r] = 1.0f / sqrtf((sh[0][r] + sh[1][r] + sh[2][r] + sh[3][r]) / (float)d + D.rms_eps);
#pragma unroll
    for (int i = 0; i < G; ++i) {
        const int k8 = t + 256 * i;
        if (k8 >= k8s) break;
        const float4 g0 = reinterpret_cast<const float4*>(gain)[2 * k8], g1 = reinterpret_cast<const float4*>(gain)[2 * k8 + 1];
        const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        if (wide) {
#pragma unroll
            for (int r = 0; r < R; ++r) {           // rows past the count hold zeros
                float y[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) y[q] = v[r][i][q] * inv[r] * gg[q];
                store_panel8(Apk, j0 + r, k8, mt_total, y, 1);
            }
            continue;
        }
#pragma unroll
        for (int term = 0; term < 2; ++term)
#pragma unroll
            for (int r = 0; r < R; ++r) {           // rows past the count hold zeros
                uint16_t o16[8];
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    const float y = v[r][i][q] * inv[r] * gg[q];
                    const uint16_t hi = f32_to_bf16_rne(y);
                    o16[q] = term == 0 ? hi : f32_to_bf16_rne(y - bf16_to_f32(hi));
                }
                Apk[packA_u4(j0 + r, k8, mt_total, term)] = *reinterpret_cast<u32x4*>(o16);
            }
    }
}

void launch_rmsnorm_pack(const Dev& D, float* h, const float* partial, int n_partial, size_t partial_stride,
                         const float* gain, u32x4* Apk, int mt_total, int gather, int bcast, int wide, hipStream_t s) {
    // eight rows per workgroup once that still gives every CU a workgroup, or when a row is too short to occupy
    // one (d <= 512: at most 64 of the 256 threads have a column group)
    if (!gather && D.d <= 4096 && mt_total * 32 > 256 && (mt_total * 4 >= 256 || D.d <= 512))
        rmsnorm_pack8_kernel<<<mt_total * 4, 256, 0, s>>>(D, h, partial, n_partial, partial_stride, gain, Apk, mt_total, wide);
    else
        rmsnorm_pack_kernel<<<mt_total * 32, 256, 0, s>>>(D, h, partial, n_partial, partial_stride, gain, Apk, mt_total, gather, bcast, wide);
}

// Few rows (block steps): the norm's row-wide sum would leave one workgroup per row with the whole row's partial tiles
// to read, and half the CUs idle.  RMSNorm's scale is one number per row and commutes with the projection that follows:
// (x / rms(x) * gain) W^T = (x * gain) W^T / rms(x).  So this kernel only adds the split-K partials to the residual,
// packs x * gain (in the panel format asked for) and leaves the sum of squares of each 2048-column block in ssq[row][block]; the kernels
// that consume the projection (bias + RoPE + cache write, SwiGLU) multiply by 1 / sqrt(sum / d + eps).  One workgroup
// per (row, block of 2048 columns), one 8-column group per thread.
#define BB_SSQ_BLOCK 2048
__global__ __launch_bounds__(256) void residual_pack_kernel(Dev D, float* __restrict__ h, const float* __restrict__ partial,
                                                            int n_partial, size_t partial_stride,
                                                            const float* __restrict__ gain, u32x4* __restrict__ Apk,
                                                            int mt_total, float* __restrict__ ssq, int nblk, int wide) {
    __shared__ float sh[4];
    const int j = blockIdx.x / nblk, b = blockIdx.x % nblk, d = D.d, k8 = b * (BB_SSQ_BLOCK / 8) + threadIdx.x;
    const bool live = k8 < (d >> 3);
    if (j >= D.counts[0]) {
        if (live) zero_panel8(Apk, j, k8, mt_total, wide);
        if (threadIdx.x == 0) ssq[j * nblk + b] = 0.f;
        return;
    }
    float ss = 0.f;
    if (live) {
        float* hr = h + (size_t)j * d;
        const float4 a = reinterpret_cast<const float4*>(hr)[2 * k8], c = reinterpret_cast<const float4*>(hr)[2 * k8 + 1];
        float4 p[2] = {make_float4(0.f, 0.f, 0.f, 0.f), make_float4(0.f, 0.f, 0.f, 0.f)};
        if (n_partial) {
            const size_t off[2] = {(size_t)j * d + k8 * 8, (size_t)j * d + k8 * 8 + 4};
            part_sum4n<2>(partial, n_partial, partial_stride, off, p);
        }
        const float v[8] = {a.x + p[0].x, a.y + p[0].y, a.z + p[0].z, a.w + p[0].w, c.x + p[1].x, c.y + p[1].y, c.z + p[1].z, c.w + p[1].w};
        if (n_partial) {
            reinterpret_cast<float4*>(hr)[2 * k8] = make_float4(v[0], v[1], v[2], v[3]);
            reinterpret_cast<float4*>(hr)[2 * k8 + 1] = make_float4(v[4], v[5], v[6], v[7]);
        }
        const float4 g0 = reinterpret_cast<const float4*>(gain)[2 * k8], g1 = reinterpret_cast<const float4*>(gain)[2 * k8 + 1];
        const float gg[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
        float y[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) { ss += v[q] * v[q]; y[q] = v[q] * gg[q]; }
        store_panel8(Apk, j, k8, mt_total, y, wide);
    }
    ss = wg_sum(ss, sh);
    if (threadIdx.x == 0) ssq[j * nblk + b] = ss;
}

int launch_residual_pack(const Dev& D, float* h, const float* partial, int n_partial, size_t partial_stride,
                         const float* gain, u32x4* Apk, int mt_total, float* ssq, int wide, hipStream_t s) {
    const int nblk = (D.d + BB_SSQ_BLOCK - 1) / BB_SSQ_BLOCK;
    residual_pack_kernel<<<mt_total * 32 * nblk, 256, 0, s>>>(D, h, partial, n_partial, partial_stride, gain, Apk, mt_total, ssq, nblk, wide);
    return nblk;
}

// 1 / rms of a row from the block sums residual_pack_kernel left (fixed order, the same in every consumer)
static __device__ __forceinline__ float row_inv_rms(const Dev& D, const float* __restrict__ ssq, int nblk, int m) {
    float t = 0.f;
    for (int b = 0; b < nblk; ++b) t += ssq[m * nblk + b];
    return 1.0f / sqrtf(t / (float)D.d + D.rms_eps);
}

static __device__ __forceinline__ void put2(half_t* hi_p, half_t* lo_p, float y) {
    const half_t hi = (half_t)y;
    *hi_p = hi;
    *lo_p = (half_t)(y - (float)hi);
}

// four consecutive values as hi / lo fp16 terms, 8 bytes each
static __device__ __forceinline__ void put2x4(half_t* hi_p, half_t* lo_p, const float* y) {
    typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
    f16x4 hi, lo;
#pragma unroll
    for (int e = 0; e < 4; ++e) { hi[e] = (half_t)y[e]; lo[e] = (half_t)(y[e] - (float)hi[e]); }
    *reinterpret_cast<f16x4*>(hi_p) = hi;
    *reinterpret_cast<f16x4*>(lo_p) = lo;
}

// QKV epilogue.  One workgroup = 16 packed rows x 128 columns (whole heads) of the fused q|k|v
// projection: sum the split-K partials (+ bias); q and k heads are rotated by the row's
// absolute position (pairs (j, j + hd/2), angles from a host-computed table) and stored as two
// fp16 terms (q for the attention kernel, k into the fragment-ordered cache page); v heads go
// through LDS so that neighbouring lanes store neighbouring tokens of one head dim, which are adjacent
// in the V fragments.
__global__ __launch_bounds__(256) void qkv_epilogue_kernel(Dev D, const float* __restrict__ qkv, int n_partial,
                                                           size_t partial_stride, const float* __restrict__ bias,
                                                           half_t* __restrict__ Q, int layer,
                                                           const float* __restrict__ ssq, int nblk) {
    __shared__ float tile[128][17];
    const int m0 = blockIdx.x * 16, c0 = blockIdx.y * 128, t = threadIdx.x;
    const int count = D.counts[0];
    if (m0 >= count) return;
    const int hd = D.hd, half = hd >> 1, nq = D.hq * hd, nk = D.hkv * hd;
    if (c0 < nq + nk) {
        // 16 rows x (128 / hd heads) x hd/8 groups of 4 pairs = 256 work items
        const int per_row = 16, r = t / per_row, m = m0 + r;
        if (m >= count) return;
        const int hh = (t % per_row) / (half >> 2), j = ((t % per_row) % (half >> 2)) * 4;
        const int ch = c0 + hh * hd;                   // first column of this head
        const size_t off = (size_t)m * D.nqkv + ch + j;
        const int pos = D.row_pos[m], phys = D.row_phys[m];
        const float4 c = *reinterpret_cast<const float4*>(&D.rope_cos[(size_t)pos * half + j]);
        const float4 sn = *reinterpret_cast<const float4*>(&D.rope_sin[(size_t)pos * half + j]);
        const size_t offs[2] = {off, off + half};
        float4 xs[2];
        part_sum4n<2>(qkv, n_partial, partial_stride, offs, xs);
        float4 x1 = xs[0], x2 = xs[1];
        if (ssq) {          // the projection's input was packed without its RMSNorm scale
            const float inv = row_inv_rms(D, ssq, nblk, m);
            x1.x *= inv; x1.y *= inv; x1.z *= inv; x1.w *= inv; x2.x *= inv; x2.y *= inv; x2.z *= inv; x2.w *= inv;
        }
        if (bias) {
            const float4 b1 = *reinterpret_cast<const float4*>(&bias[ch + j]);
            const float4 b2 = *reinterpret_cast<const float4*>(&bias[ch + j + half]);
            x1.x += b1.x; x1.y += b1.y; x1.z += b1.z; x1.w += b1.w;
            x2.x += b2.x; x2.y += b2.y; x2.z += b2.z; x2.w += b2.w;
        }
        const float a1[4] = {x1.x, x1.y, x1.z, x1.w}, a2[4] = {x2.x, x2.y, x2.z, x2.w};
        const float cc[4] = {c.x, c.y, c.z, c.w}, ss[4] = {sn.x, sn.y, sn.z, sn.w};
        float y1[4], y2[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) { y1[e] = a1[e] * cc[e] - a2[e] * ss[e]; y2[e] = a2[e] * cc[e] + a1[e] * ss[e]; }
        if (ch < nq) {
            // attention works with base-2 exponentials: fold log2(e) / sqrt(hd) into the queries
            const float qs = 1.4426950408889634f / sqrtf((float)hd);
#pragma unroll
            for (int e = 0; e < 4; ++e) { y1[e] *= qs; y2[e] *= qs; }
            half_t* dst = Q + ((size_t)m * D.hq + ch / hd) * 2 * hd;
            put2x4(dst + j, dst + hd + j, y1);
            put2x4(dst + j + half, dst + hd + j + half, y2);
        } else {
            half_t* blk = D.Kc + kv_block_off(D, layer, phys, pos / BB_PAGE, (ch - nq) / hd);
            const int tt = pos % BB_PAGE;
            put2x4(blk + k_slot(tt, j, 0, hd), blk + k_slot(tt, j, 1, hd), y1);
            put2x4(blk + k_slot(tt, j + half, 0, hd), blk + k_slot(tt, j + half, 1, hd), y2);
        }
        return;
    }
    // v columns
    {
        const int r = t / 16, cg = (t % 16) * 8, m = m0 + r;
        if (m < count) {
            const size_t off = (size_t)m * D.nqkv + c0 + cg;
            const size_t offs[2] = {off, off + 4};
            float4 vs[2];
            part_sum4n<2>(qkv, n_partial, partial_stride, offs, vs);
            float4 v0 = vs[0], v1 = vs[1];
            if (ssq) {
                const float inv = row_inv_rms(D, ssq, nblk, m);
                v0.x *= inv; v0.y *= inv; v0.z *= inv; v0.w *= inv; v1.x *= inv; v1.y *= inv; v1.z *= inv; v1.w *= inv;
            }
            if (bias) {
                const float4 b0 = *reinterpret_cast<const float4*>(&bias[c0 + cg]);
                const float4 b1 = *reinterpret_cast<const float4*>(&bias[c0 + cg + 4]);
                v0.x += b0.x; v0.y += b0.y; v0.z += b0.z; v0.w += b0.w;
                v1.x += b1.x; v1.y += b1.y; v1.z += b1.z; v1.w += b1.w;
            }
            tile[cg + 0][r] = v0.x; tile[cg + 1][r] = v0.y; tile[cg + 2][r] = v0.z; tile[cg + 3][r] = v0.w;
            tile[cg + 4][r] = v1.x; tile[cg + 5][r] = v1.y; tile[cg + 6][r] = v1.z; tile[cg + 7][r] = v1.w;
        }
    }
    __syncthreads();
    // Eight consecutive tokens of one head dim are one 16-byte piece of a V fragment.  Where the 8 rows of a
    // half tile are such a run (positions p .. p+7 with p % 8 == 0 in one cache row: always in a refresh, and
    // for block sizes that are multiples of 8) one thread stores the piece whole; otherwise element by element.
    for (int g8 = 0; g8 < 2; ++g8) {
        const int ma = m0 + 8 * g8;
        if (ma >= count) break;
        const int pa = D.row_pos[ma];
        const bool run = ma + 7 < count && (pa & 7) == 0 && D.row_pos[ma + 7] == pa + 7 && D.row_phys[ma + 7] == D.row_phys[ma] &&
                         D.row_gbr[ma + 7] == D.row_gbr[ma];
        if (run) {
            if (t < 128) {
                const int c = t, e = c0 + c - nq - nk, head = e / hd, dd = e % hd, tt = pa % BB_PAGE;
                half_t* blk = D.Vt + kv_block_off(D, layer, D.row_phys[ma], pa / BB_PAGE, head);
                typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
                f16x8 hi, lo;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const float y = tile[c][8 * g8 + j];
                    hi[j] = (half_t)y; lo[j] = (half_t)(y - (float)hi[j]);
                }
                *reinterpret_cast<f16x8*>(blk + v_slot(tt, dd, 0)) = hi;
                *reinterpret_cast<f16x8*>(blk + v_slot(tt, dd, 1)) = lo;
            }
        } else {
            for (int it = t; it < 128 * 8; it += 256) {
                const int c = it / 8, r = 8 * g8 + it % 8, m = m0 + r;
                if (m >= count) continue;
                const int e = c0 + c - nq - nk, head = e / hd, dd = e % hd;
                const int pos = D.row_pos[m], tt = pos % BB_PAGE;
                half_t* blk = D.Vt + kv_block_off(D, layer, D.row_phys[m], pos / BB_PAGE, head);
                put2(blk + v_slot(tt, dd, 0), blk + v_slot(tt, dd, 1), tile[c][r]);
            }
        }
    }
}

void launch_qkv_epilogue(const Dev& D, const float* qkv, int n_partial, size_t partial_stride, const float* bias,
                         half_t* Q, int layer, int rows_cap, const float* ssq, int nblk, hipStream_t s) {
    dim3 grid((rows_cap + 15) / 16, D.nqkv / 128);
    qkv_epilogue_kernel<<<grid, 256, 0, s>>>(D, qkv, n_partial, partial_stride, bias, Q, layer, ssq, nblk);
}

// act = SiLU(gate) * up.  The fused matrix alternates 32 gate rows with the 32 up rows of the
// same features, so feature f has its gate in column (f / 32) * 64 + f % 32 and its up 32 further.
__global__ __launch_bounds__(256) void swiglu_epilogue_kernel(Dev D, const float* __restrict__ gu, int n_partial,
                                                              size_t partial_stride, int ldp, u32x4* __restrict__ Apk,
                                                              int mt_total, int wide, const float* __restrict__ ssq, int nblk) {
    const int f8s = (D.f + 63) / 64 * 8;                   // the panel's K is padded to whole chunks of 64 with zeros
    const size_t it = (size_t)blockIdx.x * 256 + threadIdx.x;
    const int m = (int)(it / f8s), f = (int)(it % f8s) * 8;
    if (m >= mt_total * 32) return;
    if (m >= D.counts[0] || f >= D.f) {
        zero_panel8(Apk, m, f >> 3, mt_total, wide);
        return;
    }
    const size_t off = (size_t)m * ldp + (f >> 5) * 64 + (f & 31);
    const size_t offs[4] = {off, off + 4, off + 32, off + 36};
    float4 gs[4];
    part_sum4n<4>(gu, n_partial, partial_stride, offs, gs);
    const float4 g0 = gs[0], g1 = gs[1], u0 = gs[2], u1 = gs[3];
    const float g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
    const float u[8] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w};
    const float inv = ssq ? row_inv_rms(D, ssq, nblk, m) : 1.0f;      // input packed without its RMSNorm scale
    float y[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) { const float gq = g[q] * inv; y[q] = gq / (1.0f + expf(-gq)) * (u[q] * inv); }
    store_panel8(Apk, m, f >> 3, mt_total, y, wide);
}

void launch_swiglu_epilogue(const Dev& D, const float* gu, int n_partial, size_t partial_stride, int ldp, u32x4* Apk,
                            int rows_cap, int mt_total, int wide, const float* ssq, int nblk, hipStream_t s) {
    (void)rows_cap;
    const size_t items = (size_t)mt_total * 32 * ((D.f + 63) / 64 * 8);
    swiglu_epilogue_kernel<<<(unsigned)((items + 255) / 256), 256, 0, s>>>(D, gu, n_partial, partial_stride, ldp, Apk, mt_total, wide, ssq, nblk);
}

// Second half of the vocabulary reduction.  The LM-head GEMM leaves one (max, rescaled sum of exponentials,
// argmax) per row and column tile (its epilogue reduces the logits in registers: they are not read back, and not
// even written unless a test asks for them); here one wave per row merges the column tiles: each lane its tiles in
// ascending order, then the lanes pairwise.  The merge is symmetric, so every row sees the same tree wherever it
// sits.  Top-1 confidence c = max_v softmax(l)_v = 1 / sum_v exp(l_v - max); probabilities are never formed.
// Writes confidence, token and lse, also into the probability map of the row's branch (of every branch of the
// request after the initial forward).
__global__ __launch_bounds__(256) void vocab_finish_kernel(Dev D, int bcast) {
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (j >= D.counts[1]) return;
    const float4* row = D.vr_part + (size_t)j * D.vr_tiles;
    MSI t = {-INFINITY, 0.f, 0x7fffffff};
    for (int b = lane; b < D.vr_tiles; b += 64) {
        const float4 p = row[b];
        const MSI o = {p.x, p.y, __float_as_int(p.z)};
        t = msi_merge(t, o);
    }
    for (int o = 32; o > 0; o >>= 1) {
        const MSI b = {__shfl_xor(t.m, o, 64), __shfl_xor(t.s, o, 64), __shfl_xor(t.i, o, 64)};
        t = (lane & o) ? msi_merge(b, t) : msi_merge(t, b);      // both partners form the same merge
    }
    if (lane != 0) return;
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

void launch_vocab_finish(const Dev& D, int lm_cap, int bcast, hipStream_t s) {
    vocab_finish_kernel<<<(lm_cap + 3) / 4, 256, 0, s>>>(D, bcast);
}
