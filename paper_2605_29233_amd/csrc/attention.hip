// Bidirectional softmax attention of packed query rows against a branch's paged KV cache row.
//
// One workgroup = (32 flattened query rows, one kv head, one branch segment).  "Flattened"
// folds the query heads that share the kv head into the row dimension (GQA), so the K/V
// tiles a workgroup reads serve all of them.  The four waves take the row's pages round
// robin (page = 64 tokens, found through the branch's page table: shared or private
// physical row), each keeping a running max / sum / output in registers (online softmax),
// and the partial results are combined through LDS in a fixed order, so the result does not
// depend on scheduling.
//
// Q, K, V and the probabilities P each enter as two fp16 terms (hi + lo); every product keeps
// the three leading cross terms (hi.hi + lo.hi + hi.lo), i.e. ~22 bits per operand.
//
// MFMA use (fp16 inputs, fp32 accumulate, 16x16x32):
//   S^T[key][query]  = K[key][:] . Q[query][:]      A = K rows (as stored), B = Q rows
//   O^T[d][query]   += V^T[d][key] . P^T[key][query] A = V^T (cache is stored transposed),
//                                                    B = P taken straight from the S^T
//                                                    accumulators (same lane owns the same
//                                                    query), keys permuted consistently.
#include "bb_internal.h"

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

static __device__ __forceinline__ f16x8 as_f16x8(const u32x4& v) { return *reinterpret_cast<const f16x8*>(&v); }

template <int HD>
__global__ __launch_bounds__(256) void attention_kernel(Dev D, const half_t* __restrict__ Q, u32x4* __restrict__ Apk,
                                                        int layer, int mt_total, int seg_base) {
    constexpr int KS = HD / 32;         // k-steps of the score contraction
    constexpr int DT = HD / 16;         // 16-wide tiles of the output's head dimension
    __shared__ float sO[4][32][HD + 4];
    __shared__ float sM[4][32], sL[4][32];

    const int gbr = seg_base + blockIdx.z;
    const int seg_rows = D.seg_rows[gbr];
    if (seg_rows == 0) return;
    const int group = D.hq / D.hkv, nflat = seg_rows * group, tile_base = blockIdx.x * 32;
    if (tile_base >= nflat) return;
    const int kvh = blockIdx.y, seg_off = D.seg_off[gbr];
    const int L = D.hdr[gbr / D.max_br].L, n_pages = (L + BB_PAGE - 1) / BB_PAGE;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, g = lane >> 4, c = lane & 15;
    const size_t phys_rows = (size_t)D.max_req * D.phys_per_req;
    const float scale = 1.0f / sqrtf((float)HD);

    // Q fragments (B operand): lane (query c, k group g) holds 8 consecutive head dims.
    u32x4 qf[2][2][KS];                 // [query tile][term][k-step]
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        const int f = tile_base + 16 * qt + c;
        const bool ok = f < nflat;
        const int hig = ok ? f / seg_rows : 0, r = ok ? f % seg_rows : 0;
        const half_t* qp = Q + ((size_t)(seg_off + r) * D.hq + kvh * group + hig) * 2 * HD + 8 * g;
#pragma unroll
        for (int term = 0; term < 2; ++term)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                qf[qt][term][ks] = ok ? *reinterpret_cast<const u32x4*>(qp + term * HD + 32 * ks) : u32x4{0u, 0u, 0u, 0u};
    }
    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
    f32x4 o[DT][2];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) o[dt][qt] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int page = wave; page < n_pages; page += 4) {
        const int phys = D.table[(size_t)gbr * D.n_pages + page];
        const int t0 = page * BB_PAGE;
        const half_t* Kb = D.Kc + ((((size_t)layer * phys_rows + phys) * D.lpad + t0) * D.hkv + kvh) * 2 * HD;
        const half_t* Vb = D.Vt + (((size_t)layer * phys_rows + phys) * D.hkv + kvh) * 2 * HD * (size_t)D.lpad + t0;
        f32x4 s[4][2];
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
            s[kt][0] = f32x4{0.f, 0.f, 0.f, 0.f}; s[kt][1] = s[kt][0];
            const half_t* kp = Kb + (size_t)(16 * kt + c) * D.hkv * 2 * HD + 8 * g;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const f16x8 kh = as_f16x8(*reinterpret_cast<const u32x4*>(kp + 32 * ks));
                const f16x8 kl = as_f16x8(*reinterpret_cast<const u32x4*>(kp + HD + 32 * ks));
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    s[kt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kl, as_f16x8(qf[qt][0][ks]), s[kt][qt], 0, 0, 0);
                    s[kt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kh, as_f16x8(qf[qt][1][ks]), s[kt][qt], 0, 0, 0);
                    s[kt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(kh, as_f16x8(qf[qt][0][ks]), s[kt][qt], 0, 0, 0);
                }
            }
        }
        // register r of s[kt][qt]: key t0 + 16 kt + 4 g + r, query 16 qt + c
        f16x8 pf[2][2], pl[2][2];           // probabilities, hi and lo terms
#pragma unroll
        for (int qt = 0; qt < 2; ++qt) {
            float mx = -INFINITY;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int key = t0 + 16 * kt + 4 * g + r;
                    const float v = key < L ? s[kt][qt][r] * scale : -INFINITY;
                    s[kt][qt][r] = v;
                    mx = fmaxf(mx, v);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[qt], mx);           // finite: every page holds a valid key
            const float alpha = expf(m_run[qt] - m_new);        // exp(-inf) = 0 on the first page
            float sum = 0.f;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const float p = expf(s[kt][qt][r] - m_new);
                    sum += p;
                    const _Float16 ph = (_Float16)p;
                    pf[kt >> 1][qt][(kt & 1) * 4 + r] = ph;
                    pl[kt >> 1][qt][(kt & 1) * 4 + r] = (_Float16)(p - (float)ph);
                }
            l_run[qt] = l_run[qt] * alpha + sum;
            m_run[qt] = m_new;
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) o[dt][qt] *= alpha;
        }
        // P slot j of k-step kk holds key 32 kk + 4 g + j (j < 4) or 32 kk + 16 + 4 g + (j - 4)
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
            const half_t* vp = Vb + (size_t)(16 * dt + c) * D.lpad + 4 * g;
            const half_t* vq = vp + (size_t)HD * D.lpad;        // lo term
#pragma unroll
            for (int kk = 0; kk < 2; ++kk) {
                f16x8 vh, vl;
                const f16x4 h0 = *reinterpret_cast<const f16x4*>(vp + 32 * kk);
                const f16x4 h1 = *reinterpret_cast<const f16x4*>(vp + 32 * kk + 16);
                const f16x4 l0 = *reinterpret_cast<const f16x4*>(vq + 32 * kk);
                const f16x4 l1 = *reinterpret_cast<const f16x4*>(vq + 32 * kk + 16);
#pragma unroll
                for (int j = 0; j < 4; ++j) { vh[j] = h0[j]; vh[4 + j] = h1[j]; vl[j] = l0[j]; vl[4 + j] = l1[j]; }
#pragma unroll
                for (int qt = 0; qt < 2; ++qt) {
                    o[dt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vl, pf[kk][qt], o[dt][qt], 0, 0, 0);
                    o[dt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vh, pl[kk][qt], o[dt][qt], 0, 0, 0);
                    o[dt][qt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(vh, pf[kk][qt], o[dt][qt], 0, 0, 0);
                }
            }
        }
    }
    // per-wave partials -> LDS.  o[dt][qt][r] is O^T[d = 16 dt + 4 g + r][query 16 qt + c].
#pragma unroll
    for (int qt = 0; qt < 2; ++qt) {
        float l = l_run[qt];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (g == 0) { sM[wave][16 * qt + c] = m_run[qt]; sL[wave][16 * qt + c] = l; }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 4; ++r) sO[wave][16 * qt + c][16 * dt + 4 * g + r] = o[dt][qt][r];
    }
    __syncthreads();
    // fixed-order combine over the four waves, normalise, split into bf16 hi/lo, store as the
    // O-projection's packed activation panel (row = packed query row, k = head * HD + d).
    for (int item = threadIdx.x; item < 32 * (HD / 8); item += 256) {
        const int q = item / (HD / 8), d8 = item % (HD / 8);
        const int f = tile_base + q;
        if (f >= nflat) continue;
        float M = sM[0][q];
        for (int w = 1; w < 4; ++w) M = fmaxf(M, sM[w][q]);
        float wgt[4], lsum = 0.f;
        for (int w = 0; w < 4; ++w) {
            wgt[w] = sM[w][q] == -INFINITY ? 0.f : expf(sM[w][q] - M);
            lsum += wgt[w] * sL[w][q];
        }
        const float inv = 1.0f / lsum;
        float y[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float acc = 0.f;
            for (int w = 0; w < 4; ++w) acc += wgt[w] * sO[w][q][d8 * 8 + e];
            y[e] = acc * inv;
        }
        const int hig = f / seg_rows, r = f % seg_rows;
        const int m = seg_off + r, k8 = ((kvh * group + hig) * HD) / 8 + d8;
        uint16_t hi[8], lo[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            hi[e] = f32_to_bf16_rne(y[e]);
            lo[e] = f32_to_bf16_rne(y[e] - bf16_to_f32(hi[e]));
        }
        Apk[packA_u4(m, k8, mt_total, 0)] = *reinterpret_cast<u32x4*>(hi);
        Apk[packA_u4(m, k8, mt_total, 1)] = *reinterpret_cast<u32x4*>(lo);
    }
}

void launch_attention(const Dev& D, const half_t* Q, u32x4* Apk, int layer, int mt_total, int max_seg_rows,
                      int seg_base, int n_segs, hipStream_t s) {
    const int group = D.hq / D.hkv;
    dim3 grid((max_seg_rows * group + 31) / 32, D.hkv, n_segs);
    if (D.hd == 128) attention_kernel<128><<<grid, 256, 0, s>>>(D, Q, Apk, layer, mt_total, seg_base);
    else attention_kernel<64><<<grid, 256, 0, s>>>(D, Q, Apk, layer, mt_total, seg_base);
}
