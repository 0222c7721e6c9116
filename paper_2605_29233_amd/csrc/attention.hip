// Bidirectional softmax attention of packed query rows against a branch's paged KV cache row.
//
// Work is cut into tiles of 32 "flattened" query rows (the query heads that share a kv head are
// folded into the row dimension, so the K/V tiles a wave reads serve all of them), one kv head,
// one branch segment.  K and V are found page by page (64 tokens) through the branch's page
// table: shared or private physical row.  Two ways of using the four waves of a workgroup:
//   SPLITQ = false (block steps: few query rows): one tile per workgroup, the waves take the
//            row's pages round robin, each keeping a running max / sum / output (online
//            softmax), and the partial results are combined through LDS in a fixed order;
//   SPLITQ = true  (full-sequence refresh: many query rows): four tiles per workgroup, one per
//            wave; the waves walk the pages together, so the fragments the first wave pulls
//            into L2 serve the other three.
// Either way the result does not depend on scheduling.
//
// Q, K, V and the probabilities P each enter as two fp16 terms (hi + lo); every product keeps
// the three leading cross terms (hi.hi + lo.hi + hi.lo), i.e. ~22 bits per operand.
//
// MFMA use (fp16 inputs, fp32 accumulate, 32x32x16):
//   S^T[key][query]  = K[key][:] . Q[query][:]      A = K fragments (the cache stores them ready-made), B = Q rows
//   O^T[d][query]   += V^T[d][key] . P^T[key][query] A = V^T fragments (likewise),
//                                                    B = P taken straight from the S^T
//                                                    accumulators (same lane owns the same
//                                                    query), keys permuted consistently.
#include "bb_internal.h"
#include <algorithm>

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

static __device__ __forceinline__ f16x8 as_f16x8(const u32x4& v) { return *reinterpret_cast<const f16x8*>(&v); }
#define MFMA16(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0)

// One page of the online softmax for a lane's 32 scores (16 consecutive keys of each key tile, one query).
// Scores arrive in the log2 domain (the queries were scaled by log2(e) / sqrt(hd) when they were written),
// so the exponentials are single v_exp_f32.  Updates the running max / sum, rescales the output
// accumulators when some lane's max moved, and returns P as two fp16 terms in B-fragment order
// (fragment kk = 2 kt + h: slot j of lane group g holds key 32 kt + 16 g + 8 h + j).
template <int DT>
static __device__ __forceinline__ void softmax_page(f32x16 (&s)[2], bool partial_page, int t0, int L, int g, float& m_run,
                                                    float& l_run, f32x16 (&o)[DT], f16x8 (&ph)[4], f16x8 (&pl)[4]) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    if (partial_page) {
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (t0 + 32 * kt + 16 * g + r >= L) s[kt][r] = -INFINITY;
    }
    float mx = s[0][0];
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kt][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);                           // finite: every page holds a valid key
    const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);      // 2^-inf = 0 on the first page
    float sum = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt)
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
            const f32x2 p = {__builtin_amdgcn_exp2f(s[kt][r] - m_new), __builtin_amdgcn_exp2f(s[kt][r + 1] - m_new)};
            sum += p[0] + p[1];
            const f16x2 hi = __builtin_convertvector(p, f16x2);
            const f32x2 rem = p - __builtin_convertvector(hi, f32x2);
            const f16x2 lo = __builtin_convertvector(rem, f16x2);
            const int kk = 2 * kt + (r >> 3);
            ph[kk][r & 7] = hi[0]; ph[kk][(r & 7) + 1] = hi[1];
            pl[kk][r & 7] = lo[0]; pl[kk][(r & 7) + 1] = lo[1];
        }
    l_run = l_run * alpha + sum;
    m_run = m_new;
    if (__builtin_amdgcn_ballot_w64(alpha != 1.0f)) {
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) o[dt] *= alpha;
    }
}

template <int HD, bool SPLITQ>
__global__ __launch_bounds__(256, 1) void attention_kernel(Dev D, const half_t* __restrict__ Q, u32x4* __restrict__ Apk,
                                                        int layer, int mt_total, int seg_base, int n_splits,
                                                        float* __restrict__ part, int wide) {
    constexpr int KS = HD / 16;         // k-steps of the score contraction
    constexpr int DT = HD / 32;         // 32-wide tiles of the output's head dimension
    __shared__ float sO[4][32][HD + 1];
    __shared__ float sM[4][32], sL[4][32];

    // Grid = (kv head, query tile [x split], segment).  The kv head is the fastest index on purpose: workgroups go
    // to the eight XCDs round robin by linear id, so with a multiple of eight kv heads all query tiles and page
    // splits of one (branch, kv head) land on the same XCD and its L2 fetches that row's pages from HBM once.
    const int gbr = seg_base + blockIdx.z;
    const int seg_rows = D.seg_rows[gbr];
    if (seg_rows == 0) return;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, g = lane >> 5, c = lane & 31;
    const int group = D.hq / D.hkv, nflat = seg_rows * group;
    // block steps may also split a row's pages over n_splits workgroups (blockIdx.y = tile * n_splits + split)
    const int split = SPLITQ ? 0 : blockIdx.y % n_splits, qtile = SPLITQ ? blockIdx.y : blockIdx.y / n_splits;
    const int wg_base = qtile * (SPLITQ ? 128 : 32);
    if (wg_base >= nflat) return;
    const int tile_base = SPLITQ ? wg_base + 32 * wave : wg_base;     // this wave's 32 query rows
    const int kvh = blockIdx.x, seg_off = D.seg_off[gbr];
    const int L = D.hdr[gbr / D.max_br].L, n_pages = (L + BB_PAGE - 1) / BB_PAGE;

    // Q fragments (B operand).  The contraction index may be enumerated in any order as long as K uses the
    // same one: k-step ks, lane group g, slot j  <->  head dim (HD/2) g + 8 ks + j, so a lane's KS fragments
    // of a row are one contiguous run of HD/2 values.  Rows past the end repeat the last row (never stored).
    u32x4 qf[2][KS];                    // [term][k-step]
    {
        const int f = min(tile_base + c, nflat - 1);
        const int hig = f / seg_rows, r = f % seg_rows;
        const half_t* qp = Q + ((size_t)(seg_off + r) * D.hq + kvh * group + hig) * 2 * HD + (HD / 2) * g;
#pragma unroll
        for (int term = 0; term < 2; ++term)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) qf[term][ks] = *reinterpret_cast<const u32x4*>(qp + term * HD + 8 * ks);
    }
    float m_run = -INFINITY, l_run = 0.f;
    f32x16 o[DT];
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dt][r] = 0.f;

    const int pps = (n_pages + n_splits - 1) / n_splits;           // pages per split
    const int p0 = SPLITQ ? 0 : split * pps + wave, pstep = SPLITQ ? 1 : 4;
    const int p1 = (SPLITQ ? tile_base < nflat : true) ? (SPLITQ ? n_pages : min(n_pages, (split + 1) * pps)) : 0;
    // A page's K and V fragments (NF x 1 KiB each way) pass through one ring of NF registers-fragments in halves:
    // K tile 0 | K tile 1 -> V dims low | V dims high -> next page's K tile 0 | ...  Each half is requested as
    // soon as the MFMAs that read the half before it have been issued, so a wave always has 16-32 KiB in
    // flight and pays the memory latency per half page, not per fragment.
    constexpr int NF = 2 * KS * 2, H = NF / 2;      // NF = DT * 4 * 2 as well
    u32x4 kv[NF];
    auto block = [&](const half_t* cache, int page) {
        const int phys = D.table[(size_t)gbr * D.n_pages + page];
        return reinterpret_cast<const u32x4*>(cache + kv_block_off(D, layer, phys, page, kvh)) + lane;
    };
    auto fetch_half = [&](int h, const u32x4* src) {
#pragma unroll
        for (int i = 0; i < H; ++i) kv[h * H + i] = src[(h * H + i) * 64];
    };
    if (p0 < p1) { const u32x4* Kp = block(D.Kc, p0); fetch_half(0, Kp); fetch_half(1, Kp); }
    for (int page = p0; page < p1; page += pstep) {
        const int t0 = page * BB_PAGE, nxt = page + pstep;
        const u32x4* Vp = block(D.Vt, page);
        const u32x4* Kn = block(D.Kc, min(nxt, D.n_pages - 1));
        // scores: two tiles of 32 keys.  The cache stores MFMA row i of a tile as key pi(i) = i%4 + 4 (i/8) + 16 ((i/4)%2),
        // which makes the 16 accumulator registers of a lane the 16 consecutive keys t0 + 32 kt + 16 g + r
        // (query c): the order of the V^T fragments' contraction index.  Fragment (kt, ks, term) = kv[(kt KS + ks) 2 + term].
        f32x16 s[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
            for (int r = 0; r < 16; ++r) s[kt][r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const f16x8 kh = as_f16x8(kv[(kt * KS + ks) * 2 + 0]);
                const f16x8 kl = as_f16x8(kv[(kt * KS + ks) * 2 + 1]);
                s[kt] = MFMA16(kl, as_f16x8(qf[0][ks]), s[kt]);
                s[kt] = MFMA16(kh, as_f16x8(qf[1][ks]), s[kt]);
                s[kt] = MFMA16(kh, as_f16x8(qf[0][ks]), s[kt]);
            }
            __builtin_amdgcn_sched_barrier(0);
            fetch_half(kt, Vp);
            __builtin_amdgcn_sched_barrier(0);
        }
        f16x8 ph[4], pl[4];
        softmax_page<DT>(s, t0 + BB_PAGE > L, t0, L, g, m_run, l_run, o, ph, pl);
        // fragment (dt, kk, term) = kv[(dt 4 + kk) 2 + term]
#pragma unroll
        for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const f16x8 vh = as_f16x8(kv[(dt * 4 + kk) * 2 + 0]);
                const f16x8 vl = as_f16x8(kv[(dt * 4 + kk) * 2 + 1]);
                o[dt] = MFMA16(vl, ph[kk], o[dt]);
                o[dt] = MFMA16(vh, pl[kk], o[dt]);
                o[dt] = MFMA16(vh, ph[kk], o[dt]);
            }
            if (dt % (DT / 2) == DT / 2 - 1) {
                __builtin_amdgcn_sched_barrier(0);
                if (nxt < p1) fetch_half(dt / (DT / 2), Kn);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
    // per-wave results -> LDS.  o[dt][r] is O^T[d = 32 dt + 8 (r/4) + 4 g + r%4][query c].
    {
        float l = l_run + __shfl_xor(l_run, 32, 64);
        if (g == 0) { sM[wave][c] = m_run; sL[wave][c] = l; }
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
            for (int r = 0; r < 16; ++r) sO[wave][c][32 * dt + 8 * (r >> 2) + 4 * g + (r & 3)] = o[dt][r];
    }
    __syncthreads();
    // normalise (after a fixed-order combine over the four waves when they split the pages), split into
    // bf16 hi/lo and store as the O-projection's packed activation panel (row = packed query row,
    // k = head * HD + d).
    constexpr int ROWS = SPLITQ ? 128 : 32;
    if (!SPLITQ && n_splits > 1) {
        // unnormalised partial result of this split: max[32], sum[32], O[32][HD]; attention_combine_kernel finishes
        float* dst = part + ((((size_t)blockIdx.z * gridDim.x + blockIdx.x) * (gridDim.y / n_splits) + qtile) * n_splits + split) * (64 + 32 * HD);
        for (int item = threadIdx.x; item < 32 * (HD / 4); item += 256) {
            const int q = item / (HD / 4), d4 = item % (HD / 4);
            float M = sM[0][q];
            for (int w = 1; w < 4; ++w) M = fmaxf(M, sM[w][q]);
            float wgt[4], lsum = 0.f;
            for (int w = 0; w < 4; ++w) {
                wgt[w] = sM[w][q] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sM[w][q] - M);   // maxima are in the log2 domain
                lsum += wgt[w] * sL[w][q];
            }
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
            for (int w = 0; w < 4; ++w) {
                acc.x += wgt[w] * sO[w][q][d4 * 4 + 0]; acc.y += wgt[w] * sO[w][q][d4 * 4 + 1];
                acc.z += wgt[w] * sO[w][q][d4 * 4 + 2]; acc.w += wgt[w] * sO[w][q][d4 * 4 + 3];
            }
            *reinterpret_cast<float4*>(dst + 64 + q * HD + d4 * 4) = acc;
            if (d4 == 0) { dst[q] = M; dst[32 + q] = lsum; }
        }
        return;
    }
    for (int item = threadIdx.x; item < ROWS * (HD / 8); item += 256) {
        const int q = item / (HD / 8), d8 = item % (HD / 8);
        const int f = wg_base + q;
        if (f >= nflat) continue;
        float y[8];
        if (SPLITQ) {
            const int w = q >> 5, qq = q & 31;
            const float inv = 1.0f / sL[w][qq];
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = sO[w][qq][d8 * 8 + e] * inv;
        } else {
            float M = sM[0][q];
            for (int w = 1; w < 4; ++w) M = fmaxf(M, sM[w][q]);
            float wgt[4], lsum = 0.f;
            for (int w = 0; w < 4; ++w) {
                wgt[w] = sM[w][q] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(sM[w][q] - M);   // maxima are in the log2 domain
                lsum += wgt[w] * sL[w][q];
            }
            const float inv = 1.0f / lsum;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float acc = 0.f;
                for (int w = 0; w < 4; ++w) acc += wgt[w] * sO[w][q][d8 * 8 + e];
                y[e] = acc * inv;
            }
        }
        const int hig = f / seg_rows, r = f % seg_rows;
        const int m = seg_off + r, k8 = ((kvh * group + hig) * HD) / 8 + d8;
        store_panel8(Apk, m, k8, mt_total, y, wide);
    }
}

// Merge the splits of one tile in split order, normalise, and store the packed hi/lo panel.
template <int HD>
__global__ __launch_bounds__(256) void attention_combine_kernel(Dev D, const float* __restrict__ part, u32x4* __restrict__ Apk,
                                                                int mt_total, int seg_base, int n_splits, int wide) {
    const int gbr = seg_base + blockIdx.z;
    const int seg_rows = D.seg_rows[gbr];
    if (seg_rows == 0) return;
    const int group = D.hq / D.hkv, nflat = seg_rows * group, wg_base = blockIdx.y * 32;
    if (wg_base >= nflat) return;
    const int kvh = blockIdx.x, seg_off = D.seg_off[gbr];
    const float* src = part + (((size_t)blockIdx.z * gridDim.x + blockIdx.x) * gridDim.y + blockIdx.y) * n_splits * (64 + 32 * HD);
    for (int item = threadIdx.x; item < 32 * (HD / 8); item += 256) {
        const int q = item / (HD / 8), d8 = item % (HD / 8);
        const int f = wg_base + q;
        if (f >= nflat) continue;
        float M = -INFINITY;
        for (int s = 0; s < n_splits; ++s) M = fmaxf(M, src[s * (64 + 32 * HD) + q]);
        float lsum = 0.f, y[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
        for (int s = 0; s < n_splits; ++s) {
            const float* ps = src + s * (64 + 32 * HD);
            const float ms = ps[q], wgt = ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - M);
            lsum += wgt * ps[32 + q];
            const float4 a = *reinterpret_cast<const float4*>(ps + 64 + q * HD + d8 * 8);
            const float4 b = *reinterpret_cast<const float4*>(ps + 64 + q * HD + d8 * 8 + 4);
            y[0] += wgt * a.x; y[1] += wgt * a.y; y[2] += wgt * a.z; y[3] += wgt * a.w;
            y[4] += wgt * b.x; y[5] += wgt * b.y; y[6] += wgt * b.z; y[7] += wgt * b.w;
        }
        const float inv = 1.0f / lsum;
        const int hig = f / seg_rows, r = f % seg_rows;
        const int m = seg_off + r, k8 = ((kvh * group + hig) * HD) / 8 + d8;
#pragma unroll
        for (int e = 0; e < 8; ++e) y[e] *= inv;
        store_panel8(Apk, m, k8, mt_total, y, wide);
    }
}

// max_pages: pages of the longest row among the segments; part / part_elems: scratch for split partial results.
void launch_attention(const Dev& D, const half_t* Q, u32x4* Apk, int layer, int mt_total, int max_seg_rows,
                      int seg_base, int n_segs, int max_pages, float* part, size_t part_elems, int wide, hipStream_t s) {
    const int group = D.hq / D.hkv, nflat = max_seg_rows * group;
    if (nflat >= 512) {     // many query rows per segment: waves take different query tiles
        dim3 grid(D.hkv, (nflat + 127) / 128, n_segs);
        if (D.hd == 128) attention_kernel<128, true><<<grid, 256, 0, s>>>(D, Q, Apk, layer, mt_total, seg_base, 1, nullptr, wide);
        else attention_kernel<64, true><<<grid, 256, 0, s>>>(D, Q, Apk, layer, mt_total, seg_base, 1, nullptr, wide);
        return;
    }
    // few query rows: one workgroup per tile unless that leaves most of the 256 CUs idle; then the pages of a
    // row are split over several workgroups (each wave keeps at least one page) and a second kernel merges them
    const int qtiles = (nflat + 31) / 32, tiles = qtiles * D.hkv * n_segs;
    int n_splits = std::min(std::min(256 / tiles, (max_pages + 3) / 4), 16);
    while (n_splits > 1 && (size_t)tiles * n_splits * (64 + 32 * D.hd) > part_elems) --n_splits;
    if (n_splits < 1) n_splits = 1;
    dim3 grid(D.hkv, qtiles * n_splits, n_segs), cgrid(D.hkv, qtiles, n_segs);
    if (D.hd == 128) {
        attention_kernel<128, false><<<grid, 256, 0, s>>>(D, Q, Apk, layer, mt_total, seg_base, n_splits, part, wide);
        if (n_splits > 1) attention_combine_kernel<128><<<cgrid, 256, 0, s>>>(D, part, Apk, mt_total, seg_base, n_splits, wide);
    } else {
        attention_kernel<64, false><<<grid, 256, 0, s>>>(D, Q, Apk, layer, mt_total, seg_base, n_splits, part, wide);
        if (n_splits > 1) attention_combine_kernel<64><<<cgrid, 256, 0, s>>>(D, part, Apk, mt_total, seg_base, n_splits, wide);
    }
}
