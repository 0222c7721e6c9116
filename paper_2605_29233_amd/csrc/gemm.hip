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
#include <hip/hip_ext.h>
#include <type_traits>
#include <algorithm>

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define KC 4        // k-steps (of 16) per staged chunk
#define MT 4        // m-tiles (of 32 rows) per workgroup
#define DW 3        // weight chunks per wave in the register ring (two in flight ahead of the MFMAs)
#define CHUNK_U4 (KC * MT * BB_SPLIT * 64)      // uint4 per staged activation chunk (2048 = 32 KiB)
#define A_PER_THREAD (CHUNK_U4 / 256)

static __device__ __forceinline__ bf16x8 as_bf16x8(const u32x4& v) {
    return *reinterpret_cast<const bf16x8*>(&v);
}

// sched_group_barrier masks
#define SG_MFMA 0x008
#define SG_VMEM 0x020
#define SG_DSR 0x100
#define SG_DSW 0x200

// P[split][m][n] (fp32, leading dimension ldp) = this workgroup's share of the k range.
//
// One workgroup = 4 waves = one wave per SIMD; wave w owns NT weight tiles (32 rows each) and all
// four waves share the activation chunk in LDS, so the tile is 128 rows x (128 * NT) columns.
// Per chunk of 64 k a wave issues 16 * NT * 2 MFMAs, 32 LDS fragment reads, its 8 LDS writes of the
// next activation chunk and 16 global loads; with a single wave per SIMD nothing hides a stall,
// so the chunk is a software pipeline with every stream interleaved between the MFMAs:
//   k-step 0: MFMAs | LDS reads of step 1 | LDS writes of chunk c+1's activations (loaded during c-1)
//   k-step 1: MFMAs | LDS reads of step 2 | global loads of chunk c+2's activations     -> barrier
//   k-step 2: MFMAs | LDS reads of step 3 | global loads of half of chunk c+2's weights
//   k-step 3: MFMAs | LDS reads of step 0 of chunk c+1 | the other half
// Activations rotate through three LDS stages, weights through three register slots.  All loads
// are unpredicated (indices clamped, K padded with zeros to whole chunks) so the loop body is one
// straight block per chunk and the compiler's wait counts are exact.
//
// SWIGLU: the weight matrix is the fused gate/up projection (32 gate rows alternate with the 32 up rows of
// the same features, so a wave's two tiles are gate and up of one feature group); instead of P the
// kernel writes act = SiLU(gate) * up as the packed hi/lo panel Opk of the down projection (no k split).
#define EPI_PARTIAL 0
#define EPI_SWIGLU 1
#define EPI_VOCAB 2
// EPI_VOCAB: the weight matrix is the LM head; per tile every row's logits are reduced to (max, rescaled sum of
// exponentials, argmax) over the tile's columns (the mask token and padded columns excluded) and written to
// Vp[row][column tile]; a second kernel merges the column tiles of a row in a fixed order.  The logits themselves
// are stored only when keep_logits is set (tests).
template <int NT, int EPI>
__global__ __launch_bounds__(256, 1) void gemm_kernel(const u32x4* __restrict__ Wt, const u32x4* __restrict__ Apk,
                                                      float* __restrict__ P, size_t split_stride, int ldp, int mt_total,
                                                      int n_tiles, int ksteps, int chunks_per_split, int tiles_x, int tiles_y,
                                                      u32x4* __restrict__ Opk, float4* __restrict__ Vp, int mask_id,
                                                      int keep_logits) {
    constexpr bool SWIGLU = EPI == EPI_SWIGLU;
    __shared__ u32x4 lds[3][CHUNK_U4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // a workgroup walks the (column group, row group) tiles with the grid's stride: at most one round of
    // workgroups is ever launched, the rest of the tiles are taken by the same workgroups
    //
    // Workgroups go to the 8 XCDs (each with its own L2) round robin by linear id.  With a k split the
    // (column group, split) items are dealt out so that an XCD gets a contiguous run of them in split-major
    // order: its workgroups then share one or two k ranges of the activation panel, which its L2 fetches
    // once, instead of every XCD fetching the whole panel.
    int first_tile = blockIdx.x, split_id = blockIdx.z;
    if (gridDim.z > 1 && tiles_y == 1) {
        const int n = gridDim.x * gridDim.z, lin = blockIdx.x + gridDim.x * blockIdx.z, e = lin & 7;
        const int item = e * (n >> 3) + min(e, n & 7) + (lin >> 3);
        first_tile = item % gridDim.x;
        split_id = item / gridDim.x;
    }
    for (int tile = first_tile; tile < tiles_x * tiles_y; tile += gridDim.x) {
    const int bx = tile % tiles_x, by = tile / tiles_x;
    const int mt0 = by * MT;
    const int mt_cnt = min(MT, mt_total - mt0);
    const int total_chunks = ksteps / KC;
    const int c0 = split_id * chunks_per_split;
    const int c1 = min(c0 + chunks_per_split, total_chunks);
    if (c0 >= c1) continue;

    // weight stream: one pointer per tile, advanced by a chunk (KC fragments of 64 lanes) at a time
    const u32x4* wbase[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int x = min((bx * 4 + wave) * NT + t, n_tiles - 1);      // clamped loads; stores are guarded
        wbase[t] = Wt + (size_t)x * ksteps * 64 + lane;
    }
    // activation stream: per-thread offsets inside a chunk (missing m-tiles read a valid one)
    int aoff[A_PER_THREAD];
#pragma unroll
    for (int i = 0; i < A_PER_THREAD; ++i) {
        const int idx = i * 256 + threadIdx.x;
        const int k = idx / (MT * BB_SPLIT * 64), rem = idx % (MT * BB_SPLIT * 64);
        aoff[i] = (k * mt_total + min(rem / (BB_SPLIT * 64), mt_cnt - 1)) * (BB_SPLIT * 64) + rem % (BB_SPLIT * 64);
    }
    const u32x4* abase = Apk + (size_t)mt0 * (BB_SPLIT * 64);
    const size_t a_chunk = (size_t)KC * mt_total * (BB_SPLIT * 64);
    auto load_a = [&](u32x4 (&a)[A_PER_THREAD], int c) {
        const u32x4* p = abase + (size_t)min(c, c1 - 1) * a_chunk;
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) a[i] = p[aoff[i]];
    };
    auto load_w = [&](u32x4 (&w)[KC][NT], int c, int k_lo, int k_hi) {
        const size_t off = (size_t)min(c, c1 - 1) * (KC * 64);
#pragma unroll
        for (int k = k_lo; k < k_hi; ++k)
#pragma unroll
            for (int t = 0; t < NT; ++t) w[k][t] = __builtin_nontemporal_load(wbase[t] + off + k * 64);
    };
    auto read_b = [&](u32x4 (&b)[MT][BB_SPLIT], int stage, int k) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int term = 0; term < BB_SPLIT; ++term) b[mt][term] = lds[stage][((k * MT + mt) * BB_SPLIT + term) * 64 + lane];
    };

    f32x16 acc[NT][MT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][mt][r] = 0.f;
    auto mfmas = [&](const u32x4 (&w)[NT], const u32x4 (&b)[MT][BB_SPLIT]) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int term = 0; term < BB_SPLIT; ++term)
#pragma unroll
                for (int t = 0; t < NT; ++t)
                    acc[t][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(w[t]), as_bf16x8(b[mt][term]), acc[t][mt], 0, 0, 0);
    };

    u32x4 w[DW][KC][NT], a[A_PER_THREAD], b[2][MT][BB_SPLIT];
    // prologue: chunk c0 staged, chunk c0+1 in registers, weights of c0 and c0+1 in flight.  The loads are issued in
    // the order the loop issues them (activations of a chunk, then the weights of the same chunk): the wait counts at
    // the loop head are the more cautious of the two ways in, and with any other order the first chunk of every
    // pass through the unrolled loop body would wait for every load in flight.
    load_a(a, c0);
    load_w(w[0], c0, 0, KC);
#pragma unroll
    for (int i = 0; i < A_PER_THREAD; ++i) lds[0][i * 256 + threadIdx.x] = a[i];
    load_a(a, c0 + 1);
    load_w(w[1], c0 + 1, 0, KC);
    __syncthreads();
    read_b(b[0], 0, 0);

    // One chunk of the pipeline; U = (c - c0) mod 3 selects LDS stage and register slot statically.
    auto chunk = [&](auto U, int c) {
        constexpr int u = decltype(U)::value, st = u, st1 = (u + 1) % DW, slot2 = (u + 2) % DW;
        // k-step 0
        read_b(b[1], st, 1);
#pragma unroll
        for (int i = 0; i < A_PER_THREAD; ++i) lds[st1][i * 256 + threadIdx.x] = a[i];
        mfmas(w[u][0], b[0]);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            __builtin_amdgcn_sched_group_barrier(SG_MFMA, NT, 0);
            __builtin_amdgcn_sched_group_barrier(SG_DSR, 1, 0);
            __builtin_amdgcn_sched_group_barrier(SG_DSW, 1, 0);
        }
        // k-step 1
        read_b(b[0], st, 2);
        load_a(a, c + 2);
        mfmas(w[u][1], b[1]);
#pragma unroll
        for (int g = 0; g < 8; ++g) {
            __builtin_amdgcn_sched_group_barrier(SG_MFMA, NT, 0);
            __builtin_amdgcn_sched_group_barrier(SG_DSR, 1, 0);
            __builtin_amdgcn_sched_group_barrier(SG_VMEM, 1, 0);
        }
        __syncthreads();                    // chunk c+1 is staged; stage (c+2) mod 3 is free again
        // k-step 2
        read_b(b[1], st, 3);
        load_w(w[slot2], c + 2, 0, KC / 2);
        mfmas(w[u][2], b[0]);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            __builtin_amdgcn_sched_group_barrier(SG_MFMA, 2 * NT, 0);
            __builtin_amdgcn_sched_group_barrier(SG_DSR, 2, 0);
            __builtin_amdgcn_sched_group_barrier(SG_VMEM, 1, 0);
        }
        // k-step 3 (reads the first fragments of the next chunk)
        read_b(b[0], st1, 0);
        load_w(w[slot2], c + 2, KC / 2, KC);
        mfmas(w[u][3], b[1]);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            __builtin_amdgcn_sched_group_barrier(SG_MFMA, 2 * NT, 0);
            __builtin_amdgcn_sched_group_barrier(SG_DSR, 2, 0);
            __builtin_amdgcn_sched_group_barrier(SG_VMEM, 1, 0);
        }
    };
    // The steady-state loop has no branch inside a triple of chunks: with one the compiler sinks the
    // weight loads next to their uses in the later block and the prefetch distance is lost.
    int c = c0;
    for (; c + DW <= c1; c += DW) {
        chunk(std::integral_constant<int, 0>{}, c);
        chunk(std::integral_constant<int, 1>{}, c + 1);
        chunk(std::integral_constant<int, 2>{}, c + 2);
    }
    if (c < c1) chunk(std::integral_constant<int, 0>{}, c);
    if (c + 1 < c1) chunk(std::integral_constant<int, 1>{}, c + 1);
    if constexpr (SWIGLU) {
        static_assert(!SWIGLU || NT == 2, "gate and up tiles of a feature group sit in one wave");
        // Register r of lane (m = l%32, g = l/32) holds feature 8 (r/4) + 4 g + r%4 of the wave's 32.  The panel
        // wants the 8 features of group q in one lane of lane-half q%2: lane halves swap the 4-feature
        // pieces they do not own, then each lane stores the groups q = g and g + 2 (hi and lo terms).
        const int x0 = (bx * 4 + wave) * NT, g = lane >> 5;
        __syncthreads();                                    // the next tile's prologue overwrites the staged activations
        if (x0 < n_tiles) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if (mt >= mt_cnt) break;
                float act[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float gt = acc[0][mt][r], up = acc[1][mt][r];
                    act[r] = gt / (1.0f + expf(-gt)) * up;
                }
#pragma unroll
                for (int p2 = 0; p2 < 2; ++p2) {
                    float y[8];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float mine = act[4 * (2 * p2 + g) + i];            // group q = 2 p2 + g is mine
                        const float send = act[4 * (2 * p2 + 1 - g) + i];        // the other lane half owns that group
                        const float recv = __shfl_xor(send, 32, 64);
                        y[i] = g == 0 ? mine : recv;
                        y[4 + i] = g == 0 ? recv : mine;
                    }
                    uint16_t hi[8], lo[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        hi[e] = f32_to_bf16_rne(y[e]);
                        lo[e] = f32_to_bf16_rne(y[e] - bf16_to_f32(hi[e]));
                    }
                    const int m = (mt0 + mt) * 32 + (lane & 31), k8 = (x0 / 2) * 4 + 2 * p2 + g;
                    Opk[packA_u4(m, k8, mt_total, 0)] = *reinterpret_cast<u32x4*>(hi);
                    Opk[packA_u4(m, k8, mt_total, 1)] = *reinterpret_cast<u32x4*>(lo);
                }
            }
        }
        continue;
    }
    if constexpr (EPI == EPI_VOCAB) {
        static_assert(EPI != EPI_VOCAB || NT <= 2, "vocabulary epilogue is written for one or two tiles per wave");
        // Lane l holds, for activation row l % 32 of every m-tile, 16 columns of each of its weight tiles, in
        // ascending column order (register r <-> column 8 (r/4) + 4 (l/32) + r%4): a strict '>' keeps the lowest id.
        __shared__ MSI sV[4][MT * 32];
        const int x0v = (bx * 4 + wave) * NT, gv = lane >> 5;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            MSI a = {-INFINITY, 0.f, 0x7fffffff};
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if (x0v + t >= n_tiles) break;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int v = (x0v + t) * 32 + 8 * (r >> 2) + 4 * gv + (r & 3);
                    const float x = acc[t][mt][r];
                    if (v == mask_id) continue;
                    if (x > a.m) { a.s = a.s * expf(a.m - x) + 1.f; a.m = x; a.i = v; }
                    else a.s += expf(x - a.m);
                }
            }
            const MSI b = {__shfl_xor(a.m, 32, 64), __shfl_xor(a.s, 32, 64), __shfl_xor(a.i, 32, 64)};
            a = gv == 0 ? msi_merge(a, b) : msi_merge(b, a);       // both halves compute the same merge
            if (gv == 0) sV[wave][mt * 32 + (lane & 31)] = a;
        }
        __syncthreads();
        if ((int)threadIdx.x < mt_cnt * 32) {
            MSI t4 = sV[0][threadIdx.x];
#pragma unroll
            for (int w = 1; w < 4; ++w) t4 = msi_merge(t4, sV[w][threadIdx.x]);
            Vp[(size_t)(mt0 * 32 + threadIdx.x) * tiles_x + bx] = make_float4(t4.m, t4.s, __int_as_float(t4.i), 0.f);
        }
        if (!keep_logits) { __syncthreads(); continue; }
    }
    // C^T accumulator layout of the 32x32 MFMA: register r of lane l holds
    //   weight row n = 8*(r/4) + 4*(l/32) + r%4 of the tile, activation row m = l%32.
    // The tile goes through LDS (each wave its own slice, one or two m-tiles at a time) so that the global
    // stores are whole 128-byte lines of a row instead of 16-byte pieces of 32 different rows.
    constexpr int COLS = 32 * NT, LDT = COLS + 4;          // row stride in floats (16-byte aligned, conflict-free)
    constexpr int MPP = NT <= 2 ? 2 : 1;                   // m-tiles per pass: four slices of 32 MPP rows must fit the 96 KiB
    static_assert(4 * 32 * MPP * LDT * 4 <= (int)sizeof(lds), "store slices exceed the staging buffers");
    __syncthreads();                                        // all waves are done with the staged activations
    float* tl = reinterpret_cast<float*>(&lds[0][0]) + wave * (32 * MPP * LDT);
    float* Ps = P + (size_t)split_id * split_stride;
    const int x0 = (bx * 4 + wave) * NT;                    // first weight tile of this wave
#pragma unroll
    for (int pass = 0; pass < MT / MPP; ++pass) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int mh = 0; mh < MPP; ++mh)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x16& a4 = acc[t][MPP * pass + mh];
                    *reinterpret_cast<float4*>(&tl[(mh * 32 + (lane & 31)) * LDT + t * 32 + 8 * q + 4 * (lane >> 5)]) =
                        make_float4(a4[4 * q], a4[4 * q + 1], a4[4 * q + 2], a4[4 * q + 3]);
                }
        // (same wave wrote and reads: no barrier needed, the LDS counter orders them)
        constexpr int LPR = COLS / 4;                       // lanes per row
        const int rows_valid = min(32 * MPP, (mt_cnt - MPP * pass) * 32);
#pragma unroll
        for (int it = 0; it < 32 * MPP * LPR / 64; ++it) {
            const int idx = it * 64 + lane, r = idx / LPR, c4 = (idx % LPR) * 4;
            const float4 v = *reinterpret_cast<const float4*>(&tl[r * LDT + c4]);
            const int n = x0 * 32 + c4;
            if (r < rows_valid && n < n_tiles * 32)
                *reinterpret_cast<float4*>(&Ps[(size_t)((mt0 + MPP * pass) * 32 + r) * ldp + n]) = v;
        }
    }
    __syncthreads();                                        // the next tile's prologue overwrites the LDS slices
    }
}

// nt: weight tiles of 32 rows per wave (workgroup tile = 128 * nt columns); forced values <= 0 = choose.
GemmPlan gemm_plan(int m_rows, int N, int K, int forced_split, int forced_nt) {
    const int n_tiles = N / 32, mt_total = (m_rows + 31) / 32, ksteps = (K + 63) / 64 * 4;
    const int m_groups = (mt_total + MT - 1) / MT, total_chunks = ksteps / KC;
    GemmPlan p;
    p.nt = forced_nt > 0 ? forced_nt : (n_tiles >= 8 ? 2 : 1);
    if (forced_nt <= 0 && m_groups == 1 && N <= 8192) p.nt = 1;     // few columns: narrower tiles, fewer splits
    if (p.nt >= 2 && n_tiles < 4 * p.nt) p.nt = 1;
    if (forced_nt <= 0 && m_groups > 1 && p.nt == 2 && n_tiles >= 12) {
        // many rows: 384-column tiles when they need fewer rounds of workgroups (a tile costs in proportion to its width)
        auto rounds = [&](int nt) { return (long)(((n_tiles + 4 * nt - 1) / (4 * nt)) * (long)m_groups + 255) / 256 * nt; };
        if (rounds(3) < rounds(2)) p.nt = 3;
    }
    const int n_groups = (n_tiles + 4 * p.nt - 1) / (4 * p.nt), base = n_groups * m_groups;
    // One workgroup per CU (256 CUs).  Few tiles: split k so that one round of workgroups covers the chip.
    // Many tiles: split k only if filling the last round pays for writing and re-reading the extra partial tiles.
    int split = forced_split;
    if (split <= 0) {
        if (base < 256) split = 256 / base;
        else {
            double best = 1e30;
            for (int sp = 1; sp <= 4; ++sp) {
                const double units = (double)base * sp, rounds = (double)(((long)base * sp + 255) / 256);
                const double t = 4.0 * mt_total * 32 * (double)N * K / 1.4e15 * (rounds * 256 / units)
                               + (sp - 1) * 8.0 * mt_total * 32 * (double)N / 3e12;
                if (t < best) { best = t; split = sp; }
            }
        }
    }
    if (split > BB_MAX_SPLITK) split = BB_MAX_SPLITK;
    if (split > total_chunks / 4) split = total_chunks / 4;
    if (split < 1) split = 1;
    p.chunks_per_split = (total_chunks + split - 1) / split;
    p.split_k = (total_chunks + p.chunks_per_split - 1) / p.chunks_per_split;
    return p;
}

void launch_gemm(const u32x4* Wt, const u32x4* Apk, float* P, int mt_total, int N, int K, GemmPlan plan, hipStream_t s,
                 GemmEpilogue epi, LaunchStamps st) {
    const int n_tiles = N / 32, ksteps = (K + 63) / 64 * 4, m_groups = (mt_total + MT - 1) / MT;     // K padded to whole chunks
    const size_t split_stride = (size_t)mt_total * 32 * N;
    const int tiles_x = (n_tiles + 4 * plan.nt - 1) / (4 * plan.nt);
    dim3 grid(std::min(tiles_x * m_groups, 256), 1, plan.split_k);
#define GEMM_ARGS Wt, Apk, P, split_stride, N, mt_total, n_tiles, ksteps, plan.chunks_per_split, tiles_x, m_groups, epi.swiglu_out, epi.vocab_part, epi.mask_id, epi.keep_logits
    if (epi.swiglu_out)
        hipExtLaunchKernelGGL(HIP_KERNEL_NAME(gemm_kernel<2, EPI_SWIGLU>), grid, dim3(256), 0, s, st.start, st.stop, 0, GEMM_ARGS);
    else if (epi.vocab_part && plan.nt == 2)
        hipExtLaunchKernelGGL(HIP_KERNEL_NAME(gemm_kernel<2, EPI_VOCAB>), grid, dim3(256), 0, s, st.start, st.stop, 0, GEMM_ARGS);
    else if (epi.vocab_part)
        hipExtLaunchKernelGGL(HIP_KERNEL_NAME(gemm_kernel<1, EPI_VOCAB>), grid, dim3(256), 0, s, st.start, st.stop, 0, GEMM_ARGS);
    else if (plan.nt == 3)
        hipExtLaunchKernelGGL(HIP_KERNEL_NAME(gemm_kernel<3, EPI_PARTIAL>), grid, dim3(256), 0, s, st.start, st.stop, 0, GEMM_ARGS);
    else if (plan.nt == 2)
        hipExtLaunchKernelGGL(HIP_KERNEL_NAME(gemm_kernel<2, EPI_PARTIAL>), grid, dim3(256), 0, s, st.start, st.stop, 0, GEMM_ARGS);
    else
        hipExtLaunchKernelGGL(HIP_KERNEL_NAME(gemm_kernel<1, EPI_PARTIAL>), grid, dim3(256), 0, s, st.start, st.stop, 0, GEMM_ARGS);
#undef GEMM_ARGS
}

// The destination is laid out for K padded to a multiple of 64 (whole chunks); the padding must be zero.
__global__ void tile_weights_kernel(const u32x4* __restrict__ src, int rows, int k8s, u32x4* __restrict__ dst, int row0,
                                    int interleave, int ksteps_pad) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (size_t)rows * k8s) return;
    int r = (int)(i / k8s), k8 = (int)(i % k8s);
    int n = interleave ? (r / 32) * 64 + r % 32 + row0 : row0 + r;      // fused gate/up: 32 rows of one, 32 of the other
    dst[tileW_u4(n, k8, ksteps_pad)] = src[i];
}

void launch_tile_weights(const uint16_t* src, int rows, int K, u32x4* dst, int dst_row0, int interleave, hipStream_t s) {
    size_t n = (size_t)rows * (K / 8);
    tile_weights_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(reinterpret_cast<const u32x4*>(src), rows, K / 8, dst, dst_row0,
                                                                    interleave, (K + 63) / 64 * 4);
}

// fp32 row-major [M][K] -> packed hi/lo fragments; rows >= M and columns >= K (padding to whole chunks) are zero.
__global__ void pack_rows_kernel(const float* __restrict__ A, int M, int K, u32x4* __restrict__ Apk, int mt_total) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    int k8s = (K + 63) / 64 * 8;
    if (i >= (size_t)mt_total * 32 * k8s) return;
    int m = (int)(i / k8s), k8 = (int)(i % k8s);
    uint16_t hi[8], lo[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float x = m < M && k8 * 8 < K ? A[(size_t)m * K + k8 * 8 + j] : 0.f;
        hi[j] = f32_to_bf16_rne(x);
        lo[j] = f32_to_bf16_rne(x - bf16_to_f32(hi[j]));
    }
    Apk[packA_u4(m, k8, mt_total, 0)] = *reinterpret_cast<u32x4*>(hi);
    Apk[packA_u4(m, k8, mt_total, 1)] = *reinterpret_cast<u32x4*>(lo);
}

void launch_pack_rows(const float* A, int M, int K, u32x4* Apk, int mt_total, hipStream_t s) {
    size_t n = (size_t)mt_total * 32 * ((K + 63) / 64 * 8);
    pack_rows_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(A, M, K, Apk, mt_total);
}
