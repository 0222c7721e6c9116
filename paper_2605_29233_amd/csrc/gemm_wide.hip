// MFMA GEMM for passes with many activation rows (full-sequence refresh, initial forward, many requests):
//     C[m][n] = sum_k A[m][k] * W[n][k]          (fp32 accumulate)
// with the operands in the wide format of bb_internal.h: the activation as fp16 + a scaled e5m2 remainder, the
// weight as row-scaled fp16, converted in registers to e4m3 for the remainder's product.  Per 64 k and 32x32 tile
// that is four 32x32x16 fp16 MFMAs and one 32x32x64 fp8 MFMA, three quarters of the matrix work of two bf16 terms,
// and 56 KiB instead of 64 KiB fetched per workgroup and chunk (these passes are bound by what the L2 delivers to a
// CU at least as much as by the matrix pipes), at an accuracy of about 2^-16 per product.  Structure as the two-term
// kernel: C^T tiles with the weight fragment as the MFMA A-operand, one workgroup per CU, four waves that own
// 32 * NT weight rows each and share the activation chunk (128 rows x 64 k = 24 KiB) through three LDS stages;
// weights stream L2 -> registers in a ring of three chunks.  A workgroup walks its (column group, row group) tiles
// with the grid's stride.
#include "bb_internal.h"
#include <hip/hip_ext.h>
#include <type_traits>
#include <algorithm>

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef short i16x2 __attribute__((ext_vector_type(2)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

#define KC 4                                    // fp16 k-steps (of 16) per chunk = weight fragments per (tile, chunk)
#define DW 3                                    // weight chunks per wave in the register ring

#define SG_MFMA 0x008
#define SG_VMEM 0x020
#define SG_DSR 0x100
#define SG_DSW 0x200
// One scheduling group per m-tile of a phase: NT MFMAs, then this group's share of the phase's LDS reads, LDS writes
// and global loads (dealt out as evenly as possible, larger shares first).  The builtin wants constants, hence
// templates.
template <int MASK, int N> static __device__ __forceinline__ void sgb() {
    if constexpr (N > 0) __builtin_amdgcn_sched_group_barrier(MASK, N, 0);
}
template <int GROUPS, int TOTAL, int I> constexpr int sg_share() { return TOTAL / GROUPS + (I < TOTAL % GROUPS ? 1 : 0); }
template <int GROUPS, int NT, int DSR_TOTAL, int DSW_TOTAL, int VMEM_TOTAL, int I = 0>
static __device__ __forceinline__ void sched_groups() {
    if constexpr (I < GROUPS) {
        sgb<SG_MFMA, NT>();
        sgb<SG_DSR, sg_share<GROUPS, DSR_TOTAL, I>()>();
        sgb<SG_DSW, sg_share<GROUPS, DSW_TOTAL, I>()>();
        sgb<SG_VMEM, sg_share<GROUPS, VMEM_TOTAL, I>()>();
        sched_groups<GROUPS, NT, DSR_TOTAL, DSW_TOTAL, VMEM_TOTAL, I + 1>();
    }
}

#define WEPI_PARTIAL 0
#define WEPI_SWIGLU 1

static __device__ __forceinline__ f16x8 as_f16x8(const u32x4& v) { return *reinterpret_cast<const f16x8*>(&v); }
static __device__ __forceinline__ i32x8 as_i32x8(const u32x4& a, const u32x4& b) {
    i32x8 r;
    r[0] = (int)a[0]; r[1] = (int)a[1]; r[2] = (int)a[2]; r[3] = (int)a[3];
    r[4] = (int)b[0]; r[5] = (int)b[1]; r[6] = (int)b[2]; r[7] = (int)b[3];
    return r;
}
// Eight fp16 weights (already scaled by 2^S) -> eight e4m3 values of w 2^(S - BB_LO_SHIFT): the hardware conversion
// divides by its scale operand and rounds to nearest even; |w 2^S| < 2^15 keeps the result below e4m3's 448.
static __device__ __forceinline__ void to_e4m3x8(const u32x4& w, int& lo, int& hi) {
    const float sc = (float)(1 << BB_LO_SHIFT);
    // (the dwords are copied out first: a bit cast applied directly to a vector element picked element 0 every time)
    const unsigned int d0 = w[0], d1 = w[1], d2 = w[2], d3 = w[3];
    // (each conversion writes one half of its destination and keeps the other: starting from the source itself
    // saves clearing a register, the second conversion overwrites what is left of it)
    i16x2 a = __builtin_bit_cast(i16x2, d0), b = __builtin_bit_cast(i16x2, d2);
    a = __builtin_amdgcn_cvt_scalef32_pk_fp8_f16(a, __builtin_bit_cast(f16x2, d0), sc, false);
    a = __builtin_amdgcn_cvt_scalef32_pk_fp8_f16(a, __builtin_bit_cast(f16x2, d1), sc, true);
    b = __builtin_amdgcn_cvt_scalef32_pk_fp8_f16(b, __builtin_bit_cast(f16x2, d2), sc, false);
    b = __builtin_amdgcn_cvt_scalef32_pk_fp8_f16(b, __builtin_bit_cast(f16x2, d3), sc, true);
    lo = __builtin_bit_cast(int, a); hi = __builtin_bit_cast(int, b);
}

// WEPI_PARTIAL: P[split][m][n] (fp32, leading dimension ldp) = this workgroup's share of the k range.
// WEPI_SWIGLU: the weight matrix is the fused gate/up projection (32 gate rows alternate with the 32 up rows of the
// same features; NT == 2, k not split): writes SiLU(gate) * up as the wide-format panel Opk of the down projection.
//
// Chunk pipeline (one wave per SIMD, nothing else hides a stall), five phases per 64 k:
//   fp16 k-step 0: MFMAs | LDS reads of step 1 | LDS writes of chunk c+1's activations (loaded during c-1)
//   fp16 k-step 1: MFMAs | LDS reads of step 2 | global loads of chunk c+2's activations          -> barrier
//   fp16 k-step 2: MFMAs | LDS reads of step 3 | global loads of chunk c+2's weight fragments 0, 1
//   fp16 k-step 3: MFMAs | LDS reads of the fp8 fragments | weight fragments 2, 3 | this chunk's weights -> e4m3
//   fp8 step:      MFMAs | LDS reads of step 0 of chunk c+1
template <int NT, int EPI, bool STREAM, int MT>
__global__ __launch_bounds__(256, 1) void gemm_wide_kernel(const u32x4* __restrict__ Wt, const float* __restrict__ wscale,
                                                           const u32x4* __restrict__ Apk, float* __restrict__ P,
                                                           size_t split_stride, int ldp, int mt_total, int n_tiles,
                                                           int total_chunks, int chunks_per_split, int tiles_x, int tiles_y,
                                                           u32x4* __restrict__ Opk, const float* __restrict__ ssq, int nblk,
                                                           float inv_d, float eps) {
    static_assert(NT >= 1 && NT <= 3 && NT * MT <= 12, "one to three weight tiles per wave, at most 12 accumulator tiles");
    constexpr int WCHUNK_U4 = MT * BB_WFRAGS * 64;          // uint4 per staged activation chunk (6 KiB per m-tile)
    constexpr int WA_PER_THREAD = WCHUNK_U4 / 256;
    static_assert(WCHUNK_U4 % 256 == 0, "every thread stages the same number of pieces");
    __shared__ u32x4 lds[DW][WCHUNK_U4];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    // STREAM (one row group: every weight line is used once): weight loads carry the non-temporal hint, and with a k
    // split the (column group, split) items are dealt to the 8 XCDs in contiguous runs in split-major order, so that an
    // XCD's workgroups share one or two k ranges of the activation panel (as in the two-term kernel).
    int first_tile = blockIdx.x, split_id = blockIdx.z;
    if (STREAM && gridDim.z > 1 && tiles_y == 1) {
        const int n = gridDim.x * gridDim.z, lin = blockIdx.x + gridDim.x * blockIdx.z, e = lin & 7;
        const int item = e * (n >> 3) + min(e, n & 7) + (lin >> 3);
        first_tile = item % gridDim.x;
        split_id = item / gridDim.x;
    }
    for (int tile = first_tile; tile < tiles_x * tiles_y; tile += gridDim.x) {
    const int bx = tile % tiles_x, by = tile / tiles_x;
    const int mt0 = by * MT;
    const int mt_cnt = min(MT, mt_total - mt0);
    const int c0 = split_id * chunks_per_split;
    const int c1 = min(c0 + chunks_per_split, total_chunks);
    if (c0 >= c1) continue;

    const u32x4* wbase[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int x = min((bx * 4 + wave) * NT + t, n_tiles - 1);      // clamped loads; stores are guarded
        wbase[t] = Wt + (size_t)x * total_chunks * (KC * 64) + lane;
    }
    int aoff[WA_PER_THREAD];
#pragma unroll
    for (int i = 0; i < WA_PER_THREAD; ++i) {
        const int idx = i * 256 + threadIdx.x, mt = idx / (BB_WFRAGS * 64), rem = idx % (BB_WFRAGS * 64);
        aoff[i] = min(mt, mt_cnt - 1) * (BB_WFRAGS * 64) + rem;        // missing m-tiles read a valid one
    }
    const u32x4* abase = Apk + (size_t)mt0 * (BB_WFRAGS * 64);
    const size_t a_chunk = (size_t)mt_total * (BB_WFRAGS * 64);
    auto load_a = [&](u32x4 (&a)[WA_PER_THREAD], int c) {
        const u32x4* p = abase + (size_t)min(c, c1 - 1) * a_chunk;
#pragma unroll
        for (int i = 0; i < WA_PER_THREAD; ++i) a[i] = p[aoff[i]];
    };
    auto load_w = [&](u32x4 (&w)[KC][NT], int c, int f_lo, int f_hi) {
        const size_t off = (size_t)min(c, c1 - 1) * (KC * 64);
#pragma unroll
        for (int f = f_lo; f < f_hi; ++f)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                if constexpr (STREAM) w[f][t] = __builtin_nontemporal_load(wbase[t] + off + f * 64);
                else w[f][t] = wbase[t][off + f * 64];      // plain loads: the row groups of an XCD share these lines through its L2
            }
    };
    auto read_bh = [&](u32x4 (&b)[MT], int stage, int k) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) b[mt] = lds[stage][(mt * BB_WFRAGS + k) * 64 + lane];
    };
    auto read_bl = [&](u32x4 (&b)[MT][2], int stage) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int p = 0; p < 2; ++p) b[mt][p] = lds[stage][(mt * BB_WFRAGS + 4 + p) * 64 + lane];
    };

    f32x16 acc[NT][MT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][mt][r] = 0.f;
    auto mfma_hi = [&](const u32x4 (&w)[NT], const u32x4 (&b)[MT]) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                acc[t][mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(w[t]), as_f16x8(b[mt]), acc[t][mt], 0, 0, 0);
    };
    // A operand e4m3 (format 0), B operand e5m2 (format 1), both block scales 2^0
    auto mfma_lo = [&](const i32x8 (&w8)[NT], const u32x4 (&b)[MT][2]) {
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int t = 0; t < NT; ++t)
                acc[t][mt] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(w8[t], as_i32x8(b[mt][0], b[mt][1]),
                                                                            acc[t][mt], 0, 1, 0, 0x7F7F7F7F, 0, 0x7F7F7F7F);
    };
    // k-step j of a lane's fp16 weights becomes bytes 8 j .. 8 j + 7 of its fp8 operand (the panel's e5m2 fragments
    // are laid out to match)
    auto convert_w = [&](i32x8 (&w8)[NT], const u32x4 (&w)[KC][NT]) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int j = 0; j < KC; ++j) { int lo, hi; to_e4m3x8(w[j][t], lo, hi); w8[t][2 * j] = lo; w8[t][2 * j + 1] = hi; }
    };

    u32x4 w[DW][KC][NT], a[WA_PER_THREAD], bh[2][MT], bl[MT][2];
    i32x8 w8[NT];
    // prologue: chunk c0 staged, chunk c0+1 in registers, weights of c0 and c0+1 in flight; loads in the order the
    // loop issues them (activations of a chunk, then its weights), so that the wait counts at the loop head, the more
    // cautious of the two ways in, are those of the steady state
    load_a(a, c0);
    load_w(w[0], c0, 0, KC);
#pragma unroll
    for (int i = 0; i < WA_PER_THREAD; ++i) lds[0][i * 256 + threadIdx.x] = a[i];
    load_a(a, c0 + 1);
    load_w(w[1], c0 + 1, 0, KC);
    __syncthreads();
    read_bh(bh[0], 0, 0);

    auto chunk = [&](auto U, int c) {
        constexpr int u = decltype(U)::value, st = u, st1 = (u + 1) % DW, slot2 = (u + 2) % DW;
        // fp16 k-step 0
        read_bh(bh[1], st, 1);
#pragma unroll
        for (int i = 0; i < WA_PER_THREAD; ++i) lds[st1][i * 256 + threadIdx.x] = a[i];
        mfma_hi(w[u][0], bh[0]);
        sched_groups<MT, NT, MT, WA_PER_THREAD, 0>();
        // fp16 k-step 1
        read_bh(bh[0], st, 2);
        load_a(a, c + 2);
        mfma_hi(w[u][1], bh[1]);
        sched_groups<MT, NT, MT, 0, WA_PER_THREAD>();
        __syncthreads();                    // chunk c+1 is staged; stage (c+2) mod 3 is free again
        // fp16 k-step 2
        read_bh(bh[1], st, 3);
        load_w(w[slot2], c + 2, 0, 2);
        mfma_hi(w[u][2], bh[0]);
        sched_groups<MT, NT, MT, 0, 2 * NT>();
        // fp16 k-step 3 (and the conversion of this chunk's weights for the fp8 step)
        read_bl(bl, st);
        load_w(w[slot2], c + 2, 2, 4);
        convert_w(w8, w[u]);
        mfma_hi(w[u][3], bh[1]);
        sched_groups<MT, NT, 2 * MT, 0, 2 * NT>();
        // fp8 step (reads the first fp16 fragments of the next chunk)
        read_bh(bh[0], st1, 0);
        mfma_lo(w8, bl);
        sched_groups<MT, NT, MT, 0, 0>();
    };
    int c = c0;
    for (; c + DW <= c1; c += DW) {
        chunk(std::integral_constant<int, 0>{}, c);
        chunk(std::integral_constant<int, 1>{}, c + 1);
        chunk(std::integral_constant<int, 2>{}, c + 2);
    }
    if (c < c1) chunk(std::integral_constant<int, 0>{}, c);
    if (c + 1 < c1) chunk(std::integral_constant<int, 1>{}, c + 1);

    // undo the per-row weight scale: register r of lane (m = l % 32, g = l / 32) holds weight row 8 (r/4) + 4 g + r%4
    const int x0 = (bx * 4 + wave) * NT, g = lane >> 5;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int x = min(x0 + t, n_tiles - 1);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float4 s4 = *reinterpret_cast<const float4*>(&wscale[x * 32 + 8 * q + 4 * g]);
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                acc[t][mt][4 * q] *= s4.x; acc[t][mt][4 * q + 1] *= s4.y; acc[t][mt][4 * q + 2] *= s4.z; acc[t][mt][4 * q + 3] *= s4.w;
            }
        }
    }
    __syncthreads();                                        // all waves are done with the staged activations
    if constexpr (EPI == WEPI_SWIGLU) {
        static_assert(EPI != WEPI_SWIGLU || NT == 2, "gate and up tiles of a feature group sit in one wave");
        // The panel wants the 8 features of group q in one lane of lane-half q % 2: lane halves swap the 4-feature
        // pieces they do not own, then each lane stores the groups q = g and g + 2.
        if (x0 < n_tiles) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) {
                if (mt >= mt_cnt) break;
                // ssq: the activation rows were packed without their RMSNorm scale (sums of squares per block of
                // columns instead); both factors of the product take 1 / rms of this lane's row here
                float inv = 1.0f;
                if (ssq) {
                    const int m = (mt0 + mt) * 32 + (lane & 31);
                    float t = 0.f;
                    for (int b = 0; b < nblk; ++b) t += ssq[m * nblk + b];
                    inv = 1.0f / sqrtf(t * inv_d + eps);
                }
                float act[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float gt = acc[0][mt][r] * inv, up = acc[1][mt][r] * inv;
                    act[r] = gt / (1.0f + expf(-gt)) * up;
                }
#pragma unroll
                for (int p2 = 0; p2 < 2; ++p2) {
                    float y[8];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const float e0 = act[4 * (2 * p2) + i], e1 = act[4 * (2 * p2 + 1) + i];
                        const float mine = g == 0 ? e0 : e1;                     // group q = 2 p2 + g is mine
                        const float send = g == 0 ? e1 : e0;                     // the other lane half owns that group
                        const float recv = __shfl_xor(send, 32, 64);
                        y[i] = g == 0 ? mine : recv;
                        y[4 + i] = g == 0 ? recv : mine;
                    }
                    store_panel8(Opk, (mt0 + mt) * 32 + (lane & 31), (x0 / 2) * 4 + 2 * p2 + g, mt_total, y, 1);
                }
            }
        }
        continue;
    }
    // Partial tiles go out through LDS so that a wave stores whole 128-byte lines.
    constexpr int COLS = 32 * NT, LDT = COLS + 4;          // row stride in floats (16-byte aligned, conflict-free)
    constexpr int MPP = NT <= 2 ? 2 : 1;                   // m-tiles per pass: four slices of 32 MPP rows must fit the staging buffers
    static_assert(4 * 32 * MPP * LDT * 4 <= (int)sizeof(lds), "store slices exceed the staging buffers");
    float* tl = reinterpret_cast<float*>(&lds[0][0]) + wave * (32 * MPP * LDT);
    float* Ps = P + (size_t)split_id * split_stride;
#pragma unroll
    for (int pass = 0; pass < MT / MPP; ++pass) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int mh = 0; mh < MPP; ++mh)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x16& a4 = acc[t][MPP * pass + mh];
                    *reinterpret_cast<float4*>(&tl[(mh * 32 + (lane & 31)) * LDT + t * 32 + 8 * q + 4 * g]) =
                        make_float4(a4[4 * q], a4[4 * q + 1], a4[4 * q + 2], a4[4 * q + 3]);
                }
        // (the same wave wrote and reads: no barrier needed, the LDS counter orders them)
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

// Plan of a wide-format GEMM.  Up to 256 rows the two-term kernel's plan (one or two groups of 128 rows, k split so
// that one round of workgroups covers the chip).  With more rows the candidates (rows per workgroup 128 or 192, tile
// width 128 / 256 / 384 columns, k split) are priced from measured launches: the time of one 64-k chunk of a
// workgroup tile (table below: these launches are bound by what reaches the CUs, so a chunk of the 192 x 256 tile,
// 68 KiB for 12 accumulator tiles, costs less per accumulator tile than one of the 128 x 256 tile, 56 KiB for 8), a
// fixed prologue and store per tile, whole rounds of 256 workgroups, and the partial tiles, written here and read by
// the consumer launch once per k split.  fusable: the caller can take SiLU(gate) * up from the epilogue when nt == 2
// and k is not split; that candidate has no partial tiles at all.
GemmPlan gemm_plan_wide(int m_rows, int N, int K, int forced_split, int forced_nt, bool fusable) {
    const int mt_total = (m_rows + 31) / 32;
    if (mt_total <= 8 || forced_split > 0) return gemm_plan(m_rows, N, K, forced_split, forced_nt);
    const int n_tiles = N / 32, total_chunks = (K + 63) / 64;
    static const double chunk_us[2][3] = {{0.75, 1.17, 1.58}, {0.98, 1.654, 0.0}};       // [mt == 6][nt - 1]
    const double partial_us = (double)mt_total * 32 * N * 4 * 0.433e-6;     // one copy: written at ~10 TB/s, read at ~3 TB/s
    GemmPlan best = gemm_plan(m_rows, N, K, 0, forced_nt);
    double best_t = 1e30;
    for (int mt = 4; mt <= 6; mt += 2)
        for (int nt = 1; nt <= 3; ++nt) {
            if (forced_nt > 0 && nt != forced_nt) continue;
            if (nt * mt > 12 || (nt > 1 && n_tiles < 4 * nt)) continue;
            const long base = (long)((n_tiles + 4 * nt - 1) / (4 * nt)) * ((mt_total + mt - 1) / mt);
            for (int sp = 1; sp <= BB_MAX_SPLITK && sp <= std::max(1, total_chunks / 4); ++sp) {
                const int cps = (total_chunks + sp - 1) / sp, sp_eff = (total_chunks + cps - 1) / cps;
                const long rounds = (base * sp_eff + 255) / 256;
                const bool fused = fusable && nt == 2 && sp_eff == 1;
                const double t = rounds * (cps * chunk_us[mt == 6][nt - 1] + 6.0) + (fused ? 0.0 : sp_eff * partial_us + 5.0);
                if (t < best_t) { best_t = t; best.split_k = sp_eff; best.chunks_per_split = cps; best.nt = nt; best.mt = mt; }
            }
        }
    return best;
}

void launch_gemm_wide(const u32x4* Wt, const float* wscale, const u32x4* Apk, float* P, int mt_total, int N, int K,
                      GemmPlan plan, hipStream_t s, u32x4* swiglu_out, LaunchStamps st, const float* ssq, int nblk, float rms_eps) {
    const int n_tiles = N / 32, total_chunks = (K + 63) / 64, m_groups = (mt_total + plan.mt - 1) / plan.mt;
    const size_t split_stride = (size_t)mt_total * 32 * N;
    const int nt = plan.nt;
    const int tiles_x = (n_tiles + 4 * nt - 1) / (4 * nt);
    dim3 grid(std::min(tiles_x * m_groups, 256), 1, plan.split_k);
#define WARGS Wt, wscale, Apk, P, split_stride, N, mt_total, n_tiles, total_chunks, plan.chunks_per_split, tiles_x, m_groups, swiglu_out, ssq, nblk, 1.0f / (float)K, rms_eps
#define WLAUNCH(NT_, EPI_, ST_, MT_) hipExtLaunchKernelGGL(HIP_KERNEL_NAME(gemm_wide_kernel<NT_, EPI_, ST_, MT_>), grid, dim3(256), 0, s, st.start, st.stop, 0, WARGS)
    const bool stream = m_groups == 1;                  // (a single row group never takes the 192-row tile)
    if (plan.mt == 6) {
        if (swiglu_out) WLAUNCH(2, WEPI_SWIGLU, false, 6);
        else if (nt == 2) WLAUNCH(2, WEPI_PARTIAL, false, 6);
        else WLAUNCH(1, WEPI_PARTIAL, false, 6);
    }
    else if (swiglu_out) { if (stream) WLAUNCH(2, WEPI_SWIGLU, true, 4); else WLAUNCH(2, WEPI_SWIGLU, false, 4); }
    else if (nt == 3) { if (stream) WLAUNCH(3, WEPI_PARTIAL, true, 4); else WLAUNCH(3, WEPI_PARTIAL, false, 4); }
    else if (nt == 2) { if (stream) WLAUNCH(2, WEPI_PARTIAL, true, 4); else WLAUNCH(2, WEPI_PARTIAL, false, 4); }
    else { if (stream) WLAUNCH(1, WEPI_PARTIAL, true, 4); else WLAUNCH(1, WEPI_PARTIAL, false, 4); }
#undef WLAUNCH
#undef WARGS
}

// bf16 weights [rows][K] -> row-scaled fp16 in the tiled layout of the bf16 copy.  One workgroup per source row: the
// row's largest magnitude fixes its power-of-two scale 2^S (largest value into [2^14, 2^15)); fp16(w 2^S) is then
// exact unless w is below 2^-29 of the row's largest value; scale_out[row] = 2^-S.  K is padded to whole chunks of 64
// (the padding must be zero: the destination is cleared beforehand).  interleave: fused gate/up, 32 rows of one
// alternate with 32 of the other.
__global__ __launch_bounds__(256) void tile_weights_wide_kernel(const uint16_t* __restrict__ src, int K, u32x4* __restrict__ dst,
                                                                float* __restrict__ scale_out, int row0, int interleave, int ksteps_pad) {
    __shared__ float sh[4];
    const int r = blockIdx.x;
    const int n = interleave ? (r / 32) * 64 + r % 32 + row0 : row0 + r;
    const u32x4* row = reinterpret_cast<const u32x4*>(src + (size_t)r * K);
    const int k8s = K >> 3;
    float mx = 0.f;
    for (int k8 = threadIdx.x; k8 < k8s; k8 += 256) {
        const u32x4 v = row[k8];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            mx = fmaxf(mx, fabsf(bf16_to_f32((uint16_t)(v[j] & 0xFFFFu))));
            mx = fmaxf(mx, fabsf(bf16_to_f32((uint16_t)(v[j] >> 16))));
        }
    }
    for (int o = 32; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
    int S = 0;
    if (mx > 0.f && mx < INFINITY) {
        int e; (void)frexpf(mx, &e);            // mx = f 2^e, f in [0.5, 1)
        S = max(-100, min(100, 15 - e));        // mx 2^S in [2^14, 2^15)
    }
    const float up = ldexpf(1.0f, S);
    if (threadIdx.x == 0) scale_out[n] = ldexpf(1.0f, -S);
    for (int k8 = threadIdx.x; k8 < k8s; k8 += 256) {
        const u32x4 v = row[k8];
        f16x8 hi;
#pragma unroll
        for (int j = 0; j < 8; ++j) hi[j] = (half_t)(bf16_to_f32((uint16_t)((v[j >> 1] >> (16 * (j & 1))) & 0xFFFFu)) * up);
        dst[tileW_u4(n, k8, ksteps_pad)] = __builtin_bit_cast(u32x4, hi);
    }
}

void launch_tile_weights_wide(const uint16_t* src, int rows, int K, u32x4* dst, float* scale_out, int dst_row0, int interleave,
                              hipStream_t s) {
    tile_weights_wide_kernel<<<rows, 256, 0, s>>>(src, K, dst, scale_out, dst_row0, interleave, (K + 63) / 64 * 4);
}

// fp32 row-major [M][K] -> wide-format panel; rows >= M and columns >= K (padding to whole chunks) are zero.
__global__ void pack_rows_wide_kernel(const float* __restrict__ A, int M, int K, u32x4* __restrict__ Apk, int mt_total) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    int k8s = (K + 63) / 64 * 8;
    if (i >= (size_t)mt_total * 32 * k8s) return;
    int m = (int)(i / k8s), k8 = (int)(i % k8s);
    float y[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) y[j] = m < M && k8 * 8 < K ? A[(size_t)m * K + k8 * 8 + j] : 0.f;
    store_panel8(Apk, m, k8, mt_total, y, 1);
}

void launch_pack_rows_wide(const float* A, int M, int K, u32x4* Apk, int mt_total, hipStream_t s) {
    size_t n = (size_t)mt_total * 32 * ((K + 63) / 64 * 8);
    pack_rows_wide_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(A, M, K, Apk, mt_total);
}
