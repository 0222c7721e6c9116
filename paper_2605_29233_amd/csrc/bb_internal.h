// Internal declarations shared by the host code and the HIP kernels of libblockbatch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include "../../include/blockbatch.h"

typedef _Float16 half_t;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

#define BB_PAGE 64              // tokens per KV page = keys per attention tile
#define BB_SPLIT 2              // bf16 terms per activation (hi + lo) fed to the MFMA GEMMs
#define BB_MAX_SPLITK 16

// ---- device-resident request state ------------------------------------------------------
struct ReqHeader {
    int in_use, L_p, G, L, N;
    int since_refresh, refresh_due, all_done;
    int nfe_init, nfe_block, nfe_refresh;
    int initialised;            // init refresh has run
    int finished, winner, eos_pos;  // end of Alg. 1: 1 all branches done / 2 EOS winner; output branch; its EOS
    int pending[BB_MAX_BRANCHES];   // branch received logits in the latest forward
};

// One entry of a page copy list: copy page `page` of cache row src to row dst (all layers).
struct PageCopy { int src, dst, page, pad; };

// Everything a kernel needs to find its way around the workspace.
struct Dev {
    // model
    int n_layers, d, hq, hkv, hd, f, vocab, mask_id, qkv_bias;
    int nqkv;                   // (hq + 2 hkv) * hd
    float rms_eps;
    // decode
    float tau_dec, tau_merge; int tau_sync, refresh_interval, leader_rule, eos_id;
    // limits
    int max_req, max_br, lpad, n_pages, gmax, rows_cap, lm_cap;
    int phys_per_req;           // max_br + 1 (last = shared row)
    // state
    ReqHeader* hdr;             // [max_req]
    bb_branch_state* br;        // [max_req][max_br]
    int* X;                     // [max_req][max_br][lpad]
    int* table;                 // [max_req][max_br][n_pages] -> physical cache row
    // K,V are cached as two fp16 terms (hi + lo, ~22 significant bits): one fp16 term alone
    // moves the logits of a 32-layer model by more than the parity tolerance.
    half_t* Kc;                 // [n_layers][phys_rows][n_pages][hkv] blocks of MFMA fragments, see kv_block_off
    half_t* Vt;                 // same, fragments of V^T
    float* map_hf;              // [max_req][max_br][gmax][d]  final-norm hidden of the latest forward
    float* map_lse;             // [max_req][max_br][gmax]
    float* map_conf;            // [max_req][max_br][gmax]
    int*   map_pred;            // [max_req][max_br][gmax]
    // rope
    float* rope_cos; float* rope_sin;   // [lpad][hd/2]
    // per-forward row lists
    int* counts;                // [0] M_q, [1] M_lm, [2] n page copies
    int* row_tok; int* row_pos; int* row_gbr; int* row_phys;   // [rows_cap]
    int* seg_off; int* seg_rows;    // [max_req*max_br] packed rows of each branch (0 = inactive)
    int* lm_row;                // [lm_cap]
    int* out_pred; float* out_conf; float* out_lse;   // [lm_cap]
    float4* vr_part;            // [lm_cap][vr_tiles] per-column-tile (max, sum, argmax) of the vocabulary reduction
    int vr_tiles;               // column tiles of the LM-head GEMM = partial results per row
    PageCopy* copies;           // [max_req*max_br*n_pages]
    int* req_list;              // [max_req] request slots of the current call
    int* req_flags;             // [max_req] per listed request after a commit: bit 0 finished, bit 1 refresh due; bits 8.. forwards until a refresh is due
    int* commit_skip;           // [max_req] per listed request: the commit ended the request before MergeSync (EOS winner)
    float* merge_p;             // [max_req][max_br d][max_br s][gmax] P_d(i, token of row s at i) as of the start of MergeSync
    int* merge_x0;              // [max_req][max_br][gmax] the rows' generation tokens at the start of MergeSync
};

static inline __host__ __device__ size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// ---- packed activation layout --------------------------------------------------------------
// A [M][K] fp32 is stored for the GEMM as bf16 hi/lo MFMA B-fragments:
//   [k_step = k/16][m_tile = m/32][term 0..1][lane = (m%32) + 32*((k/8)%2)][k%8]
// One (k_step, m_tile, term) fragment is 64 lanes x 8 bf16 = 1 KiB, read by a wave with one
// 16-byte load per lane.  Offsets below are in units of 8 bf16 (u32x4).
static inline __host__ __device__ size_t packA_u4(int m, int k8, int mt_total, int term) {
    int kstep = k8 >> 1, mt = m >> 5, lane = (m & 31) + ((k8 & 1) << 5);
    return (((size_t)kstep * mt_total + mt) * BB_SPLIT + term) * 64 + lane;
}
// Tiled weight layout: W [N][K] bf16 -> [n_tile = n/32][k_step][lane = (n%32) + 32*((k/8)%2)][k%8].
static inline __host__ __device__ size_t tileW_u4(int n, int k8, int ksteps) {
    int kstep = k8 >> 1, nt = n >> 5, lane = (n & 31) + ((k8 & 1) << 5);
    return ((size_t)nt * ksteps + kstep) * 64 + lane;
}

// ---- wide format: fp16 + fp8 operands for the GEMMs of passes with many rows ----------------------------------
// Passes over hundreds of rows are not bound by the weight stream but by what the L2 delivers to a CU and by the
// matrix pipes, and there the second bf16 term costs a whole second pass.  Instead: activation x = hi + lo with
// hi = fp16(x) (11 bits) and the remainder (|lo| <= 2^-12 |x|) as e5m2(lo * 2^BB_LO_SHIFT), 3 bytes per element
// instead of 4; weights as fp16(w * 2^S) (exact: a bf16 value has 8 significant bits; S is chosen per weight row so
// that the row's largest value lands in [2^14, 2^15)), and for the lo term the same registers converted in the
// kernel to e4m3(w * 2^(S - BB_LO_SHIFT)), whose error (2^-4 relative) then counts 2^-16.  Per 64 k one tile costs
// four 32x32x16 fp16 MFMAs and one 32x32x64 fp8 MFMA (twice the rate): three quarters of the two-pass matrix work.
// The accumulator holds C * 2^S; the epilogue multiplies by 2^-S per weight row.
// Weights: the tiled layout of the bf16 copy (tileW_u4) with fp16 values.  Activation panel:
// [chunk = k / 64][m_tile][fragment 0..5][lane][16 bytes]:
//   fragments 0..3: fp16, k-step ks = (k % 64) / 16, lane = row % 32 + 32 ((k / 8) % 2), element k % 8;
//   fragments 4..5: e5m2, same lane, fragment 4 + ks / 2, byte 8 (ks % 2) + k % 8: a lane's 32 bytes are the
//   remainders of exactly the 32 k whose fp16 weights it holds, in the order the kernel converts those.
#define BB_WFRAGS 6
#define BB_LO_SHIFT 8
static inline __host__ __device__ size_t wideA_hi_u4(int m, int k8, int mt_total) {
    return ((((size_t)(k8 >> 3) * mt_total + (m >> 5)) * BB_WFRAGS + ((k8 & 7) >> 1)) * 64) + (m & 31) + ((k8 & 1) << 5);
}
static inline __host__ __device__ size_t wideA_lo_byte(int m, int k8, int mt_total) {      // byte offset of 8 fp8 values
    return (((((size_t)(k8 >> 3) * mt_total + (m >> 5)) * BB_WFRAGS + 4 + ((k8 & 7) >> 2)) * 64) + (m & 31) + ((k8 & 1) << 5)) * 16 + (((k8 >> 1) & 1) << 3);
}

// ---- KV cache layout ------------------------------------------------------------------------------
// One block = (layer, physical row, page, kv head): the page's 64 tokens stored as the MFMA A-fragments
// (32 rows x 16 k, 64 lanes x 8 fp16 = 1 KiB each) that attention consumes, so that a wave fetches a
// fragment with one contiguous 16-byte load per lane.
//   K block [kt = token / 32][ks][term][lane = c + 32 g][j]: token % 32 = (c&3) + 4 (c>>3) + 16 ((c>>2)&1),
//            head dim = (hd/2) g + 8 ks + j   (ks < hd/16);
//   V block [dt = dim / 32][kk][term][lane = dim % 32 + 32 g][j]: token = 32 (kk/2) + 16 g + 8 (kk%2) + j.
// The token permutation of K makes the 16 score accumulators of a lane 16 consecutive tokens, which is
// the order the V fragments need.
static inline __host__ __device__ size_t kv_block_off(const Dev& D, int layer, int phys, int page, int kvh) {
    const size_t phys_rows = (size_t)D.max_req * D.phys_per_req;
    return ((((size_t)layer * phys_rows + phys) * D.n_pages + page) * D.hkv + kvh) * ((size_t)BB_PAGE * 2 * D.hd);
}
static inline __host__ __device__ int k_slot(int tt, int d, int term, int hd) {
    const int kt = tt >> 5, kap = tt & 31, c = (kap & 3) | ((kap >> 4) << 2) | (((kap >> 2) & 3) << 3);
    const int half = hd >> 1, g = d >= half, ks = (d - g * half) >> 3, j = d & 7;
    return (((kt * (hd >> 4) + ks) * 2 + term) * 64 + c + 32 * g) * 8 + j;
}
static inline __host__ __device__ int v_slot(int tt, int d, int term) {
    const int dt = d >> 5, c = d & 31, kk = 2 * (tt >> 5) + ((tt >> 3) & 1), g = (tt >> 4) & 1, j = tt & 7;
    return (((dt * 4 + kk) * 2 + term) * 64 + c + 32 * g) * 8 + j;
}

// ---- bf16 helpers (round to nearest even, finite inputs) --------------------------------------
static inline __host__ __device__ uint16_t f32_to_bf16_rne(float x) {
    union { float f; uint32_t u; } v; v.f = x;
    uint32_t u = v.u + 0x7FFFu + ((v.u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
static inline __host__ __device__ float bf16_to_f32(uint16_t b) {
    union { float f; uint32_t u; } v; v.u = ((uint32_t)b) << 16; return v.f;
}

// ---- fp8 encodings (round to nearest even, finite inputs) ---------------------------------------------------
// e5m2 is the upper byte of an fp16 value; values beyond its largest finite one (57344) saturate.
static inline __device__ uint8_t f32_to_e5m2(float x) {
    const half_t h = (half_t)x;
    const uint16_t b = *reinterpret_cast<const uint16_t*>(&h);
    uint16_t r = (uint16_t)((b & 0x7FFFu) + 0x7Fu + ((b >> 8) & 1u)) >> 8;
    if (r > 0x7Bu) r = 0x7Bu;
    return (uint8_t)(r | ((b >> 8) & 0x80u));
}
// e4m3 (bias 7, no infinities, largest finite value 448, subnormals are multiples of 2^-9); saturates.
static inline __host__ __device__ uint8_t f32_to_e4m3(float x) {
    union { float f; uint32_t u; } v; v.f = x;
    const uint8_t sign = (uint8_t)((v.u >> 24) & 0x80u);
    v.u &= 0x7FFFFFFFu;
    if (!(v.f < 448.0f)) return sign | 0x7E;
    if (v.f < 0.015625f) return sign | (uint8_t)(int)rintf(v.f * 512.0f);       // 0..8: the subnormals, 8 = 2^-6 itself
    const uint32_t u = v.u + 0x7FFFFu + ((v.u >> 20) & 1u);                     // round the mantissa to 3 bits
    const uint32_t code = (((u >> 23) - 120u) << 3) | ((u >> 20) & 7u);         // exponent rebased from 127 to 7
    return sign | (uint8_t)(code > 0x7Eu ? 0x7Eu : code);
}

#ifdef __HIPCC__
// Eight consecutive k of one activation row into a packed panel: two bf16 terms, or (wide) fp16 + e5m2.
static __device__ __forceinline__ void store_panel8(u32x4* Apk, int m, int k8, int mt_total, const float (&y)[8], int wide) {
    if (!wide) {
        uint16_t hi[8], lo[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            hi[j] = f32_to_bf16_rne(y[j]);
            lo[j] = f32_to_bf16_rne(y[j] - bf16_to_f32(hi[j]));
        }
        Apk[packA_u4(m, k8, mt_total, 0)] = *reinterpret_cast<u32x4*>(hi);
        Apk[packA_u4(m, k8, mt_total, 1)] = *reinterpret_cast<u32x4*>(lo);
    } else {
        typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));
        f16x8_t hi;
        uint32_t lo0 = 0u, lo1 = 0u;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const float x = fminf(fmaxf(y[j], -65504.0f), 65504.0f);
            hi[j] = (half_t)x;
            const uint32_t b = f32_to_e5m2((x - (float)hi[j]) * (float)(1 << BB_LO_SHIFT));
            if (j < 4) lo0 |= b << (8 * j); else lo1 |= b << (8 * (j - 4));
        }
        Apk[wideA_hi_u4(m, k8, mt_total)] = __builtin_bit_cast(u32x4, hi);
        *reinterpret_cast<uint2*>(reinterpret_cast<char*>(Apk) + wideA_lo_byte(m, k8, mt_total)) = make_uint2(lo0, lo1);
    }
}
static __device__ __forceinline__ void zero_panel8(u32x4* Apk, int m, int k8, int mt_total, int wide) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    if (!wide) { Apk[packA_u4(m, k8, mt_total, 0)] = z; Apk[packA_u4(m, k8, mt_total, 1)] = z; }
    else {
        Apk[wideA_hi_u4(m, k8, mt_total)] = z;
        *reinterpret_cast<uint2*>(reinterpret_cast<char*>(Apk) + wideA_lo_byte(m, k8, mt_total)) = make_uint2(0u, 0u);
    }
}
#endif

// ---- running (max, rescaled sum of exponentials, argmax) of a row of logits ------------------------------
// c = max_v softmax(l)_v = 1 / sum_v exp(l_v - max) needs only these three; ties go to the lowest token id.
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

// ---- kernel launchers (each enqueues on `s`) -----------------------------------------------------
struct GemmPlan { int split_k; int chunks_per_split; int nt; int mt = 4; };      // mt: m-tiles of 32 rows per workgroup
GemmPlan gemm_plan(int m_rows, int N, int K, int forced_split, int forced_nt);
GemmPlan gemm_plan_wide(int m_rows, int N, int K, int forced_split, int forced_nt, bool fusable = false);     // wide-format kernel: may take mt = 6
// Epilogue of launch_gemm: partial tiles P[split][m][n] (default); SiLU(gate) * up as the down projection's panel
// (swiglu_out, needs nt == 2 and no k split); or the vocabulary reduction of the LM head (vocab_part: per row and
// column tile one (max, sum, argmax); needs no k split and nt <= 2; P is then written only if keep_logits).
struct GemmEpilogue { u32x4* swiglu_out = nullptr; float4* vocab_part = nullptr; int mask_id = -1; int keep_logits = 1; };
// Optional events that receive the begin and end time stamps of the launch's own dispatch packet (profiling): unlike
// events recorded around a launch they add no packets to the stream and exclude the gap before the kernel.
struct LaunchStamps { hipEvent_t start = nullptr; hipEvent_t stop = nullptr; };
void launch_gemm(const u32x4* Wt, const u32x4* Apk, float* P, int mt_total, int N, int K, GemmPlan plan, hipStream_t s,
                 GemmEpilogue epi = GemmEpilogue(), LaunchStamps st = LaunchStamps());
void launch_tile_weights(const uint16_t* src, int rows, int K, u32x4* dst, int dst_row0, int interleave, hipStream_t s);
void launch_pack_rows(const float* A, int M, int K, u32x4* Apk, int mt_total, hipStream_t s);
// The same contraction with both operands in the wide format (fp16 + fp8 terms, see above); wscale[n] = 2^-S of weight
// row n.  swiglu_out as in GemmEpilogue (a wide-format panel).  ssq (with swiglu_out): the activation rows carry no
// RMSNorm scale yet, ssq[row][nblk] holds their sums of squares per block of columns (K = the model dimension) and
// the SwiGLU epilogue applies 1 / sqrt(sum / K + rms_eps) to gate and up.
void launch_gemm_wide(const u32x4* Wt, const float* wscale, const u32x4* Apk, float* P, int mt_total, int N, int K,
                      GemmPlan plan, hipStream_t s, u32x4* swiglu_out = nullptr, LaunchStamps st = LaunchStamps(),
                      const float* ssq = nullptr, int nblk = 0, float rms_eps = 0.f);
void launch_tile_weights_wide(const uint16_t* src, int rows, int K, u32x4* dst, float* scale_out, int dst_row0, int interleave,
                              hipStream_t s);
void launch_pack_rows_wide(const float* A, int M, int K, u32x4* Apk, int mt_total, hipStream_t s);

void launch_embed(const Dev& D, const uint16_t* emb, float* h, int rows_cap, hipStream_t s);
// Panels a kernel writes are two bf16 terms, or the wide format when its `wide` argument is set.
// h += sum of split-K partials; out = packed rmsnorm(h) * gain.  gather != 0: rows are the masked (LM-head) rows.
void launch_rmsnorm_pack(const Dev& D, float* h, const float* partial, int n_partial, size_t partial_stride,
                         const float* gain, u32x4* Apk, int mt_total, int gather, int bcast, int wide, hipStream_t s);
// Few rows: h += sum of split-K partials; out = packed h * gain WITHOUT the norm's 1 / rms, whose
// ingredients go to ssq[row][block] (returns the blocks per row); the consumers below apply it after the projection.
int launch_residual_pack(const Dev& D, float* h, const float* partial, int n_partial, size_t partial_stride,
                         const float* gain, u32x4* Apk, int mt_total, float* ssq, int wide, hipStream_t s);
// q,k,v = sum of partials (* 1 / rms of the row if ssq) + bias; RoPE; q -> Q, k,v -> cache rows (two fp16 terms each)
void launch_qkv_epilogue(const Dev& D, const float* qkv, int n_partial, size_t partial_stride, const float* bias,
                         half_t* Q, int layer, int rows_cap, const float* ssq, int nblk, hipStream_t s);
// act = SiLU(gate) * up from the fused (32-row interleaved) gate/up projection -> packed panel with K = f
void launch_swiglu_epilogue(const Dev& D, const float* gu, int n_partial, size_t partial_stride, int ldp, u32x4* Apk,
                            int rows_cap, int mt_total, int wide, const float* ssq, int nblk, hipStream_t s);
void launch_attention(const Dev& D, const half_t* Q, u32x4* Apk, int layer, int mt_total, int max_seg_rows,
                      int seg_base, int n_segs, int max_pages, float* part, size_t part_elems, int wide, hipStream_t s);
void launch_vocab_finish(const Dev& D, int lm_cap, int bcast, hipStream_t s);

void launch_pack_step(const Dev& D, int n_req, hipStream_t s);
void launch_pack_refresh(const Dev& D, int n_req, int mode, hipStream_t s);
void launch_page_copies(const Dev& D, hipStream_t s);
void launch_commit_merge(const Dev& D, int n_req, const uint16_t* lm_head, hipStream_t s);
void launch_read_kv(const Dev& D, int phys_table_row_slot, int branch, int layer, float* K, float* V, int L,
                    hipStream_t s);
void launch_write_kv(const Dev& D, int phys_table_row_slot, int branch, int layer, const float* K, const float* V, int L,
                     hipStream_t s);
void launch_kv_sqdist(const Dev& D, int gbr_a, int gbr_b, const half_t* snapK, const half_t* snapV, int snap_rows, int b_row,
                      int n_pages_used, double* out, hipStream_t s);
void launch_kv_snapshot(const Dev& D, int gbr, half_t* snapK, half_t* snapV, int snap_rows, int row, int n_pages_used, hipStream_t s);
