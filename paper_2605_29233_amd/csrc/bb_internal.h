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
    float tau_dec, tau_merge; int tau_sync, refresh_interval, leader_rule;
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
    half_t* Kc;                 // [n_layers][phys_rows][lpad][hkv][term][hd]
    half_t* Vt;                 // [n_layers][phys_rows][hkv][term][hd][lpad]   (transposed)
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
    PageCopy* copies;           // [max_req*max_br*n_pages]
    int* req_list;              // [max_req] request slots of the current call
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

// ---- bf16 helpers (round to nearest even, finite inputs) --------------------------------------
static inline __host__ __device__ uint16_t f32_to_bf16_rne(float x) {
    union { float f; uint32_t u; } v; v.f = x;
    uint32_t u = v.u + 0x7FFFu + ((v.u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
static inline __host__ __device__ float bf16_to_f32(uint16_t b) {
    union { float f; uint32_t u; } v; v.u = ((uint32_t)b) << 16; return v.f;
}

// ---- kernel launchers (each enqueues on `s`) -----------------------------------------------------
struct GemmPlan { int split_k; int chunks_per_split; int nt; };
GemmPlan gemm_plan(int m_rows, int N, int K, int forced_split, int forced_nt);
void launch_gemm(const u32x4* Wt, const u32x4* Apk, float* P, int mt_total, int N, int K, GemmPlan plan, hipStream_t s);
void launch_tile_weights(const uint16_t* src, int rows, int K, u32x4* dst, int dst_row0, int interleave, hipStream_t s);
void launch_pack_rows(const float* A, int M, int K, u32x4* Apk, int mt_total, hipStream_t s);

void launch_embed(const Dev& D, const uint16_t* emb, float* h, int rows_cap, hipStream_t s);
// h += sum of split-K partials; out = packed rmsnorm(h) * gain.  gather != 0: rows are the masked (LM-head) rows.
void launch_rmsnorm_pack(const Dev& D, float* h, const float* partial, int n_partial, size_t partial_stride,
                         const float* gain, u32x4* Apk, int mt_total, int gather, int bcast, hipStream_t s);
// q,k,v = sum of partials + bias; RoPE; q -> Q, k,v -> cache rows (two fp16 terms each)
void launch_qkv_epilogue(const Dev& D, const float* qkv, int n_partial, size_t partial_stride, const float* bias,
                         half_t* Q, int layer, int rows_cap, hipStream_t s);
// act = SiLU(gate) * up from the fused (64-row interleaved) gate/up projection -> packed panel with K = f
void launch_swiglu_epilogue(const Dev& D, const float* gu, int n_partial, size_t partial_stride, int ldp, u32x4* Apk,
                            int rows_cap, int mt_total, hipStream_t s);
void launch_attention(const Dev& D, const half_t* Q, u32x4* Apk, int layer, int mt_total, int max_seg_rows,
                      int seg_base, int n_segs, int max_pages, float* part, size_t part_elems, hipStream_t s);
void launch_vocab_reduce(const Dev& D, const float* logits, int lm_cap, int bcast, hipStream_t s);

void launch_pack_step(const Dev& D, int n_req, hipStream_t s);
void launch_pack_refresh(const Dev& D, int slot, int mode, hipStream_t s);
void launch_page_copies(const Dev& D, hipStream_t s);
void launch_commit_merge(const Dev& D, int n_req, const uint16_t* lm_head, hipStream_t s);
void launch_read_kv(const Dev& D, int phys_table_row_slot, int branch, int layer, float* K, float* V, int L,
                    hipStream_t s);
