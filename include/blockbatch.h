/*
 * blockbatch.h - C ABI of the BlockBatch branch-batched denoising path for MI355X (gfx950).
 *
 * The calls follow Alg. 1 (App. D) of the paper.  One request = one prompt decoded by N
 * block-size branches; each branch owns a token row X_k, a window [start, end) and a KV
 * cache row (Sec. 5.1, App. D.1).
 *
 *   bb_refresh(BB_INIT)      InitialFullForward: one full forward on prompt + masks, the
 *                            cache shared by every branch row, logits for all G positions
 *   bb_denoise_step          GetActiveBranches + PackActiveBlocks + BatchedBlockForward
 *                            (Sec. 4.2) + top-1 confidence / argmax per masked row (Sec. 2.1)
 *   bb_merge_commit          DecodeCurrentBlock (Eq. 1), UpdateProbabilityMap,
 *                            AdvanceCompletedBlocks, MergeSync (Alg. 2), refresh cadence
 *   bb_refresh(BB_PERIODIC)  RefreshIfNeeded: K <- F(x) for every unfinished branch (App. A.1)
 *
 * Conventions
 *   - Every call returns 0 (BB_OK) or a negative error code; bb_last_error() gives a text.
 *     Nothing throws or aborts across this boundary (a failed host allocation inside a call is BB_ENOMEM).
 *   - All device work is enqueued on the HIP stream given to bb_create and is asynchronous,
 *     except where a call copies results to host memory (stated per call).
 *   - The library allocates no device memory: the caller passes one workspace of at least
 *     bb_workspace_bytes() bytes (256-byte aligned), which the context owns until bb_destroy.
 *   - Pointers named *_host are host memory, *_dev device memory.  Device pointers handed
 *     out in bb_step_view point into the workspace and stay valid until the next forward.
 *   - Branch / request state lives on the device; the host never needs to read it inside
 *     the decode loop.
 */
#ifndef BLOCKBATCH_H
#define BLOCKBATCH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BB_OK       0
#define BB_EINVAL  -1   /* bad argument or unsupported shape */
#define BB_ESTATE  -2   /* call order violated (e.g. step before the init refresh) */
#define BB_ENOMEM  -3   /* workspace too small / limits exceeded */
#define BB_EHIP    -4   /* HIP runtime error */

#define BB_INIT      0
#define BB_PERIODIC  1

#define BB_MAX_BRANCHES 8

typedef struct bb_ctx bb_ctx;

/* Model shape.  Pre-norm transformer, bidirectional attention, rotate-half RoPE, RMSNorm,
 * SwiGLU; head_dim must be 64 or 128; d_model, d_ffn multiples of 16; the row counts of all
 * projections multiples of 32; vocab a multiple of 32.  mask_id is the [M] token (Sec. 2.1);
 * its logit is treated as -inf so it is never predicted. */
typedef struct {
    int n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    float rope_base, rms_eps;
    int qkv_bias;
    int mask_id;
} bb_model_cfg;

/* Decoding hyper-parameters (Alg. 1 "Require" line; App. E.3 values tau_sync 8, tau_merge 0.5). */
typedef struct {
    float tau_dec;          /* Eq. 1: commit if confidence >= tau_dec (or most confident)   */
    float tau_merge;        /* Alg. 2: accept a merged token if P_d(i,v) >  tau_merge       */
    int   tau_sync;         /* Alg. 2: copy the leader if its lead is      >  tau_sync      */
    int   refresh_interval; /* R: block forwards between full-sequence refreshes            */
    int   leader_rule;      /* 0: most tokens decoded (Alg. 2); 1: highest mean confidence  */
    int   eos_id;           /* CheckEOS (Alg. 1): end-of-sequence token id, -1 = no EOS handling */
} bb_decode_cfg;

/* Capacity the workspace is sized for. */
typedef struct {
    int max_requests;       /* concurrently open requests                                   */
    int max_branches;       /* branches per request, <= BB_MAX_BRANCHES                     */
    int max_seq_len;        /* prompt + generation length                                   */
    int max_gen_len;        /* generation length                                            */
    int max_step_rows;      /* packed query rows of one bb_denoise_step (sum of block sizes
                               over all requests in the call)                               */
} bb_limits;

/* One weight tensor, bf16, row-major [rows][cols] ([out][in] for projections; a norm gain or
 * bias has rows = 1).  Names: tok_emb, lm_head, final_norm, and per layer i: l{i}.attn_norm,
 * l{i}.wq, l{i}.wk, l{i}.wv, l{i}.bq, l{i}.bk, l{i}.bv (only with qkv_bias), l{i}.wo,
 * l{i}.ffn_norm, l{i}.w_gate, l{i}.w_up, l{i}.w_down. */
typedef struct {
    const char* name;
    const void* data;       /* host or device memory, see on_device; caller keeps ownership */
    int on_device;
    long rows, cols;
} bb_tensor;

/* Per-branch state S_k (Alg. 1, initialisation) plus the counters Alg. 2 keeps. */
typedef struct {
    int block;              /* b_k                                                          */
    int start, end;         /* current window, absolute positions                           */
    int done;
    int tokens_decoded;     /* generation positions holding a token (as of the last commit) */
    int tokens_merged;      /* cumulative                                                   */
    int committed_threshold, committed_fallback;   /* cumulative Eq. 1 commits by arm       */
    int synced_from;        /* leader index if the last bb_merge_commit copied into this row, else -1 */
    float mean_conf;        /* mean top-1 confidence over the rows of the latest decode     */
} bb_branch_state;

/* Device-side results of the latest forward (bb_denoise_step, or bb_refresh(BB_INIT) where
 * the rows are the G generation positions of the common row).  counts_dev[0] = M_q packed
 * query rows, counts_dev[1] = M_lm rows that received logits. */
typedef struct {
    const int*   counts_dev;
    const int*   row_branch_dev;   /* [M_q] request_slot * max_branches + branch            */
    const int*   row_pos_dev;      /* [M_q] absolute position                               */
    const int*   lm_row_dev;       /* [M_lm] index into the packed rows                     */
    const int*   argmax_dev;       /* [M_lm] top-1 token                                    */
    const float* conf_dev;         /* [M_lm] top-1 probability                              */
    const float* lse_dev;          /* [M_lm] log-sum-exp of the row's logits                */
    const float* logits_dev;       /* [M_lm][vocab] fp32, mask column as computed (ignore); NULL unless
                                      bb_debug_keep_logits is on: the LM head reduces the logits of a row
                                      to (max, sum, argmax) in its epilogue and does not store them        */
    int rows_capacity;
} bb_step_view;

/* Host-side summary of one request after bb_merge_commit. */
typedef struct {
    int n_branches;
    int refresh_due;               /* R block forwards have run since the last refresh      */
    int all_done;
    int nfe_init, nfe_block, nfe_refresh;   /* one batched forward = one NFE (Sec. 5.1)      */
    int finished;                  /* 0 running; 1 every branch done; 2 an EOS-ready branch was selected */
    int winner;                    /* finished != 0: the branch whose row is the output (SelectEOSWinner, or
                                      the final argmax-progress selection of Alg. 1); else -1          */
    int eos_pos;                   /* absolute position of the winner's first EOS, -1 if it has none    */
    bb_branch_state branch[BB_MAX_BRANCHES];
} bb_request_stats;

size_t bb_workspace_bytes(const bb_model_cfg* model, const bb_limits* limits);

/* Create a context on the current device.  workspace_dev: device memory, 256-byte aligned,
 * >= bb_workspace_bytes(); hip_stream: a hipStream_t (NULL = default stream). */
int bb_create(bb_ctx** out, const bb_model_cfg* model, const bb_decode_cfg* decode,
              const bb_limits* limits, void* workspace_dev, size_t workspace_bytes, void* hip_stream);
int bb_destroy(bb_ctx* ctx);
const char* bb_last_error(const bb_ctx* ctx);

/* Copy the tensors into the workspace, re-tiled into MFMA fragment order (projections),
 * widened to fp32 (gains, biases) or as they are (embedding).  May be called several times
 * with disjoint subsets; synchronises the stream before returning so host sources can be
 * released.  Every tensor must have been loaded before the first forward. */
int bb_load_weights(bb_ctx* ctx, const bb_tensor* tensors, int n);

/* Alg. 1, initialisation: X_k = prompt + G masks for each of the N branches, windows at the end of
 * the prompt.  prompt_host: L_p token ids; block_sizes_host: N block sizes. */
int bb_request_open(bb_ctx* ctx, const int32_t* prompt_host, int L_p, int G,
                    const int* block_sizes_host, int N, int* req_id_out);
int bb_request_close(bb_ctx* ctx, int req_id);

/* Full-sequence forward(s).  BB_INIT: once per request, before anything else.  BB_PERIODIC:
 * recompute the cache row of every unfinished branch from its current tokens.  The listed requests are
 * packed into one forward as long as their rows fit the activation buffers (which hold max_branches *
 * max_seq_len rows), else into several. */
int bb_refresh(bb_ctx* ctx, const int* req_ids_host, int n, int mode);

/* One batched block forward over the current windows of all unfinished branches of the
 * listed requests; view_out (may be NULL) receives device pointers to its results. */
int bb_denoise_step(bb_ctx* ctx, const int* req_ids_host, int n, bb_step_view* view_out);

/* Commit / merge / sync on the results of the latest forward of the listed requests.
 * stats_out_host (may be NULL): n entries; when given, the call waits for the stream and
 * copies the summaries to the host; when NULL the call is asynchronous. */
int bb_merge_commit(bb_ctx* ctx, const int* req_ids_host, int n, bb_request_stats* stats_out_host);

/* Alg. 1 from start to end for requests that were opened and not yet initialised: the initial full
 * forward of each, then { block forward, commit / CheckEOS / merge / sync, refresh when due } over the
 * requests still running, until every one has finished (all branches done, or an EOS-ready branch
 * selected) or max_block_forwards batched forwards have run.  The loop reads one flags word per listed
 * request back (a single small copy) only when a refresh may fall due or the forward limit is reached:
 * in between, up to min(R, 8) forwards are enqueued back to back.  stats_out_host: n entries (may be NULL).  The output of
 * request i is row stats[i].winner of bb_get_tokens, up to stats[i].eos_pos if that is >= 0.
 * Returns BB_OK also when the forward limit stopped it (finished == 0 then). */
int bb_generate(bb_ctx* ctx, const int* req_ids_host, int n, int max_block_forwards, bb_request_stats* stats_out_host);

/* KV-consistency diagnostics of App. A.2 on the flattened cache state (all layers, keys and values) of
 * the branches of one initialised request:
 *   D_pair_host [N][N]: squared distance between the cache rows of branches i and j; *D_avg_host: their
 *                       mean over ordered pairs i != j (branch dispersion D_t);
 *   E_host [N]:         cache-consistency error ||K - F(x)||_2 of each unfinished branch (0 for finished ones).
 * E needs F(x): the call snapshots the rows into scratch_dev, runs bb_refresh(BB_PERIODIC) on the request
 * (so it counts as a refresh: K <- F(x) afterwards, refresh counters reset) and compares.  Pass E_host =
 * NULL to get the dispersion only, without scratch and without a refresh.  scratch_dev: device memory of
 * at least bb_kv_diag_scratch_bytes(), 16-byte aligned.  Synchronises the stream. */
size_t bb_kv_diag_scratch_bytes(bb_ctx* ctx, int req_id);
int bb_kv_diagnostics(bb_ctx* ctx, int req_id, void* scratch_dev, size_t scratch_bytes, double* E_host,
                      double* D_pair_host, double* D_avg_host);

/* ---- inspection and teacher forcing (tests, harness); all synchronise the stream ---- */
/* Device pointers to the results of the latest forward (what bb_denoise_step returns in
 * view_out; after bb_refresh(BB_INIT) of one request the rows are its G generation positions). */
int bb_get_view(bb_ctx* ctx, bb_step_view* view_out);
int bb_get_tokens(bb_ctx* ctx, int req_id, int32_t* X_host /* [N][L] */);
int bb_get_stats(bb_ctx* ctx, int req_id, bb_request_stats* out_host);
/* Overwrite token rows and branch windows (block sizes, counters are kept). */
int bb_set_state(bb_ctx* ctx, int req_id, const int32_t* X_host /* [N][L] */,
                 const bb_branch_state* branches_host /* [N] */);
/* Cache row of one branch in one layer as the attention of that branch sees it, widened to
 * fp32: K_host, V_host [L][n_kv_heads][head_dim]. */
int bb_get_kv(bb_ctx* ctx, int req_id, int branch, int layer, float* K_host, float* V_host);
/* Tests: overwrite the cache row of one branch in one layer with K_host, V_host [L][n_kv_heads][head_dim] (the layout
 * bb_get_kv returns; each value is stored as two fp16 terms, |value| <= 65504 or BB_EINVAL).  Pages the branch still
 * shares with the initial forward's row (App. D, Alg. 1: the broadcast cache) are first made private in every layer,
 * so no other branch sees the change.  BB_ESTATE before the request's initial forward.  Synchronises the stream. */
int bb_set_kv(bb_ctx* ctx, int req_id, int branch, int layer, const float* K_host, const float* V_host);
/* Plain device-to-host copy after a stream synchronise (for the pointers of bb_step_view). */
int bb_read_device(bb_ctx* ctx, const void* src_dev, void* dst_host, size_t bytes);
int bb_synchronize(bb_ctx* ctx);
/* ---- measurement: per-kernel-class timing with HIP events on the context's stream ---------
 * While enabled, every kernel launch of the forward is bracketed by two events (which
 * perturbs the timeline slightly: use it for per-kernel figures, not for end-to-end rates).
 * bb_profile_read waits for the stream, aggregates the recorded launches per class, copies
 * up to max_entries classes to out_host, returns their number in *n_out and resets. */
#define BB_K_GEMM_SKINNY 0   /* MFMA GEMM launches with <= 256 activation rows (weight streaming) */
#define BB_K_GEMM_WIDE   1   /* MFMA GEMM launches with  > 256 activation rows                     */
#define BB_K_ATTENTION   2
#define BB_K_GLUE        3   /* embedding, norms, RoPE/KV write, SwiGLU, vocabulary reduction, packing */
#define BB_K_POLICY      4   /* commit / merge / sync and page copies                                */
#define BB_K_CLASSES     5
typedef struct {
    int klass, launches;
    double total_ms;
    double bytes;            /* algorithmic bytes: weights streamed (GEMM), K/V read (attention)     */
    double flops;            /* algorithmic flops of the contraction (GEMM, attention)               */
} bb_profile_entry;
int bb_profile_enable(bb_ctx* ctx, int on);
int bb_profile_read(bb_ctx* ctx, bb_profile_entry* out_host, int max_entries, int* n_out);

/* C[M][N] = A[M][K] . W[N][K]^T through the same packing, tiling and MFMA kernels the
 * forward uses (kernel-level parity test).  A_host fp32, W_host bf16 bits, C_host fp32;
 * split_k = 0 lets the library choose. */
int bb_debug_gemm(bb_ctx* ctx, const float* A_host, const uint16_t* W_host, float* C_host,
                  int M, int N, int K, int split_k);
/* The same product through the kernel that passes with many rows use: activations as fp16 + a scaled e5m2 remainder,
 * weights as row-scaled fp16, converted to e4m3 in the kernel for the remainder's product (about 2^-16 relative
 * accuracy per product instead of 2^-17). */
int bb_debug_gemm_wide(bb_ctx* ctx, const float* A_host, const uint16_t* W_host, float* C_host,
                       int M, int N, int K, int split_k);
/* Tests and measurements: on == 0 makes the layer GEMMs use two bf16 activation terms like the LM head
 * (the default, on != 0, is the fp16 + fp8 operand format for them). */
int bb_debug_wide_format(bb_ctx* ctx, int on);

/* For callers that cannot allocate device memory or hand over a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): C[M][N] = A[M][K] . W[N][K]^T through the same re-tiling,
 * packing and MFMA kernels as the forward's projections, with every intermediate buffer (tiled weights, packed
 * hi/lo activation panel, split-K partial tiles) in a file-scope device array of 18 MiB that each GPU the
 * library runs on holds until the process ends.  No context is needed.
 *   A_dev fp32 row-major, W_dev bf16 bits row-major (16-byte aligned), C_dev fp32 row-major: device memory owned
 *   by the caller; hip_stream: a hipStream_t (NULL = default stream).  All work is enqueued on it; nothing is
 *   allocated, freed, memset or synchronised, so the call may be captured into a graph.
 *   Limits: 1 <= M <= 128; 32 <= N <= 4096, N % 32 == 0; 16 <= K <= 4096, K % 16 == 0; N * K64 <= 4 Mi with K64
 *   = K rounded up to 64; split_k 0 (the library chooses, at most 4) .. 4.  Beyond them: BB_ENOMEM; malformed
 *   arguments: BB_EINVAL; a HIP error: BB_EHIP (there is no context, hence no bb_last_error text).
 *   The array is shared by every call on that GPU and keeps the last call's contents (the call clears what it
 *   needs cleared): calls on different streams of one GPU that overlap in time race; serialise them.
 *   Results equal bb_debug_gemm's for the same split_k bit for bit (same kernels, same summation order). */
int bb_gemm_static(const float* A_dev, const uint16_t* W_dev, float* C_dev, int M, int N, int K, int split_k,
                   void* hip_stream);

/* Tests: on != 0 makes every later forward also store the fp32 logits of the rows that receive them (view's
 * logits_dev); off (the default) the logits exist only in the registers of the LM-head GEMM. */
int bb_debug_keep_logits(bb_ctx* ctx, int on);

/* Tuning knob: override the tile width (nt = 1: 128 columns, 2: 256, 3: 384; 0 = heuristic) and the
 * split-K factor (0 = heuristic) of one GEMM kind (1 O/down, 2 gate/up, 3 QKV; 0, the LM head, is fixed) for
 * panels of at most 128 rows.  Results are unchanged up to fp32 summation order. */
int bb_debug_set_gemm_plan(bb_ctx* ctx, int kind, int nt, int split_k);

/* Host-only query (no device is touched): the launch plan the library takes for C[M][N] = A[M][K] W[N][K]^T with
 * the heuristics on (wide != 0: the fp16 + fp8 operand kernel; fusable != 0: the caller could take SiLU(gate) * up
 * from the epilogue).  out[0] = k splits, out[1] = 64-k chunks per split, out[2] = weight tiles of 32 rows per wave
 * (workgroup tile = 128 out[2] columns), out[3] = m-tiles of 32 rows per workgroup, out[4] = workgroups launched.
 * Returns BB_EINVAL for M < 1, N < 32, K < 16, N % 32, K % 16 or out == NULL. */
int bb_debug_gemm_plan(int M, int N, int K, int wide, int fusable, int out[5]);

/* Measurement aid: copy `bytes` (a multiple of 16) from src_dev to dst_dev (device pointers, disjoint,
 * 16-byte aligned) on the context's stream with a plain kernel that moves 16 bytes per lane, the access
 * width of the library's kernels.  A known-size reference for scaling hardware traffic counters, whose
 * reading per byte depends on the request size.  Asynchronous; BB_EINVAL on misaligned arguments. */
int bb_debug_copy16(bb_ctx* ctx, const void* src_dev, void* dst_dev, size_t bytes);

/* Measurement aid: the rate at which this chip issues dense 32x32x16 bf16 MFMAs when it does nothing else (1024
 * workgroups of four waves, eight independent accumulator tiles per wave), in TFLOP/s, timed with HIP events on
 * the context's stream after a warm-up launch of the same length (about 20 ms each, so that the clocks settle under the load).  The measured denominator quoted beside the nominal 2.5 PFLOP/s.
 * Uses the activation region of the workspace as its output; synchronises the stream. */
int bb_debug_mfma_rate(bb_ctx* ctx, double* tflops_out_host);

#ifdef __cplusplus
}
#endif
#endif
