// Host side of libblockbatch: context, workspace layout, weight loading and the four calls
// of the boundary.  The host only sequences kernel launches; every step of the path runs in
// the kernels and all request state stays on the device.
#include "bb_internal.h"
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <new>
#include <algorithm>
#include <string>
#include <vector>

struct LayerW {
    u32x4 *wqkv, *wo, *wgu, *wdown;     // tiled bf16 (passes with few rows: two bf16 activation terms)
    u32x4 *wqkv_w, *wo_w, *wgu_w, *wdown_w;     // the same matrices as row-scaled fp16 (wide format, passes with many rows)
    float *s_qkv, *s_o, *s_gu, *s_down; // 2^-S per weight row of the wide-format copies
    float *g_attn, *g_ffn, *bqkv;       // fp32
};

struct HostReq { int in_use, L_p, G, L, N, blocks[BB_MAX_BRANCHES], initialised; };

struct bb_ctx {
    bb_model_cfg m; bb_decode_cfg dc; bb_limits lim;
    hipStream_t stream;
    char* ws; size_t ws_bytes;
    Dev D;
    std::vector<LayerW> layers;
    uint16_t* emb; u32x4* lm; float* g_final;
    std::vector<char> loaded;           // per tensor slot
    int n_expected;
    // activations
    float *h, *qkv, *part, *gu, *logits, *dbg, *attn_part, *wscales, *ssq;
    size_t attn_part_elems;
    u32x4 *Apk, *Apk2; half_t* Q; char* stage;     // Apk2: SwiGLU output panel (written while Apk is still being read)
    size_t qkv_elems, part_elems, gu_elems, stage_bytes, dbg_bytes;
    int refresh_rows_cap, ngu;
    int force_nt[4], force_split[4];   // tuning overrides per epilogue kind (0 = heuristic)
    std::vector<HostReq> reqs;
    std::vector<int> req_host, flags_host;   // request list as last uploaded (the caller's array is never read after the call returns)
    char* d_stats;                      // device staging for stats copies
    std::string err;
    int last_forward_rows, last_lm_cap;
    int wide_off;                       // tests: the layer GEMMs use two bf16 terms like the LM head (bb_debug_wide_format)
    int keep_logits;                    // tests: the LM head also stores its fp32 logits (bb_debug_keep_logits)
    // per-launch event timing (bb_profile_*)
    int prof_on;
    struct ProfRec { hipEvent_t a, b; int klass; double bytes, flops; bool own_a; };
    std::vector<ProfRec> prof;
    std::vector<hipEvent_t> ev_pool;
    bool prof_chain;                    // inside a forward: launches are back to back, one event per boundary
    hipEvent_t prof_prev_end;
};

// Bracket one launch with events when profiling is on.  Inside a forward the launches follow each other
// without anything in between, so the end event of one launch also serves as the start of the next:
// one event packet per kernel boundary keeps the timeline close to the unprofiled one.
//
// stamped = true (the GEMM launches): the scope's two events are not recorded around the launch but handed to it and
// receive the begin and end time stamps of its dispatch packet, i.e. the kernel's own duration as a profiler's
// dispatch records show it, with no packet added to the stream.
struct ProfScope {
    bb_ctx* c; int idx; bool stamped;
    ProfScope(bb_ctx* c_, int klass, double bytes, double flops, bool stamped_ = false) : c(c_), idx(-1), stamped(stamped_) {
        if (!c->prof_on) return;
        auto get = [&]() { hipEvent_t e; if (c->ev_pool.empty()) { if (hipEventCreate(&e) != hipSuccess) return (hipEvent_t) nullptr; }
                           else { e = c->ev_pool.back(); c->ev_pool.pop_back(); } return e; };
        const bool chain = !stamped && c->prof_chain && c->prof_prev_end;
        bb_ctx::ProfRec r{chain ? c->prof_prev_end : get(), get(), klass, bytes, flops, !chain};
        if (!r.a || !r.b) return;
        if (!chain && !stamped) (void)hipEventRecord(r.a, c->stream);
        c->prof.push_back(r); idx = (int)c->prof.size() - 1;
    }
    LaunchStamps stamps() const { LaunchStamps st; if (idx >= 0 && stamped) { st.start = c->prof[idx].a; st.stop = c->prof[idx].b; } return st; }
    ~ProfScope() {
        if (idx < 0) return;
        if (!stamped) (void)hipEventRecord(c->prof[idx].b, c->stream);
        c->prof_prev_end = c->prof[idx].b;
    }
};
#define PROF(klass, bytes, flops) ProfScope prof_scope_(c, klass, bytes, flops)
#define PROF_STAMPED(klass, bytes, flops) ProfScope prof_scope_(c, klass, bytes, flops, true)

static int fail(bb_ctx* c, int code, const std::string& msg) { if (c) c->err = msg; return code; }
#define HIPCHK(c, expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) \
    return fail(c, BB_EHIP, std::string(#expr) + ": " + hipGetErrorString(e_)); } while (0)

// ---- workspace layout (one pass computes sizes, the same pass assigns pointers) -----------------
struct Bump {
    char* base; size_t off;
    template <class T> T* take(size_t n) {
        off = align_up(off, 256);
        T* p = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += n * sizeof(T);
        return p;
    }
};

// Passes over more rows than BB_SKINNY_ROWS count as bound by the matrix pipes in the profile classes.
// The layer GEMMs of every pass take the wide format (fp16 + fp8 operands): with more than one group of 128 rows the
// matrix work sets the time and three quarters of it is 9-25 % faster; with one group the kernel streams the weights as
// fast as the two-term kernel in isolation and 6 % faster in the forward, where the chip's clock follows the matrix
// load.  The LM head keeps two bf16 terms (vocabulary reduction in the epilogue of that kernel).
// Up to BB_DEFER_ROWS rows the RMSNorm scale is applied after the projection (residual_pack_kernel).
#define BB_SKINNY_ROWS 256
#define BB_DEFER_ROWS 128

// Largest split-K output over every row count the forward may be called with.
static size_t buf_elems(int rows_cap, int N, int K, int forced_nt_wide = 0) {
    size_t best = 0;
    for (int rows = 32; rows <= (rows_cap + 31) / 32 * 32; rows += 32) {
        // (both operand formats: the wide format can be switched off at run time)
        for (int variant = 0; variant < 3; ++variant) {
            auto plan = [&](int nt) { return variant == 0 ? gemm_plan(rows, N, K, 0, nt) : gemm_plan_wide(rows, N, K, 0, nt, variant == 2); };
            GemmPlan p = plan(rows > 128 ? forced_nt_wide : 0);
            size_t e = (size_t)p.split_k * rows * N;
            if (e > best) best = e;
            if (rows > BB_DEFER_ROWS) {         // gate/up with the fused SwiGLU epilogue: two tiles per wave
                p = plan(forced_nt_wide);
                e = (size_t)p.split_k * rows * N;
                if (e > best) best = e;
            }
        }
    }
    // room for the largest split a tuning override may ask for on a skinny panel
    size_t tune = (size_t)BB_MAX_SPLITK * std::min((rows_cap + 31) / 32 * 32, 128) * N;
    return std::max(best, tune);
}

static int check_cfg(const bb_model_cfg* m, const bb_limits* l, std::string* why) {
    auto bad = [&](const char* s) { if (why) *why = s; return BB_EINVAL; };
    if (!m || !l) return bad("null config");
    if (m->head_dim != 64 && m->head_dim != 128) return bad("head_dim must be 64 or 128");
    if (m->n_q_heads % m->n_kv_heads) return bad("n_q_heads must be a multiple of n_kv_heads");
    if (m->d_model % 64 || m->d_ffn % 16) return bad("d_model must be a multiple of 64 and d_ffn of 16");
    if (m->d_model > 8192) return bad("d_model must not exceed 8192");
    if (m->d_model % 32 || (2 * m->d_ffn) % 32 || m->vocab % 32) return bad("projection row counts must be multiples of 32");
    if ((m->n_q_heads * m->head_dim) % 128 || (m->n_kv_heads * m->head_dim) % 128) return bad("q and kv widths must be multiples of 128");
    if (m->mask_id < 0 || m->mask_id >= m->vocab) return bad("mask_id out of range");
    if (l->max_branches < 1 || l->max_branches > BB_MAX_BRANCHES) return bad("max_branches out of range");
    if (l->max_requests < 1 || l->max_requests * l->max_branches > 256) return bad("max_requests * max_branches must be <= 256");
    if (l->max_gen_len < 1 || l->max_gen_len >= l->max_seq_len) return bad("max_gen_len must be in [1, max_seq_len)");
    if (l->max_step_rows < 1) return bad("max_step_rows must be positive");
    return BB_OK;
}

static void layout(bb_ctx* c, char* base, size_t* total) {
    const bb_model_cfg& m = c->m; const bb_limits& l = c->lim;
    Bump b{base, 0};
    Dev& D = c->D;
    const int lpad = (int)align_up(l.max_seq_len, BB_PAGE);
    const int nqkv = (m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim, nq = m.n_q_heads * m.head_dim;
    const int refresh_rows = l.max_branches * l.max_seq_len;
    const int rows_cap = std::max(l.max_step_rows, refresh_rows);
    const int rows_pad = (rows_cap + 31) / 32 * 32;
    const int lm_cap = std::max(l.max_step_rows, l.max_gen_len);
    const int lm_pad = (lm_cap + 31) / 32 * 32;
    const int nbr = l.max_requests * l.max_branches;
    const size_t phys_rows = (size_t)l.max_requests * (l.max_branches + 1);
    D.n_layers = m.n_layers; D.d = m.d_model; D.hq = m.n_q_heads; D.hkv = m.n_kv_heads; D.hd = m.head_dim;
    D.f = m.d_ffn; D.vocab = m.vocab; D.mask_id = m.mask_id; D.qkv_bias = m.qkv_bias; D.nqkv = nqkv;
    D.rms_eps = m.rms_eps;
    D.tau_dec = c->dc.tau_dec; D.tau_merge = c->dc.tau_merge; D.tau_sync = c->dc.tau_sync;
    D.refresh_interval = c->dc.refresh_interval; D.leader_rule = c->dc.leader_rule; D.eos_id = c->dc.eos_id;
    D.max_req = l.max_requests; D.max_br = l.max_branches; D.lpad = lpad; D.n_pages = lpad / BB_PAGE;
    D.gmax = l.max_gen_len; D.rows_cap = rows_cap; D.lm_cap = lm_cap; D.phys_per_req = l.max_branches + 1;
    c->refresh_rows_cap = refresh_rows;
    // state (zeroed at create)
    D.hdr = b.take<ReqHeader>(l.max_requests);
    D.br = b.take<bb_branch_state>(nbr);
    D.X = b.take<int>((size_t)nbr * lpad);
    D.table = b.take<int>((size_t)nbr * D.n_pages);
    D.map_hf = b.take<float>((size_t)nbr * D.gmax * m.d_model);
    D.map_lse = b.take<float>((size_t)nbr * D.gmax);
    D.map_conf = b.take<float>((size_t)nbr * D.gmax);
    D.map_pred = b.take<int>((size_t)nbr * D.gmax);
    D.rope_cos = b.take<float>((size_t)lpad * m.head_dim / 2);
    D.rope_sin = b.take<float>((size_t)lpad * m.head_dim / 2);
    D.counts = b.take<int>(16);
    D.row_tok = b.take<int>(rows_pad); D.row_pos = b.take<int>(rows_pad);
    D.row_gbr = b.take<int>(rows_pad); D.row_phys = b.take<int>(rows_pad);
    D.seg_off = b.take<int>(nbr); D.seg_rows = b.take<int>(nbr);
    D.lm_row = b.take<int>(lm_pad);
    D.out_pred = b.take<int>(lm_pad); D.out_conf = b.take<float>(lm_pad); D.out_lse = b.take<float>(lm_pad);
    D.vr_tiles = (m.vocab / 32 + (m.vocab / 32 >= 8 ? 7 : 3)) / (m.vocab / 32 >= 8 ? 8 : 4);   // column tiles of the LM-head GEMM (256 or 128 columns)
    D.vr_part = b.take<float4>((size_t)lm_pad * D.vr_tiles);
    D.copies = b.take<PageCopy>((size_t)nbr * D.n_pages);
    D.req_list = b.take<int>(l.max_requests);
    D.req_flags = b.take<int>(l.max_requests);
    D.commit_skip = b.take<int>(l.max_requests);
    D.merge_p = b.take<float>((size_t)nbr * l.max_branches * D.gmax);
    D.merge_x0 = b.take<int>((size_t)nbr * D.gmax);
    c->d_stats = b.take<char>(sizeof(ReqHeader) + sizeof(bb_branch_state) * BB_MAX_BRANCHES);
    D.Kc = b.take<half_t>((size_t)m.n_layers * phys_rows * lpad * m.n_kv_heads * m.head_dim * 2);
    D.Vt = b.take<half_t>((size_t)m.n_layers * phys_rows * lpad * m.n_kv_heads * m.head_dim * 2);
    size_t state_end = align_up(b.off, 256);
    // activations
    const int kmax = std::max(std::max(m.d_model, m.d_ffn), nq);
    c->ngu = (m.d_ffn + 63) / 64 * 128;            // fused gate/up rows: 32 gate rows alternate with the 32 up rows of the same features; f padded to 64
    c->h = b.take<float>((size_t)rows_pad * m.d_model);
    c->Apk = b.take<u32x4>((size_t)rows_pad * kmax / 8 * BB_SPLIT);
    c->Apk2 = b.take<u32x4>((size_t)rows_pad * ((m.d_ffn + 63) / 64 * 64) / 8 * BB_SPLIT);
    c->Q = b.take<half_t>((size_t)rows_pad * nq * 2);
    c->qkv_elems = buf_elems(rows_cap, nqkv, m.d_model);
    c->part_elems = std::max(buf_elems(rows_cap, m.d_model, nq), buf_elems(rows_cap, m.d_model, m.d_ffn));
    c->gu_elems = buf_elems(rows_cap, c->ngu, m.d_model, 2);
    c->qkv = b.take<float>(c->qkv_elems);
    c->part = b.take<float>(c->part_elems);
    c->gu = b.take<float>(c->gu_elems);
    c->logits = b.take<float>((size_t)lm_pad * m.vocab);
    // split-KV partial results of block-step attention: up to 8 splits of every 32-row tile
    c->attn_part_elems = ((size_t)l.max_step_rows * (m.n_q_heads / m.n_kv_heads) / 32 + nbr) * m.n_kv_heads * 8 * (64 + 32 * m.head_dim);
    c->attn_part = b.take<float>(c->attn_part_elems);
    c->ssq = b.take<float>((size_t)(BB_DEFER_ROWS + 31) / 32 * 32 * ((m.d_model + 2047) / 2048));     // block sums of squares of the rows of a block step
    c->dbg_bytes = 2 * (size_t)lpad * m.n_kv_heads * m.head_dim * sizeof(float);
    c->dbg = b.take<float>(c->dbg_bytes / sizeof(float));
    size_t biggest = (size_t)m.vocab * m.d_model;
    biggest = std::max(biggest, (size_t)m.d_ffn * m.d_model);
    biggest = std::max(biggest, (size_t)nq * m.d_model);
    c->stage_bytes = biggest * 2;
    c->stage = b.take<char>(c->stage_bytes);
    // weights
    c->emb = b.take<uint16_t>((size_t)m.vocab * m.d_model);
    c->lm = b.take<u32x4>((size_t)m.vocab * m.d_model / 8);
    c->g_final = b.take<float>(m.d_model);
    c->layers.resize(m.n_layers);
    for (auto& L : c->layers) {
        L.wqkv = b.take<u32x4>((size_t)nqkv * m.d_model / 8);
        L.wo = b.take<u32x4>((size_t)m.d_model * nq / 8);
        L.wgu = b.take<u32x4>((size_t)c->ngu * m.d_model / 8);
        L.wdown = b.take<u32x4>((size_t)m.d_model * ((m.d_ffn + 63) / 64 * 64) / 8);
        L.g_attn = b.take<float>(m.d_model); L.g_ffn = b.take<float>(m.d_model);
        L.bqkv = b.take<float>(nqkv);
    }
    // wide-format copies (fp16, tiled like the bf16 ones) and their row scales; scales first, in one run that bb_create clears
    auto wide_u4 = [](int N, int K) { return (size_t)N * ((K + 63) / 64 * 64) / 8; };
    const size_t scales_per_layer = (size_t)nqkv + 2 * (size_t)m.d_model + c->ngu;
    c->wscales = b.take<float>((size_t)m.n_layers * scales_per_layer);
    size_t so = 0;
    for (auto& L : c->layers) {
        float* sp = c->wscales ? c->wscales + so : nullptr;
        L.s_qkv = sp; L.s_o = sp ? sp + nqkv : nullptr; L.s_gu = sp ? sp + nqkv + m.d_model : nullptr;
        L.s_down = sp ? sp + nqkv + m.d_model + c->ngu : nullptr;
        so += scales_per_layer;
        L.wqkv_w = b.take<u32x4>(wide_u4(nqkv, m.d_model));
        L.wo_w = b.take<u32x4>(wide_u4(m.d_model, nq));
        L.wgu_w = b.take<u32x4>(wide_u4(c->ngu, m.d_model));
        L.wdown_w = b.take<u32x4>(wide_u4(m.d_model, m.d_ffn));
    }
    (void)state_end;
    *total = align_up(b.off, 256);
}

extern "C" size_t bb_workspace_bytes(const bb_model_cfg* model, const bb_limits* limits) {
    try {
        if (check_cfg(model, limits, nullptr) != BB_OK) return 0;
        bb_ctx tmp{};
        tmp.m = *model; tmp.lim = *limits; tmp.dc = bb_decode_cfg{};
        size_t total = 0;
        layout(&tmp, nullptr, &total);
        return total;
    } catch (...) { return 0; }
}

static int bb_create_impl(bb_ctx** out, const bb_model_cfg* model, const bb_decode_cfg* decode,
                          const bb_limits* limits, void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
    if (!out || !decode || !workspace_dev) return BB_EINVAL;
    std::string why;
    if (check_cfg(model, limits, &why) != BB_OK) return BB_EINVAL;
    if (decode->refresh_interval < 1) return BB_EINVAL;
    if (reinterpret_cast<uintptr_t>(workspace_dev) % 256) return BB_EINVAL;
    std::unique_ptr<bb_ctx> holder(new bb_ctx{});          // released to the caller only when everything succeeded
    bb_ctx* c = holder.get();
    c->m = *model; c->dc = *decode; c->lim = *limits;
    c->stream = (hipStream_t)hip_stream;
    size_t total = 0;
    layout(c, (char*)workspace_dev, &total);
    if (total > workspace_bytes) return BB_ENOMEM;
    c->ws = (char*)workspace_dev; c->ws_bytes = workspace_bytes;
    c->reqs.assign(limits->max_requests, HostReq{});
    c->n_expected = 3 + model->n_layers * (model->qkv_bias ? 12 : 9);
    c->loaded.assign(3 + model->n_layers * 12, 0);
    // zero state, caches and activations once (fp16 garbage in never-written cache tails would
    // otherwise reach 0 * NaN in the attention's P.V product)
    size_t zero_bytes = (char*)c->emb - c->ws;
    hipError_t e = hipMemsetAsync(c->ws, 0, zero_bytes, c->stream);
    if (e != hipSuccess) return BB_EHIP;
    if (model->d_ffn % 64)            // padded gate/up rows and the down projection's padded k columns must be zero
        for (auto& L : c->layers) {
            if (e == hipSuccess) e = hipMemsetAsync(L.wgu, 0, (size_t)c->ngu * model->d_model * 2, c->stream);
            if (e == hipSuccess) e = hipMemsetAsync(L.wdown, 0, (size_t)model->d_model * ((model->d_ffn + 63) / 64 * 64) * 2, c->stream);
        }
    // row scales of the wide-format weights: rows no tensor fills (padding of the fused gate/up matrix) must scale by 0
    if (e == hipSuccess)
        e = hipMemsetAsync(c->wscales, 0, sizeof(float) * model->n_layers * ((size_t)c->D.nqkv + 2 * (size_t)model->d_model + c->ngu), c->stream);
    if (model->d_ffn % 64)
        for (auto& L : c->layers) {
            const size_t gu_b = (size_t)c->ngu * model->d_model * 2;
            const size_t dn_b = (size_t)model->d_model * ((model->d_ffn + 63) / 64 * 64) * 2;
            if (e == hipSuccess) e = hipMemsetAsync(L.wgu_w, 0, gu_b, c->stream);
            if (e == hipSuccess) e = hipMemsetAsync(L.wdown_w, 0, dn_b, c->stream);
        }
    if (e != hipSuccess) return BB_EHIP;
    // rotary table in double precision on the host
    const int half = model->head_dim / 2, lpad = c->D.lpad;
    std::vector<float> cs((size_t)lpad * half), sn((size_t)lpad * half);
    for (int p = 0; p < lpad; ++p)
        for (int j = 0; j < half; ++j) {
            double th = (double)p * std::pow((double)model->rope_base, -2.0 * j / model->head_dim);
            cs[(size_t)p * half + j] = (float)std::cos(th);
            sn[(size_t)p * half + j] = (float)std::sin(th);
        }
    e = hipMemcpyAsync(c->D.rope_cos, cs.data(), cs.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = hipMemcpyAsync(c->D.rope_sin, sn.data(), sn.size() * 4, hipMemcpyHostToDevice, c->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(c->stream);
    if (e != hipSuccess) return BB_EHIP;
    *out = holder.release();
    return BB_OK;
}

static int bb_destroy_impl(bb_ctx* ctx) {
    if (!ctx) return BB_EINVAL;
    (void)hipStreamSynchronize(ctx->stream);
    for (auto& r : ctx->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (auto e : ctx->ev_pool) (void)hipEventDestroy(e);
    delete ctx;
    return BB_OK;
}

extern "C" const char* bb_last_error(const bb_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

// ---- weights ------------------------------------------------------------------------------------
__global__ void widen_bf16_kernel(const uint16_t* __restrict__ src, float* __restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = bf16_to_f32(src[i]);
}

static int load_one(bb_ctx* c, const bb_tensor& t) {
    const bb_model_cfg& m = c->m;
    const int hd = m.head_dim, nq = m.n_q_heads * hd, nkv = m.n_kv_heads * hd, d = m.d_model, f = m.d_ffn;
    std::string name = t.name ? t.name : "";
    size_t bytes = (size_t)t.rows * t.cols * 2;
    if (!t.data || t.rows <= 0 || t.cols <= 0) return fail(c, BB_EINVAL, "bad tensor " + name);
    if (bytes > c->stage_bytes) return fail(c, BB_EINVAL, "tensor larger than any expected: " + name);
    const uint16_t* src = (const uint16_t*)t.data;
    if (!t.on_device) {
        HIPCHK(c, hipMemcpyAsync(c->stage, t.data, bytes, hipMemcpyHostToDevice, c->stream));
        src = (const uint16_t*)c->stage;
    }
    auto expect = [&](long r, long k) { return t.rows == r && t.cols == k; };
    auto widen = [&](float* dst, size_t n) {
        widen_bf16_kernel<<<(unsigned)((n + 255) / 256), 256, 0, c->stream>>>(src, dst, n);
    };
    int slot = -1; bool ok = false;
    if (name == "tok_emb") {
        slot = 0; ok = expect(m.vocab, d);
        if (ok) HIPCHK(c, hipMemcpyAsync(c->emb, src, bytes, hipMemcpyDeviceToDevice, c->stream));
    } else if (name == "lm_head") {
        slot = 1; ok = expect(m.vocab, d);
        if (ok) launch_tile_weights(src, m.vocab, d, c->lm, 0, 0, c->stream);
    } else if (name == "final_norm") {
        slot = 2; ok = t.rows * t.cols == d;
        if (ok) widen(c->g_final, d);
    } else if (name.size() > 2 && name[0] == 'l') {
        size_t dot = name.find('.');
        if (dot == std::string::npos) return fail(c, BB_EINVAL, "unknown tensor " + name);
        int li = atoi(name.substr(1, dot - 1).c_str());
        if (li < 0 || li >= m.n_layers) return fail(c, BB_EINVAL, "layer out of range: " + name);
        LayerW& L = c->layers[li];
        std::string k = name.substr(dot + 1);
        const char* keys[12] = {"attn_norm", "wq", "wk", "wv", "bq", "bk", "bv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"};
        int ki = -1;
        for (int i = 0; i < 12; ++i) if (k == keys[i]) ki = i;
        if (ki < 0) return fail(c, BB_EINVAL, "unknown tensor " + name);
        slot = 3 + li * 12 + ki;
        switch (ki) {
            case 0: ok = t.rows * t.cols == d; if (ok) widen(L.g_attn, d); break;
            case 1: ok = expect(nq, d); if (ok) { launch_tile_weights(src, nq, d, L.wqkv, 0, 0, c->stream); launch_tile_weights_wide(src, nq, d, L.wqkv_w, L.s_qkv, 0, 0, c->stream); } break;
            case 2: ok = expect(nkv, d); if (ok) { launch_tile_weights(src, nkv, d, L.wqkv, nq, 0, c->stream); launch_tile_weights_wide(src, nkv, d, L.wqkv_w, L.s_qkv, nq, 0, c->stream); } break;
            case 3: ok = expect(nkv, d); if (ok) { launch_tile_weights(src, nkv, d, L.wqkv, nq + nkv, 0, c->stream); launch_tile_weights_wide(src, nkv, d, L.wqkv_w, L.s_qkv, nq + nkv, 0, c->stream); } break;
            case 4: ok = m.qkv_bias && t.rows * t.cols == nq; if (ok) widen(L.bqkv, nq); break;
            case 5: ok = m.qkv_bias && t.rows * t.cols == nkv; if (ok) widen(L.bqkv + nq, nkv); break;
            case 6: ok = m.qkv_bias && t.rows * t.cols == nkv; if (ok) widen(L.bqkv + nq + nkv, nkv); break;
            case 7: ok = expect(d, nq); if (ok) { launch_tile_weights(src, d, nq, L.wo, 0, 0, c->stream); launch_tile_weights_wide(src, d, nq, L.wo_w, L.s_o, 0, 0, c->stream); } break;
            case 8: ok = t.rows * t.cols == d; if (ok) widen(L.g_ffn, d); break;
            case 9: ok = expect(f, d); if (ok) { launch_tile_weights(src, f, d, L.wgu, 0, 1, c->stream); launch_tile_weights_wide(src, f, d, L.wgu_w, L.s_gu, 0, 1, c->stream); } break;
            case 10: ok = expect(f, d); if (ok) { launch_tile_weights(src, f, d, L.wgu, 32, 1, c->stream); launch_tile_weights_wide(src, f, d, L.wgu_w, L.s_gu, 32, 1, c->stream); } break;
            case 11: ok = expect(d, f); if (ok) { launch_tile_weights(src, d, f, L.wdown, 0, 0, c->stream); launch_tile_weights_wide(src, d, f, L.wdown_w, L.s_down, 0, 0, c->stream); } break;
        }
    } else return fail(c, BB_EINVAL, "unknown tensor " + name);
    if (!ok) return fail(c, BB_EINVAL, "shape mismatch for " + name);
    HIPCHK(c, hipGetLastError());
    if (!t.on_device) HIPCHK(c, hipStreamSynchronize(c->stream));      // staging is reused by the next tensor
    c->loaded[slot] = 1;
    return BB_OK;
}

static int bb_load_weights_impl(bb_ctx* ctx, const bb_tensor* tensors, int n) {
    if (!ctx || !tensors || n < 0) return BB_EINVAL;
    for (int i = 0; i < n; ++i) {
        int rc = load_one(ctx, tensors[i]);
        if (rc != BB_OK) return rc;
    }
    HIPCHK(ctx, hipStreamSynchronize(ctx->stream));
    return BB_OK;
}

static bool weights_complete(const bb_ctx* c) {
    int n = 0;
    for (char x : c->loaded) n += x;
    return n == c->n_expected;
}

// ---- requests ---------------------------------------------------------------------------------------
static int bb_request_open_impl(bb_ctx* c, const int32_t* prompt, int L_p, int G, const int* blocks, int N, int* req_id) {
    if (!c || !prompt || !blocks || !req_id) return BB_EINVAL;
    if (L_p < 1 || G < 1 || N < 1) return fail(c, BB_EINVAL, "bad request shape");
    if (N > c->lim.max_branches || L_p + G > c->lim.max_seq_len || G > c->lim.max_gen_len)
        return fail(c, BB_ENOMEM, "request exceeds the limits the workspace was sized for");
    int slot = -1;
    for (int i = 0; i < c->lim.max_requests; ++i) if (!c->reqs[i].in_use) { slot = i; break; }
    if (slot < 0) return fail(c, BB_ENOMEM, "no free request slot");
    const int L = L_p + G, lpad = c->D.lpad, mb = c->D.max_br;
    std::vector<int> X((size_t)mb * lpad, c->m.mask_id);
    std::vector<bb_branch_state> br(mb);
    memset(br.data(), 0, sizeof(bb_branch_state) * mb);
    for (int k = 0; k < N; ++k) {
        if (blocks[k] < 1) return fail(c, BB_EINVAL, "block size must be positive");
        for (int i = 0; i < L_p; ++i) {
            if (prompt[i] < 0 || prompt[i] >= c->m.vocab || prompt[i] == c->m.mask_id)
                return fail(c, BB_EINVAL, "prompt token out of range or equal to the mask id");
            X[(size_t)k * lpad + i] = prompt[i];
        }
        br[k].block = blocks[k]; br[k].start = L_p; br[k].end = std::min(L_p + blocks[k], L); br[k].synced_from = -1;
    }
    ReqHeader H; memset(&H, 0, sizeof(H));
    H.in_use = 1; H.L_p = L_p; H.G = G; H.L = L; H.N = N;
    HIPCHK(c, hipMemcpyAsync(c->D.X + (size_t)slot * mb * lpad, X.data(), X.size() * 4, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemcpyAsync(c->D.br + slot * mb, br.data(), sizeof(bb_branch_state) * mb, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemcpyAsync(c->D.hdr + slot, &H, sizeof(H), hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HostReq& R = c->reqs[slot];
    R = HostReq{}; R.in_use = 1; R.L_p = L_p; R.G = G; R.L = L; R.N = N;
    for (int k = 0; k < N; ++k) R.blocks[k] = blocks[k];
    *req_id = slot;
    return BB_OK;
}

static int bb_request_close_impl(bb_ctx* c, int req_id) {
    if (!c || req_id < 0 || req_id >= c->lim.max_requests || !c->reqs[req_id].in_use) return BB_EINVAL;
    HIPCHK(c, hipMemsetAsync(c->D.hdr + req_id, 0, sizeof(ReqHeader), c->stream));
    c->reqs[req_id].in_use = 0;
    return BB_OK;
}

static int check_reqs(bb_ctx* c, const int* ids, int n, bool need_init) {
    if (!c || !ids || n < 1 || n > c->lim.max_requests) return BB_EINVAL;
    for (int i = 0; i < n; ++i) {
        if (ids[i] < 0 || ids[i] >= c->lim.max_requests || !c->reqs[ids[i]].in_use) return fail(c, BB_EINVAL, "unknown request id");
        for (int j = 0; j < i; ++j) if (ids[j] == ids[i]) return fail(c, BB_EINVAL, "request listed twice");
        if (need_init && !c->reqs[ids[i]].initialised) return fail(c, BB_ESTATE, "request has not had its initial refresh");
    }
    if (!weights_complete(c)) return fail(c, BB_ESTATE, "weights not fully loaded");
    return BB_OK;
}

// ---- the forward -----------------------------------------------------------------------------------
// mode 0: block step with LM head; 1: initial full forward with LM head over lm_cap rows
// (results broadcast to all branches); 2: cache-only refresh (stops after the last K,V write).
static int forward(bb_ctx* c, int rows_cap, int lm_cap, int mode, int seg_base, int n_segs, int max_seg_rows, int max_pages) {
    const bb_model_cfg& m = c->m; const Dev& D = c->D; hipStream_t s = c->stream;
    const int d = m.d_model, nq = m.n_q_heads * m.head_dim, f = m.d_ffn, nqkv = D.nqkv, ngu = c->ngu;
    const int mt = (rows_cap + 31) / 32, rows_pad = mt * 32;
    const int gk = rows_cap <= BB_SKINNY_ROWS ? BB_K_GEMM_SKINNY : BB_K_GEMM_WIDE;
    // many rows: the layer GEMMs are bound by the matrix pipes and run in the wide format (every kernel that writes
    // a panel for them is told so); the LM head keeps two bf16 terms (its rows are the masked ones only)
    const int wide = !c->wide_off;
    const bool defer = rows_cap <= BB_DEFER_ROWS;     // block steps of at most 128 rows: every gate/up GEMM has a k split, its consumer is the SwiGLU kernel
    // kind: 0 LM head, 1 O/down, 2 gate/up, 3 QKV (index of the tuning overrides)
    // swiglu_out: where the gate/up projection may put SiLU(gate) * up itself; it does when its k range
    // is not split (then 0 is returned and no partial sums exist)
    auto gemm = [&](int kind, const u32x4* W, const u32x4* Ww, const float* wscale, const u32x4* A, float* P, int N, int K,
                    int rows, int mtt, int klass, u32x4* swiglu_out = nullptr, const float* ssq = nullptr, int nblk = 0) {
        // tile width: the fused SwiGLU epilogue pairs two tiles per wave (passes with more than 128 rows); otherwise the
        // plan picks it.  With at most 128 rows the norm's scale is deferred: the wide-format kernel's SwiGLU epilogue
        // applies it (ssq) where the plan comes out with two tiles per wave and k whole (many columns: the Dream
        // shape), the two-term kernel leaves it to the separate SwiGLU kernel.
        const int nt = c->force_nt[kind] > 0 ? c->force_nt[kind] : (swiglu_out && !defer ? 2 : 0);
        GemmPlan p = wide ? gemm_plan_wide(rows, N, K, 0, nt, swiglu_out && !defer) : gemm_plan(rows, N, K, 0, nt);
        if (c->force_split[kind] > 0 && rows <= 128) p = gemm_plan(rows, N, K, c->force_split[kind], c->force_nt[kind]);
        const bool fused = swiglu_out && (wide || !defer) && p.split_k == 1 && p.nt == 2;
        PROF_STAMPED(klass, 2.0 * N * K, 2.0 * rows * (double)N * K);
        if (wide) launch_gemm_wide(Ww, wscale, A, P, mtt, N, K, p, s, fused ? swiglu_out : nullptr, prof_scope_.stamps(),
                                   fused ? ssq : nullptr, nblk, m.rms_eps);
        else {
            GemmEpilogue epi; epi.swiglu_out = fused ? swiglu_out : nullptr;
            launch_gemm(W, A, P, mtt, N, K, p, s, epi, prof_scope_.stamps());
        }
        return fused ? 0 : p.split_k;
    };
    c->prof_chain = false;              // the first launch records its own start
    { PROF(BB_K_GLUE, 0, 0); launch_embed(D, c->emb, c->h, rows_cap, s); }
    c->prof_chain = true;
    int s_down = 0;
    const size_t pstride = (size_t)rows_pad * d;
    for (int li = 0; li < m.n_layers; ++li) {
        const LayerW& W = c->layers[li];
        // few rows: the norm's scale is applied after the projection (see residual_pack_kernel)
        const float* ssq = defer ? c->ssq : nullptr;
        int nblk = 0;
        { PROF(BB_K_GLUE, 0, 0);
          if (defer) nblk = launch_residual_pack(D, c->h, c->part, s_down, pstride, W.g_attn, c->Apk, mt, c->ssq, wide, s);
          else launch_rmsnorm_pack(D, c->h, c->part, s_down, pstride, W.g_attn, c->Apk, mt, 0, 0, wide, s); }
        const int s_qkv = gemm(3, W.wqkv, W.wqkv_w, W.s_qkv, c->Apk, c->qkv, nqkv, d, rows_cap, mt, gk);
        { PROF(BB_K_GLUE, 0, 0);
          launch_qkv_epilogue(D, c->qkv, s_qkv, (size_t)rows_pad * nqkv, m.qkv_bias ? W.bqkv : nullptr, c->Q, li, rows_cap, ssq, nblk, s); }
        if (mode == 2 && li == m.n_layers - 1) break;
        { PROF(BB_K_ATTENTION, 0, 0); launch_attention(D, c->Q, c->Apk, li, mt, max_seg_rows, seg_base, n_segs, max_pages, c->attn_part, c->attn_part_elems, wide, s); }
        const int s_o = gemm(1, W.wo, W.wo_w, W.s_o, c->Apk, c->part, d, nq, rows_cap, mt, gk);
        { PROF(BB_K_GLUE, 0, 0);
          if (defer) nblk = launch_residual_pack(D, c->h, c->part, s_o, pstride, W.g_ffn, c->Apk, mt, c->ssq, wide, s);
          else launch_rmsnorm_pack(D, c->h, c->part, s_o, pstride, W.g_ffn, c->Apk, mt, 0, 0, wide, s); }
        const int s_gu = gemm(2, W.wgu, W.wgu_w, W.s_gu, c->Apk, c->gu, ngu, d, rows_cap, mt, gk, c->Apk2, ssq, nblk);
        if (s_gu > 0) { PROF(BB_K_GLUE, 0, 0);
          launch_swiglu_epilogue(D, c->gu, s_gu, (size_t)rows_pad * ngu, ngu, c->Apk2, rows_cap, mt, wide, ssq, nblk, s); }
        s_down = gemm(1, W.wdown, W.wdown_w, W.s_down, c->Apk2, c->part, d, f, rows_cap, mt, gk);
    }
    if (mode != 2) {
        const int mt_lm = (lm_cap + 31) / 32;
        { PROF(BB_K_GLUE, 0, 0);
          launch_rmsnorm_pack(D, c->h, c->part, s_down, pstride, c->g_final, c->Apk, mt_lm, 1, mode == 1, 0, s); }
        {   // LM head with the vocabulary reduction in its epilogue: no k split, 256-column tiles (128 for tiny vocabularies)
            GemmPlan p = gemm_plan(lm_cap, m.vocab, d, 1, m.vocab / 32 >= 8 ? 2 : 1);
            GemmEpilogue epi; epi.vocab_part = D.vr_part; epi.mask_id = m.mask_id; epi.keep_logits = c->keep_logits;
            PROF_STAMPED(lm_cap <= 256 ? BB_K_GEMM_SKINNY : BB_K_GEMM_WIDE, 2.0 * m.vocab * d, 2.0 * lm_cap * (double)m.vocab * d);
            launch_gemm(c->lm, c->Apk, c->logits, mt_lm, m.vocab, d, p, s, epi, prof_scope_.stamps());
        }
        { PROF(BB_K_GLUE, 0, 0); launch_vocab_finish(D, lm_cap, mode == 1, s); }
    }
    c->prof_chain = false;
    c->last_forward_rows = rows_cap; c->last_lm_cap = lm_cap;
    HIPCHK(c, hipGetLastError());
    return BB_OK;
}

// The list of requests a call works on lives on the device; it is copied only when it differs from the one the
// previous call uploaded, and from a buffer the context owns.
static int upload_req_list(bb_ctx* c, const int* ids, int n) {
    if ((int)c->req_host.size() == n && std::equal(ids, ids + n, c->req_host.begin())) return BB_OK;
    c->req_host.assign(ids, ids + n);
    HIPCHK(c, hipMemcpyAsync(c->D.req_list, c->req_host.data(), sizeof(int) * n, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));      // the copy has left the host buffer before anything may change it
    return BB_OK;
}

static int bb_refresh_impl(bb_ctx* c, const int* ids, int n, int mode) {
    int rc = check_reqs(c, ids, n, mode == BB_PERIODIC);
    if (rc != BB_OK) return rc;
    if (mode != BB_INIT && mode != BB_PERIODIC) return fail(c, BB_EINVAL, "bad refresh mode");
    for (int i = 0; i < n; ++i)
        if (mode == BB_INIT && c->reqs[ids[i]].initialised) return fail(c, BB_ESTATE, "request already initialised");
    // The listed requests are packed into as few forwards as the activation buffers hold (they are sized for one
    // request of the largest shape): consecutive requests share a forward while their rows fit.
    const int rows_max = std::max(c->lim.max_step_rows, c->refresh_rows_cap), lm_max = c->D.lm_cap;
    for (int i = 0; i < n;) {
        int j = i, rows = 0, lm = 0, maxL = 0;
        while (j < n) {
            const HostReq& R = c->reqs[ids[j]];
            const int r = mode == BB_INIT ? R.L : R.N * R.L, g = mode == BB_INIT ? R.G : 0;
            if (j > i && (rows + r > rows_max || lm + g > lm_max)) break;
            rows += r; lm += g; maxL = std::max(maxL, R.L); ++j;
        }
        if ((rc = upload_req_list(c, ids + i, j - i)) != BB_OK) return rc;
        launch_pack_refresh(c->D, j - i, mode, c->stream);
        rc = forward(c, rows, lm, mode == BB_INIT ? 1 : 2, 0, c->D.max_req * c->D.max_br, maxL, (maxL + BB_PAGE - 1) / BB_PAGE);
        if (rc != BB_OK) return rc;
        if (mode == BB_INIT) for (int k = i; k < j; ++k) c->reqs[ids[k]].initialised = 1;
        i = j;
    }
    return BB_OK;
}

static void fill_view(bb_ctx* c, bb_step_view* v) {
    const Dev& D = c->D;
    v->counts_dev = D.counts; v->row_branch_dev = D.row_gbr; v->row_pos_dev = D.row_pos; v->lm_row_dev = D.lm_row;
    v->argmax_dev = D.out_pred; v->conf_dev = D.out_conf; v->lse_dev = D.out_lse; v->logits_dev = c->keep_logits ? c->logits : nullptr;
    v->rows_capacity = D.lm_cap;
}

static int bb_denoise_step_impl(bb_ctx* c, const int* ids, int n, bb_step_view* view) {
    int rc = check_reqs(c, ids, n, true);
    if (rc != BB_OK) return rc;
    int rows = 0, maxb = 0, maxL = 0;
    for (int i = 0; i < n; ++i) {
        const HostReq& R = c->reqs[ids[i]];
        maxL = std::max(maxL, R.L);
        for (int k = 0; k < R.N; ++k) { rows += std::min(R.blocks[k], R.G); maxb = std::max(maxb, std::min(R.blocks[k], R.G)); }
    }
    if (rows > c->lim.max_step_rows) return fail(c, BB_ENOMEM, "step rows exceed max_step_rows");
    if ((rc = upload_req_list(c, ids, n)) != BB_OK) return rc;
    { PROF(BB_K_GLUE, 0, 0); launch_pack_step(c->D, n, c->stream); }
    { PROF(BB_K_POLICY, 0, 0); launch_page_copies(c->D, c->stream); }
    rc = forward(c, rows, rows, 0, 0, c->D.max_req * c->D.max_br, maxb, (maxL + BB_PAGE - 1) / BB_PAGE);
    if (rc == BB_OK && view) fill_view(c, view);
    return rc;
}

static int read_stats(bb_ctx* c, int slot, bb_request_stats* out) {
    ReqHeader H; bb_branch_state br[BB_MAX_BRANCHES];
    HIPCHK(c, hipMemcpy(&H, c->D.hdr + slot, sizeof(H), hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(br, c->D.br + slot * c->D.max_br, sizeof(bb_branch_state) * c->D.max_br, hipMemcpyDeviceToHost));
    memset(out, 0, sizeof(*out));
    out->n_branches = H.N; out->refresh_due = H.refresh_due; out->all_done = H.all_done;
    out->nfe_init = H.nfe_init; out->nfe_block = H.nfe_block; out->nfe_refresh = H.nfe_refresh;
    out->finished = H.finished; out->winner = H.finished ? H.winner : -1; out->eos_pos = H.finished ? H.eos_pos : -1;
    for (int k = 0; k < H.N; ++k) out->branch[k] = br[k];
    return BB_OK;
}

static int bb_merge_commit_impl(bb_ctx* c, const int* ids, int n, bb_request_stats* stats) {
    int rc = check_reqs(c, ids, n, true);
    if (rc != BB_OK) return rc;
    if ((rc = upload_req_list(c, ids, n)) != BB_OK) return rc;
    { PROF(BB_K_POLICY, 0, 0); launch_commit_merge(c->D, n, reinterpret_cast<const uint16_t*>(c->lm), c->stream); }
    HIPCHK(c, hipGetLastError());
    if (stats) {
        HIPCHK(c, hipStreamSynchronize(c->stream));
        for (int i = 0; i < n; ++i) if ((rc = read_stats(c, ids[i], &stats[i])) != BB_OK) return rc;
    }
    return BB_OK;
}

// ---- Alg. 1 driver --------------------------------------------------------------------------------------
static int bb_generate_impl(bb_ctx* c, const int* ids, int n, int max_block_forwards, bb_request_stats* stats) {
    int rc = check_reqs(c, ids, n, false);
    if (rc != BB_OK) return rc;
    if (max_block_forwards < 0) return fail(c, BB_EINVAL, "max_block_forwards must not be negative");
    for (int i = 0; i < n; ++i)
        if (c->reqs[ids[i]].initialised) return fail(c, BB_ESTATE, "bb_generate wants requests that have not been initialised");
    std::vector<int> run(ids, ids + n), next, due;
    int quiet = 1;                      // forwards that may run before any listed request needs a refresh
    // One word per listed request after a commit (finished, refresh due, forwards left until a refresh is due), all
    // read back with a single copy.
    auto poll = [&](const std::vector<int>& list) -> int {
        c->flags_host.resize(list.size());
        HIPCHK(c, hipStreamSynchronize(c->stream));
        HIPCHK(c, hipMemcpy(c->flags_host.data(), c->D.req_flags, sizeof(int) * list.size(), hipMemcpyDeviceToHost));
        next.clear(); due.clear();
        quiet = c->dc.refresh_interval;
        for (size_t i = 0; i < list.size(); ++i) {
            const int f = c->flags_host[i];
            if (f & 1) continue;
            next.push_back(list[i]);
            if (f & 2) due.push_back(list[i]);             // refreshed before the next forward: a full interval ahead
            else quiet = std::min(quiet, f >> 8);
        }
        quiet = std::max(quiet, 1);
        return BB_OK;
    };
    if ((rc = bb_refresh_impl(c, run.data(), n, BB_INIT)) != BB_OK) return rc;
    if ((rc = bb_merge_commit_impl(c, run.data(), n, nullptr)) != BB_OK) return rc;
    if ((rc = poll(run)) != BB_OK) return rc;
    for (int fwd = 0; !next.empty() && fwd < max_block_forwards;) {
        run = next;
        if (!due.empty() && (rc = bb_refresh_impl(c, due.data(), (int)due.size(), BB_PERIODIC)) != BB_OK) return rc;
        // No refresh can fall due during the next `quiet` forwards, so they are enqueued without reading anything
        // back; a request that finishes on the way contributes no rows and counts no forward afterwards.
        // (and the flags are read at least every 8 forwards, so that a request that has finished is not stepped in vain for long)
        const int k = std::min(std::min(quiet, 8), max_block_forwards - fwd);
        for (int j = 0; j < k; ++j) {
            if ((rc = bb_denoise_step_impl(c, run.data(), (int)run.size(), nullptr)) != BB_OK) return rc;
            if ((rc = bb_merge_commit_impl(c, run.data(), (int)run.size(), nullptr)) != BB_OK) return rc;
        }
        fwd += k;
        if ((rc = poll(run)) != BB_OK) return rc;
    }
    if (stats) {
        HIPCHK(c, hipStreamSynchronize(c->stream));
        for (int i = 0; i < n; ++i) if ((rc = read_stats(c, ids[i], &stats[i])) != BB_OK) return rc;
    }
    return BB_OK;
}

// ---- inspection and teacher forcing ---------------------------------------------------------------------
static int check_one(bb_ctx* c, int id) {
    if (!c || id < 0 || id >= c->lim.max_requests || !c->reqs[id].in_use) return BB_EINVAL;
    return BB_OK;
}

static int bb_debug_set_gemm_plan_impl(bb_ctx* c, int kind, int nt, int split_k) {
    if (!c || kind < 0 || kind > 3 || nt < 0 || nt > 3 || split_k < 0 || split_k > BB_MAX_SPLITK) return BB_EINVAL;
    c->force_nt[kind] = nt; c->force_split[kind] = split_k;
    return BB_OK;
}

static int bb_debug_keep_logits_impl(bb_ctx* c, int on) {
    if (!c) return BB_EINVAL;
    c->keep_logits = on != 0;
    return BB_OK;
}

static int bb_profile_enable_impl(bb_ctx* c, int on) {
    if (!c) return BB_EINVAL;
    c->prof_on = on != 0;
    return BB_OK;
}

static int bb_profile_read_impl(bb_ctx* c, bb_profile_entry* out, int max_entries, int* n_out) {
    if (!c || !out || !n_out || max_entries < 1) return BB_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    bb_profile_entry acc[BB_K_CLASSES];
    for (int k = 0; k < BB_K_CLASSES; ++k) acc[k] = bb_profile_entry{k, 0, 0.0, 0.0, 0.0};
    for (auto& r : c->prof) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) == hipSuccess) {
            acc[r.klass].launches += 1; acc[r.klass].total_ms += ms; acc[r.klass].bytes += r.bytes; acc[r.klass].flops += r.flops;
        }
        if (r.own_a) c->ev_pool.push_back(r.a);
        c->ev_pool.push_back(r.b);
    }
    c->prof.clear();
    c->prof_prev_end = nullptr;
    int n = 0;
    for (int k = 0; k < BB_K_CLASSES && n < max_entries; ++k) out[n++] = acc[k];
    *n_out = n;
    return BB_OK;
}

static int bb_synchronize_impl(bb_ctx* c) {
    if (!c) return BB_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return BB_OK;
}

static int bb_read_device_impl(bb_ctx* c, const void* src, void* dst, size_t bytes) {
    if (!c || !src || !dst) return BB_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(dst, src, bytes, hipMemcpyDeviceToHost));
    return BB_OK;
}

static int bb_get_view_impl(bb_ctx* c, bb_step_view* view) {
    if (!c || !view) return BB_EINVAL;
    fill_view(c, view);
    return BB_OK;
}

static int bb_get_tokens_impl(bb_ctx* c, int id, int32_t* X) {
    if (check_one(c, id) != BB_OK || !X) return BB_EINVAL;
    const HostReq& R = c->reqs[id];
    HIPCHK(c, hipStreamSynchronize(c->stream));
    for (int k = 0; k < R.N; ++k)
        HIPCHK(c, hipMemcpy(X + (size_t)k * R.L, c->D.X + ((size_t)id * c->D.max_br + k) * c->D.lpad, R.L * 4, hipMemcpyDeviceToHost));
    return BB_OK;
}

static int bb_get_stats_impl(bb_ctx* c, int id, bb_request_stats* out) {
    if (check_one(c, id) != BB_OK || !out) return BB_EINVAL;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return read_stats(c, id, out);
}

static int bb_set_state_impl(bb_ctx* c, int id, const int32_t* X, const bb_branch_state* brs) {
    if (check_one(c, id) != BB_OK || !X || !brs) return BB_EINVAL;
    const HostReq& R = c->reqs[id];
    HIPCHK(c, hipStreamSynchronize(c->stream));
    bb_branch_state cur[BB_MAX_BRANCHES];
    HIPCHK(c, hipMemcpy(cur, c->D.br + id * c->D.max_br, sizeof(bb_branch_state) * c->D.max_br, hipMemcpyDeviceToHost));
    for (int k = 0; k < R.N; ++k) {
        if (brs[k].start < R.L_p || brs[k].end > R.L || brs[k].start > brs[k].end) return fail(c, BB_EINVAL, "window out of range");
        // the forward's row lists are sized from the block sizes: a window never holds more than one block
        if (brs[k].end - brs[k].start > std::min(R.blocks[k], R.G)) return fail(c, BB_EINVAL, "window wider than the branch's block");
        for (int i = 0; i < R.L; ++i)
            if (X[(size_t)k * R.L + i] < 0 || X[(size_t)k * R.L + i] >= c->m.vocab) return fail(c, BB_EINVAL, "token out of range");
        HIPCHK(c, hipMemcpy(c->D.X + ((size_t)id * c->D.max_br + k) * c->D.lpad, X + (size_t)k * R.L, R.L * 4, hipMemcpyHostToDevice));
        cur[k].start = brs[k].start; cur[k].end = brs[k].end; cur[k].done = brs[k].done;
        cur[k].mean_conf = brs[k].mean_conf;
    }
    HIPCHK(c, hipMemcpy(c->D.br + id * c->D.max_br, cur, sizeof(bb_branch_state) * c->D.max_br, hipMemcpyHostToDevice));
    return BB_OK;
}

static int bb_get_kv_impl(bb_ctx* c, int id, int branch, int layer, float* K, float* V) {
    if (check_one(c, id) != BB_OK || !K || !V) return BB_EINVAL;
    const HostReq& R = c->reqs[id];
    if (branch < 0 || branch >= R.N || layer < 0 || layer >= c->m.n_layers) return BB_EINVAL;
    const size_t n = (size_t)R.L * c->m.n_kv_heads * c->m.head_dim;
    float* dK = c->dbg; float* dV = c->dbg + n;
    launch_read_kv(c->D, id, branch, layer, dK, dV, R.L, c->stream);
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(K, dK, n * 4, hipMemcpyDeviceToHost));
    HIPCHK(c, hipMemcpy(V, dV, n * 4, hipMemcpyDeviceToHost));
    return BB_OK;
}

static int bb_set_kv_impl(bb_ctx* c, int id, int branch, int layer, const float* K, const float* V) {
    if (check_one(c, id) != BB_OK || !K || !V) return BB_EINVAL;
    const HostReq& R = c->reqs[id];
    if (branch < 0 || branch >= R.N || layer < 0 || layer >= c->m.n_layers) return BB_EINVAL;
    if (!R.initialised) return fail(c, BB_ESTATE, "the request has no cache yet: run bb_refresh(BB_INIT) first");
    const size_t n = (size_t)R.L * c->m.n_kv_heads * c->m.head_dim;
    for (size_t i = 0; i < n; ++i)
        if (!(std::fabs(K[i]) <= 65504.f) || !(std::fabs(V[i]) <= 65504.f)) return fail(c, BB_EINVAL, "cache value outside the fp16 range");
    float* dK = c->dbg; float* dV = c->dbg + n;
    HIPCHK(c, hipStreamSynchronize(c->stream));
    HIPCHK(c, hipMemcpy(dK, K, n * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(dV, V, n * 4, hipMemcpyHostToDevice));
    launch_write_kv(c->D, id, branch, layer, dK, dV, R.L, c->stream);
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, hipStreamSynchronize(c->stream));
    return BB_OK;
}

static int bb_debug_gemm_impl(bb_ctx* c, const float* A, const uint16_t* W, float* C, int M, int N, int K, int split_k, int wide) {
    if (!c || !A || !W || !C || M < 1 || N < 32 || K < 16 || N % 32 || K % 16 || split_k < 0 || split_k > BB_MAX_SPLITK) return BB_EINVAL;
    const int mt = (M + 31) / 32, rows_pad = mt * 32;
    GemmPlan p = wide ? gemm_plan_wide(M, N, K, split_k, 0) : gemm_plan(M, N, K, split_k, 0);
    // carve private buffers out of the activation region [h, emb): nothing else runs meanwhile
    Bump b{(char*)c->h, 0};
    float* dA = b.take<float>((size_t)M * K);
    uint16_t* dW = b.take<uint16_t>((size_t)N * K);
    const int Kp = (K + 63) / 64 * 64;
    const size_t wt_u4 = (size_t)N * Kp / 8;
    u32x4* dWt = b.take<u32x4>(wt_u4);
    u32x4* dAp = b.take<u32x4>((size_t)rows_pad * Kp / 8 * BB_SPLIT);
    float* dScale = b.take<float>(N);
    const size_t c_elems = (size_t)p.split_k * rows_pad * N;
    float* dC = b.take<float>(c_elems);
    if (b.off > (size_t)((char*)c->emb - (char*)c->h)) return fail(c, BB_ENOMEM, "debug gemm does not fit the activation region");
    HIPCHK(c, hipMemcpyAsync(dA, A, (size_t)M * K * 4, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemcpyAsync(dW, W, (size_t)N * K * 2, hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipMemsetAsync(dWt, 0, wt_u4 * sizeof(u32x4), c->stream));
    if (wide) {
        launch_tile_weights_wide(dW, N, K, dWt, dScale, 0, 0, c->stream);
        launch_pack_rows_wide(dA, M, K, dAp, mt, c->stream);
        launch_gemm_wide(dWt, dScale, dAp, dC, mt, N, K, p, c->stream);
    } else {
        launch_tile_weights(dW, N, K, dWt, 0, 0, c->stream);
        launch_pack_rows(dA, M, K, dAp, mt, c->stream);
        launch_gemm(dWt, dAp, dC, mt, N, K, p, c->stream);
    }
    HIPCHK(c, hipGetLastError());
    HIPCHK(c, hipStreamSynchronize(c->stream));
    std::vector<float> tmp(c_elems);
    HIPCHK(c, hipMemcpy(tmp.data(), dC, c_elems * 4, hipMemcpyDeviceToHost));
    for (int mrow = 0; mrow < M; ++mrow)
        for (int ncol = 0; ncol < N; ++ncol) {
            float acc = 0.f;
            for (int s = 0; s < p.split_k; ++s) acc += tmp[((size_t)s * rows_pad + mrow) * N + ncol];
            C[(size_t)mrow * N + ncol] = acc;
        }
    return BB_OK;
}

// ---- KV-consistency diagnostics -----------------------------------------------------------------------
extern "C" size_t bb_kv_diag_scratch_bytes(bb_ctx* c, int id) {      // no allocation, nothing to throw
    if (check_one(c, id) != BB_OK) return 0;
    const HostReq& R = c->reqs[id];
    const size_t pages = (R.L + BB_PAGE - 1) / BB_PAGE;
    const size_t row = (size_t)c->m.n_layers * pages * c->m.n_kv_heads * BB_PAGE * 2 * c->m.head_dim * sizeof(half_t);
    return 2 * row * R.N + align_up((size_t)c->m.n_layers * pages * sizeof(double), 256);     // K and V snapshots + partial sums
}

static int bb_kv_diagnostics_impl(bb_ctx* c, int id, void* scratch, size_t scratch_bytes, double* E, double* Dpair, double* Davg) {
    if (check_one(c, id) != BB_OK) return BB_EINVAL;
    const HostReq& R = c->reqs[id];
    if (!R.initialised) return fail(c, BB_ESTATE, "request has not had its initial refresh");
    const int pages = (R.L + BB_PAGE - 1) / BB_PAGE, n_part = c->m.n_layers * pages;
    const size_t part_bytes = align_up((size_t)n_part * sizeof(double), 256);
    if (E && (!scratch || (uintptr_t)scratch % 16 || scratch_bytes < bb_kv_diag_scratch_bytes(c, id)))
        return fail(c, BB_EINVAL, "bb_kv_diagnostics: scratch missing, misaligned or too small");
    std::vector<double> host(n_part);
    double* part = E ? reinterpret_cast<double*>(scratch) : reinterpret_cast<double*>(c->dbg);    // dbg holds 2 L hkv hd floats >= n_part doubles
    auto total = [&](double* dst) -> int {
        HIPCHK(c, hipStreamSynchronize(c->stream));
        HIPCHK(c, hipMemcpy(host.data(), part, n_part * sizeof(double), hipMemcpyDeviceToHost));
        double t = 0.0;
        for (double v : host) t += v;
        *dst = t;
        return BB_OK;
    };
    int rc;
    const int g0 = id * c->D.max_br;
    if (Dpair || Davg) {
        double sum = 0.0;
        for (int i = 0; i < R.N; ++i)
            for (int j = i; j < R.N; ++j) {
                double v = 0.0;
                if (j > i) {
                    launch_kv_sqdist(c->D, g0 + i, g0 + j, nullptr, nullptr, 0, 0, pages, part, c->stream);
                    if ((rc = total(&v)) != BB_OK) return rc;
                    sum += 2 * v;
                }
                if (Dpair) Dpair[i * R.N + j] = Dpair[j * R.N + i] = v;
            }
        if (Davg) *Davg = R.N > 1 ? sum / ((double)R.N * (R.N - 1)) : 0.0;
    }
    if (E) {
        bb_branch_state br[BB_MAX_BRANCHES];
        HIPCHK(c, hipStreamSynchronize(c->stream));
        HIPCHK(c, hipMemcpy(br, c->D.br + g0, sizeof(bb_branch_state) * c->D.max_br, hipMemcpyDeviceToHost));
        half_t* snapK = reinterpret_cast<half_t*>(reinterpret_cast<char*>(scratch) + part_bytes);
        const size_t row_halfs = (size_t)c->m.n_layers * pages * c->m.n_kv_heads * BB_PAGE * 2 * c->m.head_dim;
        half_t* snapV = snapK + row_halfs * R.N;
        bool any = false;
        for (int k = 0; k < R.N; ++k) {
            E[k] = 0.0;
            if (br[k].done) continue;
            any = true;
            launch_kv_snapshot(c->D, g0 + k, snapK, snapV, R.N, k, pages, c->stream);
        }
        if (any) {
            if ((rc = bb_refresh_impl(c, &id, 1, BB_PERIODIC)) != BB_OK) return rc;
            for (int k = 0; k < R.N; ++k) {
                if (br[k].done) continue;
                launch_kv_sqdist(c->D, g0 + k, 0, snapK, snapV, R.N, k, pages, part, c->stream);
                double v = 0.0;
                if ((rc = total(&v)) != BB_OK) return rc;
                E[k] = std::sqrt(v);
            }
        }
    }
    HIPCHK(c, hipGetLastError());
    return BB_OK;
}

// ---- traffic-counter reference ----------------------------------------------------------------------
__global__ __launch_bounds__(256) void copy16_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, size_t n) {
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

static int bb_debug_copy16_impl(bb_ctx* c, const void* src_dev, void* dst_dev, size_t bytes) {
    if (!c || !src_dev || !dst_dev) return BB_EINVAL;
    if (bytes % 16 || (uintptr_t)src_dev % 16 || (uintptr_t)dst_dev % 16) return fail(c, BB_EINVAL, "bb_debug_copy16: arguments must be multiples of 16");
    if (bytes == 0) return BB_OK;
    const size_t n = bytes / 16;
    copy16_kernel<<<(unsigned)std::min<size_t>((n + 255) / 256, 16384), 256, 0, c->stream>>>((const u32x4*)src_dev, (u32x4*)dst_dev, n);
    HIPCHK(c, hipGetLastError());
    return BB_OK;
}

// ---- MFMA issue-rate reference ------------------------------------------------------------------------
// Eight independent accumulator tiles per wave, one wave per SIMD, nothing but 32x32x16 bf16 MFMAs: what the matrix
// pipes sustain on this chip at the clocks it holds under that load (the denominator beside the nominal peak).
typedef __bf16 mr_bf16x8 __attribute__((ext_vector_type(8)));
typedef float mr_f32x16 __attribute__((ext_vector_type(16)));
__global__ __launch_bounds__(256, 1) void mfma_rate_kernel(float* __restrict__ out, int iters) {
    mr_f32x16 acc[8];
    for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    mr_bf16x8 a, b;
    for (int j = 0; j < 8; ++j) { a[j] = (__bf16)(float)((threadIdx.x + j) & 3); b[j] = (__bf16)(float)(j & 1); }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
    for (int i = 0; i < 8; ++i) for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

static int bb_debug_mfma_rate_impl(bb_ctx* c, double* tflops_out_host) {
    if (!c || !tflops_out_host) return BB_EINVAL;
    const int wgs = 1024, iters = 40000;                     // 1024 x 256 floats of output fit the activation region easily
    if ((size_t)wgs * 256 * sizeof(float) > (size_t)((char*)c->emb - (char*)c->h)) return fail(c, BB_ENOMEM, "activation region too small");
    hipEvent_t e0, e1;
    HIPCHK(c, hipEventCreate(&e0)); HIPCHK(c, hipEventCreate(&e1));
    mfma_rate_kernel<<<wgs, 256, 0, c->stream>>>(c->h, iters);            // warm-up (clocks settle under the load)
    HIPCHK(c, hipEventRecord(e0, c->stream));
    mfma_rate_kernel<<<wgs, 256, 0, c->stream>>>(c->h, iters);
    HIPCHK(c, hipEventRecord(e1, c->stream));
    HIPCHK(c, hipEventSynchronize(e1));
    float ms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    HIPCHK(c, hipGetLastError());
    *tflops_out_host = (double)wgs * 4 * iters * 8 * (2.0 * 32 * 32 * 16) / (ms * 1e-3) / 1e12;
    return BB_OK;
}

// ---- the boundary proper: nothing throws across it ----------------------------------------------------------
// The host code above uses std::vector / std::string; an allocation failure there becomes BB_ENOMEM here.
#define BB_GUARD(ctx, call) \
    try { return call; } \
    catch (const std::bad_alloc&) { bb_ctx* c_ = const_cast<bb_ctx*>(static_cast<const bb_ctx*>(ctx)); \
                                    if (c_) { try { c_->err = "out of host memory"; } catch (...) {} } return BB_ENOMEM; } \
    catch (...) { return BB_EINVAL; }

extern "C" int bb_destroy(bb_ctx* ctx) {
    BB_GUARD(ctx, bb_destroy_impl(ctx));
}

extern "C" int bb_load_weights(bb_ctx* ctx, const bb_tensor* tensors, int n) {
    BB_GUARD(ctx, bb_load_weights_impl(ctx, tensors, n));
}

extern "C" int bb_request_open(bb_ctx* c, const int32_t* prompt, int L_p, int G, const int* blocks, int N, int* req_id) {
    BB_GUARD(c, bb_request_open_impl(c, prompt, L_p, G, blocks, N, req_id));
}

extern "C" int bb_request_close(bb_ctx* c, int req_id) {
    BB_GUARD(c, bb_request_close_impl(c, req_id));
}

extern "C" int bb_refresh(bb_ctx* c, const int* ids, int n, int mode) {
    BB_GUARD(c, bb_refresh_impl(c, ids, n, mode));
}

extern "C" int bb_denoise_step(bb_ctx* c, const int* ids, int n, bb_step_view* view) {
    BB_GUARD(c, bb_denoise_step_impl(c, ids, n, view));
}

extern "C" int bb_merge_commit(bb_ctx* c, const int* ids, int n, bb_request_stats* stats) {
    BB_GUARD(c, bb_merge_commit_impl(c, ids, n, stats));
}

extern "C" int bb_generate(bb_ctx* c, const int* ids, int n, int max_block_forwards, bb_request_stats* stats) {
    BB_GUARD(c, bb_generate_impl(c, ids, n, max_block_forwards, stats));
}

extern "C" int bb_debug_set_gemm_plan(bb_ctx* c, int kind, int nt, int split_k) {
    BB_GUARD(c, bb_debug_set_gemm_plan_impl(c, kind, nt, split_k));
}

extern "C" int bb_profile_enable(bb_ctx* c, int on) {
    BB_GUARD(c, bb_profile_enable_impl(c, on));
}

extern "C" int bb_profile_read(bb_ctx* c, bb_profile_entry* out, int max_entries, int* n_out) {
    BB_GUARD(c, bb_profile_read_impl(c, out, max_entries, n_out));
}

extern "C" int bb_synchronize(bb_ctx* c) {
    BB_GUARD(c, bb_synchronize_impl(c));
}

extern "C" int bb_read_device(bb_ctx* c, const void* src, void* dst, size_t bytes) {
    BB_GUARD(c, bb_read_device_impl(c, src, dst, bytes));
}

extern "C" int bb_get_view(bb_ctx* c, bb_step_view* view) {
    BB_GUARD(c, bb_get_view_impl(c, view));
}

extern "C" int bb_get_tokens(bb_ctx* c, int id, int32_t* X) {
    BB_GUARD(c, bb_get_tokens_impl(c, id, X));
}

extern "C" int bb_get_stats(bb_ctx* c, int id, bb_request_stats* out) {
    BB_GUARD(c, bb_get_stats_impl(c, id, out));
}

extern "C" int bb_set_state(bb_ctx* c, int id, const int32_t* X, const bb_branch_state* brs) {
    BB_GUARD(c, bb_set_state_impl(c, id, X, brs));
}

extern "C" int bb_get_kv(bb_ctx* c, int id, int branch, int layer, float* K, float* V) {
    BB_GUARD(c, bb_get_kv_impl(c, id, branch, layer, K, V));
}

extern "C" int bb_set_kv(bb_ctx* c, int id, int branch, int layer, const float* K, const float* V) {
    BB_GUARD(c, bb_set_kv_impl(c, id, branch, layer, K, V));
}

extern "C" int bb_debug_gemm(bb_ctx* c, const float* A, const uint16_t* W, float* C, int M, int N, int K, int split_k) {
    BB_GUARD(c, bb_debug_gemm_impl(c, A, W, C, M, N, K, split_k, 0));
}

extern "C" int bb_debug_gemm_wide(bb_ctx* c, const float* A, const uint16_t* W, float* C, int M, int N, int K, int split_k) {
    BB_GUARD(c, bb_debug_gemm_impl(c, A, W, C, M, N, K, split_k, 1));
}

extern "C" int bb_debug_gemm_plan(int M, int N, int K, int wide, int fusable, int out[5]) {
    if (M < 1 || N < 32 || K < 16 || N % 32 || K % 16 || !out) return BB_EINVAL;
    const GemmPlan p = wide ? gemm_plan_wide(M, N, K, 0, 0, fusable != 0) : gemm_plan(M, N, K, 0, 0);
    const int mt_total = (M + 31) / 32, n_groups = (N / 32 + 4 * p.nt - 1) / (4 * p.nt), m_groups = (mt_total + p.mt - 1) / p.mt;
    out[0] = p.split_k; out[1] = p.chunks_per_split; out[2] = p.nt; out[3] = p.mt;
    out[4] = std::min(n_groups * m_groups, 256) * p.split_k;
    return BB_OK;
}

extern "C" int bb_debug_wide_format(bb_ctx* c, int on) {
    if (!c) return BB_EINVAL;
    c->wide_off = !on;
    return BB_OK;
}

extern "C" int bb_kv_diagnostics(bb_ctx* c, int id, void* scratch, size_t scratch_bytes, double* E, double* Dpair, double* Davg) {
    BB_GUARD(c, bb_kv_diagnostics_impl(c, id, scratch, scratch_bytes, E, Dpair, Davg));
}

extern "C" int bb_debug_copy16(bb_ctx* c, const void* src_dev, void* dst_dev, size_t bytes) {
    BB_GUARD(c, bb_debug_copy16_impl(c, src_dev, dst_dev, bytes));
}

extern "C" int bb_debug_mfma_rate(bb_ctx* c, double* tflops_out_host) {
    BB_GUARD(c, bb_debug_mfma_rate_impl(c, tflops_out_host));
}

extern "C" int bb_create(bb_ctx** out, const bb_model_cfg* model, const bb_decode_cfg* decode, const bb_limits* limits,
                         void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
    BB_GUARD(nullptr, bb_create_impl(out, model, decode, limits, workspace_dev, workspace_bytes, hip_stream));
}

extern "C" int bb_debug_keep_logits(bb_ctx* c, int on) {
    BB_GUARD(c, bb_debug_keep_logits_impl(c, on));
}
