// Device-side scheduling and policy kernels: packing the active windows into one row list
// (GetActiveBranches / PackActiveBlocks of Alg. 1), copy-on-write of cache pages, and the
// commit / merge / sync step (Eq. 1 and Alg. 2) on the results of the latest forward.
// All branch and request state lives in device memory, so a decode loop never has to read
// anything back.
#include "bb_internal.h"

// ---- small workgroup reductions (blockDim.x == 256) ----------------------------------------
static __device__ __forceinline__ int wg_sum_i(int v, int* sh) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return sh[0] + sh[1] + sh[2] + sh[3];
}
static __device__ __forceinline__ int wg_min_i(int v, int* sh) {
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return min(min(sh[0], sh[1]), min(sh[2], sh[3]));
}
static __device__ __forceinline__ float wg_sum_f(float v, float* sh) {
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return sh[0] + sh[1] + sh[2] + sh[3];
}

// ---- packing --------------------------------------------------------------------------------
// Block step: every unfinished branch of the listed requests contributes the rows of its
// window; rows still masked are additionally listed for the LM head.  Pages under a window
// that the branch does not own yet are queued for copy-on-write and re-pointed.
__global__ __launch_bounds__(256) void pack_step_kernel(Dev D, int n_req) {
    __shared__ int s_rows[256], s_lm[256], s_off[257], s_lmoff[257];
    const int nb_all = D.max_req * D.max_br, nb = n_req * D.max_br, t = threadIdx.x;
    const int wave = t >> 6, lane = t & 63;
    for (int i = t; i < nb_all; i += 256) D.seg_rows[i] = 0;
    if (t == 0) D.counts[2] = 0;
    for (int i = t; i < 256; i += 256) { s_rows[i] = 0; s_lm[i] = 0; }
    __syncthreads();
    // one wave per branch (round robin): window length and number of masked positions
    for (int b = wave; b < nb; b += 4) {
        const int slot = D.req_list[b / D.max_br], k = b % D.max_br;
        const ReqHeader& H = D.hdr[slot];
        const bb_branch_state& B = D.br[slot * D.max_br + k];
        int rows = 0, nlm = 0;
        if (k < H.N && !B.done) {
            const int start = B.start, end = B.end;
            rows = end - start;
            const int* Xr = D.X + ((size_t)slot * D.max_br + k) * D.lpad;
            for (int i = start + lane; i < end; i += 64) nlm += Xr[i] == D.mask_id;
            for (int o = 32; o > 0; o >>= 1) nlm += __shfl_xor(nlm, o, 64);
        }
        if (lane == 0) { s_rows[b] = rows; s_lm[b] = nlm; D.hdr[slot].pending[k] = rows > 0; }
    }
    __syncthreads();
    if (t == 0) {
        int a = 0, c = 0;
        for (int i = 0; i < nb; ++i) { s_off[i] = a; s_lmoff[i] = c; a += s_rows[i]; c += s_lm[i]; }
        D.counts[0] = a; D.counts[1] = c;
    }
    __syncthreads();
    for (int b = wave; b < nb; b += 4) {
        const int rows = s_rows[b];
        if (rows == 0) continue;
        const int slot = D.req_list[b / D.max_br], k = b % D.max_br;
        const bb_branch_state& B = D.br[slot * D.max_br + k];
        const int start = B.start, end = B.end;
        const int gbr = slot * D.max_br + k, own = slot * D.phys_per_req + k;
        const int* Xr = D.X + (size_t)gbr * D.lpad;
        if (lane == 0) { D.seg_off[gbr] = s_off[b]; D.seg_rows[gbr] = rows; }
        int c = s_lmoff[b];                          // LM rows keep the order of the positions
        for (int i0 = start; i0 < end; i0 += 64) {
            const int i = i0 + lane;
            const bool in = i < end;
            const int tok = in ? Xr[i] : 0;
            const bool masked = in && tok == D.mask_id;
            const unsigned long long bal = __ballot(masked);
            if (in) {
                const int r = s_off[b] + (i - start);
                D.row_tok[r] = tok; D.row_pos[r] = i; D.row_gbr[r] = gbr; D.row_phys[r] = own;
                if (masked) D.lm_row[c + __popcll(bal & ((1ull << lane) - 1))] = r;
            }
            c += __popcll(bal);
        }
        // pages under the window that the branch does not own yet: queue a copy-on-write and re-point
        for (int p = start / BB_PAGE + lane; p <= (end - 1) / BB_PAGE; p += 64) {
            int* e = &D.table[(size_t)gbr * D.n_pages + p];
            if (*e != own) {
                const int idx = atomicAdd(&D.counts[2], 1);
                D.copies[idx] = PageCopy{*e, own, p, 0};
                *e = own;
            }
        }
    }
    if (t < n_req) {            // a request that has already finished contributes no rows and counts no forward
        ReqHeader& H = D.hdr[D.req_list[t]];
        if (!H.finished) { H.since_refresh += 1; H.nfe_block += 1; }
    }
}

void launch_pack_step(const Dev& D, int n_req, hipStream_t s) { pack_step_kernel<<<1, 256, 0, s>>>(D, n_req); }

// Full-sequence forwards of the listed requests, packed into one row list.  mode BB_INIT: the common row of each
// request (all its branches are still identical), written to the request's shared physical row that every branch's
// page table then points to; logits for its G generation positions.  mode BB_PERIODIC: all L rows of every
// unfinished branch, each into its own physical row.
__global__ __launch_bounds__(256) void pack_refresh_kernel(Dev D, int n_req, int mode) {
    __shared__ int s_off[256 + 1], s_lm[256 + 1];       // first packed row of each (listed request, branch); first LM row of each request
    const int nb_all = D.max_req * D.max_br, t = threadIdx.x;
    for (int i = t; i < nb_all; i += 256) D.seg_rows[i] = 0;
    if (t == 0) {
        int a = 0, lm = 0;
        for (int i = 0; i < n_req; ++i) {
            const int slot = D.req_list[i];
            ReqHeader& H = D.hdr[slot];
            s_lm[i] = lm;
            for (int k = 0; k < D.max_br; ++k) {
                s_off[i * D.max_br + k] = a;
                if (mode == BB_INIT) { if (k == 0) a += H.L; }
                else if (k < H.N && !D.br[slot * D.max_br + k].done) a += H.L;
            }
            if (mode == BB_INIT) {
                lm += H.G;
                H.nfe_init += 1; H.since_refresh = 0; H.refresh_due = 0; H.initialised = 1;
                for (int k = 0; k < BB_MAX_BRANCHES; ++k) H.pending[k] = k < H.N;
            } else {
                H.nfe_refresh += 1; H.since_refresh = 0; H.refresh_due = 0;
            }
        }
        s_off[n_req * D.max_br] = a;
        D.counts[0] = a; D.counts[1] = lm; D.counts[2] = 0;
    }
    __syncthreads();
    for (int i = 0; i < n_req; ++i) {
        const int slot = D.req_list[i];
        const ReqHeader& H = D.hdr[slot];
        const int L = H.L, N = H.N;
        if (mode == BB_INIT) {
            const int gbr = slot * D.max_br, shared_row = slot * D.phys_per_req + D.max_br, r0 = s_off[i * D.max_br];
            const int* Xr = D.X + (size_t)gbr * D.lpad;
            for (int j = t; j < L; j += 256) {
                D.row_tok[r0 + j] = Xr[j]; D.row_pos[r0 + j] = j; D.row_gbr[r0 + j] = gbr; D.row_phys[r0 + j] = shared_row;
            }
            for (int j = t; j < H.G; j += 256) D.lm_row[s_lm[i] + j] = r0 + H.L_p + j;
            for (int j = t; j < N * D.n_pages; j += 256)
                D.table[(size_t)(gbr + j / D.n_pages) * D.n_pages + j % D.n_pages] = shared_row;
            if (t == 0) { D.seg_off[gbr] = r0; D.seg_rows[gbr] = L; }
            continue;
        }
        for (int k = 0; k < N; ++k) {
            const int r0 = s_off[i * D.max_br + k];
            if (s_off[i * D.max_br + k + 1] == r0) continue;
            const int gbr = slot * D.max_br + k, own = slot * D.phys_per_req + k;
            const int* Xr = D.X + (size_t)gbr * D.lpad;
            for (int j = t; j < L; j += 256) {
                D.row_tok[r0 + j] = Xr[j]; D.row_pos[r0 + j] = j; D.row_gbr[r0 + j] = gbr; D.row_phys[r0 + j] = own;
            }
            for (int pg = t; pg < D.n_pages; pg += 256) D.table[(size_t)gbr * D.n_pages + pg] = own;
            if (t == 0) { D.seg_off[gbr] = r0; D.seg_rows[gbr] = L; }
        }
    }
}

void launch_pack_refresh(const Dev& D, int n_req, int mode, hipStream_t s) {
    pack_refresh_kernel<<<1, 256, 0, s>>>(D, n_req, mode);
}

// ---- page copies (copy-on-write before a block step, row copies after a sync) ------------------
// A page of one cache row is one contiguous run of hkv blocks per layer, for K and for V.
// Work item = (list entry, layer, eighth of that run); a fixed grid strides over the items.
__global__ __launch_bounds__(256) void page_copy_kernel(Dev D) {
    const int n = D.counts[2];
    const int items = n * D.n_layers * 8;
    const int u4s = D.hkv * BB_PAGE * 2 * D.hd / 8 / 8;      // 16-byte pieces per item
    for (int it = blockIdx.x; it < items; it += gridDim.x) {
        const int e = it / (D.n_layers * 8), layer = (it / 8) % D.n_layers, part = it % 8;
        const PageCopy pc = D.copies[e];
        const size_t so = kv_block_off(D, layer, pc.src, pc.page, 0), dof = kv_block_off(D, layer, pc.dst, pc.page, 0);
        const u32x4* ks = reinterpret_cast<const u32x4*>(D.Kc + so) + (size_t)part * u4s;
        const u32x4* vs = reinterpret_cast<const u32x4*>(D.Vt + so) + (size_t)part * u4s;
        u32x4* kd = reinterpret_cast<u32x4*>(D.Kc + dof) + (size_t)part * u4s;
        u32x4* vd = reinterpret_cast<u32x4*>(D.Vt + dof) + (size_t)part * u4s;
        for (int i = threadIdx.x; i < u4s; i += 256) { kd[i] = ks[i]; vd[i] = vs[i]; }
    }
}

void launch_page_copies(const Dev& D, hipStream_t s) { page_copy_kernel<<<1024, 256, 0, s>>>(D); }


// ---- commit / merge / sync ----------------------------------------------------------------------
struct CommitShared {
    int si[4]; float sf[4];
    int decoded[BB_MAX_BRANCHES], order[BB_MAX_BRANCHES], compat[BB_MAX_BRANCHES];
    int n_order, lead, istar, merged, thr, fb, go;
    int win, win_dec, win_eos;
};

static __device__ int count_decoded(const Dev& D, const int* Xr, int L_p, int L, int* sh) {
    int c = 0;
    for (int i = L_p + threadIdx.x; i < L; i += 256) c += Xr[i] != D.mask_id;
    return wg_sum_i(c, sh);
}

// AdvanceBlock: slide the window over blocks that hold no mask; past the end -> done.
static __device__ void advance(const Dev& D, bb_branch_state* B, const int* Xr, int L, int* sh) {
    while (true) {
        __syncthreads();
        if (B->done) break;
        const int start = B->start, end = B->end;
        int c = 0;
        for (int i = start + threadIdx.x; i < end; i += 256) c += Xr[i] == D.mask_id;
        c = wg_sum_i(c, sh);
        if (c > 0) break;
        if (threadIdx.x == 0) {
            B->start = end; B->end = min(end + B->block, L);
            if (B->start >= L) { B->done = 1; B->start = B->end = L; }
        }
    }
    __syncthreads();
}

// P_d(i, v) = exp(hf . W_v - lse) with the hidden vector the destination stored for position i;
// one wave, lanes stride over the model dimension.  W is the LM head in tiled fragment order.
static __device__ float prob_of(const Dev& D, const u32x4* lm, const float* hf, float lse, int v) {
    const int lane = threadIdx.x & 63, k8s = D.d >> 3;
    float acc = 0.f;
    for (int k8 = lane; k8 < k8s; k8 += 64) {
        const u32x4 w = lm[tileW_u4(v, k8, k8s >> 1)];
        const uint16_t* wb = reinterpret_cast<const uint16_t*>(&w);
        const float* x = hf + k8 * 8;
#pragma unroll
        for (int q = 0; q < 8; ++q) acc += x[q] * bf16_to_f32(wb[q]);
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    return expf(acc - lse);
}

// prob_of by one thread, with the wave's order of additions (64 strided partial sums, then the pairwise tree as lane 0
// sees it): the same bits.  Only for a lookup that finds no row (see merge_prob).
static __device__ float prob_of_serial(const Dev& D, const u32x4* lm, const float* hf, float lse, int v) {
    const int k8s = D.d >> 3;
    float part[64];
    for (int lane = 0; lane < 64; ++lane) {
        float acc = 0.f;
        for (int k8 = lane; k8 < k8s; k8 += 64) {
            const u32x4 w = lm[tileW_u4(v, k8, k8s >> 1)];
            const uint16_t* wb = reinterpret_cast<const uint16_t*>(&w);
            const float* x = hf + k8 * 8;
#pragma unroll
            for (int q = 0; q < 8; ++q) acc += x[q] * bf16_to_f32(wb[q]);
        }
        part[lane] = acc;
    }
    for (int o = 32; o > 0; o >>= 1)
        for (int lane = 0; lane < o; ++lane) part[lane] += part[lane + o];
    return expf(part[0] - lse);
}

// MergeSync asks for P_d(i, v) only where destination row d holds a mask at i and v is the token some other row
// holds there.  Rows change during MergeSync only by taking such tokens, and a destination is written only in its
// own turn, so every probability the sequential pass can ask for is P_d(i, token of row s at i) for the rows as they
// stand when MergeSync starts.  This kernel computes them all at once, one wave per (d, s, i) with d masked and s
// not (grid = 16 positions x ordered pair (d, s) x listed request), and the diagonal pairs keep the rows' tokens:
// the pass then looks a probability up by its token.  Same dot product as before, so the same bits.
__global__ __launch_bounds__(256) void merge_probs_kernel(Dev D, const u32x4* __restrict__ lm) {
    if (D.commit_skip[blockIdx.z]) return;
    const int slot = D.req_list[blockIdx.z];
    const ReqHeader& H = D.hdr[slot];
    const int d = blockIdx.y / D.max_br, s = blockIdx.y % D.max_br;
    if (d >= H.N || s >= H.N) return;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, L_p = H.L_p, G = H.L - H.L_p;
    const int* Xd = D.X + ((size_t)slot * D.max_br + d) * D.lpad;
    const int* Xs = D.X + ((size_t)slot * D.max_br + s) * D.lpad;
    for (int q = 0; q < 4; ++q) {
        const int j = blockIdx.x * 16 + wave * 4 + q;
        if (j >= G) break;
        if (s == d) {
            if (lane == 0) D.merge_x0[((size_t)slot * D.max_br + d) * D.gmax + j] = Xd[L_p + j];
            continue;
        }
        const int v = Xs[L_p + j];
        if (Xd[L_p + j] != D.mask_id || v == D.mask_id) continue;
        const size_t mi = ((size_t)slot * D.max_br + d) * D.gmax + j;
        const float p = prob_of(D, lm, D.map_hf + mi * D.d, D.map_lse[mi], v);
        if (lane == 0) D.merge_p[(((size_t)slot * D.max_br + d) * D.max_br + s) * D.gmax + j] = p;
    }
}

// P_d(i, v), j = i - L_p, from the table of merge_probs_kernel: row s held v at the start unless it took it from
// another row since; then that row (or the one it took it from) held it.  Computed directly if no row did.
static __device__ float merge_prob(const Dev& D, const u32x4* lm, int slot, int N, int d, int s, int j, int v) {
    const int* x0 = D.merge_x0 + (size_t)slot * D.max_br * D.gmax + j;
    const float* T = D.merge_p + ((size_t)slot * D.max_br + d) * D.max_br * D.gmax + j;
    if (x0[(size_t)s * D.gmax] == v) return T[(size_t)s * D.gmax];
    for (int q = 0; q < N; ++q)
        if (q != d && x0[(size_t)q * D.gmax] == v) return T[(size_t)q * D.gmax];
    const size_t mi = ((size_t)slot * D.max_br + d) * D.gmax + j;
    return prob_of_serial(D, lm, D.map_hf + mi * D.d, D.map_lse[mi], v);
}

// phase 0: DecodeCurrentBlock, CheckEOS, AdvanceCompletedBlocks; phase 1 (after merge_probs_kernel): MergeSync and
// the end of the step.
__global__ __launch_bounds__(256) void commit_merge_kernel(Dev D, const u32x4* __restrict__ lm, int phase) {
    __shared__ CommitShared S;
    const int slot = D.req_list[blockIdx.x], t = threadIdx.x;
    ReqHeader& H = D.hdr[slot];
    const int N = H.N, L_p = H.L_p, L = H.L, mask = D.mask_id;
    bb_branch_state* B = D.br + slot * D.max_br;
    int* X = D.X + (size_t)slot * D.max_br * D.lpad;
    const size_t map0 = (size_t)slot * D.max_br * D.gmax;

    if (phase == 0) {
    if (t == 0) { D.commit_skip[blockIdx.x] = 0; if (blockIdx.x == 0) D.counts[2] = 0; }    // (the copy list is filled in phase 1)
    // -- DecodeCurrentBlock (Eq. 1) for every branch that received logits ---------------------
    for (int k = 0; k < N; ++k) {
        __syncthreads();
        if (!H.pending[k] || B[k].done) continue;
        int* Xr = X + (size_t)k * D.lpad;
        const int start = B[k].start, end = B[k].end;
        const float* conf = D.map_conf + map0 + (size_t)k * D.gmax - L_p;
        const int* pred = D.map_pred + map0 + (size_t)k * D.gmax - L_p;
        // most confident masked position, lowest position on ties
        float bc = -1.f; int bi = 0x7fffffff, nm = 0; float sc = 0.f;
        for (int i = start + t; i < end; i += 256)
            if (Xr[i] == mask) { ++nm; sc += conf[i]; if (conf[i] > bc) { bc = conf[i]; bi = i; } }
        for (int o = 32; o > 0; o >>= 1) {
            const float oc = __shfl_xor(bc, o, 64); const int oi = __shfl_xor(bi, o, 64);
            if (oc > bc || (oc == bc && oi < bi)) { bc = oc; bi = oi; }
        }
        __shared__ float w_c[4]; __shared__ int w_i[4];
        if ((t & 63) == 0) { w_c[t >> 6] = bc; w_i[t >> 6] = bi; }
        nm = wg_sum_i(nm, S.si);
        sc = wg_sum_f(sc, S.sf);
        if (t == 0) {
            float c = w_c[0]; int ii = w_i[0];
            for (int w = 1; w < 4; ++w) if (w_c[w] > c || (w_c[w] == c && w_i[w] < ii)) { c = w_c[w]; ii = w_i[w]; }
            S.istar = ii; S.thr = 0; S.fb = 0;
        }
        __syncthreads();
        if (nm == 0) continue;
        for (int i = start + t; i < end; i += 256)
            if (Xr[i] == mask) {
                const bool thr = conf[i] >= D.tau_dec;
                if (thr || i == S.istar) { Xr[i] = pred[i]; atomicAdd(thr ? &S.thr : &S.fb, 1); }
            }
        __syncthreads();
        if (t == 0) {
            B[k].committed_threshold += S.thr; B[k].committed_fallback += S.fb;
            B[k].mean_conf = sc / (float)nm;
        }
    }
    // -- CheckEOS (Alg. 1) on the branches that were just decoded: the branch's EOS is the first generation
    //    position holding the EOS token, and it is EOS-ready when nothing before that is masked.  A ready
    //    branch ends the request (most tokens decoded wins, lowest index on ties) before advance / MergeSync.
    //    Alg. 1 has CheckEOS in the body of its while loop only: the commit that follows the initial full
    //    forward (no block forward has run yet) skips it.
    if (D.eos_id >= 0 && H.nfe_block > 0) {
        __syncthreads();
        if (t == 0) S.win = -1;
        for (int k = 0; k < N; ++k) {
            __syncthreads();
            if (!H.pending[k] || B[k].done) continue;
            const int* Xr = X + (size_t)k * D.lpad;
            int e = 0x7fffffff, fm = 0x7fffffff;
            for (int i = L_p + t; i < L; i += 256) {
                if (Xr[i] == D.eos_id) e = min(e, i);
                if (Xr[i] == mask) fm = min(fm, i);
            }
            e = wg_min_i(e, S.si);
            fm = wg_min_i(fm, S.si);
            const int c = count_decoded(D, Xr, L_p, L, S.si);
            if (t == 0 && e != 0x7fffffff && fm > e && (S.win < 0 || c > S.win_dec)) { S.win = k; S.win_dec = c; S.win_eos = e; }
        }
        __syncthreads();
        if (S.win >= 0) {
            for (int k = 0; k < N; ++k) {
                const int c = count_decoded(D, X + (size_t)k * D.lpad, L_p, L, S.si);
                if (t == 0) { B[k].tokens_decoded = c; B[k].done = 1; B[k].start = B[k].end = L; }
            }
            if (t < BB_MAX_BRANCHES) H.pending[t] = 0;
            if (t == 0) {
                H.finished = 2; H.winner = S.win; H.eos_pos = S.win_eos; H.all_done = 1; H.refresh_due = 0; D.req_flags[blockIdx.x] = 1;
                D.commit_skip[blockIdx.x] = 1;
            }
            return;
        }
    }
    __syncthreads();
    if (t < BB_MAX_BRANCHES) H.pending[t] = 0;
    // -- AdvanceCompletedBlocks ----------------------------------------------------------------
    for (int k = 0; k < N; ++k) advance(D, &B[k], X + (size_t)k * D.lpad, L, S.si);
    return;
    }
    if (D.commit_skip[blockIdx.x]) return;
    // -- MergeSync (Alg. 2) ---------------------------------------------------------------------
    for (int k = 0; k < N; ++k) {
        const int c = count_decoded(D, X + (size_t)k * D.lpad, L_p, L, S.si);
        if (t == 0) { S.decoded[k] = c; B[k].synced_from = -1; }
    }
    __syncthreads();
    if (t == 0) {
        int lead = 0;
        for (int k = 1; k < N; ++k) {
            bool better;
            if (D.leader_rule == 0)
                better = S.decoded[k] > S.decoded[lead] ||
                         (S.decoded[k] == S.decoded[lead] && B[k].mean_conf > B[lead].mean_conf);
            else
                better = B[k].mean_conf > B[lead].mean_conf;
            if (better) lead = k;
        }
        S.lead = lead;
        S.go = S.decoded[lead] > 0;
        // active branches, most decoded first, index breaks ties (stable insertion sort)
        int n = 0;
        for (int k = 0; k < N; ++k) if (!B[k].done) {
            int p = n++;
            while (p > 0 && S.decoded[S.order[p - 1]] < S.decoded[k]) { S.order[p] = S.order[p - 1]; --p; }
            S.order[p] = k;
        }
        S.n_order = n;
    }
    __syncthreads();
    if (S.go) {
        const int lead = S.lead, n_order = S.n_order;
        for (int oi = 0; oi < n_order; ++oi) {
            const int d = S.order[oi];
            __syncthreads();
            if (B[d].done) continue;
            int* Xd = X + (size_t)d * D.lpad;
            // CompatibleSources, evaluated once for this destination: conflicts with every source counted in one pass
            // (conflicts are rare, so the shared counters are rarely touched; prompt rows are equal)
            if (t < BB_MAX_BRANCHES) S.compat[t] = 0;
            if (t == 0) S.merged = 0;
            __syncthreads();
            for (int i = L_p + t; i < L; i += 256) {
                const int xd = Xd[i];
                if (xd == mask) continue;
                for (int oj = 0; oj < n_order; ++oj) {
                    const int s = S.order[oj];
                    if (s == d) continue;
                    const int xs = X[(size_t)s * D.lpad + i];
                    if (xs != mask && xs != xd) atomicAdd(&S.compat[s], 1);
                }
            }
            __syncthreads();
            // (until the next destination S.compat[s] holds the number of conflicts: compatible = none, and not d itself)
            int lo = L, hi = 0;
            for (int oj = 0; oj < n_order; ++oj) {
                const int s = S.order[oj];
                if (s != d && S.compat[s] == 0) { lo = min(lo, B[s].start); hi = max(hi, B[s].end); }
            }
            // positions of the union of the sources' windows, one thread per position
            for (int i = lo + t; i < hi; i += 256) {
                if (Xd[i] != mask) continue;
                float best_p = -1.f; int best_v = -1;
                for (int oj = 0; oj < n_order; ++oj) {
                    const int s = S.order[oj];
                    if (s == d || S.compat[s] != 0 || i < B[s].start || i >= B[s].end) continue;   // in the union at all?
                    best_v = -2; break;
                }
                if (best_v != -2) continue;
                best_v = -1;
                for (int oj = 0; oj < n_order; ++oj) {
                    const int s = S.order[oj];
                    if (s == d || S.compat[s] != 0) continue;
                    const int v = X[(size_t)s * D.lpad + i];
                    if (v == mask) continue;
                    const float p = merge_prob(D, lm, slot, N, d, s, i - L_p, v);
                    if (p > best_p) { best_p = p; best_v = v; }      // strict: earliest source keeps a tie
                }
                if (best_v >= 0 && best_p > D.tau_merge) { Xd[i] = best_v; atomicAdd(&S.merged, 1); }
            }
            __syncthreads();
            if (t == 0) B[d].tokens_merged += S.merged;
            advance(D, &B[d], Xd, L, S.si);
            const int c = count_decoded(D, Xd, L_p, L, S.si);
            if (t == 0) S.decoded[d] = c;
            __syncthreads();
        }
        // hard synchronisation: copy the leader into branches that lag by more than tau_sync
        for (int d = 0; d < N; ++d) {
            __syncthreads();
            if (B[d].done || d == lead || S.decoded[lead] - S.decoded[d] <= D.tau_sync) continue;
            int* Xd = X + (size_t)d * D.lpad; const int* Xl = X + (size_t)lead * D.lpad;
            for (int i = t; i < L; i += 256) Xd[i] = Xl[i];
            const size_t md = map0 + (size_t)d * D.gmax, ml = map0 + (size_t)lead * D.gmax;
            for (int j = t; j < H.G; j += 256) {
                D.map_lse[md + j] = D.map_lse[ml + j]; D.map_conf[md + j] = D.map_conf[ml + j];
                D.map_pred[md + j] = D.map_pred[ml + j];
            }
            const float4* hs = reinterpret_cast<const float4*>(D.map_hf + ml * D.d);
            float4* hdst = reinterpret_cast<float4*>(D.map_hf + md * D.d);
            for (size_t j = t; j < (size_t)H.G * D.d / 4; j += 256) hdst[j] = hs[j];
            const int gd = slot * D.max_br + d, gl = slot * D.max_br + lead;
            const int own = slot * D.phys_per_req + d, shared_row = slot * D.phys_per_req + D.max_br;
            for (int p = t; p < (L + BB_PAGE - 1) / BB_PAGE; p += 256) {
                const int src = D.table[(size_t)gl * D.n_pages + p];
                if (src == shared_row) D.table[(size_t)gd * D.n_pages + p] = shared_row;
                else {
                    D.table[(size_t)gd * D.n_pages + p] = own;
                    D.copies[atomicAdd(&D.counts[2], 1)] = PageCopy{src, own, p, 0};
                }
            }
            __syncthreads();
            // RealignBlockWindow: block of the branch's own grid that holds the first mask
            int f = 0x7fffffff;
            for (int i = L_p + t; i < L; i += 256) if (Xd[i] == mask) f = min(f, i);
            f = wg_min_i(f, S.si);
            if (t == 0) {
                B[d].mean_conf = B[lead].mean_conf; B[d].synced_from = lead;
                if (f == 0x7fffffff) { B[d].done = 1; B[d].start = B[d].end = L; }
                else {
                    B[d].start = L_p + (f - L_p) / B[d].block * B[d].block;
                    B[d].end = min(B[d].start + B[d].block, L);
                    B[d].done = 0;
                }
                S.decoded[d] = S.decoded[lead];
            }
        }
    }
    __syncthreads();
    if (t == 0) {
        int all = 1;
        for (int k = 0; k < N; ++k) { B[k].tokens_decoded = S.decoded[k]; all &= B[k].done; }
        H.all_done = all;
        H.refresh_due = H.since_refresh >= D.refresh_interval && !all;
        S.win = -1;
        if (all && !H.finished) {       // final selection of Alg. 1: most progress, lowest index on ties
            int w = 0;
            for (int k = 1; k < N; ++k) if (S.decoded[k] > S.decoded[w]) w = k;
            S.win = w;
        }
    }
    __syncthreads();
    if (S.win >= 0) {
        const int* Xw = X + (size_t)S.win * D.lpad;
        int e = 0x7fffffff;
        if (D.eos_id >= 0)
            for (int i = L_p + t; i < L; i += 256) if (Xw[i] == D.eos_id) e = min(e, i);
        e = wg_min_i(e, S.si);
        if (t == 0) { H.finished = 1; H.winner = S.win; H.eos_pos = e == 0x7fffffff ? -1 : e; }
    }
    // one word per listed request for a driver loop: finished, refresh due, forwards left until a refresh falls due
    if (t == 0) {
        const int fin = H.finished != 0 || S.win >= 0;
        const int left = max(0, D.refresh_interval - H.since_refresh);
        D.req_flags[blockIdx.x] = fin | (H.refresh_due ? 2 : 0) | (left << 8);
    }
}

void launch_commit_merge(const Dev& D, int n_req, const uint16_t* lm_head, hipStream_t s) {
    const u32x4* lm = reinterpret_cast<const u32x4*>(lm_head);
    commit_merge_kernel<<<n_req, 256, 0, s>>>(D, lm, 0);
    merge_probs_kernel<<<dim3((D.gmax + 15) / 16, D.max_br * D.max_br, n_req), 256, 0, s>>>(D, lm);
    commit_merge_kernel<<<n_req, 256, 0, s>>>(D, lm, 1);
    page_copy_kernel<<<1024, 256, 0, s>>>(D);
}

// ---- inspection -------------------------------------------------------------------------------
__global__ void read_kv_kernel(Dev D, int gbr, int layer, float* __restrict__ K, float* __restrict__ V, int L) {
    const int krow = D.hkv * D.hd, hd = D.hd;
    const size_t n = (size_t)L * krow;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const int pos = (int)(i / krow), e = (int)(i % krow), head = e / hd, dd = e % hd;
        const int phys = D.table[(size_t)gbr * D.n_pages + pos / BB_PAGE], tt = pos % BB_PAGE;
        const size_t blk = kv_block_off(D, layer, phys, pos / BB_PAGE, head);
        K[i] = (float)D.Kc[blk + k_slot(tt, dd, 0, hd)] + (float)D.Kc[blk + k_slot(tt, dd, 1, hd)];
        V[i] = (float)D.Vt[blk + v_slot(tt, dd, 0)] + (float)D.Vt[blk + v_slot(tt, dd, 1)];
    }
}

void launch_read_kv(const Dev& D, int slot, int branch, int layer, float* K, float* V, int L, hipStream_t s) {
    read_kv_kernel<<<1024, 256, 0, s>>>(D, slot * D.max_br + branch, layer, K, V, L);
}

// Queue a copy of every page of a branch row that still lives in another physical row (all layers) and re-point the
// page table at the branch's own row: afterwards a write to this row changes no other branch's view.
__global__ void own_all_pages_kernel(Dev D, int gbr, int own, int n_pages_used) {
    if (threadIdx.x == 0) D.counts[2] = 0;
    __syncthreads();
    for (int p = threadIdx.x; p < n_pages_used; p += blockDim.x) {
        int* e = &D.table[(size_t)gbr * D.n_pages + p];
        if (*e != own) {
            const int idx = atomicAdd(&D.counts[2], 1);
            D.copies[idx] = PageCopy{*e, own, p, 0};
            *e = own;
        }
    }
}

// Overwrite one layer of a (private) cache row with caller values, each as two fp16 terms.
__global__ void write_kv_kernel(Dev D, int gbr, int layer, const float* __restrict__ K, const float* __restrict__ V, int L) {
    const int krow = D.hkv * D.hd, hd = D.hd;
    const size_t n = (size_t)L * krow;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const int pos = (int)(i / krow), e = (int)(i % krow), head = e / hd, dd = e % hd;
        const int phys = D.table[(size_t)gbr * D.n_pages + pos / BB_PAGE], tt = pos % BB_PAGE;
        const size_t blk = kv_block_off(D, layer, phys, pos / BB_PAGE, head);
        const float k = K[i], v = V[i];
        const half_t kh = (half_t)k, vh = (half_t)v;
        D.Kc[blk + k_slot(tt, dd, 0, hd)] = kh; D.Kc[blk + k_slot(tt, dd, 1, hd)] = (half_t)(k - (float)kh);
        D.Vt[blk + v_slot(tt, dd, 0)] = vh;     D.Vt[blk + v_slot(tt, dd, 1)] = (half_t)(v - (float)vh);
    }
}

void launch_write_kv(const Dev& D, int slot, int branch, int layer, const float* K, const float* V, int L, hipStream_t s) {
    const int gbr = slot * D.max_br + branch, own = slot * D.phys_per_req + branch;
    own_all_pages_kernel<<<1, 256, 0, s>>>(D, gbr, own, (L + BB_PAGE - 1) / BB_PAGE);
    page_copy_kernel<<<1024, 256, 0, s>>>(D);
    write_kv_kernel<<<1024, 256, 0, s>>>(D, gbr, layer, K, V, L);
}

// ---- KV-consistency diagnostics (App. A.2) ---------------------------------------------------------
// Squared distance between two cache rows, per (layer, page): out[(layer * n_pages + page)] = sum over the
// page's K and V blocks of ((a_hi + a_lo) - (b_hi + b_lo))^2 in fp64.  A row is either a branch's view of
// the cache (page table -> physical row) or row `b_row` of a snapshot buffer with the cache's block layout
// ([layer][row][page][kv head]).  Both sides use the same fragment order, so elements pair up by offset.
__global__ __launch_bounds__(256) void kv_sqdist_kernel(Dev D, int gbr_a, int gbr_b, const half_t* __restrict__ snapK,
                                                        const half_t* __restrict__ snapV, int snap_rows, int b_row,
                                                        int n_pages_used, double* __restrict__ out) {
    __shared__ double sh[4];
    const int layer = blockIdx.y, page = blockIdx.x;
    const int pa = D.table[(size_t)gbr_a * D.n_pages + page];
    const size_t blk = (size_t)D.hkv * BB_PAGE * 2 * D.hd;              // halfs per page of one row
    const half_t *ka = D.Kc + kv_block_off(D, layer, pa, page, 0), *va = D.Vt + kv_block_off(D, layer, pa, page, 0);
    const half_t *kb, *vb;
    bool same = false;
    if (snapK) {
        const size_t off = (((size_t)layer * snap_rows + b_row) * n_pages_used + page) * blk;
        kb = snapK + off; vb = snapV + off;
    } else {
        const int pb = D.table[(size_t)gbr_b * D.n_pages + page];
        same = pb == pa;
        kb = D.Kc + kv_block_off(D, layer, pb, page, 0); vb = D.Vt + kv_block_off(D, layer, pb, page, 0);
    }
    double acc = 0.0;
    if (!same) {
        // fragment pair f: hi term at 16-byte piece (2 f) * 64 + lane, lo term 64 pieces further
        const int n_frag = (int)(blk / 8 / 128);
        for (int it = threadIdx.x; it < n_frag * 64; it += 256) {
            const size_t q = (size_t)(it / 64) * 128 + it % 64;
            for (int op = 0; op < 2; ++op) {
                const half_t* a = (op ? va : ka) + q * 8; const half_t* b = (op ? vb : kb) + q * 8;
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const double x = ((double)(float)a[j] + (double)(float)a[j + 512]) - ((double)(float)b[j] + (double)(float)b[j + 512]);
                    acc += x * x;
                }
            }
        }
    }
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) out[(size_t)layer * n_pages_used + page] = sh[0] + sh[1] + sh[2] + sh[3];
}

// Copy a branch's view of the cache into row `row` of a snapshot buffer.
__global__ __launch_bounds__(256) void kv_snapshot_kernel(Dev D, int gbr, half_t* __restrict__ snapK, half_t* __restrict__ snapV,
                                                          int snap_rows, int row, int n_pages_used) {
    const int layer = blockIdx.y, page = blockIdx.x;
    const int phys = D.table[(size_t)gbr * D.n_pages + page];
    const size_t blk = (size_t)D.hkv * BB_PAGE * 2 * D.hd, off = (((size_t)layer * snap_rows + row) * n_pages_used + page) * blk;
    const u32x4* ks = reinterpret_cast<const u32x4*>(D.Kc + kv_block_off(D, layer, phys, page, 0));
    const u32x4* vs = reinterpret_cast<const u32x4*>(D.Vt + kv_block_off(D, layer, phys, page, 0));
    u32x4* kd = reinterpret_cast<u32x4*>(snapK + off); u32x4* vd = reinterpret_cast<u32x4*>(snapV + off);
    for (int i = threadIdx.x; i < (int)(blk / 8); i += 256) { kd[i] = ks[i]; vd[i] = vs[i]; }
}

void launch_kv_sqdist(const Dev& D, int gbr_a, int gbr_b, const half_t* snapK, const half_t* snapV, int snap_rows, int b_row,
                      int n_pages_used, double* out, hipStream_t s) {
    kv_sqdist_kernel<<<dim3(n_pages_used, D.n_layers), 256, 0, s>>>(D, gbr_a, gbr_b, snapK, snapV, snap_rows, b_row, n_pages_used, out);
}
void launch_kv_snapshot(const Dev& D, int gbr, half_t* snapK, half_t* snapV, int snap_rows, int row, int n_pages_used, hipStream_t s) {
    kv_snapshot_kernel<<<dim3(n_pages_used, D.n_layers), 256, 0, s>>>(D, gbr, snapK, snapV, snap_rows, row, n_pages_used);
}
